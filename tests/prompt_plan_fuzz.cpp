// Host-only driver for the prompt plan (tdk_prompt_plan_*), built with AddressSanitizer and
// UndefinedBehaviorSanitizer by tests/test_host_sanitizers.py: seeded random prompt sets with the shapes
// that stress the splitter (empty prompts, no separators, only separators, repeated blocks, blocks shared by
// some prompts only), every result checked for the invariants the header states.  Exit code 0 = clean.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "tdk.h"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd() {                       // splitmix64, upper half
  uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return (uint32_t)((z ^ (z >> 31)) >> 32);
}

#define REQUIRE(c) do { if (!(c)) { std::fprintf(stderr, "case %d: requirement failed: %s (line %d)\n", cs, #c, __LINE__); return 1; } } while (0)

int main() {
  const int32_t SEP = -7;
  for (int cs = 0; cs < 400; ++cs) {
    const int n_prompts = (int)(rnd() % 9);
    // a pool of block contents; short alphabets make accidental equal blocks likely
    std::vector<std::vector<int32_t>> pool(1 + rnd() % 6);
    for (auto& b : pool) { b.resize(rnd() % 5); for (auto& t : b) t = (int32_t)(rnd() % 3); }
    std::vector<std::vector<int32_t>> toks(n_prompts);
    for (auto& t : toks) {
      const int n_blocks = (int)(rnd() % 7);
      for (int k = 0; k < n_blocks; ++k) {
        const uint32_t what = rnd() % 8;
        if (what == 0) { t.push_back(SEP); continue; }                       // empty block
        if (what == 1) { for (uint32_t j = rnd() % 4; j > 0; --j) t.push_back((int32_t)(rnd() % 1000) + 10); }   // private block
        else { const auto& b = pool[rnd() % pool.size()]; t.insert(t.end(), b.begin(), b.end()); }
        if (rnd() % 5) t.push_back(SEP);
      }
    }
    std::vector<tdk_prompt> prompts(n_prompts);
    for (int i = 0; i < n_prompts; ++i) { prompts[i].tokens = toks[i].empty() ? nullptr : toks[i].data(); prompts[i].n_tokens = (int32_t)toks[i].size(); }
    tdk_prompt_plan* plan = nullptr;
    const tdk_status st = tdk_prompt_plan_create(n_prompts ? prompts.data() : nullptr, n_prompts, SEP, &plan);
    REQUIRE(st == TDK_OK && plan != nullptr);
    const int32_t n_sessions = tdk_prompt_plan_n_sessions(plan);
    REQUIRE(n_sessions >= 0 && n_sessions <= n_prompts / 2 + 1);
    REQUIRE(tdk_prompt_plan_span(plan, -1) == -1 && tdk_prompt_plan_span(plan, n_sessions) == -1);
    REQUIRE(tdk_prompt_plan_session_of(plan, -1) == -1 && tdk_prompt_plan_session_of(plan, n_prompts) == -1);
    const tdk_segment* none = nullptr;
    REQUIRE(tdk_prompt_plan_segments(plan, n_prompts, &none) == -1);
    std::vector<int> members(n_sessions, 0);
    for (int i = 0; i < n_prompts; ++i) {
      const int32_t s = tdk_prompt_plan_session_of(plan, i);
      const tdk_segment* seg = nullptr;
      const int32_t n_seg = tdk_prompt_plan_segments(plan, i, &seg);
      REQUIRE(s >= -1 && s < n_sessions);
      if (s < 0) { REQUIRE(n_seg == 0); continue; }
      ++members[s];
      const int32_t span = tdk_prompt_plan_span(plan, s);
      REQUIRE(span > 0 && n_seg > 0 && seg != nullptr);
      // the segments tile the master span exactly once and every one lies inside the prompt, on equal tokens
      std::vector<char> covered((size_t)span, 0);
      for (int32_t k = 0; k < n_seg; ++k) {
        REQUIRE(seg[k].len > 0 && seg[k].src_tok >= 0 && (int64_t)seg[k].src_tok + seg[k].len <= span);
        REQUIRE(seg[k].dst_pos >= 0 && seg[k].dst_pos + seg[k].len <= (int64_t)toks[i].size());
        REQUIRE(seg[k].diff_pos == seg[k].dst_pos);
        for (int32_t j = 0; j < seg[k].len; ++j) {
          REQUIRE(!covered[(size_t)seg[k].src_tok + j]);
          covered[(size_t)seg[k].src_tok + j] = 1;
          REQUIRE(toks[i][(size_t)seg[k].dst_pos + j] != SEP);
        }
      }
      for (char c : covered) REQUIRE(c);
    }
    for (int s = 0; s < n_sessions; ++s) REQUIRE(members[s] >= 2);
    // members of one session hold equal tokens at equal master positions
    for (int s = 0; s < n_sessions; ++s) {
      std::vector<int32_t> master((size_t)tdk_prompt_plan_span(plan, s), INT32_MIN);
      for (int i = 0; i < n_prompts; ++i) {
        if (tdk_prompt_plan_session_of(plan, i) != s) continue;
        const tdk_segment* seg = nullptr;
        const int32_t n_seg = tdk_prompt_plan_segments(plan, i, &seg);
        for (int32_t k = 0; k < n_seg; ++k)
          for (int32_t j = 0; j < seg[k].len; ++j) {
            int32_t& m = master[(size_t)seg[k].src_tok + j];
            const int32_t t = toks[i][(size_t)seg[k].dst_pos + j];
            REQUIRE(m == INT32_MIN || m == t);
            m = t;
          }
      }
    }
    tdk_prompt_plan_destroy(plan);
  }
  // argument errors
  {
    const int cs = -1;
    tdk_prompt_plan* plan = nullptr;
    tdk_prompt bad = {nullptr, 3};
    REQUIRE(tdk_prompt_plan_create(&bad, 1, 0, &plan) == TDK_ERR_INVALID_ARG && plan == nullptr);
    REQUIRE(tdk_prompt_plan_create(nullptr, 2, 0, &plan) == TDK_ERR_INVALID_ARG);
    REQUIRE(tdk_prompt_plan_create(nullptr, 0, 0, nullptr) == TDK_ERR_INVALID_ARG);
    tdk_prompt_plan_destroy(nullptr);
  }
  std::printf("prompt plan: 400 random cases clean\n");
  return 0;
}
