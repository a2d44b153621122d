// Host side of the round-aware prompt interface (Sec. 4.1) and the segment-based index that replaces
// fixed-size chunk hashing (Sec. 5): prompts are split at a reserved separator token, every block is
// indexed by a hash of its own content (verified by comparison, so a collision cannot merge two
// different blocks), and the prompts that hold the same set of shared blocks form one session whose
// layout is returned in the form tdk_round_create takes (tdk_segment lists).  No device code.
#include <algorithm>
#include <cstring>
#include <map>
#include <memory>
#include <new>
#include <string>
#include <unordered_map>
#include <vector>

#include "tdk.h"

namespace {

struct Block {
  int32_t pos;       // position of its first token in the prompt
  int32_t len;
  int32_t content;   // id of its content (equal ids = equal token sequences)
};

// FNV-1a over the token ids, 64 bits
uint64_t hash_tokens(const int32_t* t, int32_t n) {
  uint64_t h = 1469598103934665603ull;
  for (int32_t i = 0; i < n; ++i) {
    uint32_t v = (uint32_t)t[i];
    for (int b = 0; b < 4; ++b) {
      h ^= (v >> (8 * b)) & 0xffu;
      h *= 1099511628211ull;
    }
  }
  return h ^ (uint64_t)n;
}

}  // namespace

struct tdk_prompt_plan {
  std::vector<int32_t> span;                         // per session
  std::vector<int32_t> session_of;                   // per prompt, -1 = single-request path
  std::vector<std::vector<tdk_segment>> segments;    // per prompt
};

extern "C" {

tdk_status tdk_prompt_plan_create(const tdk_prompt* prompts, int32_t n_prompts, int32_t separator,
                                  tdk_prompt_plan** out) {
  if (!out) return TDK_ERR_INVALID_ARG;
  *out = nullptr;
  if (n_prompts < 0 || (n_prompts && !prompts)) return TDK_ERR_INVALID_ARG;
  for (int32_t i = 0; i < n_prompts; ++i)
    if (prompts[i].n_tokens < 0 || (prompts[i].n_tokens && !prompts[i].tokens)) return TDK_ERR_INVALID_ARG;
  try {
    // 1. blocks of every prompt, contents numbered through the hash index
    struct Rep { const int32_t* tok; int32_t len; };
    std::vector<Rep> reps;                                       // one representative per content id
    std::unordered_map<uint64_t, std::vector<int32_t>> index;    // hash -> content ids with that hash
    std::vector<std::vector<Block>> blocks(n_prompts);
    for (int32_t i = 0; i < n_prompts; ++i) {
      const int32_t* t = prompts[i].tokens;
      const int32_t n = prompts[i].n_tokens;
      int32_t start = 0;
      for (int32_t p = 0; p <= n; ++p) {
        if (p < n && t[p] != separator) continue;
        const int32_t len = p - start;
        if (len > 0) {
          auto& bucket = index[hash_tokens(t + start, len)];
          int32_t id = -1;
          for (int32_t c : bucket)
            if (reps[c].len == len && std::memcmp(reps[c].tok, t + start, sizeof(int32_t) * (size_t)len) == 0) { id = c; break; }
          if (id < 0) {
            id = (int32_t)reps.size();
            reps.push_back({t + start, len});
            bucket.push_back(id);
          }
          blocks[i].push_back({start, len, id});
        }
        start = p + 1;
      }
    }
    // 2. a content is shared if at least two prompts hold it
    std::vector<int32_t> holders(reps.size(), 0), last(reps.size(), -1);
    for (int32_t i = 0; i < n_prompts; ++i)
      for (const Block& b : blocks[i])
        if (last[b.content] != i) { last[b.content] = i; ++holders[b.content]; }
    // 3. prompts grouped by the set of shared contents they hold
    std::map<std::vector<int32_t>, std::vector<int32_t>> members;
    for (int32_t i = 0; i < n_prompts; ++i) {
      std::vector<int32_t> key;
      for (const Block& b : blocks[i])
        if (holders[b.content] >= 2) key.push_back(b.content);
      std::sort(key.begin(), key.end());
      key.erase(std::unique(key.begin(), key.end()), key.end());
      if (!key.empty()) members[key].push_back(i);
    }
    std::vector<const std::vector<int32_t>*> groups;
    for (const auto& kv : members)
      if (kv.second.size() >= 2) groups.push_back(&kv.second);
    std::sort(groups.begin(), groups.end(), [](const std::vector<int32_t>* a, const std::vector<int32_t>* b) { return (*a)[0] < (*b)[0]; });
    // 4. master order = shared blocks in the order of the group's first prompt; segments of every member
    std::unique_ptr<tdk_prompt_plan> plan(new tdk_prompt_plan());   // freed if anything below throws
    plan->session_of.assign(n_prompts, -1);
    plan->segments.resize(n_prompts);
    std::vector<int32_t> src(reps.size(), -1);
    for (size_t s = 0; s < groups.size(); ++s) {
      const std::vector<int32_t>& m = *groups[s];
      std::vector<int32_t> order;
      int64_t at = 0;
      for (const Block& b : blocks[m[0]])
        if (holders[b.content] >= 2 && src[b.content] < 0) {
          src[b.content] = (int32_t)at;
          order.push_back(b.content);
          at += b.len;
        }
      if (at >= (int64_t)1 << 31) return TDK_ERR_UNSUPPORTED;
      plan->span.push_back((int32_t)at);
      for (int32_t i : m) {
        plan->session_of[i] = (int32_t)s;
        std::vector<int32_t> where(order.size(), -1);
        for (const Block& b : blocks[i]) {
          if (src[b.content] < 0) continue;
          const size_t k = std::find(order.begin(), order.end(), b.content) - order.begin();
          if (where[k] < 0) where[k] = b.pos;                    // the first occurrence counts
        }
        for (size_t k = 0; k < order.size(); ++k)
          plan->segments[i].push_back({src[order[k]], reps[order[k]].len, where[k], where[k]});
      }
      for (int32_t c : order) src[c] = -1;
    }
    *out = plan.release();
    return TDK_OK;
  } catch (const std::bad_alloc&) {
    return TDK_ERR_NOMEM;
  } catch (...) {
    return TDK_ERR_INVALID_ARG;
  }
}

void tdk_prompt_plan_destroy(tdk_prompt_plan* p) { delete p; }

int32_t tdk_prompt_plan_n_sessions(const tdk_prompt_plan* p) { return p ? (int32_t)p->span.size() : 0; }

int32_t tdk_prompt_plan_span(const tdk_prompt_plan* p, int32_t session) {
  return p && session >= 0 && session < (int32_t)p->span.size() ? p->span[session] : -1;
}

int32_t tdk_prompt_plan_session_of(const tdk_prompt_plan* p, int32_t prompt) {
  return p && prompt >= 0 && prompt < (int32_t)p->session_of.size() ? p->session_of[prompt] : -1;
}

int32_t tdk_prompt_plan_segments(const tdk_prompt_plan* p, int32_t prompt, const tdk_segment** out) {
  if (out) *out = nullptr;
  if (!p || prompt < 0 || prompt >= (int32_t)p->segments.size()) return -1;
  if (out && !p->segments[prompt].empty()) *out = p->segments[prompt].data();
  return (int32_t)p->segments[prompt].size();
}

}  // extern "C"
