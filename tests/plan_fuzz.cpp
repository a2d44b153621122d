// Host-only driver for the round planner (csrc/tdk_plan.cpp), built with AddressSanitizer and
// UndefinedBehaviorSanitizer by tests/test_host_sanitizers.py: seeded random rounds with the shapes that stress
// the index arithmetic (spans of 0 and 1 token, spans that end on and next to page borders, sessions without
// agents, per-agent block layouts cut at page borders and inside pages, three segments on one page), every plan
// checked against a recomputation of what its tables must hold.  Exit code 0 = clean.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "tdk_plan.h"

using namespace tdk;

static uint64_t rng_state = 0x2545F4914F6CDD1Dull;
static uint32_t rnd() {                       // splitmix64, upper half
  uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return (uint32_t)((z ^ (z >> 31)) >> 32);
}
static int64_t between(int64_t lo, int64_t hi) { return lo + (int64_t)(rnd() % (uint32_t)(hi - lo + 1)); }

#define REQUIRE(c) do { if (!(c)) { std::fprintf(stderr, "case %d: requirement failed: %s (line %d)\n", cs, #c, __LINE__); return 1; } } while (0)

struct HostAgent {
  int32_t session;
  int64_t pos0, diff_pos0;
  std::vector<int32_t> table;
  std::vector<tdk_segment> segs;
};

int main() {
  int refused_three = 0, planned = 0;
  for (int cs = 0; cs < 600; ++cs) {
    tdk_model model{};
    model.num_layers = 2; model.num_kv_heads = (int32_t)between(1, 8); model.head_dim = 128;
    model.page_tokens = rnd() % 2 ? 16 : 32; model.dtype = TDK_BF16;
    model.rope_style = rnd() % 2 ? TDK_ROPE_HALF : TDK_ROPE_INTERLEAVED;
    model.rope_theta = rnd() % 2 ? 1.0e6 : 5.0e5;
    const int T = model.page_tokens;
    const int n_sessions = (int)between(0, 4);
    std::vector<tdk_session> sessions(n_sessions);
    for (auto& s : sessions) {
      const int pick = (int)(rnd() % 7);
      const int32_t spans[6] = {0, 1, T - 1, T, T + 1, 3 * T};
      s.span_tokens = pick < 6 ? spans[pick] : (int32_t)between(1, 300);
      s.master_pos0 = rnd() % 3 ? 0 : between(0, 50);
    }
    const int n_agents = n_sessions ? (int)between(0, 10) : 0;
    std::vector<HostAgent> ha(n_agents);
    bool three_on_a_page = false;
    int32_t next_page = 1;
    for (auto& a : ha) {
      a.session = (int32_t)between(0, n_sessions - 1);
      const int32_t S = sessions[a.session].span_tokens;
      a.pos0 = rnd() % 4 == 0 ? between(0, 3) * T : between(0, 2000);
      a.diff_pos0 = rnd() % 2 ? a.pos0 : between(0, 2000);
      int64_t hi = a.pos0 + S;
      if (S > 0 && rnd() % 3 == 0) {
        // a layout of its own: cut the span (often at page borders), place the pieces in a shuffled order
        std::vector<int32_t> cuts{0, S};
        const int n_cuts = (int)between(0, 4);
        for (int k = 0; k < n_cuts; ++k) {
          int32_t c = rnd() % 2 ? (int32_t)(between(0, (S + T - 1) / T) * T) : (int32_t)between(0, S);
          if (c > 0 && c < S) cuts.push_back(c);
        }
        std::sort(cuts.begin(), cuts.end());
        cuts.erase(std::unique(cuts.begin(), cuts.end()), cuts.end());
        const int n_seg = (int)cuts.size() - 1;
        std::vector<int> place(n_seg);
        for (int k = 0; k < n_seg; ++k) place[k] = k;
        for (int k = n_seg - 1; k > 0; --k) std::swap(place[k], place[rnd() % (k + 1)]);
        std::vector<int64_t> dst(n_seg);
        int64_t cursor = a.pos0;
        for (int k = 0; k < n_seg; ++k) {
          const int q = place[k];
          cursor += rnd() % 3 == 0 ? between(0, 40) : 0;          // gaps between the pieces
          dst[q] = cursor;
          cursor += cuts[q + 1] - cuts[q];
        }
        hi = cursor;
        for (int q = 0; q < n_seg; ++q)
          a.segs.push_back({cuts[q], cuts[q + 1] - cuts[q], dst[q], rnd() % 2 ? dst[q] : between(0, 3000)});
        for (int32_t p = 0; p * T < S; ++p) {
          int met = 0;
          for (int q = 0; q < n_seg; ++q) met += cuts[q] < std::min<int32_t>(S, (p + 1) * T) && cuts[q + 1] > p * T;
          three_on_a_page |= met > 2;
        }
      }
      a.table.assign((size_t)((hi + T - 1) / T) + (rnd() % 2), 0);
      for (auto& e : a.table) e = next_page++;
      if (rnd() % 5 == 0) std::reverse(a.table.begin(), a.table.end());
    }
    std::vector<tdk_agent> agents(n_agents);
    for (int i = 0; i < n_agents; ++i) {
      agents[i].session = ha[i].session; agents[i].dst_pos0 = ha[i].pos0; agents[i].diff_pos0 = ha[i].diff_pos0;
      agents[i].block_table = ha[i].table.empty() ? nullptr : ha[i].table.data();
      agents[i].block_table_len = (int32_t)ha[i].table.size();
      agents[i].n_segments = (int32_t)ha[i].segs.size();
      agents[i].segments = ha[i].segs.empty() ? nullptr : ha[i].segs.data();
    }
    RoundPlan p;
    std::string err;
    const tdk_status st = plan_round(&model, n_sessions ? sessions.data() : nullptr, n_sessions,
                                     n_agents ? agents.data() : nullptr, n_agents, p, err);
    if (three_on_a_page) {
      REQUIRE(st == TDK_ERR_UNSUPPORTED && !err.empty());
      ++refused_three;
      continue;
    }
    REQUIRE(st == TDK_OK);
    ++planned;
    // sessions and the agent order
    REQUIRE((int)p.sess.size() == n_sessions && (int)p.agents.size() == n_agents && (int)p.order.size() == n_agents);
    int64_t row0 = 0, pages_sum = 0, tokens_sum = 0;
    for (int s = 0; s < n_sessions; ++s) {
      REQUIRE(p.sess[s].master_row0 == row0 && p.sess[s].span == sessions[s].span_tokens);
      REQUIRE(p.sess[s].pages == (sessions[s].span_tokens + T - 1) / T);
      row0 += sessions[s].span_tokens;
      int members = 0;
      for (int q = 0; q < p.sess[s].n_agents; ++q) {
        const int a = p.order[(size_t)p.sess[s].order_begin + q];
        REQUIRE(a >= 0 && a < n_agents && ha[a].session == s);
        REQUIRE(q == 0 || a > p.order[(size_t)p.sess[s].order_begin + q - 1]);
        ++members;
      }
      int expect = 0;
      for (const auto& a : ha) expect += a.session == s;
      REQUIRE(members == expect);
    }
    REQUIRE(p.total_master_rows == row0);
    bool any_seg = false;
    for (const auto& a : ha) any_seg |= !a.segs.empty();
    REQUIRE(p.any_segments == any_seg);
    int64_t max_page = -1;
    for (int i = 0; i < n_agents; ++i) {
      const AgentDev& ad = p.agents[i];
      const int32_t S = sessions[ha[i].session].span_tokens;
      REQUIRE(ad.session == ha[i].session && ad.flag_off == pages_sum && ad.score_off == tokens_sum);
      pages_sum += (S + T - 1) / T;
      tokens_sum += S;
      REQUIRE(ad.bt_off >= 0 && ad.bt_len >= 0 && (size_t)ad.bt_off + (size_t)ad.bt_len <= p.bt.size());
      // position of master token m in this agent's prompt
      auto pos_of = [&](int32_t m) -> int64_t {
        if (ha[i].segs.empty()) return ha[i].pos0 + m;
        for (const auto& sg : ha[i].segs) if (m >= sg.src_tok && m < sg.src_tok + sg.len) return sg.dst_pos + (m - sg.src_tok);
        return -1;
      };
      for (int32_t m = 0; m < S; ++m) {
        const int64_t pos = pos_of(m);
        REQUIRE(pos >= 0);
        const int64_t want = (int64_t)ha[i].table[(size_t)(pos / T)] * T + pos % T;
        max_page = std::max<int64_t>(max_page, ha[i].table[(size_t)(pos / T)]);
        const int64_t lp = pos / T - ad.lp_first;
        REQUIRE(lp >= 0 && lp < ad.bt_len);
        REQUIRE((int64_t)p.bt[(size_t)ad.bt_off + (size_t)lp] * T + pos % T == want);
        if (any_seg) REQUIRE(p.rowmap[(size_t)ad.score_off + (size_t)m] == want);
      }
      // rotation tables: entry 0 is (cos, sin) of the whole delta, every entry lies on the unit circle
      const double delta = (double)(ha[i].pos0 - sessions[ha[i].session].master_pos0);
      const float* c = p.tab.data() + (size_t)i * 2 * kHalf;
      REQUIRE(c[0] == (float)std::cos(delta) && c[kHalf] == (float)std::sin(delta));
      for (int j = 0; j < kHalf; ++j) REQUIRE(std::fabs((double)c[j] * c[j] + (double)c[kHalf + j] * c[kHalf + j] - 1.0) < 1e-6);
      if (any_seg) {
        const int t0 = p.seg_off[(size_t)i], t1 = p.seg_off[(size_t)i + 1];
        const int n_seg = ha[i].segs.empty() ? (S > 0 ? 1 : 0) : (int)ha[i].segs.size();
        REQUIRE(t1 - t0 == n_seg && (size_t)t1 * 2 * kHalf <= p.segtab.size() && p.segtab.size() == p.segtab_diff.size());
        for (int32_t pg = 0; pg * T < S; ++pg) {
          const PageTab e = p.pagetab[(size_t)ad.flag_off + (size_t)pg];
          REQUIRE(e.x >= t0 && e.x < t1 && e.y >= e.x && e.y < t1 && e.y <= e.x + 1);
          for (int r = 0; r < T && pg * T + r < S; ++r) {
            const int32_t m = pg * T + r;
            int q = 0;
            if (!ha[i].segs.empty()) while (!(m >= ha[i].segs[q].src_tok && m < ha[i].segs[q].src_tok + ha[i].segs[q].len)) ++q;
            REQUIRE(t0 + q == (((e.z >> r) & 1) ? e.y : e.x));
          }
        }
      }
    }
    REQUIRE(p.total_pages == pages_sum && p.total_tokens == tokens_sum && p.max_phys_page == max_page);
    // work lists: every (agent, page) exactly once, whatever the group size; the queues hold the same items
    for (int trial = 0; trial < 4; ++trial) {
      const int group = trial == 0 ? plan_auto_group(p.sessions) : trial == 1 ? plan_auto_group(p.sessions, true) : (int)between(1, kMaxGroup);
      REQUIRE(group >= 1 && group <= kMaxGroup);
      std::vector<WorkItem> work, queued;
      plan_work(p.sessions, group, rnd() % 2, work);
      REQUIRE(work.size() <= p.work_capacity);
      std::vector<int> seen((size_t)pages_sum, 0);
      for (const auto& w : work) {
        REQUIRE(w.session >= 0 && w.session < n_sessions && w.page >= 0 && w.page < p.sess[w.session].pages);
        REQUIRE(w.ag_count >= 1 && w.ag_count <= kMaxGroup);
        REQUIRE(w.ag_begin >= p.sess[w.session].order_begin &&
                w.ag_begin + w.ag_count <= p.sess[w.session].order_begin + p.sess[w.session].n_agents);
        for (int g = 0; g < w.ag_count; ++g) ++seen[(size_t)p.agents[p.order[(size_t)w.ag_begin + g]].flag_off + (size_t)w.page];
      }
      for (int v : seen) REQUIRE(v == 1);
      int32_t q_begin[9];
      plan_queues(work, queued, q_begin);
      REQUIRE(queued.size() == work.size() && q_begin[0] == 0 && q_begin[8] == (int32_t)work.size());
      for (int x = 0; x < 8; ++x) {
        REQUIRE(q_begin[x + 1] - q_begin[x] == (int32_t)((work.size() + 7 - x) / 8));
        for (int32_t k = q_begin[x]; k < q_begin[x + 1]; ++k) {
          const WorkItem& a = queued[(size_t)k];
          const WorkItem& b = work[(size_t)x + 8 * (size_t)(k - q_begin[x])];
          REQUIRE(a.session == b.session && a.page == b.page && a.ag_begin == b.ag_begin && a.ag_count == b.ag_count);
        }
      }
    }
  }
  // argument errors
  {
    const int cs = -1;
    RoundPlan p;
    std::string err;
    tdk_model m{2, 8, 128, 16, TDK_BF16, TDK_ROPE_HALF, 1.0e6};
    tdk_session s{40, 0};
    int32_t table[4] = {3, 1, 2, 0};
    tdk_agent a{0, 5, table, 3, 5, 0, nullptr};
    REQUIRE(plan_round(&m, &s, 1, &a, 1, p, err) == TDK_OK);
    REQUIRE(plan_round(nullptr, &s, 1, &a, 1, p, err) == TDK_ERR_INVALID_ARG);
    tdk_agent bad = a;
    bad.block_table_len = 2;                                            // 5 + 40 tokens need 3 pages
    REQUIRE(plan_round(&m, &s, 1, &bad, 1, p, err) == TDK_ERR_INVALID_ARG);
    bad = a; bad.session = 1;
    REQUIRE(plan_round(&m, &s, 1, &bad, 1, p, err) == TDK_ERR_INVALID_ARG);
    bad = a; bad.dst_pos0 = -1;
    REQUIRE(plan_round(&m, &s, 1, &bad, 1, p, err) == TDK_ERR_INVALID_ARG);
    int32_t neg[3] = {0, -1, 2};
    bad = a; bad.block_table = neg;
    REQUIRE(plan_round(&m, &s, 1, &bad, 1, p, err) == TDK_ERR_INVALID_ARG);
    tdk_segment overlap[2] = {{0, 20, 5, 5}, {20, 20, 10, 10}};         // destinations overlap
    bad = a; bad.n_segments = 2; bad.segments = overlap;
    REQUIRE(plan_round(&m, &s, 1, &bad, 1, p, err) == TDK_ERR_INVALID_ARG);
    tdk_segment gap[1] = {{0, 30, 5, 5}};                                // does not cover the span
    bad = a; bad.n_segments = 1; bad.segments = gap;
    REQUIRE(plan_round(&m, &s, 1, &bad, 1, p, err) == TDK_ERR_INVALID_ARG);
    tdk_model wrong = m; wrong.head_dim = 64;
    REQUIRE(plan_round(&wrong, &s, 1, &a, 1, p, err) == TDK_ERR_UNSUPPORTED);
    tdk_session negs{-1, 0};
    REQUIRE(plan_round(&m, &negs, 1, nullptr, 0, p, err) == TDK_ERR_INVALID_ARG);
  }
  std::printf("round planner: %d rounds planned, %d refused for three segments on a page, clean\n", planned, refused_three);
  return planned > 300 && refused_three > 3 ? 0 : 2;
}
