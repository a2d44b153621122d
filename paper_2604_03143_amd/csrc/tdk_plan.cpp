// Host planner of a round (see tdk_plan.h).  No HIP here.
#include "tdk_plan.h"

#include <algorithm>
#include <cmath>
#include <cstdint>

namespace tdk {

tdk_status plan_check_model(const tdk_model* m, std::string& err) {
  auto refuse = [&](tdk_status st, const char* msg) { err = msg; return st; };
  if (!m) return refuse(TDK_ERR_INVALID_ARG, "model is NULL");
  if (m->num_layers <= 0 || m->num_kv_heads <= 0 || m->head_dim <= 0 || m->page_tokens <= 0)
    return refuse(TDK_ERR_INVALID_ARG, "model: sizes must be positive");
  if (!(m->rope_theta > 0.0) || !std::isfinite(m->rope_theta))
    return refuse(TDK_ERR_INVALID_ARG, "model: rope_theta must be positive and finite");
  if (m->rope_style != TDK_ROPE_HALF && m->rope_style != TDK_ROPE_INTERLEAVED)
    return refuse(TDK_ERR_INVALID_ARG, "model: unknown rope_style");
  if (m->dtype != TDK_BF16) return refuse(TDK_ERR_UNSUPPORTED, "model: only bf16 caches are supported");
  if (m->head_dim != kHeadDim) return refuse(TDK_ERR_UNSUPPORTED, "model: only head_dim 128 is supported");
  if (m->num_kv_heads > 8) return refuse(TDK_ERR_UNSUPPORTED, "model: at most 8 KV heads per device are supported");
  if (m->page_tokens != 16 && m->page_tokens != 32)
    return refuse(TDK_ERR_UNSUPPORTED, "model: page_tokens must be 16 or 32");
  return TDK_OK;
}


tdk_status plan_round(const tdk_model* model, const tdk_session* sessions, int32_t n_sessions,
                      const tdk_agent* agents, int32_t n_agents, RoundPlan& out, std::string& err) {
  auto refuse = [&](tdk_status st, const char* msg) { err = msg; return st; };
  out = RoundPlan();
  tdk_status st = plan_check_model(model, err);
  if (st != TDK_OK) return st;
  if (n_sessions < 0 || n_agents < 0) return refuse(TDK_ERR_INVALID_ARG, "negative session or agent count");
  if ((n_sessions && !sessions) || (n_agents && !agents)) return refuse(TDK_ERR_INVALID_ARG, "sessions / agents is NULL");
  const int T = model->page_tokens;
  out.sess.resize(n_sessions);
  out.agents.resize(n_agents);
  out.tab.resize((size_t)n_agents * 2 * kHalf);
  out.tab_diff.resize((size_t)n_agents * 2 * kHalf);
  out.sessions.resize(n_sessions);
  int64_t row0 = 0;
  for (int32_t s = 0; s < n_sessions; ++s) {
    if (sessions[s].span_tokens < 0) { return refuse(TDK_ERR_INVALID_ARG, "session: negative span_tokens"); }
    if (sessions[s].master_pos0 < 0) { return refuse(TDK_ERR_INVALID_ARG, "session: negative master_pos0"); }
    PlanSession& hs = out.sessions[s];
    hs.span = sessions[s].span_tokens;
    hs.pages = (hs.span + T - 1) / T;
    hs.master_pos0 = sessions[s].master_pos0;
    hs.master_row0 = row0;
    row0 += hs.span;
    out.sess[s] = {hs.master_row0, hs.span, hs.pages, 0, 0};
    out.total_master_pages += hs.pages;
  }
  out.total_master_rows = row0;
  int64_t flag_off = 0, score_off = 0;
  for (int32_t i = 0; i < n_agents; ++i) out.any_segments |= agents[i].n_segments > 0;
  bool seg_moved = false;                  // some segment's stored diff sits at another position
  for (int32_t i = 0; i < n_agents; ++i) {
    const tdk_agent& a = agents[i];
    if (a.session < 0 || a.session >= n_sessions) { return refuse(TDK_ERR_INVALID_ARG, "agent: session index out of range"); }
    if (a.dst_pos0 < 0) { return refuse(TDK_ERR_INVALID_ARG, "agent: negative dst_pos0"); }
    if (a.dst_pos0 >= (int64_t)1 << 31) { return refuse(TDK_ERR_INVALID_ARG, "agent: positions beyond 2^31"); }
    PlanSession& hs = out.sessions[a.session];
    const int64_t S = hs.span;
    if (a.n_segments < 0 || (a.n_segments > 0 && !a.segments)) { return refuse(TDK_ERR_INVALID_ARG, "agent: bad segment list"); }
    // the logical pages the shared span touches: one range for the identity layout, the hull of the
    // segments otherwise
    int64_t pos_lo = a.dst_pos0, pos_hi = a.dst_pos0 + S;   // [lo, hi)
    if (a.n_segments > 0) {
      int64_t next = 0;
      pos_lo = INT64_MAX; pos_hi = 0;
      for (int32_t q = 0; q < a.n_segments; ++q) {
        const tdk_segment& sg = a.segments[q];
        if (sg.diff_pos < 0 || sg.diff_pos >= (int64_t)1 << 31) { return refuse(TDK_ERR_INVALID_ARG, "agent: segment diff_pos out of range"); }
        if (sg.src_tok != next || sg.len <= 0 || sg.dst_pos < 0) { return refuse(TDK_ERR_INVALID_ARG, "agent: segments must be sorted, contiguous in the master and non-empty"); }
        for (int32_t o = 0; o < q; ++o) {
          const tdk_segment& og = a.segments[o];
          if (sg.dst_pos < og.dst_pos + og.len && og.dst_pos < sg.dst_pos + sg.len) { return refuse(TDK_ERR_INVALID_ARG, "agent: segment destinations overlap"); }
        }
        next += sg.len;
        pos_lo = std::min<int64_t>(pos_lo, sg.dst_pos);
        pos_hi = std::max<int64_t>(pos_hi, sg.dst_pos + sg.len);
      }
      if (next != S) { return refuse(TDK_ERR_INVALID_ARG, "agent: segments do not cover the span"); }
    }
    if (pos_hi + T >= (int64_t)1 << 31) { return refuse(TDK_ERR_INVALID_ARG, "agent: positions beyond 2^31"); }
    const int64_t lp_first = S > 0 ? pos_lo / T : a.dst_pos0 / T;
    const int64_t lp_last = S > 0 ? (pos_hi - 1) / T : lp_first - 1;
    if (S > 0) {
      if (!a.block_table) { return refuse(TDK_ERR_INVALID_ARG, "agent: block_table is NULL"); }
      if ((int64_t)a.block_table_len <= lp_last) { return refuse(TDK_ERR_INVALID_ARG, "agent: block_table too short for its span"); }
    }
    AgentDev& ad = out.agents[i];
    ad.pos0 = (int32_t)a.dst_pos0;
    ad.bt_off = (int32_t)out.bt.size();
    ad.lp_first = (int32_t)lp_first;
    ad.bt_len = (int32_t)(lp_last - lp_first + 1);
    ad.session = a.session;
    ad.flag_off = (int32_t)flag_off;
    ad.score_off = (int32_t)score_off;
    if (a.n_segments == 0 && a.diff_pos0 < 0) { return refuse(TDK_ERR_INVALID_ARG, "agent: negative diff_pos0"); }
    ad.diff_rot = a.n_segments ? 0 : a.diff_pos0 != a.dst_pos0;
    for (int32_t q = 0; q < a.n_segments; ++q) ad.diff_rot |= a.segments[q].diff_pos != a.segments[q].dst_pos;
    if (ad.diff_rot) out.diff_moved = true;
    score_off += S;
    {
      // only pages that hold shared tokens count (the hull of a permuted layout may contain others)
      auto touch = [&](int64_t lo, int64_t hi) -> bool {
        for (int64_t lp = lo / T; lp <= (hi - 1) / T; ++lp) {
          if (a.block_table[lp] < 0) return false;
          out.max_phys_page = std::max<int64_t>(out.max_phys_page, a.block_table[lp]);
        }
        return true;
      };
      bool ok = true;
      if (S > 0 && a.n_segments == 0) ok = touch(pos_lo, pos_hi);
      for (int32_t q = 0; q < a.n_segments && ok; ++q) ok = touch(a.segments[q].dst_pos, a.segments[q].dst_pos + a.segments[q].len);
      if (!ok) { return refuse(TDK_ERR_INVALID_ARG, "agent: negative page number in block_table"); }
    }
    for (int64_t lp = lp_first; lp <= lp_last; ++lp) out.bt.push_back(a.block_table[lp]);
    // layout tables (only if some agent of the round has segments)
    if (out.any_segments) {
      tdk_segment whole{0, (int32_t)S, a.dst_pos0, a.diff_pos0};
      const tdk_segment* segs = a.n_segments ? a.segments : &whole;
      const int32_t nseg = a.n_segments ? a.n_segments : (S > 0 ? 1 : 0);
      const int32_t tab0 = (int32_t)(out.segtab.size() / (2 * kHalf));
      out.seg_off.push_back(tab0);
      for (int32_t q = 0; q < nseg; ++q) {
        out.seg_src.push_back(segs[q].src_tok);
        seg_moved |= segs[q].dst_pos != segs[q].diff_pos;
        const double delta = (double)(segs[q].dst_pos - (hs.master_pos0 + segs[q].src_tok));
        for (int j = 0; j < kHalf; ++j) {
          const double inv_freq = std::pow(model->rope_theta, -(double)(2 * j) / (double)model->head_dim);
          out.segtab.push_back((float)std::cos(delta * inv_freq));
        }
        for (int j = 0; j < kHalf; ++j) {
          const double inv_freq = std::pow(model->rope_theta, -(double)(2 * j) / (double)model->head_dim);
          out.segtab.push_back((float)std::sin(delta * inv_freq));
        }
        const double moved = (double)(segs[q].dst_pos - segs[q].diff_pos);
        for (int j = 0; j < kHalf; ++j) {
          const double inv_freq = std::pow(model->rope_theta, -(double)(2 * j) / (double)model->head_dim);
          out.segtab_diff.push_back((float)std::cos(moved * inv_freq));
        }
        for (int j = 0; j < kHalf; ++j) {
          const double inv_freq = std::pow(model->rope_theta, -(double)(2 * j) / (double)model->head_dim);
          out.segtab_diff.push_back((float)std::sin(moved * inv_freq));
        }
        for (int32_t m = segs[q].src_tok; m < segs[q].src_tok + segs[q].len; ++m) {
          const int64_t pos = segs[q].dst_pos + (m - segs[q].src_tok);
          out.rowmap.push_back((int32_t)((int64_t)a.block_table[pos / T] * T + pos % T));
        }
      }
      int32_t q = 0;
      for (int32_t p = 0; p < hs.pages; ++p) {
        const int32_t m_lo = p * T, m_hi = (int32_t)std::min<int64_t>(S, (int64_t)(p + 1) * T);
        while (segs[q].src_tok + segs[q].len <= m_lo) ++q;
        PageTab e{tab0 + q, tab0 + q, 0, 0};
        int32_t q2 = q;
        for (int32_t m = m_lo; m < m_hi; ++m) {
          while (segs[q2].src_tok + segs[q2].len <= m) ++q2;
          if (q2 > q + 1) { return refuse(TDK_ERR_UNSUPPORTED, "agent: a master page meets more than two segments"); }
          if (q2 == q + 1) { e.y = tab0 + q2; e.z |= 1 << (m - m_lo); }
        }
        // which of the two runs sat elsewhere when the stored diff was encoded
        e.w = (segs[e.x - tab0].dst_pos != segs[e.x - tab0].diff_pos ? 1 : 0) |
              (segs[e.y - tab0].dst_pos != segs[e.y - tab0].diff_pos ? 2 : 0);
        out.pagetab.push_back(e);
      }
    }
    flag_off += hs.pages;
    if (flag_off >= (int64_t)1 << 31 || score_off >= (int64_t)1 << 31 || out.bt.size() >= (size_t)1 << 31) { return refuse(TDK_ERR_UNSUPPORTED, "round too large"); }
    hs.agents.push_back(i);

    // rotation tables of this agent: master frame -> its offset, and the frame its stored diff values
    // were encoded in -> its offset.  Angles in double, one rounding to fp32.
    const double deltas[2] = {(double)(a.dst_pos0 - hs.master_pos0), (double)(a.dst_pos0 - a.diff_pos0)};
    float* tabs[2] = {out.tab.data() + (size_t)i * 2 * kHalf, out.tab_diff.data() + (size_t)i * 2 * kHalf};
    for (int which = 0; which < 2; ++which) {
      float* c = tabs[which];
      float* sn = c + kHalf;
      for (int j = 0; j < kHalf; ++j) {
        const double inv_freq = std::pow(model->rope_theta, -(double)(2 * j) / (double)model->head_dim);
        const double phi = deltas[which] * inv_freq;
        c[j] = (float)std::cos(phi);
        sn[j] = (float)std::sin(phi);
      }
    }
  }
  out.total_pages = flag_off;
  if (out.any_segments) out.seg_off.push_back((int32_t)out.seg_src.size());
  out.seg_moved = seg_moved;
  for (int32_t i = 0; out.any_segments && i < n_agents; ++i) out.max_segments = std::max(out.max_segments, out.seg_off[i + 1] - out.seg_off[i]);
  if (out.any_segments && (out.max_phys_page + 1) * T >= (int64_t)1 << 31)
    return refuse(TDK_ERR_UNSUPPORTED, "segmented layouts address pool rows with 32 bits: page numbers too large");
  out.order.reserve(n_agents);
  for (size_t q = 0; q < out.sessions.size(); ++q) {
    const auto& hs = out.sessions[q];
    out.sess[q].order_begin = (int32_t)out.order.size();
    out.sess[q].n_agents = (int32_t)hs.agents.size();
    out.order.insert(out.order.end(), hs.agents.begin(), hs.agents.end());
  }
  out.total_tokens = score_off;

  // worst case for the work list: every agent its own group
  size_t work_cap = 0;
  for (const auto& hs : out.sessions) work_cap += (size_t)hs.pages * hs.agents.size();
  out.work_capacity = work_cap;

  return TDK_OK;
}

// Work list: one item per (master page, agent group).  Items that share a master page are given
// workgroup ids that are congruent modulo 8, so that (with round-robin dispatch of workgroups to
// the 8 XCDs) they run on the same XCD and the re-read of the master page hits that XCD's L2.
// taper: the pages at the end of the list are cut into smaller groups (a third of the group size over
// the last tenth of the work, single agents over the last fiftieth), so that the launch does not end
// with a few long items running on an otherwise idle chip.
void plan_work(const std::vector<PlanSession>& sessions, int group, bool taper, std::vector<WorkItem>& work) {
  work.clear();
  std::vector<int32_t> order_begin(sessions.size(), 0);
  int32_t cursor = 0;
  int64_t total = 0, done = 0;
  for (size_t s = 0; s < sessions.size(); ++s) {
    order_begin[s] = cursor;
    cursor += (int32_t)sessions[s].agents.size();
    total += (int64_t)sessions[s].pages * (int64_t)sessions[s].agents.size();
  }
  for (size_t s = 0; s < sessions.size(); ++s) {
    const int n = (int)sessions[s].agents.size();
    if (!n) continue;
    const int32_t pages = sessions[s].pages;
    for (int32_t q0 = 0; q0 < pages; q0 += 8) {
      const int32_t qn = std::min<int32_t>(8, pages - q0);
      // every block of 8 pages has one group count
      int g_eff = group;
      if (taper && total > 0) {
        if (done * 50 >= total * 49) g_eff = 1;
        else if (done * 10 >= total * 9) g_eff = std::max(1, (group + 2) / 3);
      }
      const int G = (n + g_eff - 1) / g_eff;
      for (int g = 0; g < G; ++g) {
        // balanced split: the first (n % G) groups get one agent more
        const int base = n / G, extra = n % G;
        const int begin = g * base + std::min(g, extra);
        const int cnt = base + (g < extra ? 1 : 0);
        for (int32_t q = 0; q < qn; ++q)
          work.push_back({(int32_t)s, q0 + q, order_begin[s] + begin, cnt});
      }
      done += (int64_t)qn * n;
    }
  }
}

int plan_auto_group(const std::vector<PlanSession>& sessions, bool read_kernels) {
  // Measured on MI355X: about 9 agents per work item is the best trade between re-reads of the
  // master page (one per work item, served by the XCD's L2) and the number of work items; rounds
  // too small to give ~2800 items that way are split further (a launch of one workgroup per item then runs
  // three to four rounds of the chip's workgroup slots instead of one and a bit: the 25-agent session
  // steps in 15.31 ms with 3 agents per item, 2817 items, against 15.48 ms with 9 agents, 939 items).
  // The kernels that only read have their own list: every item re-reads its master page, which costs them more
  // than the coarser end of their launch (the same session: compare kernel 87 us with 9 agents per item, 91 with 3),
  // so they stop splitting at ~900 items.
  const int64_t target = read_kernels ? 900 : 2800;
  int best = 9;
  for (int g = 9; g >= 1; --g) {
    int64_t items = 0;
    for (const auto& s : sessions) {
      const int n = (int)s.agents.size();
      if (n) items += (int64_t)s.pages * ((n + g - 1) / g);
    }
    best = g;
    if (items >= target) break;
  }
  return best;
}

void plan_queues(const std::vector<WorkItem>& work, std::vector<WorkItem>& queued, int32_t (&q_begin)[9]) {
  queued.clear();
  queued.reserve(work.size());
  for (int x = 0; x < 8; ++x) {
    q_begin[x] = (int32_t)queued.size();
    for (size_t i = x; i < work.size(); i += 8) queued.push_back(work[i]);
  }
  q_begin[8] = (int32_t)queued.size();
}

}  // namespace tdk
