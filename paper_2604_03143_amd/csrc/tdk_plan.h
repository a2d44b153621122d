// The host planner of a round: argument validation, rotation tables, block-table slices, layout tables and the
// work list, as host vectors.  Nothing here touches the GPU or includes HIP, so the whole planner runs (and is
// fuzzed under AddressSanitizer / UBSan) on machines without one; tdk_api.cpp uploads what it returns.
#pragma once

#include <stdint.h>

#include <string>
#include <vector>

#include "tdk.h"
#include "tdk_types.h"

namespace tdk {

struct PlanSession {
  int32_t span = 0, pages = 0;
  int64_t master_pos0 = 0, master_row0 = 0;
  std::vector<int32_t> agents;   // ids of its agents, in descriptor order
};

struct RoundPlan {
  std::vector<PlanSession> sessions;
  // what the device gets
  std::vector<SessionDev> sess;
  std::vector<AgentDev>   agents;
  std::vector<int32_t>    order;      // agent ids grouped by session
  std::vector<int32_t>    bt;         // block-table slices that cover the shared spans, concatenated
  std::vector<float>      tab;        // [n_agents][2][64]: cos then sin of dst_pos0 - master_pos0
  std::vector<float>      tab_diff;   // the same for dst_pos0 - diff_pos0
  bool any_segments = false;          // some agent has its own block layout: the vectors below are filled
  std::vector<int32_t>    rowmap;     // pool row of (agent, master token)
  std::vector<PageTab>    pagetab;    // per (agent, master page)
  std::vector<float>      segtab, segtab_diff;   // one table per (agent, segment)
  std::vector<int32_t>    seg_off, seg_src;      // per agent the range of its segments, their first master tokens
  // totals
  int64_t max_phys_page = -1;         // largest page number any shared span maps to
  int64_t total_pages = 0;            // sum over agents of their session's page count
  int64_t total_master_pages = 0, total_master_rows = 0;
  int64_t total_tokens = 0;           // sum over agents of their session's span
  int32_t max_segments = 1;           // most segments any agent has (1 for identity layouts)
  bool seg_moved = false;             // a segmented agent's stored diff sits at other positions
  bool diff_moved = false;            // some agent's stored diff sits at other positions (segmented or not)
  size_t work_capacity = 0;           // work items in the worst case (every agent its own group)
};

// Every function returns TDK_OK or the status to hand to the caller, with the reason in `err`.
tdk_status plan_check_model(const tdk_model* m, std::string& err);
tdk_status plan_round(const tdk_model* model, const tdk_session* sessions, int32_t n_sessions,
                      const tdk_agent* agents, int32_t n_agents, RoundPlan& p, std::string& err);

// Work list for `group` agents per item in the order of a static launch (item i runs on XCD i % 8), and the same
// items grouped by that XCD (queue x = queued[q_begin[x] .. q_begin[x + 1])).
void plan_work(const std::vector<PlanSession>& sessions, int group, bool taper, std::vector<WorkItem>& work);
void plan_queues(const std::vector<WorkItem>& work, std::vector<WorkItem>& queued, int32_t (&q_begin)[9]);
int  plan_auto_group(const std::vector<PlanSession>& sessions, bool read_kernels = false);   // agents per work item when the caller names none

}  // namespace tdk
