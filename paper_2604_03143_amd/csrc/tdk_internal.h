// Internal declarations shared by the host planner (tdk_api.cpp) and the kernels (tdk_kernels.hip).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tdk.h"
#include "tdk_types.h"

namespace tdk {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte access
struct RoundDev {
  const WorkItem*   work;    // one item per workgroup of a static launch: item i runs on XCD i % 8
  const WorkItem*   qwork;   // the same items grouped by that XCD: the queues of a queued launch
  const SessionDev* sess;
  const AgentDev*   agents;
  const int32_t*    order;   // agent ids grouped by session
  const int32_t*    bt;      // block-table slices, concatenated
  const float*      tab;     // [n_agents][2][64]: cos then sin of the agent's delta
  const float*      tab_diff;  // [n_agents][2][64]: same for dst_pos0 - diff_pos0 (payload re-rotation)
  // general block layouts (some agent has its own order of the shared blocks); all NULL otherwise
  const int32_t*    rowmap;    // [sum_i S_i]: pool row of (agent, master token), agents in order
  const PageTab*    pagetab;   // [sum_i pages_i]: {first table, second table, row mask of the second,
                               //  bit t: table t's run moved since the stored diff was encoded}
  const float*      segtab;    // [n tables][2][64]: cos then sin, one table per (agent, segment)
  const float*      segtab_diff;  // same indexing: dst_pos - diff_pos of the segment (payload re-rotation)
  const int32_t*    seg_off;   // [n_agents + 1]: agent i's segments (and tables) are seg_off[i] .. seg_off[i + 1]
  const int32_t*    seg_src;   // first master token of each segment (ascending within an agent, first is 0)
  uint8_t*          flags;   // [sum_i pages_i] scratch of encode
  unsigned long long* stamps;  // measurement only: [2 x work items] start / end clock of every work item, or NULL
  int32_t*          q_state; // [16] work queues: [0..7] next item of each XCD's queue, [8] workgroups that have left, [12] next item of a static launch's shared tail; all zero between launches
  int64_t           agent_pages;           // sum over agents of their session's page count: the length of a page-kernel launch
  const WorkItem*   rwork;                 // the work list of the kernels that only read (compare, key difference): it may be coarser
  int32_t           n_rwork;
  int32_t           dyn_begin, dyn_count;  // static launches of the write kernels: workgroups [dyn_begin, dyn_begin + dyn_count) take the items from dyn_begin on in the order they start (set per launch; dyn_begin = n_work, dyn_count = 0: none)
  int32_t           q_begin[9];  // XCD x's queue is work[q_begin[x] .. q_begin[x + 1])
  int32_t           n_cus;
  int32_t n_work, n_agents, n_sessions;
  int32_t heads;             // H
  int32_t page_tokens;       // T
  int32_t interleaved;       // rope style
  int32_t nontemporal;
  int32_t seg;               // 1: rowmap / pagetab / segtab describe the layout
  int64_t master_rows;       // rows of master_k / master_v (all sessions)
};

struct LayerDev {
  const u32x4* master_k;
  const u32x4* master_v;
  u32x4*       pool_k;
  u32x4*       pool_v;
};

struct DiffDev {
  int32_t* count;
  int64_t* offset;
  int32_t* idx;
  u32x4*   payload;
  int64_t  capacity;
  int32_t* overflow;
};

// Outputs of the check-layer pass (all device pointers).
struct PlanDev {
  float*   score;        // [sum_i S_i]
  int32_t* important;    // [n_agents][k_stride]
  int32_t* n_important;  // [n_agents]
  float*   total;        // [n_agents]
  int32_t* master;       // [n_sessions]
  int32_t  k_stride;
  float    ratio;
  float    min_score;
};

// Attention over the shared span from master + diff (tdk_attend.hip).
struct AttendDev {
  const void* q;        // bf16 [n_agents][n_q][n_q_heads][128]
  void*       qrot;     // workspace: the same rows rotated back by each agent's offset
  void*       qdiff;    // workspace: the rows as the listed pages meet them (turned back by dst - diff position)
  float*      part_o;   // workspace: [rows][n_parts][128] un-normalised partial outputs
  float*      part_m;   // workspace: [rows][n_parts] running maxima
  float*      part_l;   // workspace: [rows][n_parts] partial sums
  float*      out;      // [rows][128]
  float*      lse;      // [rows]
  int32_t n_q, n_q_heads, group;     // group = query heads per KV head
  int32_t chunk_tokens;              // master tokens per workgroup of the master pass (multiple of 32 and of T)
  int32_t n_chunks;                  // chunks of the longest span
  int32_t n_parts;                   // n_chunks + n_pieces: the chunks' partial results, then those of the listed pages
  int32_t n_pieces;                  // partial results of the listed-pages pass per query row
  int32_t piece_tokens;              // listed tokens per piece
  int32_t piece_grid;                // wavefronts launched per list: wavefront z takes the pieces z, z + piece_grid, ...
  int32_t max_seg;                   // copies of every query row in qrot: one per segment of its agent's layout
  int32_t diff_seg;                  // copies of every query row in qdiff: max_seg if a segmented round's stored
                                     // diffs sit at other positions (each segment moved by its own distance), else 1
  float   scale;                     // magnitude of the caller's scale, at least 1e-30
  int32_t q_flip;                    // the caller's scale was negative: the query copies carry the sign
};

// launchers (tdk_kernels.hip); each enqueues exactly one kernel
hipError_t launch_rerotate(const RoundDev& rd, const LayerDev& io, hipStream_t st);
hipError_t launch_flag(const RoundDev& rd, const LayerDev& io, float eps, int planes, hipStream_t st);
hipError_t launch_compact(const RoundDev& rd, const DiffDev& d, hipStream_t st);
hipError_t launch_gather(const RoundDev& rd, const LayerDev& io, const DiffDev& d, int planes, int grid, hipStream_t st);
hipError_t launch_decode(const RoundDev& rd, const LayerDev& io, const DiffDev& d, int planes, int scatter_blocks, bool* scattered,
                         hipStream_t st);
hipError_t launch_scatter(const RoundDev& rd, const LayerDev& io, const DiffDev& d, int planes, int grid, hipStream_t st);
hipError_t launch_keydiff(const RoundDev& rd, const LayerDev& io, const PlanDev& pl, hipStream_t st);
hipError_t launch_select(const RoundDev& rd, const PlanDev& pl, hipStream_t st);
hipError_t launch_master(const RoundDev& rd, const PlanDev& pl, hipStream_t st);
hipError_t launch_copy(u32x4* dst, const u32x4* src, size_t n16, hipStream_t st);
hipError_t launch_fill(u32x4* dst, uint32_t word, size_t n16, hipStream_t st);

hipError_t launch_attend_qrot(const RoundDev& rd, const AttendDev& at, hipStream_t st);
hipError_t launch_attend_master(const RoundDev& rd, const LayerDev& io, const DiffDev& d, const AttendDev& at,
                                int max_rows, hipStream_t st);
hipError_t launch_attend_diff(const RoundDev& rd, const DiffDev& d, const AttendDev& at, hipStream_t st);
hipError_t launch_attend_merge(const RoundDev& rd, const DiffDev& d, const AttendDev& at, hipStream_t st);
// master pass and listed-pages pass in one launch (identity layouts, stored diffs not moved, few rows per agent)
hipError_t launch_attend_fused(const RoundDev& rd, const LayerDev& io, const DiffDev& d, const AttendDev& at,
                               int max_rows, hipStream_t st);
int attend_piece_tokens(int64_t lists, int n_cus);   // listed tokens per piece of the listed-pages pass; lists = agents x KV heads

hipError_t launch_page_fill(u32x4* dst, const int32_t* ids, int n_pages, int page_u4, uint32_t word, hipStream_t st);
hipError_t launch_page_read(const u32x4* src, const int32_t* ids, int n_pages, int page_u4, u32x4* sink, hipStream_t st);
hipError_t launch_page_fill_product(u32x4* pk, u32x4* pv, const int32_t* ids, int n_pages, int group, int heads, int page_tokens,
                                    uint32_t word, hipStream_t st);
hipError_t launch_page_read_product(const u32x4* pk, const u32x4* pv, const int32_t* ids, int n_pages, int group, int heads,
                                    int page_tokens, u32x4* sink, hipStream_t st);

}  // namespace tdk
