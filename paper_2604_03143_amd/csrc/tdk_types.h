// Plain descriptor types of a round, shared by the host planner (no HIP needed) and the kernels.
#pragma once

#include <stdint.h>

namespace tdk {

constexpr int kMaxGroup = 32;     // agents that share one read of a master page
constexpr int kBlock = 256;       // threads per workgroup (4 wavefronts of 64)
constexpr int kWaves = kBlock / 64;
constexpr int kHeadDim = 128;
constexpr int kHalf = kHeadDim / 2;

// One unit of work of the page kernels: a master page and a group of agents of its session.
struct WorkItem {
  int32_t session;
  int32_t page;        // master page number
  int32_t ag_begin;    // range in RoundDev::order
  int32_t ag_count;    // 1..kMaxGroup
};

struct SessionDev {
  int64_t master_row0;  // first row of this session in master_k / master_v
  int32_t span;         // S
  int32_t pages;        // ceil(S / T)
  int32_t order_begin;  // its agents are RoundDev::order[order_begin .. order_begin + n_agents)
  int32_t n_agents;
};

struct AgentDev {
  int32_t pos0;         // dst_pos0 (validated < 2^31)
  int32_t bt_off;       // start of this agent's block-table slice in RoundDev::bt
  int32_t lp_first;     // logical page number of slice entry 0 (= pos0 / T)
  int32_t bt_len;       // entries in the slice
  int32_t session;
  int32_t flag_off;     // start of this agent's per-page flags in the flag scratch
  int32_t score_off;    // start of this agent's per-token scores (sum of the spans of earlier agents)
  int32_t diff_rot;     // 1: payload K rows of this agent were stored at another position (re-rotate on restore)
};

// Per (agent, master page) of a round with per-agent block layouts: the rotation tables of the (at most two)
// segments the page meets, which rows use the second, and which of the two runs moved since the stored diff
// was encoded.  Read by the kernels as one 16-byte word.
struct alignas(16) PageTab {
  int32_t x;   // first table
  int32_t y;   // second table (= x if the page lies in one segment)
  int32_t z;   // bit r: row r uses the second table
  int32_t w;   // bit t: table t's run sat at another position when the stored diff was encoded
};

}  // namespace tdk
