// HIP kernels of libtdk for gfx950 (MI355X): collective RoPE re-rotation, per-page compare,
// ballot/prefix compaction, payload gather and fused diff restore.
//
// Data movement plan shared by the three page kernels (rerotate, flag, decode):
//   - a workgroup of 4 wavefronts owns one master page (T rows of H*D bf16, K and V) and a group
//     of up to 32 agents of that page's session;
//   - the master page is read from HBM once, 16 bytes per lane, and stays in registers while the
//     workgroup walks its agents (Sec. 4.2: the cost of a shared block is paid once per group);
//   - the per-agent cos/sin tables, the two physical pages a master page can land on and the
//     page's row offset are staged in LDS once per workgroup;
//   - a wavefront always handles whole rows: lane l holds 8 consecutive elements of the low half
//     and the 8 matching elements of the high half of head l/8, so both members of every rotation
//     pair sit in the same lane and each load/store instruction covers whole 128-byte segments.
#include "tdk_internal.h"

#include <algorithm>
#include <map>
#include <mutex>
#include <type_traits>

namespace tdk {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------------------------
// bf16 <-> fp32
// ---------------------------------------------------------------------------------------------

__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// two fp32 -> packed bf16 (a in the low half), round-to-nearest-even
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

// y_a = fma(x_a, c, -(x_b * s)), y_b = fma(x_b, c, x_a * s): one rounded product, one fma.
__device__ __forceinline__ void rot(float xa, float xb, float c, float s, float& ya, float& yb) {
  float t = __fmul_rn(xb, s);
  float u = __fmul_rn(xa, s);
  ya = __builtin_fmaf(xa, c, -t);
  yb = __builtin_fmaf(xb, c, u);
}

// Rotates the 16 elements a lane holds.  Half style: lo[e] pairs with hi[e], table entry e.
// Interleaved style: each 32-bit word is one pair; lo uses entries 0..3, hi entries 4..7.
template <bool IL>
__device__ __forceinline__ void rotate16(const u32x4 lo, const u32x4 hi, const float (&c)[8],
                                         const float (&s)[8], u32x4& olo, u32x4& ohi) {
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    if (!IL) {
      float yl0, yh0, yl1, yh1;
      rot(bf_lo(lo[w]), bf_lo(hi[w]), c[2 * w], s[2 * w], yl0, yh0);
      rot(bf_hi(lo[w]), bf_hi(hi[w]), c[2 * w + 1], s[2 * w + 1], yl1, yh1);
      olo[w] = pack_bf16(yl0, yl1);
      ohi[w] = pack_bf16(yh0, yh1);
    } else {
      float ya, yb;
      rot(bf_lo(lo[w]), bf_hi(lo[w]), c[w], s[w], ya, yb);
      olo[w] = pack_bf16(ya, yb);
      rot(bf_lo(hi[w]), bf_hi(hi[w]), c[4 + w], s[4 + w], ya, yb);
      ohi[w] = pack_bf16(ya, yb);
    }
  }
}

// Streaming store: system-scope, non-temporal (sc0 sc1 nt).  The line is written through instead of
// staying dirty in L2 for a later kernel to flush; measured best for the page kernels' scattered
// 32 KB writes when they run back to back with the compare kernel.
template <bool NT>
__device__ __forceinline__ void st16(u32x4* p, u32x4 v) {
  // The two idle cycles keep a following VALU write of the data registers clear of the store's read
  // of them (16-byte stores need two wait states on gfx940+; the compiler cannot see into the asm).
  if (NT) asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
  else *p = v;
}

template <bool NT>
__device__ __forceinline__ u32x4 ld16(const u32x4* p) {
  return NT ? __builtin_nontemporal_load(p) : *p;
}

// ---------------------------------------------------------------------------------------------
// per-workgroup staging
// ---------------------------------------------------------------------------------------------

struct GroupShared {
  float   tab[kMaxGroup][2 * kHalf];  // cos[64], sin[64] of each agent of the group
  int32_t pg0[kMaxGroup];             // physical page holding the master page's first token
  int32_t pg1[kMaxGroup];             // the next logical page's physical page (or -1)
  int32_t off[kMaxGroup];             // row of the first token inside pg0
  int32_t aux[kMaxGroup];             // flag kernel: OR of the waves; decode: payload slot or -1
  int32_t agent[kMaxGroup];
};

// The same for rounds with per-agent block layouts: a master page can meet two segments of an agent
// (two position deltas), and its rows can land anywhere, so the pool row of every row is staged.
struct GroupSharedSeg {
  float    tab[kMaxGroup][2][2 * kHalf];
  int32_t  row[kMaxGroup][32];       // pool row of each row of the page
  uint32_t sel[kMaxGroup];           // bit r set: row r uses the second table
  int32_t  aux[kMaxGroup];
  int32_t  agent[kMaxGroup];
};

template <int T>
__device__ __forceinline__ void stage_group(const RoundDev& rd, const WorkItem& w, GroupSharedSeg& sh) {
  const int tid = threadIdx.x;
  for (int i = tid; i < w.ag_count * 64; i += kBlock) {
    const int g = i >> 6, which = (i >> 5) & 1, q = i & 31;
    const AgentDev ad = rd.agents[rd.order[w.ag_begin + g]];
    const PageTab pt = rd.pagetab[ad.flag_off + w.page];
    const int t = which ? pt.y : pt.x;
    reinterpret_cast<float4*>(sh.tab[g][which])[q] =
        reinterpret_cast<const float4*>(rd.segtab + (size_t)t * (2 * kHalf))[q];
  }
  const SessionDev sd = rd.sess[w.session];
  for (int i = tid; i < w.ag_count * T; i += kBlock) {
    const int g = i / T, r = i - g * T;
    const AgentDev ad = rd.agents[rd.order[w.ag_begin + g]];
    const int m = w.page * T + r;
    sh.row[g][r] = m < sd.span ? rd.rowmap[ad.score_off + m] : 0;
  }
  if (tid < w.ag_count) {
    const int a = rd.order[w.ag_begin + tid];
    sh.sel[tid] = (uint32_t)rd.pagetab[rd.agents[a].flag_off + w.page].z;
    sh.aux[tid] = 0;
    sh.agent[tid] = a;
  }
}

template <int T>
__device__ __forceinline__ void stage_group(const RoundDev& rd, const WorkItem& w, GroupShared& sh) {
  const int tid = threadIdx.x;
  for (int i = tid; i < w.ag_count * 32; i += kBlock) {
    const int g = i >> 5, q = i & 31;
    const int a = rd.order[w.ag_begin + g];
    reinterpret_cast<float4*>(sh.tab[g])[q] =
        reinterpret_cast<const float4*>(rd.tab + (size_t)a * (2 * kHalf))[q];
  }
  if (tid < w.ag_count) {
    const int a = rd.order[w.ag_begin + tid];
    const AgentDev ad = rd.agents[a];
    const int a0 = ad.pos0 + w.page * T;
    const int lp = a0 / T - ad.lp_first;
    sh.pg0[tid] = rd.bt[ad.bt_off + lp];
    sh.pg1[tid] = (lp + 1 < ad.bt_len) ? rd.bt[ad.bt_off + lp + 1] : -1;
    sh.off[tid] = a0 % T;
    sh.aux[tid] = 0;
    sh.agent[tid] = a;
  }
}

// lane geometry inside a row of H heads x 128 bf16 (= H*16 chunks of 16 bytes)
struct Lane {
  int klo, khi;      // chunk index of this lane's low-half / high-half K chunk
  int v0, v1;        // chunk indices of its two V chunks
  bool kok, v0ok, v1ok;
  int jb;            // which 8-element block of the half this lane rotates
};

__device__ __forceinline__ Lane lane_geometry(int H) {
  const int lane = threadIdx.x & 63;
  Lane L;
  L.jb = lane & 7;
  L.klo = (lane >> 3) * 16 + L.jb;
  L.khi = L.klo + 8;
  L.kok = (lane >> 3) < H;
  L.v0 = lane;
  L.v1 = lane + 64;
  L.v0ok = L.v0 < H * 16;
  L.v1ok = L.v1 < H * 16;
  return L;
}

__device__ __forceinline__ const float* tab_of(const GroupShared& sh, int g, int) { return sh.tab[g]; }
__device__ __forceinline__ const float* tab_of(const GroupSharedSeg& sh, int g, int r) {
  return sh.tab[g][(sh.sel[g] >> r) & 1u];
}

// cos/sin a lane needs for row r of agent g (r matters only with per-agent block layouts)
template <bool IL, class Shared>
__device__ __forceinline__ void load_tab(const Shared& sh, int g, int r, int jb, float (&c)[8], float (&s)[8]) {
  const float* t = tab_of(sh, g, r);
  if (!IL) {
#pragma unroll
    for (int e = 0; e < 8; ++e) { c[e] = t[jb * 8 + e]; s[e] = t[kHalf + jb * 8 + e]; }
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      c[e] = t[jb * 4 + e];          s[e] = t[kHalf + jb * 4 + e];
      c[4 + e] = t[32 + jb * 4 + e]; s[4 + e] = t[kHalf + 32 + jb * 4 + e];
    }
  }
}

template <int RPW>
struct MasterRows {
  u32x4 kl[RPW], kh[RPW], v0[RPW], v1[RPW];
  bool  valid[RPW];
};

template <int RPW, bool LOADV = true, bool LOADK = true>
__device__ __forceinline__ void load_master(const RoundDev& rd, const LayerDev& io, const WorkItem& w,
                                            const Lane& L, MasterRows<RPW>& M) {
  constexpr int T = RPW * kWaves;
  const SessionDev sd = rd.sess[w.session];
  const int wave = threadIdx.x >> 6;
  const int64_t row_u4 = (int64_t)rd.heads * 16;
#pragma unroll
  for (int k = 0; k < RPW; ++k) {
    const int m = w.page * T + wave + kWaves * k;
    M.valid[k] = m < sd.span;
    const u32x4 z = {0, 0, 0, 0};
    M.kl[k] = z; M.kh[k] = z; M.v0[k] = z; M.v1[k] = z;
    if (M.valid[k]) {
      const u32x4* rk = io.master_k + (sd.master_row0 + m) * row_u4;
      const u32x4* rv = io.master_v + (sd.master_row0 + m) * row_u4;
      if (LOADK && L.kok) { M.kl[k] = rk[L.klo]; M.kh[k] = rk[L.khi]; }
      if (LOADV && L.v0ok) M.v0[k] = rv[L.v0];
      if (LOADV && L.v1ok) M.v1[k] = rv[L.v1];
    }
  }
}

template <int T>
__device__ __forceinline__ int64_t dest_row(const GroupSharedSeg& sh, int g, int r) { return sh.row[g][r]; }

// physical pool row of row r (0..T-1) of the master page for agent g of the group
template <int T>
__device__ __forceinline__ int64_t dest_row(const GroupShared& sh, int g, int r) {
  const int q = sh.off[g] + r;
  const int pg = q < T ? sh.pg0[g] : sh.pg1[g];
  return (int64_t)pg * T + (q & (T - 1));
}

// ---------------------------------------------------------------------------------------------
// rerotate: pool_k <- bf16(R(delta_i) master_k), pool_v <- master_v       [Sec. 4.2]
// ---------------------------------------------------------------------------------------------

constexpr int kPrefetchBlocks = 1024;   // workgroups that take part in the master sweep (about one dispatch wave)

// The workgroups that start first sweep the masters once, in address order, before any of them
// writes: the reads then come from DRAM as one sequential stream into the memory-side cache instead
// of arriving one page at a time among the writes (a read among writes costs DRAM a bus turnaround;
// measured at about twice its byte share).
__device__ __forceinline__ void sweep_masters(const RoundDev& rd, const LayerDev& io, bool k, bool v) {
  if (blockIdx.x >= kPrefetchBlocks) return;
  const size_t n16 = (size_t)rd.master_rows * rd.heads * 16;
  const unsigned nb = min((unsigned)gridDim.x, (unsigned)kPrefetchBlocks);
  u32x4 acc = {0, 0, 0, 0};
  for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n16; i += (size_t)nb * kBlock) {
    if (k) acc ^= io.master_k[i];
    if (v) acc ^= io.master_v[i];
  }
  asm volatile("" : : "v"(acc));      // keeps the loads alive; the values are not used
}

// Optional timeline of a launch (measurement only): when the round carries a stamp buffer, the clock is
// recorded when a work item is taken up and when the last wavefront has issued its last access for it.
__device__ __forceinline__ int xcd_id() { return (int)(__builtin_amdgcn_s_getreg((3 << 11) | 20) & 7u); }   // XCC_ID, bits 3:0

__device__ __forceinline__ void stamp_begin(const RoundDev& rd, int item) {
  // (the low four bits carry the XCD the workgroup runs on)
  if (rd.stamps && threadIdx.x == 0) rd.stamps[4 * (size_t)item] = (wall_clock64() & ~15ull) | (unsigned)xcd_id();
}
__device__ __forceinline__ void stamp_end(const RoundDev& rd, int item) {
  if (rd.stamps && (threadIdx.x & 63) == 0) atomicMax(&rd.stamps[4 * (size_t)item + 1], (unsigned long long)wall_clock64());
}
// which = 2: the item's staging is in LDS; which = 3: the first wavefront has handled its rows of the first agent
__device__ __forceinline__ void stamp_mid(const RoundDev& rd, int item, int which) {
  if (rd.stamps && threadIdx.x == 0) rd.stamps[4 * (size_t)item + which] = wall_clock64();
}

// Which work items a workgroup processes.
//   Static: workgroup b owns item b, dispatched by the hardware round-robin over the XCDs.
//   Queued (TDK_TUNE_XCD_QUEUES, the kernels that write): the launch holds two workgroups per compute unit, and each
//   takes items until none is left: first from the queue of the XCD it runs on (the items that the static form
//   would have run there, so re-reads of a master page still meet in that XCD's L2), then from the other XCDs'
//   queues.  The XCDs do not write to memory at the same rate (measured: four of the eight finish a static
//   rerotate launch 15 % earlier and then idle); with queues the fast ones take over what the slow ones have left.
// Queue state in device memory: next[8], then the count of workgroups that have left the loop; the last one to
// leave puts everything back to zero, so every launch finds the state as the round's creation left it.
// Barrier for data exchanged through LDS only: waits for this wavefront's LDS traffic, not for its global stores
// (__syncthreads() would also wait until every store issued so far has been acknowledged by memory, which stalls
// a wavefront for microseconds at every item border while the chip is writing at full rate).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <bool queued>
struct Items {
  int home, k, ahead;
  __device__ __forceinline__ Items() : home(queued ? xcd_id() : 0), k(0), ahead(-1) {}

  // The first item of every workgroup is fixed by its number (workgroup b starts with entry b / 8 of queue b % 8, the
  // XCD the hardware places it on): no atomic stands between the launch and the first access, and the queues hand
  // out what lies behind those entries.
  __device__ __forceinline__ int reserved(int x) const { return ((int)gridDim.x - x + 7) >> 3; }   // workgroups b with b % 8 == x

  // thread 0 only: the next item for this workgroup, or -1 when every queue is empty
  __device__ __forceinline__ int fetch(const RoundDev& rd) {
    while (k < 8) {
      const int x = (home + k) & 7;
      const int n = rd.q_begin[x + 1] - rd.q_begin[x] - reserved(x);
      const int i = n > 0 ? atomicAdd(&rd.q_state[x], 1) : 0;
      if (i < n) return rd.q_begin[x] + reserved(x) + i;
      ++k;             // that queue is empty for good
    }
    return -1;
  }

  // Asks for the item after the current one (thread 0; an atomic whose answer is a round trip to memory among
  // the writes).  Called once per item, after the item's own loads have been issued: answers come back in issue
  // order, so a load issued behind the atomic would wait for it, while the stores of the data phase do not.
  __device__ __forceinline__ void prefetch(const RoundDev& rd) {
    if (queued) { if (threadIdx.x == 0) ahead = fetch(rd); }
  }

  // Hands the prefetched item to the whole workgroup.
  __device__ __forceinline__ int publish(int* s_item) {
    lds_barrier();     // every wavefront is through with the previous item: its staging in LDS may be replaced
    if (threadIdx.x == 0) *s_item = ahead;
    lds_barrier();
    return *s_item;
  }

  __device__ __forceinline__ int first(const RoundDev& rd, int* s_item) {
    if (!queued) {
      // Static launch: workgroup b owns item b, except for a shared tail (TDK_TUNE_SHARED_TAIL): the last items
      // go, in order, to whichever of the launch's last workgroups start first (there are twice as many of those
      // as items left, the late ones leave at once).  An XCD that writes faster gets through its share of the
      // workgroup ids sooner and so takes more of the tail, which evens out the end of a launch too short for
      // the looping form.  Every such workgroup does one atomic; the one that draws the last ticket puts the
      // counter back to zero.
      const int b = (int)blockIdx.x;
      if (b < rd.dyn_begin) return b;
      if (b >= rd.dyn_begin + rd.dyn_count) return -1;
      if (threadIdx.x == 0) {
        const int i = atomicAdd(&rd.q_state[12], 1);
        if (i == rd.dyn_count - 1) atomicExch(&rd.q_state[12], 0);
        *s_item = rd.dyn_begin + i < rd.n_work ? rd.dyn_begin + i : -1;
      }
      lds_barrier();
      return *s_item;
    }
    const int x = (int)blockIdx.x & 7, i = (int)blockIdx.x >> 3;
    return i < rd.q_begin[x + 1] - rd.q_begin[x] ? rd.q_begin[x] + i : -1;
  }
  __device__ __forceinline__ int next(const RoundDev& rd, int* s_item) {
    if (!queued) return -1;
    return publish(s_item);
  }
  __device__ __forceinline__ const WorkItem& at(const RoundDev& rd, int item) const { return queued ? rd.qwork[item] : rd.work[item]; }
  __device__ __forceinline__ void leave(const RoundDev& rd) {
    if (queued) if (threadIdx.x == 0) {
      const int gone = atomicAdd(&rd.q_state[8], 1);
      if (gone == (int)gridDim.x - 1) {       // nobody takes items any more
#pragma unroll
        for (int x = 0; x < 8; ++x) atomicExch(&rd.q_state[x], 0);
        __threadfence();
        atomicExch(&rd.q_state[8], 0);
      }
    }
  }
};

template <int RPW, bool IL, bool NT, bool SEG, bool Q>
__global__ __launch_bounds__(kBlock) void tdk_rerotate_kernel(const RoundDev rd, const LayerDev io) {
  constexpr int T = RPW * kWaves;
  __shared__ std::conditional_t<SEG, GroupSharedSeg, GroupShared> sh;
  __shared__ int s_item;
  const Lane L = lane_geometry(rd.heads);
  if (rd.nontemporal & 32) sweep_masters(rd, io, true, true);
  const int wave = threadIdx.x >> 6;
  const int64_t row_u4 = (int64_t)rd.heads * 16;
  u32x4* pk = io.pool_k;
  u32x4* pv = io.pool_v;
  Items<Q> items;
  for (int item = items.first(rd, &s_item); item >= 0; item = items.next(rd, &s_item)) {
    stamp_begin(rd, item);
    const WorkItem w = items.at(rd, item);
    stage_group<T>(rd, w, sh);
    MasterRows<RPW> M;
    load_master<RPW>(rd, io, w, L, M);
    lds_barrier();
    items.prefetch(rd);
    stamp_mid(rd, item, 2);
    for (int g = 0; g < w.ag_count; ++g) {
      if (g == 1) stamp_mid(rd, item, 3);
      float c[8], s[8];
      if (!SEG) load_tab<IL>(sh, g, 0, L.jb, c, s);
#pragma unroll
      for (int k = 0; k < RPW; ++k) {
        if (!M.valid[k]) continue;
        const int64_t base = dest_row<T>(sh, g, wave + kWaves * k) * row_u4;
        if (L.kok) {
          if (SEG) load_tab<IL>(sh, g, wave + kWaves * k, L.jb, c, s);
          u32x4 olo, ohi;
          rotate16<IL>(M.kl[k], M.kh[k], c, s, olo, ohi);
          st16<NT>(pk + base + L.klo, olo);
          st16<NT>(pk + base + L.khi, ohi);
        }
        if (L.v0ok) st16<NT>(pv + base + L.v0, M.v0[k]);
        if (L.v1ok) st16<NT>(pv + base + L.v1, M.v1[k]);
      }
    }
    stamp_end(rd, item);
  }
  items.leave(rd);
}

// ---------------------------------------------------------------------------------------------
// flag: per (agent, master page) compare against the re-rotated master     [Sec. 4.3]
// ---------------------------------------------------------------------------------------------

// differ <=> not (|a - ref| <= eps) in fp32; NaN on either side differs
__device__ __forceinline__ bool word_differs(uint32_t a, uint32_t r, float eps) {
  const bool lo = !(__builtin_fabsf(bf_lo(a) - bf_lo(r)) <= eps);
  const bool hi = !(__builtin_fabsf(bf_hi(a) - bf_hi(r)) <= eps);
  return lo | hi;
}

__device__ __forceinline__ bool chunk_differs(const u32x4 a, const u32x4 r, float eps) {
  bool d = false;
#pragma unroll
  for (int w = 0; w < 4; ++w) d |= word_differs(a[w], r[w], eps);
  return d;
}

__device__ __forceinline__ uint32_t chunk_xor(const u32x4 a, const u32x4 r) {
  const u32x4 x = a ^ r;
  return x[0] | x[1] | x[2] | x[3];
}

// true if some bf16 in the chunk is non-finite or so large (|x| >= 2^126) that a rotation could
// overflow: only then can a reference that is bit-identical to the agent's value still "differ"
// (|inf - inf| and NaN compare false), so such rows always take the full fp32 compare.
__device__ __forceinline__ bool chunk_special(const u32x4 m) {
  bool sp = false;
#pragma unroll
  for (int w = 0; w < 4; ++w)
    sp |= ((m[w] & 0x7f80u) >= 0x7e80u) | ((m[w] & 0x7f800000u) >= 0x7e800000u);
  return sp;
}

// PM: planes that take part (bit 0 = K, bit 1 = V); 3 is the paired diff, 1 / 2 the single-plane diffs
template <int RPW, bool IL, int PM, bool SEG, bool NTL>
__global__ __launch_bounds__(kBlock) void tdk_flag_kernel(const RoundDev rd, const LayerDev io, const float eps) {
  constexpr int T = RPW * kWaves;
  constexpr bool DOK = (PM & 1) != 0, DOV = (PM & 2) != 0;
  __shared__ std::conditional_t<SEG, GroupSharedSeg, GroupShared> sh;
  const Lane L = lane_geometry(rd.heads);
  const int wave = threadIdx.x >> 6;
  const int64_t row_u4 = (int64_t)rd.heads * 16;
  const u32x4* pk = io.pool_k;
  const u32x4* pv = io.pool_v;
  const int item = blockIdx.x;
  stamp_begin(rd, item);
  const WorkItem w = rd.rwork[item];
  stage_group<T>(rd, w, sh);
  MasterRows<RPW> M;
  load_master<RPW, DOV, DOK>(rd, io, w, L, M);
  bool special[RPW];
#pragma unroll
  for (int k = 0; k < RPW; ++k)
    special[k] = ((int)chunk_special(M.kl[k]) | (int)chunk_special(M.kh[k]) | (int)chunk_special(M.v0[k]) | (int)chunk_special(M.v1[k])) != 0;
  lds_barrier();
  // Rolling requests (see tdk_keydiff_kernel): the rows of the next agent are asked for as the rows of this one
  // are used up; no branch stands around a load, a request with nothing to fetch reads the first row of the
  // master page and its result is ignored.
  const int64_t first_row = (rd.sess[w.session].master_row0 + (int64_t)w.page * T) * row_u4;
  const u32x4* idle_k = DOK ? io.master_k + first_row + L.jb : nullptr;
  const u32x4* idle_v = DOV ? io.master_v + first_row + (threadIdx.x & 15) : nullptr;
  const u32x4 z = {0, 0, 0, 0};
  u32x4 akl[RPW], akh[RPW], av0[RPW], av1[RPW];
  auto request = [&](int g, int k) {
    const int64_t base = dest_row<T>(sh, max(min(g, w.ag_count - 1), 0), wave + kWaves * k) * row_u4;
    const bool ok = g < w.ag_count && M.valid[k];
    akl[k] = z; akh[k] = z; av0[k] = z; av1[k] = z;
    if (DOK) {
      akl[k] = ld16<NTL>(ok && L.kok ? pk + base + L.klo : idle_k);
      akh[k] = ld16<NTL>(ok && L.kok ? pk + base + L.khi : idle_k + 8);
    }
    if (DOV) {
      av0[k] = ld16<NTL>(ok && L.v0ok ? pv + base + L.v0 : idle_v);
      av1[k] = ld16<NTL>(ok && L.v1ok ? pv + base + L.v1 : idle_v);
    }
  };
#pragma unroll
  for (int k = 0; k < RPW; ++k) { request(0, k); __builtin_amdgcn_sched_barrier(0); }   // in the order the loop uses them
  for (int g = 0; g < w.ag_count; ++g) {
    float c[8], s[8];
    if (DOK && !SEG) load_tab<IL>(sh, g, 0, L.jb, c, s);
    bool differs = false;
#pragma unroll
    for (int k = 0; k < RPW; ++k) {
      if (M.valid[k]) {
        u32x4 rlo = z, rhi = z;
        if (DOK && SEG) load_tab<IL>(sh, g, wave + kWaves * k, L.jb, c, s);
        if (DOK) rotate16<IL>(M.kl[k], M.kh[k], c, s, rlo, rhi);
        // rows whose bits all match the reference (the common case) need no fp32 compare
        uint32_t x = 0;
        if (DOV) x |= (L.v0ok ? chunk_xor(av0[k], M.v0[k]) : 0u) | (L.v1ok ? chunk_xor(av1[k], M.v1[k]) : 0u);
        if (DOK) x |= L.kok ? chunk_xor(akl[k], rlo) | chunk_xor(akh[k], rhi) : 0u;
        if (__any((int)(x != 0) | (int)special[k])) {
          if (DOK && L.kok) {
            differs |= chunk_differs(akl[k], rlo, eps);
            differs |= chunk_differs(akh[k], rhi, eps);
          }
          if (DOV && L.v0ok) differs |= chunk_differs(av0[k], M.v0[k], eps);
          if (DOV && L.v1ok) differs |= chunk_differs(av1[k], M.v1[k], eps);
        }
      }
      request(g + 1, k);
    }
    if (__any(differs) && (threadIdx.x & 63) == 0) atomicOr(&sh.aux[g], 1);
  }
  lds_barrier();
  if (threadIdx.x < w.ag_count) {
    const AgentDev ad = rd.agents[sh.agent[threadIdx.x]];
    rd.flags[ad.flag_off + w.page] = (uint8_t)sh.aux[threadIdx.x];
  }
  stamp_end(rd, item);
}

// ---------------------------------------------------------------------------------------------
// compaction: count, exclusive prefix, ascending index list                [Sec. 5]
// One launch.  A workgroup of 16 wavefronts takes 16 consecutive agents, one per wavefront: ballot over
// 64 page flags at a time, popcount, prefix by lane mask.  The flag bytes of all agents lie one after
// another in agent order, so the number of listed pages of all earlier agents (the exclusive prefix the
// offsets need) is the number of non-zero bytes before the workgroup's first agent: every workgroup
// counts that range itself with 16-byte loads (the flags of a round are a few hundred KB, L2-resident),
// and no workgroup waits for another.
// ---------------------------------------------------------------------------------------------

constexpr int kCompactBlock = 1024;
constexpr int kCompactWaves = kCompactBlock / 64;

__device__ __forceinline__ int nonzero_bytes(uint32_t w) {
  const uint32_t t = (((w & 0x7f7f7f7fu) + 0x7f7f7f7fu) | w) & 0x80808080u;
  return __popc(t);
}

__global__ __launch_bounds__(kCompactBlock) void tdk_compact_kernel(const RoundDev rd, const DiffDev d) {
  __shared__ int64_t s_part[kCompactWaves];
  __shared__ int32_t s_cnt[kCompactWaves];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (rd.n_agents == 0) {
    if (blockIdx.x == 0 && threadIdx.x == 0) { d.offset[0] = 0; d.overflow[0] = 0; }
    return;
  }
  const int a0 = blockIdx.x * kCompactWaves;
  const int a = a0 + wave;
  // listed pages of all agents before a0: non-zero bytes of flags[0, flag_off(a0))
  const int64_t n_before = rd.agents[a0].flag_off;
  const uint8_t* fl = rd.flags;
  int64_t part = 0;
  const int64_t n16 = n_before >> 4;
  for (int64_t i = threadIdx.x; i < n16; i += kCompactBlock) {
    const u32x4 w = reinterpret_cast<const u32x4*>(fl)[i];
    part += nonzero_bytes(w[0]) + nonzero_bytes(w[1]) + nonzero_bytes(w[2]) + nonzero_bytes(w[3]);
  }
  for (int64_t i = (n16 << 4) + threadIdx.x; i < n_before; i += kCompactBlock) part += fl[i] != 0;
#pragma unroll
  for (int sft = 32; sft > 0; sft >>= 1) part += __shfl_xor(part, sft);
  // this wavefront's agent: its count
  int n = 0;
  int P = 0, flag_off = 0;
  if (a < rd.n_agents) {
    const AgentDev ad = rd.agents[a];
    P = rd.sess[ad.session].pages;
    flag_off = ad.flag_off;
    for (int p0 = 0; p0 < P; p0 += 64) {
      const int p = p0 + lane;
      const bool f = p < P && fl[flag_off + p] != 0;
      n += __popcll(__ballot(f));
    }
  }
  if (lane == 0) { s_part[wave] = part; s_cnt[wave] = n; }
  __syncthreads();
  int64_t base = 0;
#pragma unroll
  for (int q = 0; q < kCompactWaves; ++q) { base += s_part[q]; if (q < wave) base += s_cnt[q]; }
  if (a >= rd.n_agents) return;
  if (lane == 0) {
    d.count[a] = n;
    d.offset[a] = base;
    if (a == rd.n_agents - 1) {
      const int64_t total = base + n;
      d.offset[a + 1] = total;
      d.overflow[0] = total > d.capacity ? 1 : 0;
    }
  }
  int64_t run = base;
  for (int p0 = 0; p0 < P; p0 += 64) {
    const int p = p0 + lane;
    const bool f = p < P && fl[flag_off + p] != 0;
    const uint64_t b = __ballot(f);
    const int rank = __popcll(b & ((1ull << lane) - 1ull));
    if (f && run + rank < d.capacity) d.idx[run + rank] = p;
    run += __popcll(b);
  }
}

// ---------------------------------------------------------------------------------------------
// gather: K/V values of the listed pages, as they sit in the agent's cache   [Sec. 5]
// A workgroup copies one plane (K or V) of one payload slot; grid-stride over the slots that
// exist, so the host never needs the count.
// ---------------------------------------------------------------------------------------------

// Shared by gather and scatter.  A workgroup moves one payload slot (K plane, then V plane).
// Prologue: all threads search offset[] in parallel for the agent that owns the slot (one memory
// round trip per 256 agents instead of a serial binary search), then T threads resolve the pool
// row of each row of the page through the block table.
struct SlotShared {
  int32_t owner;
  int64_t row[32];     // pool row of each row of the page, -1 past the span / not listed
};

__device__ __forceinline__ void find_owner(const DiffDev& d, int A, int64_t slot, SlotShared& sh) {
  for (int a = threadIdx.x; a < A; a += kBlock)
    if (d.offset[a] <= slot && slot < d.offset[a + 1]) sh.owner = a;
}

constexpr int kCopyBatch = 4;   // 16-byte accesses per thread in flight in gather / scatter

// planes: bit 0 = K, bit 1 = V; a slot holds the selected planes back to back
__global__ __launch_bounds__(kBlock) void tdk_gather_kernel(const RoundDev rd, const LayerDev io, const DiffDev d,
                                                            const int planes) {
  __shared__ SlotShared sh;
  const int T = rd.page_tokens;
  const int A = rd.n_agents;
  if (A == 0) return;
  int64_t total = d.offset[A];
  if (total > d.capacity) total = d.capacity;
  const int row_u4 = rd.heads * 16;
  const int page_u4 = T * row_u4;
  for (int64_t slot = blockIdx.x; slot < total; slot += gridDim.x) {
    find_owner(d, A, slot, sh);
    __syncthreads();
    if (threadIdx.x < T) {
      const AgentDev ad = rd.agents[sh.owner];
      const int m = d.idx[slot] * T + threadIdx.x;
      int64_t row = -1;
      if (m < rd.sess[ad.session].span) {
        const int a0 = ad.pos0 + m;
        row = rd.seg ? (int64_t)rd.rowmap[ad.score_off + m]
                     : (int64_t)rd.bt[ad.bt_off + a0 / T - ad.lp_first] * T + a0 % T;
      }
      sh.row[threadIdx.x] = row;
    }
    __syncthreads();
    const int n_planes = planes == 3 ? 2 : 1;
#pragma unroll 1
    for (int plane = 0; plane < 2; ++plane) {
      if (!((planes >> plane) & 1)) continue;
      const u32x4* src = plane ? io.pool_v : io.pool_k;
      u32x4* dst = d.payload + (slot * n_planes + (planes == 3 ? plane : 0)) * (int64_t)page_u4;
      for (int i0 = threadIdx.x; i0 < page_u4; i0 += kBlock * kCopyBatch) {
        u32x4 v[kCopyBatch];
#pragma unroll
        for (int j = 0; j < kCopyBatch; ++j) {
          const int i = i0 + j * kBlock;
          const u32x4 z = {0, 0, 0, 0};
          v[j] = z;
          if (i < page_u4) {
            const int r = i / row_u4;
            const int64_t row = sh.row[r];
            if (row >= 0) v[j] = (rd.nontemporal & 16) ? __builtin_nontemporal_load(src + row * row_u4 + (i - r * row_u4))
                                                       : src[row * row_u4 + (i - r * row_u4)];
          }
        }
#pragma unroll
        for (int j = 0; j < kCopyBatch; ++j) {
          const int i = i0 + j * kBlock;
          if (i < page_u4) {
            if (rd.nontemporal & 16) st16<true>(dst + i, v[j]);
            else dst[i] = v[j];
          }
        }
      }
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------------
// decode: diff pages from the payload, all others from the re-rotated master   [Sec. 4.4, Alg. 1]
// ---------------------------------------------------------------------------------------------

// The "correct" half of skip-or-correct: pages listed in a diff are copied from the payload to the
// agent's rows (the mirror image of the gather kernel).  Every pool row is written exactly once by
// either this kernel or the page kernel above, so their order does not matter.
struct ScatterShared {
  SlotShared sh;
  float s_tab[2][2 * kHalf];    // cos/sin of the payload re-rotation: up to two segments meet a page
  uint32_t s_sel, s_moved;      // bit r of s_sel: row r uses table 1; bit t of s_moved: table t is not the identity
};

// Workgroup `first` of `stride` workgroups: walks the payload slots first, first + stride, ...
template <bool IL>
__device__ __forceinline__ void scatter_slots(const RoundDev& rd, const LayerDev& io, const DiffDev& d, const int planes,
                                              ScatterShared& ss, const int64_t first, const int64_t stride) {
  SlotShared& sh = ss.sh;
  float (&s_tab)[2][2 * kHalf] = ss.s_tab;
  uint32_t& s_sel = ss.s_sel;
  uint32_t& s_moved = ss.s_moved;
  const int T = rd.page_tokens;
  const int A = rd.n_agents;
  if (A == 0) return;
  int64_t total = d.offset[A];
  if (total > d.capacity) total = d.capacity;
  const int row_u4 = rd.heads * 16;
  const int page_u4 = T * row_u4;
  const Lane L = lane_geometry(rd.heads);
  for (int64_t slot = first; slot < total; slot += stride) {
    if (threadIdx.x == 0) sh.owner = -1;
    __syncthreads();
    find_owner(d, A, slot, sh);
    __syncthreads();
    bool rot = false;
    int t0 = 0, t1 = 0;
    const float* tabs = rd.tab_diff;
    if (sh.owner >= 0 && rd.agents[sh.owner].diff_rot != 0) {
      // which stored-frame -> current-frame rotations this page needs
      const AgentDev ad = rd.agents[sh.owner];
      const int p = d.idx[slot];
      uint32_t sel = 0, moved = 1;
      t0 = t1 = sh.owner;
      if (rd.seg) {
        moved = 0;
        if (p >= 0 && p < rd.sess[ad.session].pages) {
          const PageTab pt = rd.pagetab[ad.flag_off + p];
          t0 = pt.x; t1 = pt.y; sel = (uint32_t)pt.z; moved = (uint32_t)pt.w;
          tabs = rd.segtab_diff;
        }
      }
      rot = moved != 0;
      if (threadIdx.x == 0) { s_sel = sel; s_moved = moved; }
    }
    if (threadIdx.x < T) {
      int64_t row = -1;
      if (sh.owner >= 0) {                       // an inconsistent offset[] leaves the slot unowned
        const AgentDev ad = rd.agents[sh.owner];
        const SessionDev sd = rd.sess[ad.session];
        const int p = d.idx[slot];
        const int m = p * T + threadIdx.x;
        if (p >= 0 && p < sd.pages && m < sd.span) {   // anything else is not an index this round produces
          const int a0 = ad.pos0 + m;
          row = rd.seg ? (int64_t)rd.rowmap[ad.score_off + m]
                       : (int64_t)rd.bt[ad.bt_off + a0 / T - ad.lp_first] * T + a0 % T;
        }
      }
      sh.row[threadIdx.x] = row;
    }
    if (rot) {
      const int which = threadIdx.x >> 7, e = threadIdx.x & (2 * kHalf - 1);
      s_tab[which][e] = tabs[(size_t)(which ? t1 : t0) * (2 * kHalf) + e];
    }
    __syncthreads();
    const int n_planes = planes == 3 ? 2 : 1;
#pragma unroll 1
    for (int plane = 0; plane < 2; ++plane) {
      if (!((planes >> plane) & 1)) continue;
      u32x4* dst = plane ? io.pool_v : io.pool_k;
      const u32x4* src = d.payload + (slot * n_planes + (planes == 3 ? plane : 0)) * (int64_t)page_u4;
      if (plane == 0 && rot) {
        // stored at another position: K rows are re-rotated, a wavefront per row, both members of a
        // pair in one lane (the page kernels' lane layout)
        for (int r = threadIdx.x >> 6; r < T; r += kWaves) {
          const int64_t row = sh.row[r];
          if (row < 0 || !L.kok) continue;
          const int which = (s_sel >> r) & 1u;
          u32x4 olo = src[r * row_u4 + L.klo], ohi = src[r * row_u4 + L.khi];
          if ((s_moved >> which) & 1u) {           // a run that did not move is a bit copy
            const float* t = s_tab[which];
            float c[8], sn[8];
            if (!IL) {
#pragma unroll
              for (int e = 0; e < 8; ++e) { c[e] = t[L.jb * 8 + e]; sn[e] = t[kHalf + L.jb * 8 + e]; }
            } else {
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                c[e] = t[L.jb * 4 + e];          sn[e] = t[kHalf + L.jb * 4 + e];
                c[4 + e] = t[32 + L.jb * 4 + e]; sn[4 + e] = t[kHalf + 32 + L.jb * 4 + e];
              }
            }
            rotate16<IL>(olo, ohi, c, sn, olo, ohi);
          }
          dst[row * row_u4 + L.klo] = olo;
          dst[row * row_u4 + L.khi] = ohi;
        }
        continue;
      }
      for (int i0 = threadIdx.x; i0 < page_u4; i0 += kBlock * kCopyBatch) {
        u32x4 v[kCopyBatch];
#pragma unroll
        for (int j = 0; j < kCopyBatch; ++j) {
          const int i = i0 + j * kBlock;
          const u32x4 z = {0, 0, 0, 0};
          v[j] = z;
          if (i < page_u4) v[j] = (rd.nontemporal & 8) ? __builtin_nontemporal_load(src + i) : src[i];
        }
#pragma unroll
        for (int j = 0; j < kCopyBatch; ++j) {
          const int i = i0 + j * kBlock;
          if (i < page_u4) {
            const int r = i / row_u4;
            const int64_t row = sh.row[r];
            if (row >= 0) {
              if (rd.nontemporal & 8) st16<true>(dst + row * row_u4 + (i - r * row_u4), v[j]);
              else dst[row * row_u4 + (i - r * row_u4)] = v[j];
            }
          }
        }
      }
    }
    __syncthreads();
  }
}

template <bool IL>
__global__ __launch_bounds__(kBlock) void tdk_scatter_kernel(const RoundDev rd, const LayerDev io, const DiffDev d,
                                                             const int planes) {
  __shared__ ScatterShared ss;
  scatter_slots<IL>(rd, io, d, planes, ss, blockIdx.x, gridDim.x);
}

template <int RPW, bool IL, bool NT, int PM, bool SEG, bool Q>
__global__ __launch_bounds__(kBlock) void tdk_decode_kernel(const RoundDev rd, const LayerDev io, const DiffDev d,
                                                            const int n_scatter) {
  constexpr int T = RPW * kWaves;
  __shared__ std::conditional_t<SEG, GroupSharedSeg, GroupShared> sh;
  __shared__ int s_item;
  constexpr bool DOK = (PM & 1) != 0, DOV = (PM & 2) != 0;
  if (!Q && (int)blockIdx.x >= rd.dyn_begin + rd.dyn_count) {
    // Small rounds only (static launches that do not fill the chip for long): the workgroups that copy the listed
    // pages from the payload ride behind the page items of the same launch, n_scatter of them, and run while the
    // page items drain, instead of paying for a launch of their own.  (On large rounds two launches are faster:
    // payload reads among the page items' writes cost more than the second launch.)
    __shared__ ScatterShared ss;
    scatter_slots<IL>(rd, io, d, PM, ss, (int64_t)blockIdx.x - (rd.dyn_begin + rd.dyn_count), n_scatter);
    return;
  }
  const Lane L = lane_geometry(rd.heads);
  if (rd.nontemporal & 64) sweep_masters(rd, io, DOK, DOV);
  const int wave = threadIdx.x >> 6;
  const int64_t row_u4 = (int64_t)rd.heads * 16;
  u32x4* pk = io.pool_k;
  u32x4* pv = io.pool_v;
  Items<Q> items;
  for (int item = items.first(rd, &s_item); item >= 0; item = items.next(rd, &s_item)) {
    stamp_begin(rd, item);
    const WorkItem w = items.at(rd, item);
    stage_group<T>(rd, w, sh);
    MasterRows<RPW> M;
    load_master<RPW, DOV, DOK>(rd, io, w, L, M);
    if (threadIdx.x < w.ag_count) {
      // skip-or-correct decision per block: is this page in the agent's index list?
      const int a = rd.order[w.ag_begin + threadIdx.x];
      int64_t lo = d.offset[a];
      int64_t hi = lo + d.count[a];
      if (lo < 0) lo = 0;
      if (hi > d.capacity) hi = d.capacity;
      int64_t slot = -1;
      while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        const int v = d.idx[mid];
        if (v == w.page) { slot = mid; break; }
        if (v < w.page) lo = mid + 1; else hi = mid;
      }
      sh.aux[threadIdx.x] = (int32_t)slot;
    }
    lds_barrier();
    items.prefetch(rd);
    for (int g = 0; g < w.ag_count; ++g) {
      if (sh.aux[g] >= 0) continue;   // listed in the diff: the scatter kernel writes this page
      float c[8], s[8];
      if (DOK && !SEG) load_tab<IL>(sh, g, 0, L.jb, c, s);
#pragma unroll
      for (int k = 0; k < RPW; ++k) {
        if (!M.valid[k]) continue;
        const int64_t base = dest_row<T>(sh, g, wave + kWaves * k) * row_u4;
        if (DOK && L.kok) {
          if (SEG) load_tab<IL>(sh, g, wave + kWaves * k, L.jb, c, s);
          u32x4 olo, ohi;
          rotate16<IL>(M.kl[k], M.kh[k], c, s, olo, ohi);
          st16<NT>(pk + base + L.klo, olo);
          st16<NT>(pk + base + L.khi, ohi);
        }
        if (DOV && L.v0ok) st16<NT>(pv + base + L.v0, M.v0[k]);
        if (DOV && L.v1ok) st16<NT>(pv + base + L.v1, M.v1[k]);
      }
    }
    stamp_end(rd, item);
  }
  items.leave(rd);
}

// ---------------------------------------------------------------------------------------------
// plain copy / fill (bandwidth ceiling and traffic-counter reference)
// ---------------------------------------------------------------------------------------------

// Plain copy with the streaming policy on both sides (the fastest copy measured on this chip).
__global__ __launch_bounds__(kBlock) void tdk_copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src, size_t n) {
  for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock)
    st16<true>(dst + i, ld16<true>(src + i));
}

__global__ __launch_bounds__(kBlock) void tdk_fill_kernel(u32x4* __restrict__ dst, uint32_t word, size_t n) {
  const u32x4 v = {word, word, word, word};
  for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock) dst[i] = v;
}

// ---------------------------------------------------------------------------------------------
// check layer: batched key-difference pass, important positions, master choice   [Sec. 4.2]
// ---------------------------------------------------------------------------------------------

// Sum of v over the 64 lanes of a wavefront with DPP row shifts and row broadcasts (no LDS
// traffic); the total is valid in lane 63 only.
__device__ __forceinline__ float wave_sum_to_lane63(float v) {
  auto dpp = [](float x, auto ctrl, auto row_mask) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value,
                                                                   decltype(row_mask)::value, 0xf, false));
  };
  v += dpp(v, std::integral_constant<int, 0x111>{}, std::integral_constant<int, 0xf>{});   // row_shr:1
  v += dpp(v, std::integral_constant<int, 0x112>{}, std::integral_constant<int, 0xf>{});   // row_shr:2
  v += dpp(v, std::integral_constant<int, 0x114>{}, std::integral_constant<int, 0xf>{});   // row_shr:4
  v += dpp(v, std::integral_constant<int, 0x118>{}, std::integral_constant<int, 0xf>{});   // row_shr:8 -> lane 15 of each row
  v += dpp(v, std::integral_constant<int, 0x142>{}, std::integral_constant<int, 0xa>{});   // row_bcast:15 into rows 1, 3
  v += dpp(v, std::integral_constant<int, 0x143>{}, std::integral_constant<int, 0xc>{});   // row_bcast:31 into rows 2, 3
  return v;
}

// Per (agent, token): sum over the row of (fresh K - rotated cached K)^2, fp32.  Same traversal as
// the compare kernel, K plane only.  Twice the arithmetic per byte of the compare kernel and only half a
// page per agent in flight, so the loads of one agent must overlap the arithmetic of the one before: see the
// rolling requests below (482 -> 415 us on 250 agents x 5000 tokens; at a budget of 128 registers the compiler
// spills, and a reload from scratch waits for every load issued before it, so the kernel runs at 3 waves per SIMD).
template <int RPW, bool IL, bool SEG, bool NTL>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(RPW == 4 ? 3 : 1))) void tdk_keydiff_kernel(const RoundDev rd, const LayerDev io, const PlanDev pl) {
  constexpr int T = RPW * kWaves;
  __shared__ std::conditional_t<SEG, GroupSharedSeg, GroupShared> sh;
  __shared__ float s_score[kMaxGroup][T];
  const Lane L = lane_geometry(rd.heads);
  const int wave = threadIdx.x >> 6;
  const int64_t row_u4 = (int64_t)rd.heads * 16;
  const u32x4* pk = io.pool_k;
  const WorkItem w = rd.rwork[blockIdx.x];
  stage_group<T>(rd, w, sh);
  MasterRows<RPW> M;
  load_master<RPW, false>(rd, io, w, L, M);
  if (threadIdx.x < w.ag_count) sh.aux[threadIdx.x] = rd.agents[sh.agent[threadIdx.x]].score_off;   // (own entry of sh.agent)
  lds_barrier();
  // Rolling requests: row k of the next agent is asked for as soon as row k of this one has been used, into the
  // registers that just became free, so a wavefront keeps its eight 16-byte loads per lane in flight all the
  // time instead of only between two arithmetic phases.  The loop body has no branch around a load: a request
  // that has nothing to fetch (a row past the span, a lane past the heads, the agent after the last) reads the
  // first row of the master page instead, and its result is not used; with straight-line code the compiler
  // counts the outstanding loads exactly and waits for the oldest pair only.
  const u32x4* idle = io.master_k + (rd.sess[w.session].master_row0 + (int64_t)w.page * T) * row_u4 + L.jb;
  u32x4 akl[RPW], akh[RPW];
  auto request = [&](int g, int k) {
    const int64_t base = dest_row<T>(sh, max(min(g, w.ag_count - 1), 0), wave + kWaves * k) * row_u4;
    const bool ok = g < w.ag_count && M.valid[k] && L.kok;
    const u32x4* lo = ok ? pk + base + L.klo : idle;
    const u32x4* hi = ok ? pk + base + L.khi : idle + 8;
    akl[k] = ld16<NTL>(lo); akh[k] = ld16<NTL>(hi);
  };
#pragma unroll
  for (int k = 0; k < RPW; ++k) { request(0, k); __builtin_amdgcn_sched_barrier(0); }   // in the order the loop uses them
  for (int g = 0; g < w.ag_count; ++g) {
    float c[8], s[8];
    if (!SEG) load_tab<IL>(sh, g, 0, L.jb, c, s);
#pragma unroll
    for (int k = 0; k < RPW; ++k) {
      if (SEG) load_tab<IL>(sh, g, wave + kWaves * k, L.jb, c, s);
      u32x4 rlo, rhi;
      rotate16<IL>(M.kl[k], M.kh[k], c, s, rlo, rhi);
      float acc = 0.f;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float d0 = bf_lo(akl[k][q]) - bf_lo(rlo[q]), d1 = bf_hi(akl[k][q]) - bf_hi(rlo[q]);
        float d2 = bf_lo(akh[k][q]) - bf_lo(rhi[q]), d3 = bf_hi(akh[k][q]) - bf_hi(rhi[q]);
        acc = __builtin_fmaf(d0, d0, acc); acc = __builtin_fmaf(d1, d1, acc);
        acc = __builtin_fmaf(d2, d2, acc); acc = __builtin_fmaf(d3, d3, acc);
      }
      request(g + 1, k);
      acc = wave_sum_to_lane63(L.kok ? acc : 0.f);
      if ((threadIdx.x & 63) == 63) s_score[g][wave + kWaves * k] = acc;   // (no store to memory among the loads: the count of outstanding accesses stays exact)
    }
  }
  lds_barrier();
  const int rows = min(T, rd.sess[w.session].span - w.page * T);
  for (int i = threadIdx.x; i < w.ag_count * T; i += kBlock) {
    const int g = i / T, r = i - g * T;
    if (r < rows) pl.score[sh.aux[g] + w.page * T + r] = s_score[g][r];
  }
}

// rank of a set flag among the set flags of the workgroup (threads in order) and their total
__device__ __forceinline__ int block_rank(bool f, int* s_wave, int& total) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const uint64_t b = __ballot(f);
  const int in_wave = __popcll(b & ((1ull << lane) - 1ull));
  __syncthreads();
  if (lane == 0) s_wave[wave] = __popcll(b);
  __syncthreads();
  int before = 0;
  total = 0;
#pragma unroll
  for (int q = 0; q < kWaves; ++q) { const int c = s_wave[q]; if (q < wave) before += c; total += c; }
  return before + in_wave;
}

// Important positions of one agent: the k = ceil(ratio * S) tokens with the largest score among those
// with !(score <= min_score), ties towards the lower token index, listed in ascending token order.
// Radix select on the fp32 bit patterns (non-negative floats order like unsigned integers; NaN sorts
// above everything), then an ordered compaction.  Also the agent's total deviation.
__global__ __launch_bounds__(kBlock) void tdk_select_kernel(const RoundDev rd, const PlanDev pl) {
  static_assert(kBlock == 256, "one thread per radix bin: hist[threadIdx.x] and the suffix scan assume 256 threads");
  __shared__ uint32_t hist[256];
  __shared__ int s_wave[kWaves];
  __shared__ float s_sum[kWaves];
  __shared__ uint32_t s_prefix, s_need;
  const int a = blockIdx.x;
  const AgentDev ad = rd.agents[a];
  const int S = rd.sess[ad.session].span;
  const float* sc = pl.score + ad.score_off;
  const float min_score = pl.min_score;
  auto key_of = [&](int m) -> uint32_t {
    const float v = sc[m];
    return !(v <= min_score) ? (__float_as_uint(v) & 0x7fffffffu) : 0u;
  };
  // total deviation and the number of candidates
  float part = 0.f;
  int cand = 0;
  for (int m = threadIdx.x; m < S; m += kBlock) { part += sc[m]; cand += key_of(m) != 0u; }
#pragma unroll
  for (int sft = 32; sft > 0; sft >>= 1) { part += __shfl_xor(part, sft); cand += __shfl_xor(cand, sft); }
  if ((threadIdx.x & 63) == 0) { s_sum[threadIdx.x >> 6] = part; s_wave[threadIdx.x >> 6] = cand; }
  __syncthreads();
  float total = 0.f;
  int n_cand = 0;
#pragma unroll
  for (int q = 0; q < kWaves; ++q) { total += s_sum[q]; n_cand += s_wave[q]; }
  if (threadIdx.x == 0) pl.total[a] = total;
  int64_t k = (int64_t)ceil((double)pl.ratio * (double)S);
  if (k > S) k = S;
  if (k > pl.k_stride) k = pl.k_stride;
  if (k > n_cand) k = n_cand;
  if (k <= 0) {
    if (threadIdx.x == 0) pl.n_important[a] = 0;
    return;
  }
  // radix select: the key of the k-th largest candidate, 8 bits at a time from the top
  if (threadIdx.x == 0) { s_prefix = 0u; s_need = (uint32_t)k; }
  uint32_t mask = 0u;
  for (int shift = 24; shift >= 0; shift -= 8) {
    hist[threadIdx.x] = 0u;
    __syncthreads();
    const uint32_t prefix = s_prefix;
    for (int m = threadIdx.x; m < S; m += kBlock) {
      const uint32_t key = key_of(m);
      if (key != 0u && (key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    {
      // the bin that holds the need-th largest key: thread t looks after bin t and knows, from a suffix scan
      // over the 256 counts, how many keys lie in the bins above it; exactly one bin has above < need <= above + own
      const uint32_t need = s_need, own = hist[threadIdx.x];
      const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
      uint32_t inc = own;                                   // own + the higher bins of this wavefront
#pragma unroll
      for (int sft = 1; sft < 64; sft <<= 1) {
        const uint32_t v = __shfl_down(inc, sft);
        if (lane + sft < 64) inc += v;
      }
      if (lane == 0) s_wave[wv] = (int)inc;                 // the wavefront's total
      __syncthreads();
      uint32_t above = inc - own;
#pragma unroll
      for (int q = 0; q < kWaves; ++q)
        if (q > wv) above += (uint32_t)s_wave[q];
      if (above < need && above + own >= need) {
        s_need = need - above;
        s_prefix = prefix | ((uint32_t)threadIdx.x << shift);
      }
    }
    mask |= 255u << shift;
    __syncthreads();
  }
  const uint32_t tkey = s_prefix;
  const int need_eq = (int)s_need;     // how many tokens equal to the threshold key are taken (the first ones)
  int done_eq = 0, done_sel = 0;
  int32_t* out = pl.important + (int64_t)a * pl.k_stride;
  for (int m0 = 0; m0 < S; m0 += kBlock) {
    const int m = m0 + threadIdx.x;
    const uint32_t key = m < S ? key_of(m) : 0u;
    const bool gt = key > tkey, eq = key != 0u && key == tkey;
    int tot_eq, tot_sel;
    const int r_eq = block_rank(eq, s_wave, tot_eq);
    const bool sel = gt | (eq && done_eq + r_eq < need_eq);
    const int r_sel = block_rank(sel, s_wave, tot_sel);
    if (sel) out[done_sel + r_sel] = m;
    done_eq += tot_eq;
    done_sel += tot_sel;
  }
  if (threadIdx.x == 0) pl.n_important[a] = done_sel;
}

// Master of each session: the agent with the lowest total deviation (NaN counts as +inf; ties go to
// the agent listed first).  One wavefront per session.
__global__ __launch_bounds__(kBlock) void tdk_master_kernel(const RoundDev rd, const PlanDev pl) {
  const int s = blockIdx.x * kWaves + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (s >= rd.n_sessions) return;
  const SessionDev sd = rd.sess[s];
  float best = __builtin_inff();
  int best_i = 0x7fffffff;
  for (int q = lane; q < sd.n_agents; q += 64) {
    const int a = rd.order[sd.order_begin + q];
    float t = pl.total[a];
    if (t != t) t = __builtin_inff();
    if (t < best || (t == best && a < best_i)) { best = t; best_i = a; }
  }
#pragma unroll
  for (int sft = 32; sft > 0; sft >>= 1) {
    const float ob = __shfl_xor(best, sft);
    const int oi = __shfl_xor(best_i, sft);
    if (ob < best || (ob == best && oi < best_i)) { best = ob; best_i = oi; }
  }
  if (lane == 0) pl.master[s] = sd.n_agents ? best_i : -1;
}

// Access-pattern probes: the page kernels' memory accesses with no arithmetic and no master.
// Plain form: one workgroup per page, contiguous 4 KB per step, ordinary stores / dependent loads.
__global__ __launch_bounds__(kBlock) void tdk_page_fill_kernel(u32x4* __restrict__ dst, const int32_t* __restrict__ ids,
                                                              int page_u4, uint32_t word) {
  const u32x4 v = {word, word, word, word};
  u32x4* p = dst + (size_t)ids[blockIdx.x] * page_u4;
  for (int i = threadIdx.x; i < page_u4; i += kBlock) p[i] = v;
}

__global__ __launch_bounds__(kBlock) void tdk_page_read_kernel(const u32x4* __restrict__ src, const int32_t* __restrict__ ids,
                                                              int page_u4, u32x4* __restrict__ sink) {
  const u32x4* p = src + (size_t)ids[blockIdx.x] * page_u4;
  u32x4 acc = {0, 0, 0, 0};
  for (int i = threadIdx.x; i < page_u4; i += kBlock) acc ^= p[i];
  // never true for the probe's fill pattern; keeps the loads alive
  if (acc[0] == 0x9e3779b9u && acc[1] == 0x7f4a7c15u) sink[0] = acc;
}

// Product form: exactly the traversal of the page kernels.  A workgroup takes `group` pages of the id list (as
// a work item takes a group of agents); its four wavefronts own interleaved rows; a lane touches the two
// halves of a head row in the K plane and two chunks 1 KB apart in the V plane; streaming stores / non-temporal
// loads; all 16 accesses of a wavefront's rows of one page are issued before anything waits for them.
template <int RPW>
__global__ __launch_bounds__(kBlock) void tdk_page_fill_product_kernel(u32x4* __restrict__ pk, u32x4* __restrict__ pv,
                                                                      const int32_t* __restrict__ ids, int n_pages, int group,
                                                                      int heads, uint32_t word) {
  constexpr int T = RPW * kWaves;
  const Lane L = lane_geometry(heads);
  const int wave = threadIdx.x >> 6;
  const int64_t row_u4 = (int64_t)heads * 16;
  const u32x4 v = {word, word ^ threadIdx.x, word, blockIdx.x};
  for (int g = 0; g < group; ++g) {
    const int64_t q = (int64_t)blockIdx.x * group + g;
    if (q >= n_pages) break;
    const int64_t page = ids[q];
#pragma unroll
    for (int k = 0; k < RPW; ++k) {
      const int64_t base = (page * T + wave + kWaves * k) * row_u4;
      if (L.kok) { st16<true>(pk + base + L.klo, v); st16<true>(pk + base + L.khi, v); }
      if (L.v0ok) st16<true>(pv + base + L.v0, v);
      if (L.v1ok) st16<true>(pv + base + L.v1, v);
    }
  }
}

template <int RPW>
__global__ __launch_bounds__(kBlock) void tdk_page_read_product_kernel(const u32x4* __restrict__ pk, const u32x4* __restrict__ pv,
                                                                      const int32_t* __restrict__ ids, int n_pages, int group,
                                                                      int heads, u32x4* __restrict__ sink) {
  constexpr int T = RPW * kWaves;
  const Lane L = lane_geometry(heads);
  const int wave = threadIdx.x >> 6;
  const int64_t row_u4 = (int64_t)heads * 16;
  u32x4 acc = {0, 0, 0, 0};
  for (int g = 0; g < group; ++g) {
    const int64_t q = (int64_t)blockIdx.x * group + g;
    if (q >= n_pages) break;
    const int64_t page = ids[q];
    u32x4 a[RPW][4];
    const u32x4 z = {0, 0, 0, 0};
#pragma unroll
    for (int k = 0; k < RPW; ++k) {
      const int64_t base = (page * T + wave + kWaves * k) * row_u4;
      a[k][0] = z; a[k][1] = z; a[k][2] = z; a[k][3] = z;
      if (L.kok) { a[k][0] = ld16<true>(pk + base + L.klo); a[k][1] = ld16<true>(pk + base + L.khi); }
      if (L.v0ok) a[k][2] = ld16<true>(pv + base + L.v0);
      if (L.v1ok) a[k][3] = ld16<true>(pv + base + L.v1);
    }
#pragma unroll
    for (int k = 0; k < RPW; ++k) acc ^= a[k][0] ^ a[k][1] ^ a[k][2] ^ a[k][3];
  }
  if (acc[0] == 0x9e3779b9u && acc[1] == 0x7f4a7c15u) sink[0] = acc;
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------

// Launch of a page kernel that writes (rerotate, decode).  Static distribution: one workgroup per work item.
// Queued (TDK_TUNE_XCD_QUEUES, and only when every resident workgroup gets at least four items: below that the
// launch is over before an imbalance between the XCDs can build up, and the hardware's own dispatch of fresh
// workgroups fills freed wavefront slots sooner than a looping workgroup does): two workgroups per compute unit
// that loop over the items (see below).  `queued_kernel` / `static_kernel` are the two instantiations.
// `extra` static workgroups behind the page items (decode's payload copies on small rounds); returns whether they
// were launched (only the static form takes them).
template <class KernelQ, class KernelS, class... Args>
static bool launch_write_pages(const RoundDev& rd, KernelQ queued_kernel, KernelS static_kernel, int extra, hipStream_t st, Args... args) {
  int n = 0;
  {
    static std::mutex mu;
    static std::map<const void*, int> per_cu;
    std::lock_guard<std::mutex> lock(mu);
    const void* id = reinterpret_cast<const void*>(queued_kernel);
    auto it = per_cu.find(id);
    if (it == per_cu.end()) {
      if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, queued_kernel, kBlock, 0) != hipSuccess || n < 1) n = 2;
      per_cu[id] = n;
    } else {
      n = it->second;
    }
  }
  const int64_t resident = (int64_t)n * std::max(rd.n_cus, 1);
  // long enough for the looping form: at least four items and at least 32 (agent, page) pairs per resident
  // workgroup (a round cut into many small items, such as one agent per item, is no longer than its pairs)
  const bool large = (int64_t)rd.n_work >= 4 * resident && rd.agent_pages >= 32 * resident;
  if ((rd.nontemporal & 128) && (large || (rd.nontemporal & 512))) {
    // Two looping workgroups per compute unit, although three fit: memory is saturated with one per unit already,
    // and the fewer pages are being written at a time, the better DRAM takes it (batched250: decode 876 us with
    // three per unit, 868 with two, 860 with one; rerotate 958 / 953 / 962; `long` loses 7 % with one).
    const int64_t looping = std::min<int64_t>(resident, 2 * (int64_t)std::max(rd.n_cus, 1));
    hipLaunchKernelGGL(queued_kernel, dim3((unsigned)std::min<int64_t>(rd.n_work, looping)), dim3(kBlock), 0, st, rd, args...);
    return false;
  }
  const bool ride = extra > 0 && !large && (rd.nontemporal & 1024);
  RoundDev rs = rd;
  rs.dyn_begin = rd.n_work;
  rs.dyn_count = 0;
  if ((rd.nontemporal & 2048) && rd.n_work >= 64) {
    // the last fifth of the items is shared (see Items::first); twice as many workgroups as items stand by for it
    const int tail = rd.n_work / 5;
    rs.dyn_begin = rd.n_work - tail;
    rs.dyn_count = 2 * tail;
  }
  hipLaunchKernelGGL(static_kernel, dim3((unsigned)(rs.dyn_begin + rs.dyn_count) + (ride ? (unsigned)extra : 0u)), dim3(kBlock), 0, st, rs, args...);
  return ride;
}

template <int V> using ic = std::integral_constant<int, V>;

template <class F> static void with_rpw(int page_tokens, F f) { if (page_tokens == 16) f(ic<4>{}); else f(ic<8>{}); }
template <class F> static void with_bool(bool b, F f) { if (b) f(std::true_type{}); else f(std::false_type{}); }
template <class F> static void with_planes(int planes, F f) {
  if (planes == 1) f(ic<1>{}); else if (planes == 2) f(ic<2>{}); else f(ic<3>{});
}

hipError_t launch_rerotate(const RoundDev& rd, const LayerDev& io, hipStream_t st) {
  if (rd.n_work == 0) return hipSuccess;
  with_rpw(rd.page_tokens, [&](auto rpw) { with_bool(rd.interleaved != 0, [&](auto il) { with_bool((rd.nontemporal & 1) != 0, [&](auto nt) {
    with_bool(rd.seg != 0, [&](auto sg) {
      launch_write_pages(rd, tdk_rerotate_kernel<decltype(rpw)::value, decltype(il)::value, decltype(nt)::value, decltype(sg)::value, true>,
                         tdk_rerotate_kernel<decltype(rpw)::value, decltype(il)::value, decltype(nt)::value, decltype(sg)::value, false>, 0, st, io);
    });
  }); }); });
  return hipGetLastError();
}

hipError_t launch_flag(const RoundDev& rd, const LayerDev& io, float eps, int planes, hipStream_t st) {
  if (rd.n_work == 0) return hipSuccess;
  with_rpw(rd.page_tokens, [&](auto rpw) { with_bool(rd.interleaved != 0, [&](auto il) { with_planes(planes, [&](auto pm) {
    with_bool(rd.seg != 0, [&](auto sg) { with_bool((rd.nontemporal & 4) != 0, [&](auto ntl) {
      hipLaunchKernelGGL((tdk_flag_kernel<decltype(rpw)::value, decltype(il)::value, decltype(pm)::value, decltype(sg)::value, decltype(ntl)::value>),
                         dim3(rd.n_rwork), dim3(kBlock), 0, st, rd, io, eps);
    }); });
  }); }); });
  return hipGetLastError();
}

hipError_t launch_compact(const RoundDev& rd, const DiffDev& d, hipStream_t st) {
  const dim3 grid(rd.n_agents ? (rd.n_agents + kCompactWaves - 1) / kCompactWaves : 1);
  hipLaunchKernelGGL(tdk_compact_kernel, grid, dim3(kCompactBlock), 0, st, rd, d);
  return hipGetLastError();
}

hipError_t launch_gather(const RoundDev& rd, const LayerDev& io, const DiffDev& d, int planes, int grid_size, hipStream_t st) {
  if (rd.n_agents == 0 || d.capacity == 0 || grid_size <= 0) return hipSuccess;
  hipLaunchKernelGGL(tdk_gather_kernel, dim3(grid_size), dim3(kBlock), 0, st, rd, io, d, planes);
  return hipGetLastError();
}

// scatter_blocks > 0: so many workgroups may ride behind the page items to copy the listed pages; *scattered says
// whether they did (then no separate scatter launch is needed)
hipError_t launch_decode(const RoundDev& rd, const LayerDev& io, const DiffDev& d, int planes, int scatter_blocks, bool* scattered,
                         hipStream_t st) {
  *scattered = false;
  if (rd.n_work == 0) return hipSuccess;
  if (rd.n_agents == 0 || d.capacity == 0) scatter_blocks = 0;
  with_rpw(rd.page_tokens, [&](auto rpw) { with_bool(rd.interleaved != 0, [&](auto il) { with_bool((rd.nontemporal & 2) != 0, [&](auto nt) {
    with_planes(planes, [&](auto pm) { with_bool(rd.seg != 0, [&](auto sg) {
      *scattered = launch_write_pages(rd, tdk_decode_kernel<decltype(rpw)::value, decltype(il)::value, decltype(nt)::value, decltype(pm)::value, decltype(sg)::value, true>,
                                      tdk_decode_kernel<decltype(rpw)::value, decltype(il)::value, decltype(nt)::value, decltype(pm)::value, decltype(sg)::value, false>,
                                      scatter_blocks, st, io, d, scatter_blocks);
    }); });
  }); }); });
  return hipGetLastError();
}

hipError_t launch_scatter(const RoundDev& rd, const LayerDev& io, const DiffDev& d, int planes, int grid_size, hipStream_t st) {
  if (rd.n_agents == 0 || d.capacity == 0 || grid_size <= 0) return hipSuccess;
  if (rd.interleaved) hipLaunchKernelGGL(tdk_scatter_kernel<true>, dim3(grid_size), dim3(kBlock), 0, st, rd, io, d, planes);
  else hipLaunchKernelGGL(tdk_scatter_kernel<false>, dim3(grid_size), dim3(kBlock), 0, st, rd, io, d, planes);
  return hipGetLastError();
}

hipError_t launch_keydiff(const RoundDev& rd, const LayerDev& io, const PlanDev& pl, hipStream_t st) {
  if (rd.n_work == 0) return hipSuccess;
  with_rpw(rd.page_tokens, [&](auto rpw) { with_bool(rd.interleaved != 0, [&](auto il) { with_bool(rd.seg != 0, [&](auto sg) {
    with_bool((rd.nontemporal & 4) != 0, [&](auto ntl) {
      hipLaunchKernelGGL((tdk_keydiff_kernel<decltype(rpw)::value, decltype(il)::value, decltype(sg)::value, decltype(ntl)::value>),
                         dim3(rd.n_rwork), dim3(kBlock), 0, st, rd, io, pl);
    });
  }); }); });
  return hipGetLastError();
}

hipError_t launch_select(const RoundDev& rd, const PlanDev& pl, hipStream_t st) {
  if (rd.n_agents == 0) return hipSuccess;
  hipLaunchKernelGGL(tdk_select_kernel, dim3(rd.n_agents), dim3(kBlock), 0, st, rd, pl);
  return hipGetLastError();
}

hipError_t launch_master(const RoundDev& rd, const PlanDev& pl, hipStream_t st) {
  if (rd.n_sessions == 0) return hipSuccess;
  hipLaunchKernelGGL(tdk_master_kernel, dim3((rd.n_sessions + kWaves - 1) / kWaves), dim3(kBlock), 0, st, rd, pl);
  return hipGetLastError();
}

hipError_t launch_copy(u32x4* dst, const u32x4* src, size_t n16, hipStream_t st) {
  if (n16 == 0) return hipSuccess;
  // one 4 KB chunk per workgroup while the grid allows: workgroups are dispatched in order, so the chip
  // sweeps memory in one narrow sequential window, which is what DRAM serves fastest
  size_t blocks = (n16 + kBlock - 1) / kBlock;
  if (blocks > ((size_t)1 << 30)) blocks = (size_t)1 << 30;
  hipLaunchKernelGGL(tdk_copy_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, st,
                     dst, src, n16);
  return hipGetLastError();
}

hipError_t launch_fill(u32x4* dst, uint32_t word, size_t n16, hipStream_t st) {
  if (n16 == 0) return hipSuccess;
  size_t blocks = (n16 + kBlock - 1) / kBlock;
  if (blocks > ((size_t)1 << 30)) blocks = (size_t)1 << 30;
  hipLaunchKernelGGL(tdk_fill_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, st,
                     dst, word, n16);
  return hipGetLastError();
}

hipError_t launch_page_fill(u32x4* dst, const int32_t* ids, int n_pages, int page_u4, uint32_t word, hipStream_t st) {
  if (n_pages <= 0) return hipSuccess;
  hipLaunchKernelGGL(tdk_page_fill_kernel, dim3(n_pages), dim3(kBlock), 0, st, dst, ids, page_u4, word);
  return hipGetLastError();
}

hipError_t launch_page_read(const u32x4* src, const int32_t* ids, int n_pages, int page_u4, u32x4* sink, hipStream_t st) {
  if (n_pages <= 0) return hipSuccess;
  hipLaunchKernelGGL(tdk_page_read_kernel, dim3(n_pages), dim3(kBlock), 0, st, src, ids, page_u4, sink);
  return hipGetLastError();
}

hipError_t launch_page_fill_product(u32x4* pk, u32x4* pv, const int32_t* ids, int n_pages, int group, int heads, int page_tokens,
                                    uint32_t word, hipStream_t st) {
  if (n_pages <= 0) return hipSuccess;
  const dim3 grid((n_pages + group - 1) / group);
  if (page_tokens == 16) hipLaunchKernelGGL(tdk_page_fill_product_kernel<4>, grid, dim3(kBlock), 0, st, pk, pv, ids, n_pages, group, heads, word);
  else hipLaunchKernelGGL(tdk_page_fill_product_kernel<8>, grid, dim3(kBlock), 0, st, pk, pv, ids, n_pages, group, heads, word);
  return hipGetLastError();
}

hipError_t launch_page_read_product(const u32x4* pk, const u32x4* pv, const int32_t* ids, int n_pages, int group, int heads,
                                    int page_tokens, u32x4* sink, hipStream_t st) {
  if (n_pages <= 0) return hipSuccess;
  const dim3 grid((n_pages + group - 1) / group);
  if (page_tokens == 16) hipLaunchKernelGGL(tdk_page_read_product_kernel<4>, grid, dim3(kBlock), 0, st, pk, pv, ids, n_pages, group, heads, sink);
  else hipLaunchKernelGGL(tdk_page_read_product_kernel<8>, grid, dim3(kBlock), 0, st, pk, pv, ids, n_pages, group, heads, sink);
  return hipGetLastError();
}

}  // namespace tdk
