// Attention of new query tokens over the shared span of every mirror, computed from master + diff
// with no restored copy (Sec. 4.4, last paragraphs: the diff applied as attention tiles are loaded;
// Fig. 9: skip-or-correct per block).
//
// RoPE rotations are orthogonal, so q . (R(delta) k) = (R(-delta) q) . k: instead of rotating the
// master's keys once per agent, each agent's few query rows are rotated back by its offset and all
// agents of a session then attend to the SAME un-rotated master keys.  The query rows of a session
// (agents x query tokens x query heads of one KV head) become the N side of one dense product with
// the master's K and V tiles, which is MFMA work, and the master is read once per session instead of
// once per agent (the master pass).  Pages that an agent's diff lists are masked out of that product for
// that agent's rows and come from the payload instead, with the same tile arithmetic (the listed-pages
// pass, the "correct" half); a last kernel merges the partial results with their log-sum-exp weights.
// For the decode case (identity layouts, stored diffs not moved, at most 32 rows per agent and KV head)
// the two passes share one launch, which also rotates the query rows itself; other rounds run
// tdk_attend_qrot_kernel, tdk_attend_master_kernel and tdk_attend_diff(16)_kernel one after another.
#include "tdk_internal.h"

#include <type_traits>

namespace tdk {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2a __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2a __attribute__((ext_vector_type(2)));

namespace {

constexpr int kTile = 32;            // tokens per MFMA tile
constexpr int kRowsPerWave = 32;     // query rows per wavefront (the N side of the 32x32 MFMA)
constexpr int kRowsPerBlock = kRowsPerWave * kWaves;
constexpr int kKsStride = kHeadDim + 8;   // bf16 elements per staged K row (+16 bytes: spreads LDS banks)
constexpr int kBigTile = 2 * kTile;       // tokens per step of the master pass
constexpr int kVsStride = kHeadDim + 16;  // bf16 elements per staged V row (+32 bytes: four consecutive rows' 32-byte
                                          // pieces then fall into different LDS banks for the transposing reads)

__device__ __forceinline__ uint32_t pack2(float a, float b) {
  f32x2a v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2a));
}

// position of a query row inside its session's row list, and where its data lives
struct RowRef {
  int agent;      // agent id, -1 for a padding row
  int64_t out;    // index of the row in q / out / lse: ((agent * n_q + qi) * Hq + hq)
};

__device__ __forceinline__ RowRef row_ref(const RoundDev& rd, const SessionDev& sd, const AttendDev& at, int h, int row) {
  RowRef r;
  const int per_agent = at.n_q * at.group;
  const int a_local = row / per_agent;
  if (a_local >= sd.n_agents) { r.agent = -1; r.out = 0; return r; }
  const int rem = row - a_local * per_agent;
  const int qi = rem / at.group, g = rem - qi * at.group;
  r.agent = rd.order[sd.order_begin + a_local];
  r.out = ((int64_t)r.agent * at.n_q + qi) * at.n_q_heads + h * at.group + g;
  return r;
}

// Running softmax of one query row (the lane pair n, n + 32 shares a row) and its output accumulators:
// oacc[b][i] is element 32 b + 8 (i / 4) + 4 hh + i % 4 of the row's un-normalised output.
struct RowState {
  float m_run, l_run;
  f32x16 oacc[4];
};

__device__ __forceinline__ void row_state_init(RowState& st) {
  st.m_run = -INFINITY;
  st.l_run = 0.f;
#pragma unroll
  for (int b = 0; b < 4; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) st.oacc[b][i] = 0.f;
}

// Orders the LDS traffic of one wavefront (its lanes exchange data through a staging area no other
// wavefront touches): no hardware barrier, only a point the compiler may not move memory accesses across.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The same for a 64-token step held in LDS (two independent score tiles): their MFMA chains interleave,
// the LDS reads of one hide behind the products of the other, and the softmax bookkeeping (exchange with
// the partner lane, reference point, rescale test) is paid once per 64 tokens.  Score i of a lane is token
// 32 (i / 16) + 8 ((i % 16) / 4) + 4 hh + i % 4 of the step.
// scores of a 64-token step for the wavefront's 32 rows: two independent MFMA chains
template <bool AHEAD>
__device__ __forceinline__ void scores64(const uint16_t* Ks, const bf16x8 (&qf)[8], int n, int hh, f32x16& s0, f32x16& s1) {
#pragma unroll
  for (int i = 0; i < 16; ++i) { s0[i] = 0.f; s1[i] = 0.f; }
  if (!AHEAD) {                                             // the form that needs few registers
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const u32x4 a0 = *reinterpret_cast<const u32x4*>(Ks + n * kKsStride + 16 * kk + 8 * hh);
      const u32x4 a1 = *reinterpret_cast<const u32x4*>(Ks + (kTile + n) * kKsStride + 16 * kk + 8 * hh);
      s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a0), qf[kk], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a1), qf[kk], s1, 0, 0, 0);
    }
    return;
  }
  // all sixteen A operands are requested before the first product: the LDS round trips overlap instead of
  // each pair of products waiting for its own
  u32x4 a[16];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    a[2 * kk] = *reinterpret_cast<const u32x4*>(Ks + n * kKsStride + 16 * kk + 8 * hh);
    a[2 * kk + 1] = *reinterpret_cast<const u32x4*>(Ks + (kTile + n) * kKsStride + 16 * kk + 8 * hh);
  }
  __builtin_amdgcn_sched_group_barrier(0x100, 16, 0);       // the 16 LDS reads first
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[2 * kk]), qf[kk], s0, 0, 0, 0);
    s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[2 * kk + 1]), qf[kk], s1, 0, 0, 0);
  }
  __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);       // then the 16 products
}

// O^T += V^T P^T for a 64-token step whose V rows sit row-major in LDS (Vs[token][d]).  The A operand of
// product (kk, b) is V^T[d = 32 b + n][tokens 16 kk + 8 hf + 4 hh + j], hf = 0, 1, j = 0..3: each half comes from
// one ds_read_b64_tr_b16.  Within a block of 16 lanes that instruction treats the 8-byte pieces the lanes
// address as the rows of a 16 x 4 matrix of 16-bit values and hands lane i the values (i / 4 + 4 j, i % 4),
// j = 0..3; with lane i addressing (token i / 4 of the four, d-quad i % 4 of its block's sixteen d) lane i gets
// element d = 16 (block % 2) + i of tokens 0..3 -- its own row of V^T.  p[i] is the weight of token
// 32 (i / 16) + 8 ((i % 16) / 4) + 4 hh + i % 4.
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

template <int NK>                             // NK products of 16 tokens each: 4 for a 64-token step, 2 for a 32-token tile
__device__ __forceinline__ void pv_tr(const uint16_t* Vs, const float (&p)[8 * NK], int lane, RowState& st) {
  const int i16 = lane & 15, blk = lane >> 4;
  const uint16_t* base = Vs + (4 * (blk >> 1) + (i16 >> 2)) * kVsStride + 16 * (blk & 1) + 4 * (i16 & 3);
  u32x4 va[4 * NK];
#pragma unroll
  for (int kk = 0; kk < NK; ++kk)
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(base + (16 * kk) * kVsStride + 32 * b));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(base + (16 * kk + 8) * kVsStride + 32 * b));
      const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
      va[4 * kk + b] = u32x4{l2.x, l2.y, h2.x, h2.y};
    }
#pragma unroll
  for (int kk = 0; kk < NK; ++kk) {
    u32x4 pw;
#pragma unroll
    for (int e = 0; e < 4; ++e) pw[e] = pack2(p[8 * kk + 2 * e], p[8 * kk + 2 * e + 1]);
    const bf16x8 pb = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
    for (int b = 0; b < 4; ++b)
      st.oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, va[4 * kk + b]), pb, st.oacc[b], 0, 0, 0);
  }
}

// One 32-token tile for the 32 query rows of a wavefront, K rows in registers: k[kk] holds, for lane (n, hh),
// elements 16 kk + 8 hh .. + 7 of the K row of token n.  S^T (tokens x rows) = K Q^T: lane (n, hh) then holds,
// for query row n, the scores of tokens 8 (i / 4) + 4 hh + i % 4; bit i of `live` says whether that token counts.
__device__ __forceinline__ void scores32(const u32x4 (&k)[8], const bf16x8 (&qf)[8], f32x16& sacc) {
#pragma unroll
  for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
  for (int kk = 0; kk < 8; ++kk)
    sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, k[kk]), qf[kk], sacc, 0, 0, 0);
}

__device__ __forceinline__ void softmax_pv32(const uint16_t* Vs, const f32x16& sacc, float scale, uint32_t live, int lane,
                                             RowState& st) {
  float p[16];
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    p[i] = ((live >> i) & 1u) ? sacc[i] * scale : -INFINITY;
    mx = fmaxf(mx, p[i]);
  }
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  constexpr float kLazy = 8.f;
  const float m_new = mx > st.m_run + kLazy || st.m_run == -INFINITY ? fmaxf(st.m_run, mx) : st.m_run;
  const float m_ref = m_new == -INFINITY ? 0.f : m_new;
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) { p[i] = __expf(p[i] - m_ref); sum += p[i]; }
  if (__any(m_new != st.m_run)) {
    const float alpha = __expf(st.m_run - m_ref);      // 1 for the rows whose reference stays
    st.l_run *= alpha;
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) st.oacc[b][i] *= alpha;
  }
  st.l_run += sum;
  st.m_run = m_new;
  pv_tr<2>(Vs, p, lane, st);
}

__device__ __forceinline__ void softmax_pv64(const uint16_t* Vs, const f32x16& s0, const f32x16& s1, float scale,
                                             uint32_t live, int lane, RowState& st) {
  float p[32];
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    p[i] = ((live >> i) & 1u) ? s0[i] * scale : -INFINITY;
    p[16 + i] = ((live >> (16 + i)) & 1u) ? s1[i] * scale : -INFINITY;
    mx = fmaxf(mx, fmaxf(p[i], p[16 + i]));
  }
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  constexpr float kLazy = 8.f;
  const float m_new = mx > st.m_run + kLazy || st.m_run == -INFINITY ? fmaxf(st.m_run, mx) : st.m_run;
  const float m_ref = m_new == -INFINITY ? 0.f : m_new;
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 32; ++i) { p[i] = __expf(p[i] - m_ref); sum += p[i]; }
  if (__any(m_new != st.m_run)) {
    const float alpha = __expf(st.m_run - m_ref);
    st.l_run *= alpha;
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) st.oacc[b][i] *= alpha;
  }
  st.l_run += sum;
  st.m_run = m_new;
  pv_tr<4>(Vs, p, lane, st);
}

// The same with whole 16-token groups switched off instead of single tokens, for a positive scale: score i
// of a lane belongs to group i / 8 and bit g of m4 says whether group g takes part (four lane masks, one
// select per score); the scale and the reference point go into one fused multiply-add in base-2 units in
// front of v_exp_f32.  m_run stays in natural-log units of the scaled scores.
__device__ __forceinline__ void softmax_pv64_groups(const uint16_t* Vs, const f32x16& s0, const f32x16& s1, float scale,
                                                    uint32_t m4, int lane, RowState& st) {
  constexpr float kLog2e = 1.4426950408889634f;
  const bool on[4] = {(m4 & 1u) != 0, (m4 & 2u) != 0, (m4 & 4u) != 0, (m4 & 8u) != 0};
  float p[32];
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    p[i] = on[i >> 3] ? s0[i] : -INFINITY;
    p[16 + i] = on[2 + (i >> 3)] ? s1[i] : -INFINITY;
    // (the NaN-propagating maximum: v_maximum3_f32, with no quieting of its operands first)
    mx = __builtin_elementwise_maximum(mx, __builtin_elementwise_maximum(p[i], p[16 + i]));
  }
  mx = fmaxf(mx, __shfl_xor(mx, 32)) * scale;
  constexpr float kLazy = 8.f;
  const float m_new = mx > st.m_run + kLazy || st.m_run == -INFINITY ? fmaxf(st.m_run, mx) : st.m_run;
  const float m_ref = m_new == -INFINITY ? 0.f : m_new;
  const float c2 = scale * kLog2e, m2 = -m_ref * kLog2e;
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 32; ++i) { p[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(p[i], c2, m2)); sum += p[i]; }
  if (__any(m_new != st.m_run)) {
    const float alpha = __expf(st.m_run - m_ref);
    st.l_run *= alpha;
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) st.oacc[b][i] *= alpha;
  }
  st.l_run += sum;
  st.m_run = m_new;
  pv_tr<4>(Vs, p, lane, st);
}

// ---- the same tile for 16 query rows per wavefront (v_mfma_f32_16x16x32_bf16): for passes whose row
// blocks are nearly empty (the listed pages of one agent meet only its own few rows), a quarter of the
// scores per lane.  Lane (n, g) = (lane % 16, lane / 16) owns row n; of a 32-token tile it holds the scores
// of tokens 16 tt + 4 g + i (tt = 0, 1; i = 0..3) as p[4 tt + i], and elements 16 b + 4 g + i of the output.
typedef float f32x4a __attribute__((ext_vector_type(4)));

struct RowState16 {
  float m_run, l_run;
  f32x4a oacc[8];
};

__device__ __forceinline__ void row_state16_init(RowState16& st) {
  st.m_run = -INFINITY;
  st.l_run = 0.f;
#pragma unroll
  for (int b = 0; b < 8; ++b)
#pragma unroll
    for (int i = 0; i < 4; ++i) st.oacc[b][i] = 0.f;
}

// k[2 kk + tt] holds, for lane (n, g), elements 32 kk + 8 g .. + 7 of the K row of token 16 tt + n
__device__ __forceinline__ void scores16(const u32x4 (&k)[8], const bf16x8 (&qf)[4], f32x4a& s0, f32x4a& s1) {
#pragma unroll
  for (int i = 0; i < 4; ++i) { s0[i] = 0.f; s1[i] = 0.f; }
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k[2 * kk]), qf[kk], s0, 0, 0, 0);
    s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k[2 * kk + 1]), qf[kk], s1, 0, 0, 0);
  }
}

// Vs holds the tile's V rows row-major (kVsStride); the A operands come from transposing reads as in pv_tr:
// lane i of a block of 16 addresses (token i / 4 of the block's four, d-quad i % 4) and receives d = 16 b + i.
__device__ __forceinline__ void softmax_pv16(const uint16_t* Vs, const f32x4a& s0, const f32x4a& s1, float scale, uint32_t live,
                                             int n, int g, RowState16& st) {
  float p[8];
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    p[i] = ((live >> i) & 1u) ? s0[i] * scale : -INFINITY;
    p[4 + i] = ((live >> (4 + i)) & 1u) ? s1[i] * scale : -INFINITY;
    mx = fmaxf(mx, fmaxf(p[i], p[4 + i]));
  }
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  constexpr float kLazy = 8.f;
  const float m_new = mx > st.m_run + kLazy || st.m_run == -INFINITY ? fmaxf(st.m_run, mx) : st.m_run;
  const float m_ref = m_new == -INFINITY ? 0.f : m_new;
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) { p[i] = __expf(p[i] - m_ref); sum += p[i]; }
  if (__any(m_new != st.m_run)) {
    const float alpha = __expf(st.m_run - m_ref);
    st.l_run *= alpha;
#pragma unroll
    for (int b = 0; b < 8; ++b)
#pragma unroll
      for (int i = 0; i < 4; ++i) st.oacc[b][i] *= alpha;
  }
  st.l_run += sum;
  st.m_run = m_new;
  u32x4 pw;
#pragma unroll
  for (int e = 0; e < 4; ++e) pw[e] = pack2(p[2 * e], p[2 * e + 1]);
  const bf16x8 pb = __builtin_bit_cast(bf16x8, pw);
  const uint16_t* base = Vs + (4 * g + (n >> 2)) * kVsStride + 4 * (n & 3);
#pragma unroll
  for (int b = 0; b < 8; ++b) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(base + 16 * b));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(base + 16 * kVsStride + 16 * b));
    const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
    const u32x4 a = {l2.x, l2.y, h2.x, h2.y};
    st.oacc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), pb, st.oacc[b], 0, 0, 0);
  }
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// q' = bf16(R(-delta_i) q): one wavefront per query row (all heads of one token of one agent)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void tdk_attend_qrot_kernel(const RoundDev rd, const AttendDev at) {
  const int64_t row = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);   // (agent, qi, hq)
  const int64_t n_rows = (int64_t)rd.n_agents * at.n_q * at.n_q_heads;
  if (row >= n_rows) return;
  const int lane = threadIdx.x & 63;
  const int agent = (int)(row / ((int64_t)at.n_q * at.n_q_heads));
  const uint16_t* src = reinterpret_cast<const uint16_t*>(at.q) + row * kHeadDim;
  const int ia = rd.interleaved ? 2 * lane : lane;
  const int ib = rd.interleaved ? 2 * lane + 1 : lane + kHalf;
  // the kernels after this one work with |scale|: a negative scale flips the sign of every query copy (exact)
  const uint32_t flip = at.q_flip ? 0x8000u : 0u;
  const float xa = __uint_as_float((uint32_t)(src[ia] ^ flip) << 16), xb = __uint_as_float((uint32_t)(src[ib] ^ flip) << 16);
  // one copy per segment of the agent's layout (one for an identity layout): every segment has its own offset
  const int seg0 = rd.seg ? rd.seg_off[agent] : agent;
  const int nseg = rd.seg ? rd.seg_off[agent + 1] - seg0 : 1;
  const float* tabs = rd.seg ? rd.segtab : rd.tab;
  for (int k = 0; k < nseg; ++k) {
    const float* tab = tabs + (size_t)(seg0 + k) * (2 * kHalf);
    uint16_t* dst = reinterpret_cast<uint16_t*>(at.qrot) + (row * at.max_seg + k) * kHeadDim;
    const float c = tab[lane], s = tab[kHalf + lane];
    // rotation by -delta: y_a = x_a cos + x_b sin, y_b = x_b cos - x_a sin
    dst[ia] = (uint16_t)(pack2(__builtin_fmaf(xa, c, __fmul_rn(xb, s)), 0.f) & 0xffffu);
    dst[ib] = (uint16_t)(pack2(__builtin_fmaf(xb, c, -__fmul_rn(xa, s)), 0.f) & 0xffffu);
  }
  // the queries the listed pages meet: as they are, or turned back by the distance the stored values
  // have moved since they were encoded
  // (a segmented round whose stored diffs moved keeps one such copy per segment: diff_seg copies per row)
  for (int k = 0; k < (at.diff_seg > 1 ? nseg : 1); ++k) {
    uint16_t* dst2 = reinterpret_cast<uint16_t*>(at.qdiff) + (row * at.diff_seg + k) * kHeadDim;
    uint16_t za = (uint16_t)(src[ia] ^ flip), zb = (uint16_t)(src[ib] ^ flip);
    const float* td = nullptr;
    if (!rd.seg && rd.agents[agent].diff_rot) td = rd.tab_diff + (size_t)agent * (2 * kHalf);
    if (rd.seg && at.diff_seg > 1) td = rd.segtab_diff + (size_t)(seg0 + k) * (2 * kHalf);   // identity tables copy exactly
    if (td) {
      const float c2 = td[lane], s2 = td[kHalf + lane];
      if (c2 != 1.f || s2 != 0.f || !rd.seg) {
        za = (uint16_t)(pack2(__builtin_fmaf(xa, c2, __fmul_rn(xb, s2)), 0.f) & 0xffffu);
        zb = (uint16_t)(pack2(__builtin_fmaf(xb, c2, -__fmul_rn(xa, s2)), 0.f) & 0xffffu);
      }
    }
    dst2[ia] = za;
    dst2[ib] = zb;
  }
}

// ---------------------------------------------------------------------------------------------
// master pass: S^T = K Q'^T and O^T += V^T P^T per 32-token tile, online softmax per query row
// grid: one linear id = KV head + heads * (block of 128 query rows + row blocks * (session * n_chunks + chunk))
// ---------------------------------------------------------------------------------------------
constexpr int kMasterKs = kBigTile * kKsStride, kMasterVs = kBigTile * kVsStride;      // bf16 elements of the two tiles
constexpr int kMaskWords = 2;                                                          // 64-bit words of a row's page mask: 128 pages per chunk
constexpr int kMasterLds = (kMasterKs + kMasterVs) * 2 + kRowsPerBlock * kMaskWords * 8;   // bytes, with the page masks

// One workgroup of the master pass: KV head h, chunk number `sc` = session * n_chunks + chunk, row block zb.
// lds: kMasterLds bytes, 16-byte aligned.
// QDIRECT (identity layouts only): the query rows are rotated back here, from the caller's q, instead of
// being read from the copies the qrot kernel leaves (same arithmetic, so the same bits).
template <bool SEG, bool QDIRECT = false>
__device__ __forceinline__ void attend_master_body(const RoundDev& rd, const LayerDev& io, const DiffDev& d, const AttendDev& at,
                                                   unsigned char* lds, int h, int sc, int zb) {
  static_assert(!(SEG && QDIRECT), "one rotation per row only");
  uint16_t* Ks = reinterpret_cast<uint16_t*>(lds);
  uint16_t* Vs = Ks + kMasterKs;
  uint64_t* s_mask = reinterpret_cast<uint64_t*>(Vs + kMasterVs);   // bit p: page p of this chunk is listed in the row's agent's diff

  const int session = sc / at.n_chunks, chunk = sc - session * at.n_chunks;
  const SessionDev sd = rd.sess[session];
  const int tok_begin = chunk * at.chunk_tokens;
  if (tok_begin >= sd.span || sd.n_agents == 0) return;
  const int rows = sd.n_agents * at.n_q * at.group;
  const int row_begin = zb * kRowsPerBlock;
  if (row_begin >= rows) return;
  const int T = rd.page_tokens;
  const int tok_end = min(sd.span, tok_begin + at.chunk_tokens);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 31, hh = lane >> 5;

  // which pages of this chunk each row's agent lists in its diff (those tokens belong to the other kernel)
  if (threadIdx.x < kRowsPerBlock) {
    uint64_t mask[kMaskWords] = {0, 0};
    const RowRef rr = row_ref(rd, sd, at, h, row_begin + threadIdx.x);
    if (rr.agent >= 0) {
      int64_t lo = d.offset[rr.agent], hi = lo + d.count[rr.agent];
      if (lo < 0) lo = 0;
      if (hi > d.capacity) hi = d.capacity;
      const int pg0 = tok_begin / T, pg1 = (tok_end - 1) / T;
      int64_t a = lo, b = hi;
      while (a < b) {                      // first listed page >= pg0
        const int64_t mid = (a + b) >> 1;
        if (d.idx[mid] < pg0) a = mid + 1; else b = mid;
      }
      for (; a < hi; ++a) {
        const int p = d.idx[a];
        if (p > pg1 || p < pg0) break;
        const int rel_p = p - pg0;
        if (rel_p < 64) mask[0] |= (uint64_t)1 << rel_p; else mask[1] |= (uint64_t)1 << (rel_p - 64);
      }
    }
    s_mask[kMaskWords * threadIdx.x] = mask[0];
    s_mask[kMaskWords * threadIdx.x + 1] = mask[1];
  }

  // this lane's query row: its B operands (8 steps of 16 along the head dimension) stay in registers.
  // With per-agent block layouts every segment has its own copy of the row (rotated back by that
  // segment's offset); seg_k follows the segment that holds the current token.
  const RowRef mine = row_ref(rd, sd, at, h, row_begin + wave * kRowsPerWave + n);
  const uint16_t* q_rows = reinterpret_cast<const uint16_t*>(at.qrot) + mine.out * at.max_seg * kHeadDim;
  auto load_q = [&](int k, bool on, bf16x8 (&f)[8]) {
    const u32x4* qp = reinterpret_cast<const u32x4*>(q_rows + (size_t)k * kHeadDim);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      u32x4 v = {0, 0, 0, 0};
      if (on) v = qp[2 * kk + hh];
      f[kk] = __builtin_bit_cast(bf16x8, v);
    }
  };
  bf16x8 qf[8];
  int seg_base = 0, seg_n = 1, seg_k = 0;
  if (SEG && mine.agent >= 0) {
    seg_base = rd.seg_off[mine.agent];
    seg_n = rd.seg_off[mine.agent + 1] - seg_base;
    while (seg_k + 1 < seg_n && rd.seg_src[seg_base + seg_k + 1] <= tok_begin) ++seg_k;
  }
  if (!SEG && !QDIRECT) {
    const u32x4* qp = reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(at.qrot) + mine.out * kHeadDim);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      u32x4 v = {0, 0, 0, 0};
      if (mine.agent >= 0) v = qp[2 * kk + hh];
      qf[kk] = __builtin_bit_cast(bf16x8, v);
    }
  }
  if (QDIRECT) {
    // fragment kk of a lane = elements 16 kk + 8 hh .. + 7 of its row.  Rotation by -delta of the pair (a, b):
    // y_a = x_a cos + x_b sin, y_b = x_b cos - x_a sin, with pair j = (j, j + 64) or (2 j, 2 j + 1).
    u32x4 raw[8];
    const u32x4* qp = reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(at.q) + mine.out * kHeadDim);
    const uint32_t flip = at.q_flip ? 0x80008000u : 0u;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      u32x4 v = {0, 0, 0, 0};
      if (mine.agent >= 0) v = qp[2 * kk + hh];
      raw[kk] = u32x4{v.x ^ flip, v.y ^ flip, v.z ^ flip, v.w ^ flip};
    }
    const float* tab = rd.tab + (size_t)(mine.agent >= 0 ? mine.agent : 0) * (2 * kHalf);
    auto lo16 = [](uint32_t w) { return __uint_as_float(w << 16); };
    auto hi16 = [](uint32_t w) { return __uint_as_float(w & 0xffff0000u); };
    u32x4 rot[8];
    if (!rd.interleaved) {
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {           // fragments kk (elements a) and kk + 4 (elements b = a + 64)
        u32x4 ya, yb;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const int j = 16 * kk + 8 * hh + 2 * w;
          const float c0 = tab[j], s0 = tab[kHalf + j], c1 = tab[j + 1], s1 = tab[kHalf + j + 1];
          const float a0 = lo16(raw[kk][w]), a1 = hi16(raw[kk][w]), b0 = lo16(raw[kk + 4][w]), b1 = hi16(raw[kk + 4][w]);
          ya[w] = pack2(__builtin_fmaf(a0, c0, __fmul_rn(b0, s0)), __builtin_fmaf(a1, c1, __fmul_rn(b1, s1)));
          yb[w] = pack2(__builtin_fmaf(b0, c0, -__fmul_rn(a0, s0)), __builtin_fmaf(b1, c1, -__fmul_rn(a1, s1)));
        }
        rot[kk] = ya; rot[kk + 4] = yb;
      }
    } else {
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {           // word w of a fragment holds the pair j = 8 kk + 4 hh + w
        u32x4 y;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const int j = 8 * kk + 4 * hh + w;
          const float c = tab[j], sn = tab[kHalf + j];
          const float a = lo16(raw[kk][w]), b = hi16(raw[kk][w]);
          y[w] = pack2(__builtin_fmaf(a, c, __fmul_rn(b, sn)), __builtin_fmaf(b, c, -__fmul_rn(a, sn)));
        }
        rot[kk] = y;
      }
    }
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) qf[kk] = __builtin_bit_cast(bf16x8, rot[kk]);
  }
  __syncthreads();
  const uint64_t* my_masks = s_mask + kMaskWords * (wave * kRowsPerWave + n);   // (read per step: two registers less)

  RowState rs;
  row_state_init(rs);

  const int64_t head_u4 = 16;                                  // 128 bf16 = 16 chunks of 16 bytes
  const int64_t row_u4 = (int64_t)rd.heads * head_u4;
  // staging: sixteen lanes per token row (coalesced 256-byte reads of one head's K and V), four rows per
  // wavefront instruction; both tiles are kept row-major in LDS (the V operands are read with transposing loads)
  const int st_tok = threadIdx.x >> 4, st_pc = threadIdx.x & 15;

  // 64 tokens per step: the next step's rows travel from HBM to registers while this one is multiplied.
  // kp / vp follow this thread's piece of the rows of the chunk (thread t: token t / 16 of each group of 16,
  // piece t % 16); a step whose 64 tokens all lie inside the span needs no bounds checks.
  u32x4 kv[8];
  const int64_t row16 = 16 * row_u4;                           // sixteen token rows, in 16-byte units
  const u32x4* kp = io.master_k + (sd.master_row0 + tok_begin + st_tok) * row_u4 + h * head_u4 + st_pc;
  const u32x4* vp = io.master_v + (sd.master_row0 + tok_begin + st_tok) * row_u4 + h * head_u4 + st_pc;
  auto fetch = [&](int t0) {                                   // advances kp / vp past the step
    if (t0 + kBigTile <= tok_end) {
#pragma unroll
      for (int e = 0; e < 4; ++e) { kv[e] = __builtin_nontemporal_load(kp + e * row16); kv[4 + e] = __builtin_nontemporal_load(vp + e * row16); }
    } else {
      const u32x4 z = {0, 0, 0, 0};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        kv[e] = z; kv[4 + e] = z;
        if (t0 + 16 * e + st_tok < tok_end) { kv[e] = __builtin_nontemporal_load(kp + e * row16); kv[4 + e] = __builtin_nontemporal_load(vp + e * row16); }
      }
    }
    kp += 4 * row16; vp += 4 * row16;
  };
  fetch(tok_begin);
  uint32_t touch = 0;
  // thread t looks after line t % 2 of the K (t % 4 < 2) or V row of token t / 4, two steps ahead
  const u32x4* tp = ((threadIdx.x & 2) ? io.master_v : io.master_k) +
                    (sd.master_row0 + tok_begin + 2 * kBigTile + (threadIdx.x >> 2)) * row_u4 + h * head_u4 + (threadIdx.x & 1) * 8;
  // one 64-token step; WHOLE: all 64 tokens lie inside the span (every step but a ragged last one)
  auto step = [&](int t0, auto whole_tag) {
    constexpr bool WHOLE = decltype(whole_tag)::value;
    __syncthreads();                                           // the previous step has been consumed
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      *reinterpret_cast<u32x4*>(Ks + (16 * e + st_tok) * kKsStride + 8 * st_pc) = kv[e];
      *reinterpret_cast<u32x4*>(Vs + (16 * e + st_tok) * kVsStride + 8 * st_pc) = kv[4 + e];
    }
    __syncthreads();
    if (WHOLE && t0 + kBigTile < tok_end) fetch(t0 + kBigTile);
    // The step after that is called into the caches now: one 4-byte read per 128-byte line of its K and V
    // rows (64 tokens x 2 lines x 2 planes = one line per thread), so that its rows, fetched a step from
    // now, come from L2 instead of HBM.  The value is not used.
    if (WHOLE) {
      if (t0 + 2 * kBigTile + (int)(threadIdx.x >> 2) < tok_end) touch = *reinterpret_cast<const uint32_t*>(tp);
      tp += 4 * row16;
    }
    // which of this lane's 32 scores take part: 16-token groups follow the page mask of the row's agent
    // (m4: bit g set = the g-th group of 16 tokens of this step takes part)
    uint32_t m4;
    {
      const uint32_t rel = (uint32_t)(t0 - tok_begin);
      if (T == 16) {
        const uint32_t pg = rel >> 4;                                        // four pages of 16 tokens
        m4 = ~(uint32_t)(my_masks[pg >> 6] >> (pg & 63u)) & 0xfu;
      } else {
        const uint32_t pg = rel >> 5;                                        // two pages of 32 tokens
        const uint32_t m2 = ~(uint32_t)(my_masks[pg >> 6] >> (pg & 63u)) & 0x3u;
        m4 = ((m2 & 1u) ? 0x3u : 0u) | ((m2 & 2u) ? 0xcu : 0u);
      }
      if (mine.agent < 0) m4 = 0;
    }
    f32x16 s0, s1;
    if (!SEG) {
      scores64<true>(Ks, qf, n, hh, s0, s1);
    } else {
      // The step may run over several segments of this row's agent: the scores are computed once per
      // segment met (each with that segment's copy of the query row) and every token keeps the one of the
      // segment it belongs to.  Rows differ in where their segments end; the loop runs while any row has one left.
#pragma unroll
      for (int i = 0; i < 16; ++i) { s0[i] = 0.f; s1[i] = 0.f; }
      const int t_end = t0 + kBigTile;
      bool more = mine.agent >= 0;
      int k = seg_k;
      while (__any(more)) {
        load_q(k, more, qf);
        f32x16 p0, p1;
        scores64<false>(Ks, qf, n, hh, p0, p1);
        const int lo = more ? rd.seg_src[seg_base + k] : 0;
        const int hi = more ? (k + 1 < seg_n ? rd.seg_src[seg_base + k + 1] : sd.span) : 0;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int ta = t0 + 8 * (i >> 2) + 4 * hh + (i & 3), tb2 = ta + kTile;
          if (ta >= lo && ta < hi) s0[i] = p0[i];
          if (tb2 >= lo && tb2 < hi) s1[i] = p1[i];
        }
        more = more && hi < t_end && k + 1 < seg_n;
        if (more) ++k;
      }
      seg_k = k;                                  // the segment that holds the last token of this step
      if (mine.agent >= 0 && seg_k + 1 < seg_n && rd.seg_src[seg_base + seg_k + 1] <= t_end) ++seg_k;
    }
    if (WHOLE) {
      softmax_pv64_groups(Vs, s0, s1, at.scale, m4, lane, rs);
    } else {
      uint32_t live = ((m4 & 1u) ? 0x000000ffu : 0u) | ((m4 & 2u) ? 0x0000ff00u : 0u) |
                      ((m4 & 4u) ? 0x00ff0000u : 0u) | ((m4 & 8u) ? 0xff000000u : 0u);
#pragma unroll
      for (int i = 0; i < 32; ++i)                                           // ragged end of the span
        if (t0 + 32 * (i >> 4) + 8 * ((i & 15) >> 2) + 4 * hh + (i & 3) >= tok_end) live &= ~(1u << i);
      softmax_pv64(Vs, s0, s1, at.scale, live, lane, rs);
    }
  };
  const int whole_end = tok_begin + (tok_end - tok_begin) / kBigTile * kBigTile;
  for (int t0 = tok_begin; t0 < whole_end; t0 += kBigTile) step(t0, std::true_type{});
  if (whole_end < tok_end) step(whole_end, std::false_type{});
  asm volatile("" : : "v"(touch));                             // keeps the reads above alive

  const float l_tot = rs.l_run + __shfl_xor(rs.l_run, 32);
  if (mine.agent >= 0) {
    const int64_t slot = mine.out * at.n_parts + chunk;
    float4* po = reinterpret_cast<float4*>(at.part_o + slot * kHeadDim);
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
        po[(32 * b + 8 * q4 + 4 * hh) >> 2] = make_float4(rs.oacc[b][4 * q4], rs.oacc[b][4 * q4 + 1], rs.oacc[b][4 * q4 + 2], rs.oacc[b][4 * q4 + 3]);
    if (hh == 0) { at.part_m[slot] = rs.m_run; at.part_l[slot] = l_tot; }
  }
}

template <bool SEG>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(2, 2))) void tdk_attend_master_kernel(const RoundDev rd, const LayerDev io, const DiffDev d,
                                                                   const AttendDev at, const int row_blocks) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[kMasterLds];
  // one linear id (grid dimensions y and z stop at 65535): KV head fastest, then the row block, then the chunk
  const int h = blockIdx.x % rd.heads, rest = blockIdx.x / rd.heads;
  attend_master_body<SEG>(rd, io, d, at, lds, h, rest / row_blocks, rest % row_blocks);
}

// ---------------------------------------------------------------------------------------------
// diff pass: the pages an agent's diff lists, from the payload (the "correct" half of skip-or-correct).
// One wavefront per (agent, KV head, piece): a piece is piece_tokens / 32 consecutive 32-token tiles of the agent's
// listed tokens and has its own partial result, so there is nothing to combine inside the kernel; workgroups
// whose piece lies past the end of the agent's list leave at once (the merge knows how many pieces an agent
// has).  The K rows go straight from the payload into the MFMA operand registers, the V rows through one
// row-major tile in LDS.  32 query rows at a time; more rows walk the piece again.
// ---------------------------------------------------------------------------------------------
constexpr int kPieceTiles = 16;                // 512 listed tokens per piece at most (small rounds use shorter pieces)

// Vs: this wavefront's V tile, kTile * kVsStride bf16 elements; lane: 0..63.  QDIRECT (stored diffs not moved):
// the listed pages meet the caller's rows as they are (but for the sign), no copies from the qrot kernel.
template <bool SEGMOVED, bool QDIRECT = false>
__device__ __forceinline__ bool attend_diff32_piece(const RoundDev& rd, const DiffDev& d, const AttendDev& at, uint16_t* Vs,
                                                   int h, int agent, int piece, int lane) {
  const int T = rd.page_tokens;
  int64_t lo = d.offset[agent], hi = lo + d.count[agent];
  if (lo < 0) lo = 0;
  if (hi > d.capacity) hi = d.capacity;
  const int n_tok = hi > lo ? (int)((hi - lo) * T) : 0;
  const int n_tiles = (n_tok + kTile - 1) / kTile;
  const int piece_tiles = at.piece_tokens / kTile;
  const int tile_begin = piece * piece_tiles, tile_end = min(n_tiles, tile_begin + piece_tiles);
  if (tile_begin >= tile_end) return false;     // past the end of the list: so are the pieces after this one
  const int per_agent = at.n_q * at.group;
  const AgentDev ad = rd.agents[agent];
  const SessionDev sd = rd.sess[ad.session];
  const int n = lane & 31, hh = lane >> 5;
  const int64_t row_e = (int64_t)rd.heads * kHeadDim, page_e = (int64_t)T * row_e;
  const uint16_t* pay = reinterpret_cast<const uint16_t*>(d.payload);
  const int seg_base = SEGMOVED ? rd.seg_off[agent] : 0;
  const int seg_n = SEGMOVED ? rd.seg_off[agent + 1] - seg_base : 1;
  // (offsets inside the agent's part of the payload fit 32 bits: at most 2 P pages of 64 KB or less)
  const uint16_t* apay = pay + lo * 2 * page_e;
  const uint32_t row_u = (uint32_t)row_e, page_u = (uint32_t)page_e, tile_u = (uint32_t)(kTile / T) * 2u * page_u;
  auto tok_off = [&](int tk) { return (uint32_t)(tk / T) * 2u * page_u + (uint32_t)(tk % T) * row_u + (uint32_t)(h * kHeadDim); };
  const int st_row = lane >> 4, st_pc = lane & 15;

  for (int r0 = 0; r0 < per_agent; r0 += kRowsPerWave) {
    // this lane's query row of the block
    const int rem = r0 + n;
    const bool row_ok = rem < per_agent;
    const int qi = row_ok ? rem / at.group : 0, g = row_ok ? rem - qi * at.group : 0;
    const int64_t out = ((int64_t)agent * at.n_q + qi) * at.n_q_heads + h * at.group + g;
    bf16x8 qf[8];
    auto load_q = [&](int k) {
      const u32x4* qp = QDIRECT ? reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(at.q) + out * kHeadDim)
                                : reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(at.qdiff) +
                                                                 (out * at.diff_seg + k) * kHeadDim);
      const uint32_t flip = QDIRECT && at.q_flip ? 0x80008000u : 0u;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        u32x4 v = {0, 0, 0, 0};
        if (row_ok) v = qp[2 * kk + hh];
        qf[kk] = __builtin_bit_cast(bf16x8, u32x4{v.x ^ flip, v.y ^ flip, v.z ^ flip, v.w ^ flip});
      }
    };
    if (!SEGMOVED) load_q(0);
    RowState rs;
    row_state_init(rs);
    // The next tile travels from the payload to registers while the current one is multiplied.  K: lane
    // (n, hh) loads what it multiplies, elements 16 kk + 8 hh .. + 7 of the row of token n.  V: sixteen lanes
    // per 256-byte row, four rows per instruction.  The payload address of a listed token depends on its place
    // in the list alone, so the rows are requested together with the page number; what the page number decides
    // (does the token lie inside the span, which segment holds it) is settled when the tile is used.
    u32x4 kreg[8], vreg[8];
    int p_next = -1;                             // master page of token lane % 32 of the fetched tile (-1: no such token)
    auto fetch = [&](int tile) {
      const int t = tile * kTile + n;
      const bool there = t < n_tok;
      p_next = there ? d.idx[lo + t / T] : -1;
      const u32x4 z = {0, 0, 0, 0};
      const uint32_t tile_off = (uint32_t)tile * tile_u;
      const uint32_t off = tile_off + tok_off(n) + 8u * hh;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        kreg[kk] = z;
        if (there) kreg[kk] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(apay + off + 16 * kk));
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        vreg[j] = z;
        if (tile * kTile + 4 * j + st_row < n_tok)
          vreg[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(apay + tile_off + tok_off(4 * j + st_row) + page_u + 8u * st_pc));
      }
    };
    fetch(tile_begin);
    for (int tile = tile_begin; tile < tile_end; ++tile) {
      wave_sync();                               // the previous tile has been consumed
      // bit t of valid: token t of the tile exists and lies inside the span (lanes 32..63 repeat lanes 0..31)
      int seg_cur = 0;
      bool ok = false;
      {
        const int rr = (tile * kTile + n) % T, p = p_next;
        if (p >= 0 && p < sd.pages && p * T + rr < sd.span) {
          ok = true;
          if (SEGMOVED)
            while (seg_cur + 1 < seg_n && rd.seg_src[seg_base + seg_cur + 1] <= p * T + rr) ++seg_cur;
        }
      }
      const uint32_t valid = (uint32_t)__ballot(ok);
      if (valid != 0xffffffffu) {                // rows of tokens that do not count are staged as zeros
        const u32x4 z = {0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (!((valid >> (4 * j + st_row)) & 1u)) vreg[j] = z;     // (their scores are switched off below)
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) *reinterpret_cast<u32x4*>(Vs + (4 * j + st_row) * kVsStride + 8 * st_pc) = vreg[j];
      f32x16 sacc;
      if (!SEGMOVED) {
        scores32(kreg, qf, sacc);
      } else {
        // the tile's tokens come from up to four segments (two pages, two segments each), stored at
        // different distances from today's positions: the scores are computed once per segment present,
        // with the queries turned back by that segment's distance, and every token keeps its own
        int sid[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) sid[i] = __shfl(seg_cur, 8 * (i >> 2) + 4 * hh + (i & 3));
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
        int done = -1;
        while (true) {
          int cand = (lane < kTile && ((valid >> lane) & 1u) && seg_cur > done) ? seg_cur : 0x7fffffff;
#pragma unroll
          for (int sft = 32; sft > 0; sft >>= 1) cand = min(cand, __shfl_xor(cand, sft));
          if (cand == 0x7fffffff) break;
          load_q(cand);
          f32x16 pacc;
          scores32(kreg, qf, pacc);
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (sid[i] == cand) sacc[i] = pacc[i];
          done = cand;
        }
      }
      wave_sync();                               // the V tile is complete
      if (tile + 1 < tile_end) fetch(tile + 1);  // the K registers are free: the scores are taken
      // score i of a lane belongs to token 8 (i / 4) + 4 hh + i % 4: four nibbles of `valid`
      const uint32_t vs = valid >> (4 * hh);
      uint32_t live = (vs & 0xfu) | ((vs >> 4) & 0xf0u) | ((vs >> 8) & 0xf00u) | ((vs >> 12) & 0xf000u);
      if (!row_ok) live = 0;
      softmax_pv32(Vs, sacc, at.scale, live, lane, rs);
    }
    // this piece's partial result for the block's rows: lane (n, hh) holds elements 32 b + 8 q + 4 hh + (0..3) of row n
    const float l_tot = rs.l_run + __shfl_xor(rs.l_run, 32);
    if (row_ok) {
      const int64_t slot = out * at.n_parts + at.n_chunks + piece;
      float4* po = reinterpret_cast<float4*>(at.part_o + slot * kHeadDim);
#pragma unroll
      for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
          po[(32 * b + 8 * q4 + 4 * hh) >> 2] = make_float4(rs.oacc[b][4 * q4], rs.oacc[b][4 * q4 + 1], rs.oacc[b][4 * q4 + 2], rs.oacc[b][4 * q4 + 3]);
      if (hh == 0) { at.part_m[slot] = rs.m_run; at.part_l[slot] = l_tot; }
    }
    wave_sync();                                 // before the next block's first tile overwrites the V tile
  }
  return true;
}

// the pieces z, z + piece_grid, ... of one list, until one lies past its end
template <bool SEGMOVED, bool QDIRECT = false>
__device__ __forceinline__ void attend_diff32_body(const RoundDev& rd, const DiffDev& d, const AttendDev& at, uint16_t* Vs,
                                                   int h, int agent, int piece0, int lane) {
  for (int piece = piece0; piece < at.n_pieces; piece += at.piece_grid)
    if (!attend_diff32_piece<SEGMOVED, QDIRECT>(rd, d, at, Vs, h, agent, piece, lane)) break;
}

template <bool SEGMOVED>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2, 2))) void tdk_attend_diff_kernel(const RoundDev rd, const DiffDev d, const AttendDev at) {
  __shared__ __attribute__((aligned(16))) uint16_t Vs[kTile * kVsStride];
  // one linear id: KV head fastest, then the agent, then the wavefront's number among those of its list
  const int h = blockIdx.x % rd.heads, rest = blockIdx.x / rd.heads;
  attend_diff32_body<SEGMOVED>(rd, d, at, Vs, h, rest % rd.n_agents, rest / rd.n_agents, threadIdx.x);
}

// The same pass with 16 query rows per wavefront: used when an agent brings at most 16 rows per KV head
// (decode: query tokens x heads per KV head), where the 32-row tiles would be five sixths padding.

// Vs: this wavefront's V tile, kTile * kVsStride bf16 elements (the K rows go straight from the payload into
// the MFMA operand registers); lane: 0..63
template <bool SEGMOVED, bool QDIRECT = false>
__device__ __forceinline__ bool attend_diff16_piece(const RoundDev& rd, const DiffDev& d, const AttendDev& at, uint16_t* Vs,
                                                   int h, int agent, int piece, int lane) {
  const int T = rd.page_tokens;
  int64_t lo = d.offset[agent], hi = lo + d.count[agent];
  if (lo < 0) lo = 0;
  if (hi > d.capacity) hi = d.capacity;
  const int n_tok = hi > lo ? (int)((hi - lo) * T) : 0;
  const int n_tiles = (n_tok + kTile - 1) / kTile;
  const int piece_tiles = at.piece_tokens / kTile;
  const int tile_begin = piece * piece_tiles, tile_end = min(n_tiles, tile_begin + piece_tiles);
  if (tile_begin >= tile_end) return false;     // past the end of the list: so are the pieces after this one
  const int per_agent = at.n_q * at.group;     // at most 16: one row block
  const AgentDev ad = rd.agents[agent];
  const SessionDev sd = rd.sess[ad.session];
  const int n = lane & 15, g4 = lane >> 4;
  const int64_t row_e = (int64_t)rd.heads * kHeadDim, page_e = (int64_t)T * row_e;
  const uint16_t* pay = reinterpret_cast<const uint16_t*>(d.payload);

  // this lane's query row
  const bool row_ok = n < per_agent;
  const int qi = row_ok ? n / at.group : 0, g = row_ok ? n - qi * at.group : 0;
  const int64_t out = ((int64_t)agent * at.n_q + qi) * at.n_q_heads + h * at.group + g;
  bf16x8 qf[4];
  auto load_q = [&](int k) {
    // QDIRECT (stored diffs not moved): the listed pages meet the caller's rows as they are (but for the sign)
    const u32x4* qp = QDIRECT ? reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(at.q) + out * kHeadDim)
                              : reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(at.qdiff) +
                                                               (out * at.diff_seg + k) * kHeadDim);
    const uint32_t flip = QDIRECT && at.q_flip ? 0x80008000u : 0u;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      u32x4 v = {0, 0, 0, 0};
      if (row_ok) v = qp[4 * kk + g4];
      qf[kk] = __builtin_bit_cast(bf16x8, u32x4{v.x ^ flip, v.y ^ flip, v.z ^ flip, v.w ^ flip});
    }
  };
  if (!SEGMOVED) load_q(0);
  const int seg_base = SEGMOVED ? rd.seg_off[agent] : 0;
  const int seg_n = SEGMOVED ? rd.seg_off[agent + 1] - seg_base : 1;
  RowState16 rs;
  row_state16_init(rs);
  // The next tile travels from the payload to registers while the current one is multiplied.
  // K: lane (n, g) loads what it multiplies -- elements 32 kk + 8 g .. + 7 of the rows of tokens n and 16 + n
  // (the A operands of the two 16-token score products).  V: sixteen lanes per 256-byte row, four rows per
  // instruction, staged row-major in LDS for the transposing reads.
  u32x4 kreg[8], vreg[8];
  int p_next = -1;                             // master page of token lane % 32 of the fetched tile (-1: no such token)
  const int st_row = lane >> 4, st_pc = lane & 15;
  // The payload address of a listed token depends on its place in the list alone, so the rows are requested
  // together with the page number; what the page number decides (does the token lie inside the span, which
  // segment holds it) is settled when the tile is used.
  // (offsets inside the agent's part of the payload fit 32 bits: at most 2 P pages of 64 KB or less)
  const uint16_t* apay = pay + lo * 2 * page_e;
  const uint32_t row_u = (uint32_t)row_e, page_u = (uint32_t)page_e, tile_u = (uint32_t)(kTile / T) * 2u * page_u;
  auto tok_off = [&](int tk) { return (uint32_t)(tk / T) * 2u * page_u + (uint32_t)(tk % T) * row_u + (uint32_t)(h * kHeadDim); };
  auto fetch = [&](int tile) {
    const int t = tile * kTile + (lane & 31);
    p_next = t < n_tok ? d.idx[lo + t / T] : -1;
    const u32x4 z = {0, 0, 0, 0};
    const uint32_t tile_off = (uint32_t)tile * tile_u;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const bool there = tile * kTile + 16 * tt + n < n_tok;
      const uint32_t off = tile_off + tok_off(16 * tt + n) + 8u * g4;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        kreg[2 * kk + tt] = z;
        if (there) kreg[2 * kk + tt] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(apay + off + 32 * kk));
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      vreg[j] = z;
      if (tile * kTile + 4 * j + st_row < n_tok)
        vreg[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(apay + tile_off + tok_off(4 * j + st_row) + page_u + 8u * st_pc));
    }
  };
  fetch(tile_begin);
  for (int tile = tile_begin; tile < tile_end; ++tile) {
    wave_sync();                               // the previous tile has been consumed
    // bit t of valid: token t of the tile exists and lies inside the span (lanes 32..63 repeat lanes 0..31)
    int seg_cur = 0;
    bool ok = false;
    {
      const int rr = (tile * kTile + (lane & 31)) % T, p = p_next;
      if (p >= 0 && p < sd.pages && p * T + rr < sd.span) {
        ok = true;
        if (SEGMOVED)
          while (seg_cur + 1 < seg_n && rd.seg_src[seg_base + seg_cur + 1] <= p * T + rr) ++seg_cur;
      }
    }
    const uint32_t valid = (uint32_t)__ballot(ok);
    if (valid != 0xffffffffu) {                // rows of tokens that do not count are staged as zeros
      const u32x4 z = {0, 0, 0, 0};
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (!((valid >> (4 * j + st_row)) & 1u)) vreg[j] = z;       // (their scores are switched off below)
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) *reinterpret_cast<u32x4*>(Vs + (4 * j + st_row) * kVsStride + 8 * st_pc) = vreg[j];
    // scores 0..3 of a lane belong to tokens 4 g + i, scores 4..7 to tokens 16 + 4 g + i
    f32x4a s0, s1;
    if (!SEGMOVED) {
      scores16(kreg, qf, s0, s1);
    } else {
      // the tile's tokens come from up to four segments stored at different distances from today's
      // positions: scores once per segment present, with the queries turned back by that distance
      int sid[8];
#pragma unroll
      for (int i = 0; i < 4; ++i) { sid[i] = __shfl(seg_cur, 4 * g4 + i); sid[4 + i] = __shfl(seg_cur, 16 + 4 * g4 + i); }
#pragma unroll
      for (int i = 0; i < 4; ++i) { s0[i] = 0.f; s1[i] = 0.f; }
      int done = -1;
      while (true) {
        int cand = (lane < kTile && ((valid >> lane) & 1u) && seg_cur > done) ? seg_cur : 0x7fffffff;
#pragma unroll
        for (int sft = 32; sft > 0; sft >>= 1) cand = min(cand, __shfl_xor(cand, sft));
        if (cand == 0x7fffffff) break;
        load_q(cand);
        f32x4a p0, p1;
        scores16(kreg, qf, p0, p1);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (sid[i] == cand) s0[i] = p0[i];
          if (sid[4 + i] == cand) s1[i] = p1[i];
        }
        done = cand;
      }
    }
    wave_sync();                               // the V tile is complete
    if (tile + 1 < tile_end) fetch(tile + 1);  // the K registers are free: the scores are taken
    const uint32_t vs = valid >> (4 * g4);
    uint32_t live = (vs & 0xfu) | ((vs >> 12) & 0xf0u);
    if (!row_ok) live = 0;
    softmax_pv16(Vs, s0, s1, at.scale, live, n, g4, rs);
  }
  // this piece's partial result: lane (n, g) holds elements 16 b + 4 g + i of row n
  float l_tot = rs.l_run + __shfl_xor(rs.l_run, 16);
  l_tot += __shfl_xor(l_tot, 32);
  if (row_ok) {
    const int64_t slot = out * at.n_parts + at.n_chunks + piece;
    float4* po = reinterpret_cast<float4*>(at.part_o + slot * kHeadDim);
#pragma unroll
    for (int b = 0; b < 8; ++b) po[4 * b + g4] = make_float4(rs.oacc[b][0], rs.oacc[b][1], rs.oacc[b][2], rs.oacc[b][3]);
    if (g4 == 0) { at.part_m[slot] = rs.m_run; at.part_l[slot] = l_tot; }
  }
  return true;
}

// the pieces z, z + piece_grid, ... of one list, until one lies past its end
template <bool SEGMOVED, bool QDIRECT = false>
__device__ __forceinline__ void attend_diff16_body(const RoundDev& rd, const DiffDev& d, const AttendDev& at, uint16_t* Vs,
                                                   int h, int agent, int piece0, int lane) {
  for (int piece = piece0; piece < at.n_pieces; piece += at.piece_grid)
    if (!attend_diff16_piece<SEGMOVED, QDIRECT>(rd, d, at, Vs, h, agent, piece, lane)) break;
}

template <bool SEGMOVED>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2, 2))) void tdk_attend_diff16_kernel(const RoundDev rd, const DiffDev d, const AttendDev at) {
  __shared__ __attribute__((aligned(16))) uint16_t Vs[kTile * kVsStride];
  // one linear id: KV head fastest, then the agent, then the wavefront's number among those of its list
  const int h = blockIdx.x % rd.heads, rest = blockIdx.x / rd.heads;
  attend_diff16_body<SEGMOVED>(rd, d, at, Vs, h, rest % rd.n_agents, rest / rd.n_agents, threadIdx.x);
}

// Both passes in one launch, for rounds with identity layouts whose stored diffs have not moved and few query
// rows per agent: one ramp and one drain instead of two, and the listed-pages pass (bound by HBM) streams while
// the master pass (bound by arithmetic and LDS latency) computes.  A workgroup of the listed-pages kind = four
// wavefronts = four KV heads of one agent's piece; the pieces past 0, most of which leave at once, come last.
// Where the kinds run (measured with clock stamps and the hardware ids of the compute units): the device deals
// consecutive workgroup ids to the 8 XCDs, inside an XCD to its 4 shader engines in turn, inside an engine to its
// compute units in turn, and the two slots of a compute unit receive ids 256 apart.  With the kinds alternating
// in groups of 8 ids every engine holds one kind only; alternating in blocks of 32 puts both kinds on every
// engine but still never on one compute unit; blocks of 256 pair one workgroup of each kind on every compute
// unit.  The launch takes the same time in all three (the master workgroups slow down by what the listed ones
// gain: both wait for memory, whose latency under this launch's own 60 MB in flight is 5 to 9 us), so the
// simplest form stays.
struct FusedGrid {
  int32_t n_master;      // workgroups of the master pass: heads * (sessions * chunks) * row blocks
  int32_t row_blocks;    // blocks of 128 query rows per session and KV head
  int32_t n_diff0;       // workgroups of the listed-pages pass per piece: agents * head_groups
  int32_t head_groups;   // ceil(heads / 4)
};

constexpr int kFusedLds = kMasterLds > kWaves * kTile * kVsStride * 2 ? kMasterLds : kWaves * kTile * kVsStride * 2;

template <bool ROWS32>    // the listed-pages kind with 32-row tiles (17 to 32 rows per agent and KV head) or 16-row tiles
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(2, 2))) void tdk_attend_fused_kernel(const RoundDev rd, const LayerDev io, const DiffDev d,
                                                                  const AttendDev at, const FusedGrid fg) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[kFusedLds];
  const int bid = blockIdx.x;
  // ids alternate between the kinds in groups of eight while both last (consecutive ids go to different XCDs,
  // so both kinds reach every XCD, on different shader engines), then come the master workgroups that are left,
  // then the other kind's
  const int groups = min(fg.n_master, fg.n_diff0) >> 3;
  int m_id = -1, d_id = -1;
  if (bid < 16 * groups) {
    const int at8 = (bid >> 4) * 8 + (bid & 7);
    if (bid & 8) d_id = at8; else m_id = at8;
  } else {
    const int r = bid - 16 * groups, m_left = fg.n_master - 8 * groups;
    if (r < m_left) m_id = 8 * groups + r; else d_id = 8 * groups + (r - m_left);
  }
  if (m_id >= 0) {
    const int h = m_id % rd.heads, rest = m_id / rd.heads;
    // the row blocks of one (chunk, KV head) get ids 8 apart: same XCD, one after the other, so the second
    // finds the tiles in that XCD's L2
    attend_master_body<false, true>(rd, io, d, at, lds, h, rest / fg.row_blocks, rest % fg.row_blocks);
  } else {
    const int piece = d_id / fg.n_diff0, rem = d_id - piece * fg.n_diff0;
    const int agent = rem / fg.head_groups, h = (rem - agent * fg.head_groups) * kWaves + (threadIdx.x >> 6);
    if (h >= rd.heads) return;
    uint16_t* Vs = reinterpret_cast<uint16_t*>(lds) + (threadIdx.x >> 6) * (kTile * kVsStride);
    if (ROWS32) attend_diff32_body<false, true>(rd, d, at, Vs, h, agent, piece, threadIdx.x & 63);
    else attend_diff16_body<false, true>(rd, d, at, Vs, h, agent, piece, threadIdx.x & 63);
  }
}

// ---------------------------------------------------------------------------------------------
// merge: out = sum_c o_c e^(m_c - M) / sum_c l_c e^(m_c - M), lse = M + log(that sum); one wavefront per row
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void tdk_attend_merge_kernel(const RoundDev rd, const DiffDev d, const AttendDev at) {
  const int64_t row = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
  const int64_t n_rows = (int64_t)rd.n_agents * at.n_q * at.n_q_heads;
  if (row >= n_rows) return;
  const int lane = threadIdx.x & 63;
  const int agent = (int)(row / ((int64_t)at.n_q * at.n_q_heads));
  const int span = rd.sess[rd.agents[agent].session].span;
  const int chunks = (span + at.chunk_tokens - 1) / at.chunk_tokens;
  // the chunks of this row's span, then the pieces of its agent's listed pages
  int pieces;
  {
    int64_t lo = d.offset[agent], hi = lo + d.count[agent];
    if (lo < 0) lo = 0;
    if (hi > d.capacity) hi = d.capacity;
    const int64_t n_tok = hi > lo ? (hi - lo) * rd.page_tokens : 0;
    pieces = (int)min<int64_t>((n_tok + at.piece_tokens - 1) / at.piece_tokens, at.n_pieces);   // (a count beyond the session's pages)
  }
  const int used = chunks + pieces;
  const int64_t base = row * at.n_parts;
  auto part_of = [&](int c) { return c < chunks ? c : at.n_chunks + (c - chunks); };
  // a lane per part for the maxima and the weights, then a lane per output element
  float M = -INFINITY;
  for (int c0 = 0; c0 < used; c0 += 64) {
    const int c = c0 + lane;
    if (c < used) M = fmaxf(M, at.part_m[base + part_of(c)]);
  }
#pragma unroll
  for (int sft = 32; sft > 0; sft >>= 1) M = fmaxf(M, __shfl_xor(M, sft));
  // lane l keeps output elements 2 l and 2 l + 1; the parts' rows are requested eight at a time, before any is used
  float L = 0.f, a0 = 0.f, a1 = 0.f;
  for (int c0 = 0; c0 < used; c0 += 64) {
    const int c = c0 + lane;
    float w = 0.f;
    if (c < used) {
      const float m = at.part_m[base + part_of(c)];
      if (m != -INFINITY) { w = __expf(m - M); L = __builtin_fmaf(at.part_l[base + part_of(c)], w, L); }
    }
    const int cnt = min(64, used - c0);
    for (int j0 = 0; j0 < cnt; j0 += 8) {
      f32x2a v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        v[j] = f32x2a{0.f, 0.f};
        if (j0 + j < cnt)
          v[j] = __builtin_nontemporal_load(reinterpret_cast<const f32x2a*>(at.part_o + (base + part_of(c0 + j0 + j)) * kHeadDim) + lane);
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float wj = __shfl(w, (j0 + j) & 63);           // 0 for a part that does not exist or is empty
        if (j0 + j < cnt && wj != 0.f) {                     // (an empty part's row was never written)
          a0 = __builtin_fmaf(v[j].x, wj, a0);
          a1 = __builtin_fmaf(v[j].y, wj, a1);
        }
      }
    }
  }
#pragma unroll
  for (int sft = 32; sft > 0; sft >>= 1) L += __shfl_xor(L, sft);
  const float inv = L > 0.f ? 1.f / L : 0.f;
  reinterpret_cast<float2*>(at.out + row * kHeadDim)[lane] = make_float2(a0 * inv, a1 * inv);
  if (lane == 0) at.lse[row] = L > 0.f ? M + __logf(L) : -INFINITY;
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
hipError_t launch_attend_qrot(const RoundDev& rd, const AttendDev& at, hipStream_t st) {
  const int64_t rows = (int64_t)rd.n_agents * at.n_q * at.n_q_heads;
  if (rows == 0) return hipSuccess;
  hipLaunchKernelGGL(tdk_attend_qrot_kernel, dim3((unsigned)((rows + kWaves - 1) / kWaves)), dim3(kBlock), 0, st, rd, at);
  return hipGetLastError();
}

hipError_t launch_attend_master(const RoundDev& rd, const LayerDev& io, const DiffDev& d, const AttendDev& at,
                                int max_rows, hipStream_t st) {
  if (rd.n_sessions == 0 || at.n_chunks == 0 || max_rows == 0) return hipSuccess;
  // the KV heads of one chunk get consecutive workgroup ids: they start together and read neighbouring
  // 256-byte pieces of the same master rows
  // and the row blocks of a chunk follow each other (the second finds the tiles in L2)
  const int row_blocks = (max_rows + kRowsPerBlock - 1) / kRowsPerBlock;
  const int64_t blocks = (int64_t)rd.heads * row_blocks * rd.n_sessions * at.n_chunks;
  if (blocks >= ((int64_t)1 << 31)) return hipErrorInvalidConfiguration;
  const dim3 grid((unsigned)blocks);
  if (rd.seg) hipLaunchKernelGGL(tdk_attend_master_kernel<true>, grid, dim3(kBlock), 0, st, rd, io, d, at, row_blocks);
  else hipLaunchKernelGGL(tdk_attend_master_kernel<false>, grid, dim3(kBlock), 0, st, rd, io, d, at, row_blocks);
  return hipGetLastError();
}

hipError_t launch_attend_diff(const RoundDev& rd, const DiffDev& d, const AttendDev& at, hipStream_t st) {
  if (rd.n_agents == 0) return hipSuccess;
  // piece_grid wavefronts per list (agent, KV head): wavefront z takes the pieces z, z + piece_grid, ...
  const int64_t blocks = (int64_t)rd.heads * rd.n_agents * at.piece_grid;
  if (blocks >= ((int64_t)1 << 31)) return hipErrorInvalidConfiguration;
  const dim3 grid((unsigned)blocks);
  if (at.n_q * at.group <= 16) {
    if (at.diff_seg > 1) hipLaunchKernelGGL(tdk_attend_diff16_kernel<true>, grid, dim3(64), 0, st, rd, d, at);
    else hipLaunchKernelGGL(tdk_attend_diff16_kernel<false>, grid, dim3(64), 0, st, rd, d, at);
  } else {
    if (at.diff_seg > 1) hipLaunchKernelGGL(tdk_attend_diff_kernel<true>, grid, dim3(64), 0, st, rd, d, at);
    else hipLaunchKernelGGL(tdk_attend_diff_kernel<false>, grid, dim3(64), 0, st, rd, d, at);
  }
  return hipGetLastError();
}

int attend_piece_tokens(int64_t lists, int n_cus) {
  // lists = agents x KV heads.  A piece is 512 tokens, unless the round is so small (at most one list per compute
  // unit) that its few wavefronts would each walk ten or more tiles one after another while most
  // of the chip idles: then 128.  (Shorter pieces in larger rounds cost more in start-up than they gain: the
  // 100-agent long round 138 -> 162 us with pieces of 256 tokens.)
  return (lists > n_cus ? kPieceTiles : kPieceTiles / 4) * kTile;
}

hipError_t launch_attend_fused(const RoundDev& rd, const LayerDev& io, const DiffDev& d, const AttendDev& at,
                               int max_rows, hipStream_t st) {
  FusedGrid fg;
  fg.row_blocks = (max_rows + kRowsPerBlock - 1) / kRowsPerBlock;
  fg.n_master = rd.heads * rd.n_sessions * at.n_chunks * fg.row_blocks;
  fg.head_groups = (rd.heads + kWaves - 1) / kWaves;
  fg.n_diff0 = rd.n_agents * fg.head_groups;
  const int64_t blocks = (int64_t)fg.n_master + (int64_t)fg.n_diff0 * at.piece_grid;
  if (blocks == 0) return hipSuccess;
  if (at.n_q * at.group > 16) hipLaunchKernelGGL(tdk_attend_fused_kernel<true>, dim3((unsigned)blocks), dim3(kBlock), 0, st, rd, io, d, at, fg);
  else hipLaunchKernelGGL(tdk_attend_fused_kernel<false>, dim3((unsigned)blocks), dim3(kBlock), 0, st, rd, io, d, at, fg);
  return hipGetLastError();
}

hipError_t launch_attend_merge(const RoundDev& rd, const DiffDev& d, const AttendDev& at, hipStream_t st) {
  const int64_t rows = (int64_t)rd.n_agents * at.n_q * at.n_q_heads;
  if (rows == 0) return hipSuccess;
  hipLaunchKernelGGL(tdk_attend_merge_kernel, dim3((unsigned)((rows + kWaves - 1) / kWaves)), dim3(kBlock), 0, st, rd, d, at);
  return hipGetLastError();
}

}  // namespace tdk
