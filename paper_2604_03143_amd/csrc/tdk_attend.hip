// Attention of new query tokens over the shared span of every mirror, computed from master + diff
// with no restored copy (Sec. 4.4, last paragraphs: the diff applied as attention tiles are loaded;
// Fig. 9: skip-or-correct per block).
//
// RoPE rotations are orthogonal, so q . (R(delta) k) = (R(-delta) q) . k: instead of rotating the
// master's keys once per agent, each agent's few query rows are rotated back by its offset and all
// agents of a session then attend to the SAME un-rotated master keys.  The query rows of a session
// (agents x query tokens x query heads of one KV head) become the N side of one dense product with
// the master's K and V tiles, which is MFMA work, and the master is read once per session instead of
// once per agent.  Pages that an agent's diff lists are masked out of that product for that agent's
// rows and handled by a second, small kernel from the payload (the "correct" half); a third kernel
// merges the partial results with their log-sum-exp weights.
#include "tdk_internal.h"

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
constexpr int kVtStride = kTile + 4;      // bf16 elements per staged V^T row

__device__ __forceinline__ float bfl(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bfh(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
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
  const float* tab = rd.tab + (size_t)agent * (2 * kHalf);
  const uint16_t* src = reinterpret_cast<const uint16_t*>(at.q) + row * kHeadDim;
  uint16_t* dst = reinterpret_cast<uint16_t*>(at.qrot) + row * kHeadDim;
  const int ia = rd.interleaved ? 2 * lane : lane;
  const int ib = rd.interleaved ? 2 * lane + 1 : lane + kHalf;
  const float xa = __uint_as_float((uint32_t)src[ia] << 16), xb = __uint_as_float((uint32_t)src[ib] << 16);
  const float c = tab[lane], s = tab[kHalf + lane];
  // rotation by -delta: y_a = x_a cos + x_b sin, y_b = x_b cos - x_a sin
  const float ya = __builtin_fmaf(xa, c, __fmul_rn(xb, s));
  const float yb = __builtin_fmaf(xb, c, -__fmul_rn(xa, s));
  dst[ia] = (uint16_t)(pack2(ya, 0.f) & 0xffffu);
  dst[ib] = (uint16_t)(pack2(yb, 0.f) & 0xffffu);
}

// ---------------------------------------------------------------------------------------------
// master pass: S^T = K Q'^T and O^T += V^T P^T per 32-token tile, online softmax per query row
// grid: x = session * n_chunks + chunk, y = KV head, z = block of 128 query rows
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void tdk_attend_master_kernel(const RoundDev rd, const LayerDev io, const DiffDev d,
                                                                   const AttendDev at) {
  __shared__ __attribute__((aligned(16))) uint16_t Ks[kTile * kKsStride];
  __shared__ __attribute__((aligned(16))) uint16_t Vt[kHeadDim * kVtStride];
  __shared__ uint32_t s_mask[kRowsPerBlock];    // bit p: page p of this chunk is listed in the row's agent's diff

  const int session = blockIdx.x / at.n_chunks, chunk = blockIdx.x - session * at.n_chunks;
  const SessionDev sd = rd.sess[session];
  const int tok_begin = chunk * at.chunk_tokens;
  if (tok_begin >= sd.span || sd.n_agents == 0) return;
  const int rows = sd.n_agents * at.n_q * at.group;
  const int row_begin = blockIdx.z * kRowsPerBlock;
  if (row_begin >= rows) return;
  const int h = blockIdx.y;
  const int T = rd.page_tokens;
  const int tok_end = min(sd.span, tok_begin + at.chunk_tokens);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 31, hh = lane >> 5;

  // which pages of this chunk each row's agent lists in its diff (those tokens belong to the other kernel)
  if (threadIdx.x < kRowsPerBlock) {
    uint32_t mask = 0;
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
        mask |= 1u << (p - pg0);
      }
    }
    s_mask[threadIdx.x] = mask;
  }

  // this lane's query row: its B operands (8 steps of 16 along the head dimension) stay in registers
  const RowRef mine = row_ref(rd, sd, at, h, row_begin + wave * kRowsPerWave + n);
  bf16x8 qf[8];
  {
    const u32x4* qp = reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(at.qrot) + mine.out * kHeadDim);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      u32x4 v = {0, 0, 0, 0};
      if (mine.agent >= 0) v = qp[2 * kk + hh];
      qf[kk] = __builtin_bit_cast(bf16x8, v);
    }
  }
  __syncthreads();
  const uint32_t my_mask = s_mask[wave * kRowsPerWave + n];

  f32x16 oacc[4];
#pragma unroll
  for (int b = 0; b < 4; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[b][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const int64_t head_u4 = 16;                                  // 128 bf16 = 16 chunks of 16 bytes
  const int64_t row_u4 = (int64_t)rd.heads * head_u4;
  const int st_tok = threadIdx.x >> 3, st_part = threadIdx.x & 7;   // staging: 8 threads per token, 32 bytes each

  for (int t0 = tok_begin; t0 < tok_end; t0 += kTile) {
    __syncthreads();                                           // the previous tile has been consumed
    {
      const int m = t0 + st_tok;
      u32x4 k0 = {0, 0, 0, 0}, k1 = k0, v0 = k0, v1 = k0;
      if (m < tok_end) {
        const int64_t base = (sd.master_row0 + m) * row_u4 + h * head_u4 + st_part * 2;
        k0 = io.master_k[base]; k1 = io.master_k[base + 1];
        v0 = io.master_v[base]; v1 = io.master_v[base + 1];
      }
      u32x4* kd = reinterpret_cast<u32x4*>(Ks + st_tok * kKsStride + st_part * 16);
      kd[0] = k0; kd[1] = k1;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int dd = st_part * 16 + 2 * e;
        Vt[(dd + 0) * kVtStride + st_tok] = (uint16_t)(v0[e] & 0xffffu);
        Vt[(dd + 1) * kVtStride + st_tok] = (uint16_t)(v0[e] >> 16);
        Vt[(dd + 8) * kVtStride + st_tok] = (uint16_t)(v1[e] & 0xffffu);
        Vt[(dd + 9) * kVtStride + st_tok] = (uint16_t)(v1[e] >> 16);
      }
    }
    __syncthreads();

    // S^T (tokens x rows) = K (tokens x d) * Q'^T (d x rows)
    f32x16 sacc;
#pragma unroll
    for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const u32x4 a = *reinterpret_cast<const u32x4*>(Ks + n * kKsStride + 16 * kk + 8 * hh);
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), qf[kk], sacc, 0, 0, 0);
    }
    // this lane holds, for its query row, the tokens 8 (i / 4) + 4 hh + i % 4 of the tile
    float p[16];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int m = t0 + 8 * (i >> 2) + 4 * hh + (i & 3);
      const bool masked = m >= tok_end || ((my_mask >> ((m - tok_begin) / T)) & 1u) || mine.agent < 0;
      p[i] = masked ? -INFINITY : sacc[i] * at.scale;
      mx = fmaxf(mx, p[i]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float m_ref = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __expf(m_run - m_ref);
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) { p[i] = __expf(p[i] - m_ref); sum += p[i]; }
    l_run = l_run * alpha + sum;
    m_run = m_new;
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[b][i] *= alpha;

    // O^T (d x rows) += V^T (d x tokens) * P^T (tokens x rows); the contraction runs over the tokens in the
    // order this lane holds them, so P^T needs no exchange between lanes
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      u32x4 pw;
#pragma unroll
      for (int e = 0; e < 4; ++e) pw[e] = pack2(p[8 * kk + 2 * e], p[8 * kk + 2 * e + 1]);
      const bf16x8 pb = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const uint16_t* vr = Vt + (32 * b + n) * kVtStride + 16 * kk + 4 * hh;
        const uint2 lo = *reinterpret_cast<const uint2*>(vr);
        const uint2 hi = *reinterpret_cast<const uint2*>(vr + 8);
        const u32x4 a = {lo.x, lo.y, hi.x, hi.y};
        oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), pb, oacc[b], 0, 0, 0);
      }
    }
  }

  // partial result of this chunk: un-normalised output, running maximum and sum
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (mine.agent >= 0) {
    const int64_t slot = mine.out * at.n_parts + chunk;
    float4* po = reinterpret_cast<float4*>(at.part_o + slot * kHeadDim);
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
        po[(32 * b + 8 * q4 + 4 * hh) >> 2] = make_float4(oacc[b][4 * q4], oacc[b][4 * q4 + 1], oacc[b][4 * q4 + 2], oacc[b][4 * q4 + 3]);
    if (hh == 0) { at.part_m[slot] = m_run; at.part_l[slot] = l_tot; }
  }
}

// ---------------------------------------------------------------------------------------------
// diff pass: the pages an agent's diff lists, from the payload (fp32 arithmetic, no MFMA: a few
// hundred tokens per agent).  One workgroup per (agent, KV head, block of up to 8 query rows).
// ---------------------------------------------------------------------------------------------
constexpr int kDiffRows = 8;

__global__ __launch_bounds__(kBlock) void tdk_attend_diff_kernel(const RoundDev rd, const DiffDev d, const AttendDev at) {
  __shared__ float s_q[kDiffRows][kHeadDim];
  __shared__ float s_p[kDiffRows][kBlock];
  __shared__ float s_red[kDiffRows][kWaves];
  __shared__ float s_o[kDiffRows][kHeadDim];

  const int agent = blockIdx.x, h = blockIdx.y;
  const int per_agent = at.n_q * at.group;
  const int r0 = blockIdx.z * kDiffRows;
  if (r0 >= per_agent) return;
  const int nrows = min(kDiffRows, per_agent - r0);
  const AgentDev ad = rd.agents[agent];
  const SessionDev sd = rd.sess[ad.session];
  const int T = rd.page_tokens;
  int64_t lo = d.offset[agent], hi = lo + d.count[agent];
  if (lo < 0) lo = 0;
  if (hi > d.capacity) hi = d.capacity;
  const int64_t n_tok = hi > lo ? (hi - lo) * T : 0;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

  // query rows in fp32; if the stored values sit at another position than today's, the queries are
  // rotated back by that distance instead of rotating every stored key forward
  for (int i = tid; i < nrows * kHalf; i += kBlock) {
    const int r = i / kHalf, j = i - r * kHalf;
    const int rem = r0 + r, qi = rem / at.group, g = rem - qi * at.group;
    const uint16_t* src = reinterpret_cast<const uint16_t*>(at.q) +
                          (((int64_t)agent * at.n_q + qi) * at.n_q_heads + h * at.group + g) * kHeadDim;
    const int ia = rd.interleaved ? 2 * j : j, ib = rd.interleaved ? 2 * j + 1 : j + kHalf;
    float xa = __uint_as_float((uint32_t)src[ia] << 16), xb = __uint_as_float((uint32_t)src[ib] << 16);
    if (ad.diff_rot) {
      const float c = rd.tab_diff[(size_t)agent * (2 * kHalf) + j], s = rd.tab_diff[(size_t)agent * (2 * kHalf) + kHalf + j];
      const float ya = __builtin_fmaf(xa, c, __fmul_rn(xb, s)), yb = __builtin_fmaf(xb, c, -__fmul_rn(xa, s));
      xa = ya; xb = yb;
    }
    s_q[r][ia] = xa; s_q[r][ib] = xb;
  }
  float m_run[kDiffRows], l_run[kDiffRows], o0[kDiffRows];   // this thread: d = tid % 128, one half of each block of tokens
#pragma unroll
  for (int r = 0; r < kDiffRows; ++r) { m_run[r] = -INFINITY; l_run[r] = 0.f; o0[r] = 0.f; }
  __syncthreads();

  const int64_t row_e = (int64_t)rd.heads * kHeadDim;                  // bf16 elements per token row
  const int64_t page_e = (int64_t)T * row_e;
  const uint16_t* pay = reinterpret_cast<const uint16_t*>(d.payload);
  for (int64_t tb = 0; tb < n_tok; tb += kBlock) {
    // scores of one token per thread
    const int64_t t = tb + tid;
    float sc[kDiffRows];
#pragma unroll
    for (int r = 0; r < kDiffRows; ++r) sc[r] = -INFINITY;
    if (t < n_tok) {
      const int64_t slot = lo + t / T;
      const int rr = (int)(t % T);
      const int p = d.idx[slot];
      if (p >= 0 && p < sd.pages && p * T + rr < sd.span) {
        const u32x4* kr = reinterpret_cast<const u32x4*>(pay + (slot * 2) * page_e + rr * row_e + h * kHeadDim);
        float acc[kDiffRows];
#pragma unroll
        for (int r = 0; r < kDiffRows; ++r) acc[r] = 0.f;
        for (int c = 0; c < 16; ++c) {
          const u32x4 kv = kr[c];
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            const float k0 = bfl(kv[w]), k1 = bfh(kv[w]);
#pragma unroll
            for (int r = 0; r < kDiffRows; ++r)
              if (r < nrows) acc[r] = __builtin_fmaf(s_q[r][c * 8 + 2 * w + 1], k1, __builtin_fmaf(s_q[r][c * 8 + 2 * w], k0, acc[r]));
          }
        }
#pragma unroll
        for (int r = 0; r < kDiffRows; ++r)
          if (r < nrows) sc[r] = acc[r] * at.scale;
      }
    }
    // block-wide maximum per row, then the weights of this block of tokens
#pragma unroll
    for (int r = 0; r < kDiffRows; ++r) {
      float v = sc[r];
#pragma unroll
      for (int sft = 32; sft > 0; sft >>= 1) v = fmaxf(v, __shfl_xor(v, sft));
      if (lane == 0) s_red[r][wave] = v;
    }
    __syncthreads();
    float alpha[kDiffRows];
#pragma unroll
    for (int r = 0; r < kDiffRows; ++r) {
      const float mx = fmaxf(fmaxf(s_red[r][0], s_red[r][1]), fmaxf(s_red[r][2], s_red[r][3]));
      const float m_new = fmaxf(m_run[r], mx);
      const float m_ref = m_new == -INFINITY ? 0.f : m_new;
      alpha[r] = __expf(m_run[r] - m_ref);
      m_run[r] = m_new;
      s_p[r][tid] = __expf(sc[r] - m_ref);
    }
    __syncthreads();
    // weighted V: thread = (element d, half of the block's tokens)
    const int dd = tid & (kHeadDim - 1), half = tid >> 7;
#pragma unroll
    for (int r = 0; r < kDiffRows; ++r) { o0[r] *= alpha[r]; l_run[r] *= alpha[r]; }
    const int64_t t_lo = tb + half * (kBlock / 2);
    for (int j = 0; j < kBlock / 2; ++j) {
      const int64_t tt = t_lo + j;
      if (tt >= n_tok) break;
      const int64_t slot = lo + tt / T;
      const int rr = (int)(tt % T);
      const float v = __uint_as_float((uint32_t)pay[(slot * 2 + 1) * page_e + rr * row_e + h * kHeadDim + dd] << 16);
#pragma unroll
      for (int r = 0; r < kDiffRows; ++r) {
        const float w = s_p[r][half * (kBlock / 2) + j];
        o0[r] = __builtin_fmaf(w, v, o0[r]);
        l_run[r] += w;          // every thread of a half sums the same weights: l of that half
      }
    }
    __syncthreads();
  }
  // combine the two halves and store the partial result in the last slot of each row
  if (tid >= kHeadDim) {
#pragma unroll
    for (int r = 0; r < kDiffRows; ++r) { s_o[r][tid - kHeadDim] = o0[r]; if (tid == kHeadDim) s_red[r][0] = l_run[r]; }
  }
  __syncthreads();
  if (tid < kHeadDim) {
#pragma unroll
    for (int r = 0; r < kDiffRows; ++r) {
      if (r >= nrows) continue;
      const int rem = r0 + r, qi = rem / at.group, g = rem - qi * at.group;
      const int64_t out = ((int64_t)agent * at.n_q + qi) * at.n_q_heads + h * at.group + g;
      const int64_t slot = out * at.n_parts + (at.n_parts - 1);
      at.part_o[slot * kHeadDim + tid] = o0[r] + s_o[r][tid];
      if (tid == 0) { at.part_m[slot] = m_run[r]; at.part_l[slot] = l_run[r] + s_red[r][0]; }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// merge: out = sum_c o_c e^(m_c - M) / sum_c l_c e^(m_c - M), lse = M + log(that sum); one wavefront per row
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void tdk_attend_merge_kernel(const RoundDev rd, const AttendDev at) {
  const int64_t row = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
  const int64_t n_rows = (int64_t)rd.n_agents * at.n_q * at.n_q_heads;
  if (row >= n_rows) return;
  const int lane = threadIdx.x & 63;
  const int agent = (int)(row / ((int64_t)at.n_q * at.n_q_heads));
  const int span = rd.sess[rd.agents[agent].session].span;
  const int chunks = (span + at.chunk_tokens - 1) / at.chunk_tokens;
  float M = -INFINITY;
  for (int c = 0; c <= chunks; ++c) {
    const int part = c < chunks ? c : at.n_parts - 1;
    M = fmaxf(M, at.part_m[row * at.n_parts + part]);
  }
  float L = 0.f, a0 = 0.f, a1 = 0.f;
  if (M != -INFINITY) {
    for (int c = 0; c <= chunks; ++c) {
      const int part = c < chunks ? c : at.n_parts - 1;
      const int64_t slot = row * at.n_parts + part;
      const float m = at.part_m[slot];
      if (m == -INFINITY) continue;
      const float w = __expf(m - M);
      L = __builtin_fmaf(at.part_l[slot], w, L);
      a0 = __builtin_fmaf(at.part_o[slot * kHeadDim + lane], w, a0);
      a1 = __builtin_fmaf(at.part_o[slot * kHeadDim + 64 + lane], w, a1);
    }
  }
  const float inv = L > 0.f ? 1.f / L : 0.f;
  at.out[row * kHeadDim + lane] = a0 * inv;
  at.out[row * kHeadDim + 64 + lane] = a1 * inv;
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
  const dim3 grid((unsigned)(rd.n_sessions * at.n_chunks), (unsigned)rd.heads,
                  (unsigned)((max_rows + kRowsPerBlock - 1) / kRowsPerBlock));
  hipLaunchKernelGGL(tdk_attend_master_kernel, grid, dim3(kBlock), 0, st, rd, io, d, at);
  return hipGetLastError();
}

hipError_t launch_attend_diff(const RoundDev& rd, const DiffDev& d, const AttendDev& at, hipStream_t st) {
  if (rd.n_agents == 0) return hipSuccess;
  const int per_agent = at.n_q * at.group;
  const dim3 grid((unsigned)rd.n_agents, (unsigned)rd.heads, (unsigned)((per_agent + kDiffRows - 1) / kDiffRows));
  hipLaunchKernelGGL(tdk_attend_diff_kernel, grid, dim3(kBlock), 0, st, rd, d, at);
  return hipGetLastError();
}

hipError_t launch_attend_merge(const RoundDev& rd, const AttendDev& at, hipStream_t st) {
  const int64_t rows = (int64_t)rd.n_agents * at.n_q * at.n_q_heads;
  if (rows == 0) return hipSuccess;
  hipLaunchKernelGGL(tdk_attend_merge_kernel, dim3((unsigned)((rows + kWaves - 1) / kWaves)), dim3(kBlock), 0, st, rd, at);
  return hipGetLastError();
}

}  // namespace tdk
