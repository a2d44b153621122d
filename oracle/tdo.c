/*
 * tdo.c -- plain CPU oracle (TEST INFRASTRUCTURE ONLY; see tdo.h).
 *
 * Scalar loops, one definition per function, no blocking or fusion.  The only
 * parallelism is an OpenMP loop over agents.  Build: gcc -O2 -fopenmp
 * -ffp-contract=off (no implicit fused multiply-adds: the fp32 path below pins
 * its operation order explicitly).
 */
#include "tdo.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- bf16 storage format: upper 16 bits of an IEEE fp32 ------------------ */

static float bf16_to_f32(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return f;
}

/* round-to-nearest-even; NaN stays NaN (quieted) */
static uint16_t f32_to_bf16(float f) {
  uint32_t u;
  memcpy(&u, &f, sizeof u);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

/* double -> bf16 with a single rounding: go through fp32, but when that first
 * rounding was inexact and landed exactly on a bf16 tie, nudge the fp32 value
 * off the tie towards the true value so the second rounding goes the right way. */
static uint16_t f64_to_bf16(double d) {
  float f = (float)d;
  uint32_t u;
  memcpy(&u, &f, sizeof u);
  if ((u & 0x7fffffffu) >= 0x7f800000u) return f32_to_bf16(f);
  if ((double)f != d && (u & 0xffffu) == 0x8000u) {
    if (fabs((double)f) < fabs(d)) u |= 1u; else u -= 1u;
    memcpy(&f, &u, sizeof f);
  }
  return f32_to_bf16(f);
}

/* ---- RoPE tables: phi_j = delta * theta^(-2j/D)  [Sec. 2.2] -------------- */

int tdo_rope_table_f64(double theta, int32_t head_dim, int64_t delta, double* c, double* s) {
  if (!c || !s || head_dim <= 0 || (head_dim & 1) || !(theta > 0.0)) return -1;
  for (int32_t j = 0; j < head_dim / 2; ++j) {
    double inv_freq = pow(theta, -(double)(2 * j) / (double)head_dim);
    double phi = (double)delta * inv_freq;
    c[j] = cos(phi);
    s[j] = sin(phi);
  }
  return 0;
}

int tdo_rope_table_f32(double theta, int32_t head_dim, int64_t delta, float* c, float* s) {
  if (!c || !s || head_dim <= 0 || (head_dim & 1) || !(theta > 0.0)) return -1;
  double* t = (double*)malloc(sizeof(double) * (size_t)head_dim);
  if (!t) return -2;
  tdo_rope_table_f64(theta, head_dim, delta, t, t + head_dim / 2);
  for (int32_t j = 0; j < head_dim / 2; ++j) {
    c[j] = (float)t[j];
    s[j] = (float)t[head_dim / 2 + j];
  }
  free(t);
  return 0;
}

static int geom_ok(const tdo_geom* g) {
  return g && g->num_kv_heads > 0 && g->head_dim > 0 && !(g->head_dim & 1) && g->page_tokens > 0 &&
         (g->rope_style == TDO_ROPE_HALF || g->rope_style == TDO_ROPE_INTERLEAVED) &&
         g->rope_theta > 0.0 && (g->math == TDO_MATH_F32 || g->math == TDO_MATH_F64);
}

typedef struct {
  int32_t half;
  float*  cf; float*  sf;   /* fp32 tables (TDO_MATH_F32) */
  double* cd; double* sd;   /* fp64 tables (TDO_MATH_F64) */
} rope_tab;

static int tab_init(rope_tab* t, const tdo_geom* g, int64_t delta) {
  t->half = g->head_dim / 2;
  t->cd = (double*)malloc(sizeof(double) * 2 * (size_t)t->half);
  t->cf = (float*)malloc(sizeof(float) * 2 * (size_t)t->half);
  if (!t->cd || !t->cf) { free(t->cd); free(t->cf); return -2; }
  t->sd = t->cd + t->half;
  t->sf = t->cf + t->half;
  tdo_rope_table_f64(g->rope_theta, g->head_dim, delta, t->cd, t->sd);
  tdo_rope_table_f32(g->rope_theta, g->head_dim, delta, t->cf, t->sf);
  return 0;
}

static void tab_free(rope_tab* t) { free(t->cd); free(t->cf); }

/* index of the two members of pair j inside a head */
static void pair_index(const tdo_geom* g, int32_t j, int32_t* a, int32_t* b) {
  if (g->rope_style == TDO_ROPE_HALF) { *a = j; *b = j + g->head_dim / 2; }
  else { *a = 2 * j; *b = 2 * j + 1; }
}

/* y_a = x_a cos - x_b sin ; y_b = x_b cos + x_a sin.
 * fp32 path, fixed order: one rounded product, then one fused multiply-add. */
static void rot_f32(float xa, float xb, float c, float s, float* ya, float* yb) {
  float t = xb * s;
  float u = xa * s;
  *ya = fmaf(xa, c, -t);
  *yb = fmaf(xb, c, u);
}

/* one [H][D] row, fp32 in / fp32 out */
static void rotate_row_f32io(const tdo_geom* g, const rope_tab* t, const float* x, float* y) {
  for (int32_t h = 0; h < g->num_kv_heads; ++h)
    for (int32_t j = 0; j < t->half; ++j) {
      int32_t a, b;
      pair_index(g, j, &a, &b);
      a += h * g->head_dim; b += h * g->head_dim;
      if (g->math == TDO_MATH_F32) {
        rot_f32(x[a], x[b], t->cf[j], t->sf[j], &y[a], &y[b]);
      } else {
        double xa = x[a], xb = x[b];
        y[a] = (float)(xa * t->cd[j] - xb * t->sd[j]);
        y[b] = (float)(xb * t->cd[j] + xa * t->sd[j]);
      }
    }
}

/* one [H][D] row, bf16 in / bf16 out */
static void rotate_row_bf16(const tdo_geom* g, const rope_tab* t, const uint16_t* x, uint16_t* y) {
  for (int32_t h = 0; h < g->num_kv_heads; ++h)
    for (int32_t j = 0; j < t->half; ++j) {
      int32_t a, b;
      pair_index(g, j, &a, &b);
      a += h * g->head_dim; b += h * g->head_dim;
      float xa = bf16_to_f32(x[a]), xb = bf16_to_f32(x[b]);
      if (g->math == TDO_MATH_F32) {
        float ya, yb;
        rot_f32(xa, xb, t->cf[j], t->sf[j], &ya, &yb);
        y[a] = f32_to_bf16(ya);
        y[b] = f32_to_bf16(yb);
      } else {
        y[a] = f64_to_bf16((double)xa * t->cd[j] - (double)xb * t->sd[j]);
        y[b] = f64_to_bf16((double)xb * t->cd[j] + (double)xa * t->sd[j]);
      }
    }
}

int tdo_rotate_rows_f32(const tdo_geom* g, int64_t delta, int64_t n_rows, const float* in, float* out) {
  if (!geom_ok(g) || n_rows < 0 || (n_rows && (!in || !out))) return -1;
  rope_tab t;
  if (tab_init(&t, g, delta)) return -2;
  int64_t re = (int64_t)g->num_kv_heads * g->head_dim;
  for (int64_t r = 0; r < n_rows; ++r) rotate_row_f32io(g, &t, in + r * re, out + r * re);
  tab_free(&t);
  return 0;
}

/* fp32 in, bf16 out: the rotation of tdo_rotate_rows_f32 followed by the storage rounding */
int tdo_rotate_rows_f32_bf16(const tdo_geom* g, int64_t delta, int64_t n_rows, const float* in, uint16_t* out) {
  if (!geom_ok(g) || n_rows < 0 || (n_rows && (!in || !out))) return -1;
  rope_tab t;
  if (tab_init(&t, g, delta)) return -2;
  int64_t re = (int64_t)g->num_kv_heads * g->head_dim;
  float* y = (float*)malloc((size_t)re * sizeof(float));
  if (!y) { tab_free(&t); return -2; }
  for (int64_t r = 0; r < n_rows; ++r) {
    rotate_row_f32io(g, &t, in + r * re, y);
    for (int64_t e = 0; e < re; ++e) out[r * re + e] = f32_to_bf16(y[e]);
  }
  free(y);
  tab_free(&t);
  return 0;
}

int tdo_rotate_rows_bf16(const tdo_geom* g, int64_t delta, int64_t n_rows, const uint16_t* in, uint16_t* out) {
  if (!geom_ok(g) || n_rows < 0 || (n_rows && (!in || !out))) return -1;
  rope_tab t;
  if (tab_init(&t, g, delta)) return -2;
  int64_t re = (int64_t)g->num_kv_heads * g->head_dim;
  for (int64_t r = 0; r < n_rows; ++r) rotate_row_bf16(g, &t, in + r * re, out + r * re);
  tab_free(&t);
  return 0;
}

/* ---- round helpers ------------------------------------------------------- */

/* ---- layout of the shared blocks in an agent's prompt  [Sec. 2.1, Eq. 2] ---- */

static int has_segments(const tdo_round* r, int32_t i) {
  return r->seg_offset && r->seg_offset[i + 1] > r->seg_offset[i];
}

/* absolute position of master token m in agent i's prompt */
static int64_t token_pos(const tdo_round* r, int32_t i, int64_t m) {
  if (!has_segments(r, i)) return r->agent_pos0[i] + m;
  for (int64_t q = r->seg_offset[i]; q < r->seg_offset[i + 1]; ++q)
    if (m >= r->seg_src[q] && m < (int64_t)r->seg_src[q] + r->seg_len[q]) return r->seg_dst[q] + (m - r->seg_src[q]);
  return -1;
}

/* the same at the time the stored diff was encoded */
static int64_t token_diff_pos(const tdo_round* r, int32_t i, int64_t m) {
  if (!has_segments(r, i)) return (r->agent_diff_pos0 ? r->agent_diff_pos0[i] : r->agent_pos0[i]) + m;
  if (!r->seg_diff_dst) return token_pos(r, i, m);
  for (int64_t q = r->seg_offset[i]; q < r->seg_offset[i + 1]; ++q)
    if (m >= r->seg_src[q] && m < (int64_t)r->seg_src[q] + r->seg_len[q]) return r->seg_diff_dst[q] + (m - r->seg_src[q]);
  return -1;
}

/* keeps *t equal to the table of `delta` (rebuilt only when delta changes: once per segment) */
static int tab_for(rope_tab* t, int* have, int64_t* cur, const tdo_geom* g, int64_t delta) {
  if (*have && *cur == delta) return 0;
  if (*have) tab_free(t);
  *have = 0;
  if (tab_init(t, g, delta)) return -1;
  *have = 1;
  *cur = delta;
  return 0;
}

static int segments_ok(const tdo_geom* g, const tdo_round* r, int32_t i, int64_t S, int64_t bt_len, int64_t pool_pages) {
  const int64_t T = g->page_tokens;
  int64_t next = 0;
  for (int64_t q = r->seg_offset[i]; q < r->seg_offset[i + 1]; ++q) {
    if (r->seg_src[q] != next || r->seg_len[q] <= 0 || r->seg_dst[q] < 0) return 0;
    if (r->seg_diff_dst && r->seg_diff_dst[q] < 0) return 0;
    next += r->seg_len[q];
    for (int64_t p = r->seg_offset[i]; p < q; ++p)       /* destinations must not overlap */
      if (r->seg_dst[q] < r->seg_dst[p] + r->seg_len[p] && r->seg_dst[p] < r->seg_dst[q] + r->seg_len[q]) return 0;
    for (int64_t lp = r->seg_dst[q] / T; lp <= (r->seg_dst[q] + r->seg_len[q] - 1) / T; ++lp) {
      if (lp >= bt_len) return 0;
      int32_t pp = r->bt_flat[r->bt_offset[i] + lp];
      if (pp < 0 || pp >= pool_pages) return 0;
    }
  }
  return next == S;
}


static int round_ok(const tdo_geom* g, const tdo_round* r, int64_t pool_pages) {
  if (!geom_ok(g) || !r || r->n_sessions < 0 || r->n_agents < 0 || pool_pages < 0) return 0;
  if (r->n_sessions && (!r->span_tokens || !r->master_pos0)) return 0;
  if (r->n_agents && (!r->agent_session || !r->agent_pos0 || !r->bt_flat || !r->bt_offset)) return 0;
  for (int32_t s = 0; s < r->n_sessions; ++s) if (r->span_tokens[s] < 0) return 0;
  for (int32_t i = 0; i < r->n_agents; ++i) {
    int32_t s = r->agent_session[i];
    if (s < 0 || s >= r->n_sessions || r->agent_pos0[i] < 0) return 0;
    if (r->agent_diff_pos0 && r->agent_diff_pos0[i] < 0) return 0;
    int64_t len = r->bt_offset[i + 1] - r->bt_offset[i];
    int64_t S = r->span_tokens[s];
    if (has_segments(r, i)) {
      if (!r->seg_src || !r->seg_len || !r->seg_dst || !segments_ok(g, r, i, S, len, pool_pages)) return 0;
      continue;
    }
    if (S > 0) {
      int64_t need = (r->agent_pos0[i] + S - 1) / g->page_tokens + 1;
      if (len < need) return 0;
      for (int64_t lp = r->agent_pos0[i] / g->page_tokens; lp < need; ++lp) {
        int32_t pp = r->bt_flat[r->bt_offset[i] + lp];
        if (pp < 0 || pp >= pool_pages) return 0;
      }
    }
  }
  return 1;
}

static int64_t session_row0(const tdo_round* r, int32_t s) {
  int64_t row = 0;
  for (int32_t q = 0; q < s; ++q) row += r->span_tokens[q];
  return row;
}

/* slot map: physical pool row of master token m for agent i  [Alg. 1, "slot map S"] */
static int64_t slot_row(const tdo_geom* g, const tdo_round* r, int32_t i, int64_t m) {
  int64_t a = token_pos(r, i, m);
  int64_t T = g->page_tokens;
  return (int64_t)r->bt_flat[r->bt_offset[i] + a / T] * T + a % T;
}

static int64_t span_pages(const tdo_geom* g, int64_t S) { return (S + g->page_tokens - 1) / g->page_tokens; }

/* ---- collective rerotate  [Sec. 4.2] ------------------------------------ */

int tdo_rerotate_round(const tdo_geom* g, const tdo_round* r,
                       const uint16_t* master_k, const uint16_t* master_v,
                       uint16_t* pool_k, uint16_t* pool_v, int64_t pool_pages) {
  if (!round_ok(g, r, pool_pages) || !master_k || !master_v || !pool_k || !pool_v) return -1;
  const int64_t re = (int64_t)g->num_kv_heads * g->head_dim;
  int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t i = 0; i < r->n_agents; ++i) {
    int32_t s = r->agent_session[i];
    int64_t S = r->span_tokens[s];
    int64_t row0 = session_row0(r, s);
    rope_tab t;
    int have = 0;
    int64_t cur = 0;
    for (int64_t m = 0; m < S; ++m) {
      /* position delta of this token: where it lands minus where the master holds it */
      int64_t delta = token_pos(r, i, m) - (r->master_pos0[s] + m);
      if (tab_for(&t, &have, &cur, g, delta)) { err = 1; break; }
      int64_t dst = slot_row(g, r, i, m);
      rotate_row_bf16(g, &t, master_k + (row0 + m) * re, pool_k + dst * re);
      memcpy(pool_v + dst * re, master_v + (row0 + m) * re, (size_t)re * sizeof(uint16_t));
    }
    if (have) tab_free(&t);
  }
  return err ? -2 : 0;
}

/* ---- block-sparse diff encode  [Sec. 4.3; Sec. 5] ------------------------ */

/* differ  <=>  not (|a - ref| <= eps), evaluated in fp32; a NaN on either side differs */
static int differs(uint16_t a, uint16_t ref, float eps) {
  float d = fabsf(bf16_to_f32(a) - bf16_to_f32(ref));
  return !(d <= eps);
}

/* planes: bit 0 = K, bit 1 = V.  3 = the paired diff (one list, both planes stored); 1 or 2 = a
 * single-plane diff (only that plane is compared and stored, one plane per payload slot). */
static int encode_impl(const tdo_geom* g, const tdo_round* r,
                       const uint16_t* master_k, const uint16_t* master_v,
                       const uint16_t* pool_k, const uint16_t* pool_v, int64_t pool_pages,
                       float eps, int planes,
                       int32_t* count, int64_t* offset, int32_t* idx, uint16_t* payload,
                       int64_t capacity_pages, int32_t* overflow) {
  if (!round_ok(g, r, pool_pages) || !master_k || !master_v || !pool_k || !pool_v) return -1;
  if (!count || !offset || !overflow || capacity_pages < 0 || (capacity_pages && (!idx || !payload))) return -1;
  if (!(eps >= 0.0f)) return -1;
  const int64_t T = g->page_tokens;
  const int64_t re = (int64_t)g->num_kv_heads * g->head_dim;
  const int32_t A = r->n_agents;
  int32_t** lists = (int32_t**)calloc((size_t)(A > 0 ? A : 1), sizeof(int32_t*));
  if (!lists) return -2;
  int err = 0;

  /* 1. per-page compare of each Mirror against its Master (rotated to the Mirror's offset) */
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t i = 0; i < A; ++i) {
    int32_t s = r->agent_session[i];
    int64_t S = r->span_tokens[s];
    int64_t P = span_pages(g, S);
    int64_t row0 = session_row0(r, s);
    rope_tab t;
    int have = 0;
    int64_t cur = 0;
    uint16_t* ref = (uint16_t*)malloc((size_t)re * sizeof(uint16_t));
    lists[i] = (int32_t*)malloc((size_t)(P > 0 ? P : 1) * sizeof(int32_t));
    if (!ref || !lists[i]) { err = 1; free(ref); count[i] = 0; continue; }
    int32_t n = 0;
    for (int64_t p = 0; p < P; ++p) {
      int flag = 0;
      for (int64_t q = 0; q < T; ++q) {
        int64_t m = p * T + q;
        if (m >= S) break;                       /* rows past the span are not part of the page */
        int64_t src = slot_row(g, r, i, m);
        if (tab_for(&t, &have, &cur, g, token_pos(r, i, m) - (r->master_pos0[s] + m))) { err = 1; break; }
        rotate_row_bf16(g, &t, master_k + (row0 + m) * re, ref);
        for (int64_t e = 0; e < re; ++e) {
          if ((planes & 1) && differs(pool_k[src * re + e], ref[e], eps)) flag = 1;
          if ((planes & 2) && differs(pool_v[src * re + e], master_v[(row0 + m) * re + e], eps)) flag = 1;
        }
      }
      if (flag) lists[i][n++] = (int32_t)p;
    }
    count[i] = n;
    free(ref);
    if (have) tab_free(&t);
  }

  /* 2. exclusive prefix over agents */
  offset[0] = 0;
  for (int32_t i = 0; i < A; ++i) offset[i + 1] = offset[i] + count[i];
  *overflow = offset[A] > capacity_pages ? 1 : 0;

  /* 3. index list and K/V values of the differing pages, as they sit in the agent's cache */
  if (!err) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t i = 0; i < A; ++i) {
      int64_t S = r->span_tokens[r->agent_session[i]];
      for (int32_t k = 0; k < count[i]; ++k) {
        int64_t slot = offset[i] + k;
        if (slot >= capacity_pages) break;
        int64_t p = lists[i][k];
        idx[slot] = (int32_t)p;
        const int n_planes = planes == 3 ? 2 : 1;
        uint16_t* pk = payload + slot * n_planes * T * re;          /* K values (if stored) come first */
        uint16_t* pv = planes == 3 ? pk + T * re : pk;
        for (int64_t q = 0; q < T; ++q) {
          int64_t m = p * T + q;
          if (m < S) {
            int64_t src = slot_row(g, r, i, m);
            if (planes & 1) memcpy(pk + q * re, pool_k + src * re, (size_t)re * sizeof(uint16_t));
            if (planes & 2) memcpy(pv + q * re, pool_v + src * re, (size_t)re * sizeof(uint16_t));
          } else {
            if (planes & 1) memset(pk + q * re, 0, (size_t)re * sizeof(uint16_t));
            if (planes & 2) memset(pv + q * re, 0, (size_t)re * sizeof(uint16_t));
          }
        }
      }
    }
  }
  for (int32_t i = 0; i < A; ++i) free(lists[i]);
  free(lists);
  return err ? -2 : 0;
}

int tdo_diff_encode(const tdo_geom* g, const tdo_round* r,
                    const uint16_t* master_k, const uint16_t* master_v,
                    const uint16_t* pool_k, const uint16_t* pool_v, int64_t pool_pages,
                    float eps,
                    int32_t* count, int64_t* offset, int32_t* idx, uint16_t* payload,
                    int64_t capacity_pages, int32_t* overflow) {
  return encode_impl(g, r, master_k, master_v, pool_k, pool_v, pool_pages, eps, 3,
                     count, offset, idx, payload, capacity_pages, overflow);
}

int tdo_diff_encode_plane(const tdo_geom* g, const tdo_round* r,
                          const uint16_t* master_k, const uint16_t* master_v,
                          const uint16_t* pool_k, const uint16_t* pool_v, int64_t pool_pages,
                          float eps, int32_t plane,
                          int32_t* count, int64_t* offset, int32_t* idx, uint16_t* payload,
                          int64_t capacity_pages, int32_t* overflow) {
  if (plane != 1 && plane != 2) return -1;
  return encode_impl(g, r, master_k, master_v, pool_k, pool_v, pool_pages, eps, plane,
                     count, offset, idx, payload, capacity_pages, overflow);
}

/* ---- fused diff restore  [Sec. 4.4, Alg. 1] ------------------------------ */

static int decode_impl(const tdo_geom* g, const tdo_round* r,
                       const uint16_t* master_k, const uint16_t* master_v,
                       uint16_t* pool_k, uint16_t* pool_v, int64_t pool_pages, int planes,
                       const int32_t* count, const int64_t* offset, const int32_t* idx, const uint16_t* payload) {
  if (!round_ok(g, r, pool_pages) || !master_k || !master_v || !pool_k || !pool_v) return -1;
  if (!count || !offset) return -1;
  const int64_t T = g->page_tokens;
  const int64_t re = (int64_t)g->num_kv_heads * g->head_dim;
  int err = 0;
  for (int32_t i = 0; i < r->n_agents; ++i) {
    int64_t P = span_pages(g, r->span_tokens[r->agent_session[i]]);
    if (count[i] < 0 || (count[i] && (!idx || !payload))) return -1;
    for (int32_t k = 0; k < count[i]; ++k) {
      int32_t p = idx[offset[i] + k];
      if (p < 0 || p >= P || (k && p <= idx[offset[i] + k - 1])) return -1;
    }
  }
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t i = 0; i < r->n_agents; ++i) {
    int32_t s = r->agent_session[i];
    int64_t S = r->span_tokens[s];
    int64_t P = span_pages(g, S);
    int64_t row0 = session_row0(r, s);
    rope_tab t, td;
    int have = 0, have_d = 0;
    int64_t cur = 0, cur_d = 0;
    for (int64_t p = 0; p < P && !err; ++p) {
      /* is page p in this Mirror's diff? (plain linear search of its index list) */
      int64_t slot = -1;
      for (int32_t k = 0; k < count[i]; ++k)
        if (idx[offset[i] + k] == p) slot = offset[i] + k;
      for (int64_t q = 0; q < T; ++q) {
        int64_t m = p * T + q;
        if (m >= S) break;
        int64_t dst = slot_row(g, r, i, m);
        int64_t delta = token_pos(r, i, m) - (r->master_pos0[s] + m);
        /* the diff values sit in the frame of the position they were encoded at */
        int64_t delta_diff = token_pos(r, i, m) - token_diff_pos(r, i, m);
        if (tab_for(&t, &have, &cur, g, delta) || tab_for(&td, &have_d, &cur_d, g, delta_diff)) { err = 1; break; }
        if (slot >= 0) {
          const int n_planes = planes == 3 ? 2 : 1;
          const uint16_t* pk = payload + slot * n_planes * T * re;
          const uint16_t* pv = planes == 3 ? pk + T * re : pk;
          if (planes & 1) {
            if (delta_diff == 0) memcpy(pool_k + dst * re, pk + q * re, (size_t)re * sizeof(uint16_t));
            else rotate_row_bf16(g, &td, pk + q * re, pool_k + dst * re);
          }
          if (planes & 2) memcpy(pool_v + dst * re, pv + q * re, (size_t)re * sizeof(uint16_t));
        } else {
          if (planes & 1) rotate_row_bf16(g, &t, master_k + (row0 + m) * re, pool_k + dst * re);
          if (planes & 2) memcpy(pool_v + dst * re, master_v + (row0 + m) * re, (size_t)re * sizeof(uint16_t));
        }
      }
    }
    if (have) tab_free(&t);
    if (have_d) tab_free(&td);
  }
  return err ? -2 : 0;
}

int tdo_diff_decode(const tdo_geom* g, const tdo_round* r,
                    const uint16_t* master_k, const uint16_t* master_v,
                    uint16_t* pool_k, uint16_t* pool_v, int64_t pool_pages,
                    const int32_t* count, const int64_t* offset, const int32_t* idx, const uint16_t* payload) {
  return decode_impl(g, r, master_k, master_v, pool_k, pool_v, pool_pages, 3, count, offset, idx, payload);
}

int tdo_diff_decode_plane(const tdo_geom* g, const tdo_round* r,
                          const uint16_t* master_k, const uint16_t* master_v,
                          uint16_t* pool_k, uint16_t* pool_v, int64_t pool_pages, int32_t plane,
                          const int32_t* count, const int64_t* offset, const int32_t* idx, const uint16_t* payload) {
  if (plane != 1 && plane != 2) return -1;
  return decode_impl(g, r, master_k, master_v, pool_k, pool_v, pool_pages, plane, count, offset, idx, payload);
}

/* ---- attention over a Mirror that is never restored  [Sec. 4.4, last paragraphs: the diff applied as
 * attention tiles are loaded; Fig. 9: skip-or-correct per block] ----------------------------------- */

/* one [D] head of a key in double, rotated by delta (exact angles, no rounding of the result) */
static void rotate_head_f64(const tdo_geom* g, int64_t delta, const double* x, double* y) {
  for (int32_t j = 0; j < g->head_dim / 2; ++j) {
    int32_t a, b;
    pair_index(g, j, &a, &b);
    double phi = (double)delta * pow(g->rope_theta, -(double)(2 * j) / (double)g->head_dim);
    double c = cos(phi), sn = sin(phi);
    y[a] = x[a] * c - x[b] * sn;
    y[b] = x[b] * c + x[a] * sn;
  }
}

/* For every agent i, query row (qi, hq): softmax(scale * q . K_i[m]) over the S tokens of the shared span,
 * where the Mirror's K_i[m], V_i[m] are, token by token: the payload rows if page m / T is in the agent's diff
 * (K brought from the position it was stored at to the current one), else the master's K rotated to the
 * agent's offset (exactly: no bf16 rounding in between) and the master's V.  Query head hq reads KV head
 * hq / (n_q_heads / H).  out = sum_m p_m V_i[m]; lse = log sum_m exp(scale * q . K_i[m]) (-inf, out 0 if S = 0). */
int tdo_attend_shared(const tdo_geom* g, const tdo_round* r,
                      const uint16_t* master_k, const uint16_t* master_v,
                      const int32_t* count, const int64_t* offset, const int32_t* idx, const uint16_t* payload,
                      const uint16_t* q, int32_t n_q, int32_t n_q_heads, double scale,
                      double* out, double* lse) {
  if (!round_ok(g, r, INT64_MAX) || !master_k || !master_v) return -1;   /* no pool here: any page number passes */
  if (!count || !offset || !q || !out || !lse || n_q <= 0 || n_q_heads <= 0 || n_q_heads % g->num_kv_heads) return -1;
  const int64_t T = g->page_tokens;
  const int32_t D = g->head_dim;
  const int64_t re = (int64_t)g->num_kv_heads * D;
  const int32_t G = n_q_heads / g->num_kv_heads;
  for (int32_t i = 0; i < r->n_agents; ++i)
    if (count[i] < 0 || (count[i] && (!idx || !payload))) return -1;
  int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t i = 0; i < r->n_agents; ++i) {
    int32_t s = r->agent_session[i];
    int64_t S = r->span_tokens[s];
    int64_t row0 = session_row0(r, s);
    double* kk = (double*)malloc(sizeof(double) * (size_t)(2 * D + (S > 0 ? S : 1)));
    if (!kk) { err = 1; continue; }
    double* kr = kk + D;            /* rotated key head */
    double* sc = kk + 2 * D;        /* scores of one query row */
    for (int32_t qi = 0; qi < n_q; ++qi)
      for (int32_t hq = 0; hq < n_q_heads; ++hq) {
        const int32_t h = hq / G;
        const uint16_t* qrow = q + (((int64_t)i * n_q + qi) * n_q_heads + hq) * D;
        double* o = out + (((int64_t)i * n_q + qi) * n_q_heads + hq) * D;
        double* l = lse + ((int64_t)i * n_q + qi) * n_q_heads + hq;
        for (int32_t d = 0; d < D; ++d) o[d] = 0.0;
        double mx = -INFINITY;
        for (int64_t m = 0; m < S; ++m) {
          int64_t slot = -1;
          for (int32_t k = 0; k < count[i]; ++k)
            if (idx[offset[i] + k] == m / T) slot = offset[i] + k;
          const uint16_t* krow = slot >= 0 ? payload + (slot * 2 * T + m % T) * re + (int64_t)h * D
                                           : master_k + (row0 + m) * re + (int64_t)h * D;
          int64_t delta = slot >= 0 ? token_pos(r, i, m) - token_diff_pos(r, i, m)
                                    : token_pos(r, i, m) - (r->master_pos0[s] + m);
          for (int32_t d = 0; d < D; ++d) kk[d] = (double)bf16_to_f32(krow[d]);
          rotate_head_f64(g, delta, kk, kr);
          double acc = 0.0;
          for (int32_t d = 0; d < D; ++d) acc += (double)bf16_to_f32(qrow[d]) * kr[d];
          sc[m] = scale * acc;
          if (sc[m] > mx) mx = sc[m];
        }
        double sum = 0.0;
        for (int64_t m = 0; m < S; ++m) sum += exp(sc[m] - mx);
        *l = S > 0 ? mx + log(sum) : -INFINITY;
        for (int64_t m = 0; m < S; ++m) {
          int64_t slot = -1;
          for (int32_t k = 0; k < count[i]; ++k)
            if (idx[offset[i] + k] == m / T) slot = offset[i] + k;
          const uint16_t* vrow = slot >= 0 ? payload + ((slot * 2 + 1) * T + m % T) * re + (int64_t)h * D
                                           : master_v + (row0 + m) * re + (int64_t)h * D;
          double pm = exp(sc[m] - mx) / sum;
          for (int32_t d = 0; d < D; ++d) o[d] += pm * (double)bf16_to_f32(vrow[d]);
        }
      }
    free(kk);
  }
  return err ? -2 : 0;
}

/* ---- check layer: key-difference pass, important positions, master  [Sec. 4.2; Sec. 2.2] -------- */

/* deviation of agent i at master token m: sum over the K row of (fresh - rotated cached)^2,
 * accumulated in double.  score is agent-major: agent i's S_i scores follow those of agent i-1. */
int tdo_key_deviation(const tdo_geom* g, const tdo_round* r,
                      const uint16_t* master_k, const uint16_t* pool_k, int64_t pool_pages, double* score) {
  if (!round_ok(g, r, pool_pages) || !master_k || !pool_k || !score) return -1;
  const int64_t re = (int64_t)g->num_kv_heads * g->head_dim;
  int64_t* base = (int64_t*)malloc(sizeof(int64_t) * (size_t)(r->n_agents + 1));
  if (!base) return -2;
  base[0] = 0;
  for (int32_t i = 0; i < r->n_agents; ++i) base[i + 1] = base[i] + r->span_tokens[r->agent_session[i]];
  int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t i = 0; i < r->n_agents; ++i) {
    int32_t s = r->agent_session[i];
    int64_t S = r->span_tokens[s];
    int64_t row0 = session_row0(r, s);
    rope_tab t;
    int have = 0;
    int64_t cur = 0;
    uint16_t* ref = (uint16_t*)malloc((size_t)re * sizeof(uint16_t));
    if (!ref) { err = 1; continue; }
    for (int64_t m = 0; m < S; ++m) {
      if (tab_for(&t, &have, &cur, g, token_pos(r, i, m) - (r->master_pos0[s] + m))) { err = 1; break; }
      rotate_row_bf16(g, &t, master_k + (row0 + m) * re, ref);
      const uint16_t* fresh = pool_k + slot_row(g, r, i, m) * re;
      double acc = 0.0;
      for (int64_t e = 0; e < re; ++e) {
        double d = (double)bf16_to_f32(fresh[e]) - (double)bf16_to_f32(ref[e]);
        acc += d * d;
      }
      score[base[i] + m] = acc;
    }
    free(ref);
    if (have) tab_free(&t);
  }
  free(base);
  return err ? -2 : 0;
}

typedef struct { float v; int32_t m; } scored;

static int by_score_desc_then_index(const void* a, const void* b) {
  const scored* x = (const scored*)a; const scored* y = (const scored*)b;
  /* NaN ranks above everything */
  int xn = x->v != x->v, yn = y->v != y->v;
  if (xn != yn) return yn - xn;
  if (!xn && x->v != y->v) return x->v > y->v ? -1 : 1;
  return x->m < y->m ? -1 : (x->m > y->m);
}

static int by_index(const void* a, const void* b) {
  int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return x < y ? -1 : (x > y);
}

/* the k = ceil(ratio * S) tokens with the largest score among those with !(score <= min_score),
 * ties to the lower token number; written in ascending token order.  Plain sort. */
int tdo_select_important(const float* score, int64_t S, float ratio, float min_score,
                         int32_t* out, int32_t* n_out) {
  if (S < 0 || (S && !score) || !n_out || !(ratio > 0.0f) || !(ratio <= 1.0f)) return -1;
  int64_t k = (int64_t)ceil((double)ratio * (double)S);
  if (k > S) k = S;
  scored* c = (scored*)malloc(sizeof(scored) * (size_t)(S > 0 ? S : 1));
  if (!c) return -2;
  int64_t n = 0;
  for (int64_t m = 0; m < S; ++m)
    if (!(score[m] <= min_score)) { c[n].v = score[m]; c[n].m = (int32_t)m; ++n; }
  qsort(c, (size_t)n, sizeof(scored), by_score_desc_then_index);
  if (k > n) k = n;
  for (int64_t q = 0; q < k; ++q) out[q] = c[q].m;
  qsort(out, (size_t)k, sizeof(int32_t), by_index);
  *n_out = (int32_t)k;
  free(c);
  return 0;
}

/* master of each session = the agent with the lowest total deviation (NaN = +inf, first on ties) */
int tdo_choose_master(const tdo_round* r, const float* total, int32_t* master) {
  if (!r || (r->n_agents && !total) || (r->n_sessions && !master)) return -1;
  for (int32_t s = 0; s < r->n_sessions; ++s) {
    master[s] = -1;
    float best = INFINITY;
    for (int32_t i = 0; i < r->n_agents; ++i) {
      if (r->agent_session[i] != s) continue;
      float t = total[i];
      if (t != t) t = INFINITY;
      if (master[s] < 0 || t < best) { best = t; master[s] = i; }
    }
  }
  return 0;
}

/* ---- layerwise restore of all layers  [Sec. 4.4, Alg. 1] ------------------
 * The algorithm as stated: two buffers alternate between "load" and "compute"; per layer the master
 * chunks are loaded into the load buffer, the buffers swap, and the compute buffer is corrected with
 * the layer's diff, position-recovered and written to paged memory through the slot map. */
int tdo_restore_layers(const tdo_geom* g, const tdo_round* r, int32_t n_layers,
                       const uint16_t* const* master_k, const uint16_t* const* master_v,
                       uint16_t* const* pool_k, uint16_t* const* pool_v, int64_t pool_pages,
                       const int32_t* const* count, const int64_t* const* offset,
                       const int32_t* const* idx, const uint16_t* const* payload) {
  if (!geom_ok(g) || !r || n_layers < 0) return -1;
  if (n_layers && (!master_k || !master_v || !pool_k || !pool_v || !count || !offset || !idx || !payload)) return -1;
  int64_t rows = 0;
  for (int32_t s = 0; s < r->n_sessions; ++s) rows += r->span_tokens[s];
  const size_t bytes = (size_t)rows * g->num_kv_heads * g->head_dim * sizeof(uint16_t);
  uint16_t* buf_k[2] = {(uint16_t*)malloc(bytes ? bytes : 1), (uint16_t*)malloc(bytes ? bytes : 1)};
  uint16_t* buf_v[2] = {(uint16_t*)malloc(bytes ? bytes : 1), (uint16_t*)malloc(bytes ? bytes : 1)};
  int rc = 0;
  if (!buf_k[0] || !buf_k[1] || !buf_v[0] || !buf_v[1]) rc = -2;
  int load = 0, comp = 1;
  for (int32_t l = 0; l < n_layers && rc == 0; ++l) {
    memcpy(buf_k[load], master_k[l], bytes);            /* load master chunks of layer l */
    memcpy(buf_v[load], master_v[l], bytes);
    { int t = load; load = comp; comp = t; }            /* sync; swap */
    rc = tdo_diff_decode(g, r, buf_k[comp], buf_v[comp], pool_k[l], pool_v[l], pool_pages,
                         count[l], offset[l], idx[l], payload[l]);
  }
  free(buf_k[0]); free(buf_k[1]); free(buf_v[0]); free(buf_v[1]);
  return rc;
}

/* ---- storage arithmetic  [Sec. 6.4] -------------------------------------- */

double tdo_dense_bytes(const tdo_geom* g, int64_t span_tokens) {
  return (double)span_tokens * 2.0 * (double)g->num_kv_heads * (double)g->head_dim * 2.0;
}

double tdo_diff_bytes(const tdo_geom* g, int64_t diff_pages) {
  double page = 2.0 * (double)g->page_tokens * (double)g->num_kv_heads * (double)g->head_dim * 2.0;
  return (double)diff_pages * page + 4.0 * (double)diff_pages + 4.0 + 8.0;  /* values + idx + count + offset */
}

double tdo_mirror_ratio(const tdo_geom* g, int64_t span_tokens, int64_t diff_pages) {
  return tdo_dense_bytes(g, span_tokens) / tdo_diff_bytes(g, diff_pages);
}

double tdo_family_cost(int64_t n_agents, double ratio) {
  return 1.0 + (double)(n_agents - 1) / ratio;
}

int tdo_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Number of threads the agent loops may use from now on (timing only; results do not depend on it). */
void tdo_set_threads(int n) {
#ifdef _OPENMP
  if (n >= 1) omp_set_num_threads(n);
#else
  (void)n;
#endif
}
