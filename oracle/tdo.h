/*
 * tdo -- plain CPU oracle for the collective KV-reuse step (TEST INFRASTRUCTURE ONLY).
 *
 * This is the slow, obviously-correct definition the HIP library is checked
 * against.  It is not part of the product: nothing outside the test-suite, the
 * smoke check and the benchmark's CPU-baseline leg may call it, and it shares no
 * code, table or helper with the HIP path.
 *
 * What it defines (paper passages in brackets):
 *   - RoPE re-rotation of cached keys by a position delta            [Sec. 2.2; Alg. 1 "RoPERecover"]
 *   - one collective rerotate step for a whole round                 [Sec. 4.2 "Layerwise Collective Reuse"]
 *   - the block-sparse Master/Mirror diff: indices + K/V values      [Sec. 4.3; Sec. 5 "Diff-Aware Storage"]
 *   - restore of every Mirror from Master + diff via the slot map    [Sec. 4.4, Alg. 1]
 *   - compression-ratio / capacity arithmetic                        [Sec. 6.4]
 *
 * All pointers are HOST pointers.  bf16 values are passed as uint16_t bit patterns.
 * Every function returns 0 on success and a negative value on an invalid argument.
 */
#ifndef TDO_H
#define TDO_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TDO_ROPE_HALF        0   /* pair (j, j + D/2) inside a head   */
#define TDO_ROPE_INTERLEAVED 1   /* pair (2j, 2j + 1) inside a head   */

#define TDO_MATH_F32 0  /* tables rounded to fp32, fp32 products/fma in a fixed order (the kernel's precision) */
#define TDO_MATH_F64 1  /* everything in double, one final rounding                                             */

typedef struct {
  int32_t num_kv_heads;   /* H */
  int32_t head_dim;       /* D, even */
  int32_t page_tokens;    /* T */
  int32_t rope_style;     /* TDO_ROPE_* */
  double  rope_theta;
  int32_t math;           /* TDO_MATH_* */
} tdo_geom;

/* A round: n_sessions masters, n_agents mirrors.
 *   span_tokens[s]   S_s, shared tokens of session s
 *   master_pos0[s]   absolute position the master's token 0 was rotated for
 *   agent_session[i] session of agent i
 *   agent_pos0[i]    absolute position of agent i's first shared token (its history length)
 *   bt_flat / bt_offset[i..i+1]  agent i's block table (logical page -> physical page),
 *                    covering at least logical pages 0 .. (pos0+S-1)/T
 * Master rows of session s start at row sum_{s'<s} S_s' of master_k / master_v
 * ([rows][H][D] bf16).  Pools are [pool_pages][T][H][D] bf16. */
typedef struct {
  int32_t        n_sessions;
  const int32_t* span_tokens;
  const int64_t* master_pos0;
  int32_t        n_agents;
  const int32_t* agent_session;
  const int64_t* agent_pos0;
  const int32_t* bt_flat;
  const int64_t* bt_offset;
  const int64_t* agent_diff_pos0; /* optional (NULL = agent_pos0): position of the agent's first shared token
                                     when the diff given to tdo_diff_decode was encoded (an earlier round) */
  /* optional layout of the shared blocks per agent (Eq. 2, the scheduler-defined layout Pi_i): agent i's
   * segments are seg_*[seg_offset[i] .. seg_offset[i+1]); segment q places master tokens
   * [seg_src[q], seg_src[q] + seg_len[q]) at positions seg_dst[q] ..; sorted by seg_src, covering
   * [0, S) exactly once, destinations disjoint.  NULL seg_offset (or an empty range) = the identity
   * layout agent_pos0 + m.  seg_diff_dst (optional) = the same for the stored diff's frame. */
  const int64_t* seg_offset;
  const int32_t* seg_src;
  const int32_t* seg_len;
  const int64_t* seg_dst;
  const int64_t* seg_diff_dst;
} tdo_round;

/* cos/sin of phi_j = delta * theta^(-2j/D), j = 0 .. D/2-1 */
int tdo_rope_table_f64(double theta, int32_t head_dim, int64_t delta, double* cos_out, double* sin_out);
int tdo_rope_table_f32(double theta, int32_t head_dim, int64_t delta, float* cos_out, float* sin_out);

/* Rotate n_rows rows of [H][D] by delta.  fp32 in/out (no storage rounding), fp32 in / bf16 out
 * (rotation + storage rounding, TDO_MATH_F32 arithmetic) and bf16 in/out. */
int tdo_rotate_rows_f32 (const tdo_geom* g, int64_t delta, int64_t n_rows, const float* in, float* out);
int tdo_rotate_rows_f32_bf16(const tdo_geom* g, int64_t delta, int64_t n_rows, const float* in, uint16_t* out);
int tdo_rotate_rows_bf16(const tdo_geom* g, int64_t delta, int64_t n_rows, const uint16_t* in, uint16_t* out);

/* pool_k[slot_i(m)] = bf16(R(delta_i) master_k[m]); pool_v[slot_i(m)] = master_v[m]; nothing else is written. */
int tdo_rerotate_round(const tdo_geom* g, const tdo_round* r,
                       const uint16_t* master_k, const uint16_t* master_v,
                       uint16_t* pool_k, uint16_t* pool_v, int64_t pool_pages);

/* Block-sparse diff of every agent against its master.
 *   count[n_agents], offset[n_agents+1] (exclusive prefix of count), idx[capacity_pages] (ascending master
 *   page numbers, agent-major), payload[capacity_pages][2][T][H][D] (agent's K rows then V rows, rows past
 *   the span zero).  *overflow = 1 if sum(count) > capacity_pages; count/offset stay complete, and nothing
 *   at or beyond capacity_pages is written. */
int tdo_diff_encode(const tdo_geom* g, const tdo_round* r,
                    const uint16_t* master_k, const uint16_t* master_v,
                    const uint16_t* pool_k, const uint16_t* pool_v, int64_t pool_pages,
                    float eps,
                    int32_t* count, int64_t* offset, int32_t* idx, uint16_t* payload,
                    int64_t capacity_pages, int32_t* overflow);

/* Restore every agent's shared span: diff pages from the payload, all other pages from the rotated master.
 * Payload K rows were stored at position agent_diff_pos0 + m; they are re-rotated by
 * agent_pos0 - agent_diff_pos0 (Alg. 1 "RoPERecover(P_old, P_new)"; nothing to do when that is 0), V copied. */
int tdo_diff_decode(const tdo_geom* g, const tdo_round* r,
                    const uint16_t* master_k, const uint16_t* master_v,
                    uint16_t* pool_k, uint16_t* pool_v, int64_t pool_pages,
                    const int32_t* count, const int64_t* offset, const int32_t* idx, const uint16_t* payload);

/* Single-plane diffs (Sec. 5: separate block-index lists for K and V unless both touch the same blocks).
 * plane = 1 (K) or 2 (V): only that plane is compared, listed, stored (payload [capacity][T][H][D]) and restored. */
int tdo_diff_encode_plane(const tdo_geom* g, const tdo_round* r,
                          const uint16_t* master_k, const uint16_t* master_v,
                          const uint16_t* pool_k, const uint16_t* pool_v, int64_t pool_pages,
                          float eps, int32_t plane,
                          int32_t* count, int64_t* offset, int32_t* idx, uint16_t* payload,
                          int64_t capacity_pages, int32_t* overflow);
int tdo_diff_decode_plane(const tdo_geom* g, const tdo_round* r,
                          const uint16_t* master_k, const uint16_t* master_v,
                          uint16_t* pool_k, uint16_t* pool_v, int64_t pool_pages, int32_t plane,
                          const int32_t* count, const int64_t* offset, const int32_t* idx, const uint16_t* payload);

/* Attention of new query tokens over the shared span of every Mirror, computed from Master + diff with no
 * restored copy (Sec. 4.4: the diff applied as attention tiles are loaded; Fig. 9 skip-or-correct per block).
 * q: bf16 [n_agents][n_q][n_q_heads][D], already rotated for the queries' own positions.  Keys of pages not in
 * the diff are the master's, rotated exactly (double) to the agent's offset; pages in the diff come from the
 * payload (paired layout; K moved from the position it was stored at).  out [n_agents][n_q][n_q_heads][D] and
 * lse [n_agents][n_q][n_q_heads] in double: the normalised output over the span and the log of the softmax
 * denominator, so that the caller can merge it with attention over the private tokens. */
int tdo_attend_shared(const tdo_geom* g, const tdo_round* r,
                      const uint16_t* master_k, const uint16_t* master_v,
                      const int32_t* count, const int64_t* offset, const int32_t* idx, const uint16_t* payload,
                      const uint16_t* q, int32_t n_q, int32_t n_q_heads, double scale,
                      double* out, double* lse);

/* Check layer (Sec. 4.2): per-token key deviation of every agent (double, agent-major), the selection of
 * important positions from fp32 scores, and the master choice from fp32 totals. */
int tdo_key_deviation(const tdo_geom* g, const tdo_round* r,
                      const uint16_t* master_k, const uint16_t* pool_k, int64_t pool_pages, double* score);
int tdo_select_important(const float* score, int64_t S, float ratio, float min_score,
                         int32_t* out, int32_t* n_out);
int tdo_choose_master(const tdo_round* r, const float* total, int32_t* master);

/* Alg. 1 over n_layers layers: per-layer arrays of pointers (masters, pools and diffs of each layer). */
int tdo_restore_layers(const tdo_geom* g, const tdo_round* r, int32_t n_layers,
                       const uint16_t* const* master_k, const uint16_t* const* master_v,
                       uint16_t* const* pool_k, uint16_t* const* pool_v, int64_t pool_pages,
                       const int32_t* const* count, const int64_t* const* offset,
                       const int32_t* const* idx, const uint16_t* const* payload);

/* Sec. 6.4 arithmetic. */
double tdo_dense_bytes (const tdo_geom* g, int64_t span_tokens);               /* one layer of one cache    */
double tdo_diff_bytes  (const tdo_geom* g, int64_t diff_pages);                /* payload + index metadata  */
double tdo_mirror_ratio(const tdo_geom* g, int64_t span_tokens, int64_t diff_pages);
double tdo_family_cost (int64_t n_agents, double ratio);                       /* in full caches            */

int tdo_max_threads(void);
void tdo_set_threads(int n);   /* timing only: results do not depend on the thread count */

#ifdef __cplusplus
}
#endif
#endif
