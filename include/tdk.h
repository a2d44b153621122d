/*
 * tdk.h -- C ABI of libtdk: the data-parallel hot path of collective KV-cache reuse and
 * diff-aware storage for multi-agent "All-Gather" rounds, for AMD MI355X (gfx950).
 *
 * One round = n_sessions masters (the K/V of the shared output blocks, cached once, rotated for
 * positions master_pos0 ..) and n_agents mirrors (agent sub-requests).  Every agent's prompt is its
 * private history followed by the shared blocks (Sec. 2.1, Eq. 2), so agent i sees the shared span
 * at absolute positions dst_pos0_i .. dst_pos0_i + S - 1.  Per layer the library offers three
 * collective steps over the whole round:
 *
 *   tdk_rerotate_round   Sec. 4.2 "Layerwise Collective Reuse": one batched RoPE pass for the
 *                        group; cached K re-rotated by the position delta, V copied.
 *   tdk_diff_encode      Sec. 4.3 "Block-Sparse Diff Representation", Sec. 5 "Diff-Aware Storage":
 *                        each mirror becomes {touched page indices, K/V values of those pages}.
 *   tdk_diff_decode      Sec. 4.4 / Algorithm 1 "Fused Diff Restore": apply diff, recover RoPE
 *                        positions, write through the slot map; no dense mirror is materialised.
 *
 * Conventions
 *   - Pointers marked DEV are device pointers owned by the caller; HOST are host pointers.  The
 *     library borrows DEV buffers for the duration of the enqueued work and never frees them.
 *   - The three step calls validate on the host, enqueue kernels on the given HIP stream
 *     (hipStream_t passed as void*, NULL = default stream) and return without synchronising.
 *     They allocate nothing.  tdk_round_create / tdk_round_destroy allocate / free the library's
 *     own device memory (tables, descriptors, per-page flag scratch) and are synchronous.
 *   - Errors are return codes; tdk_last_error() gives thread-local detail.  Anything the host can
 *     detect fails before any work is enqueued.  No exception leaves the library.  A round belongs to
 *     the device that was current when it was created; step calls made with another device current
 *     fail with INVALID_ARG.
 *   - Results are deterministic: same inputs, same bits, including index order and payload placement.
 *   - Not checked (preconditions): physical pages of different agents do not overlap (a precondition of
 *     grouping requests, Sec. 4.2); buffers are not written concurrently; calls on one
 *     round are issued in stream order on one stream at a time (encode uses the round's own flag
 *     scratch, restore its events), different rounds are independent.
 *
 * Arithmetic: bf16 storage; cos/sin of phi_j = delta * theta^(-2j/D) evaluated in double on the
 * host and rounded once to fp32; per pair (a, b): y_a = fma(x_a, cos, -(x_b * sin)),
 * y_b = fma(x_b, cos, x_a * sin) in fp32; round-to-nearest-even to bf16.
 */
#ifndef TDK_H
#define TDK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TDK_OK = 0,
  TDK_ERR_INVALID_ARG = 1,   /* NULL, out-of-range or inconsistent argument           */
  TDK_ERR_UNSUPPORTED = 2,   /* a valid request this build has no kernel for          */
  TDK_ERR_CAPACITY = 3,      /* the round exceeds a fixed limit of the call (tdk_diff_encode_static); a diff
                                buffer that is too small is reported on the device (tdk_diff.overflow)  */
  TDK_ERR_HIP = 4,           /* a HIP runtime call failed (no GPU, launch error, ...)  */
  TDK_ERR_NOMEM = 5          /* host or device allocation failed                      */
} tdk_status;

#define TDK_BF16 0
#define TDK_ROPE_HALF 0          /* pair (j, j + D/2) inside a head */
#define TDK_ROPE_INTERLEAVED 1   /* pair (2j, 2j + 1) inside a head */

const char* tdk_status_str(tdk_status s);   /* static string                                   */
const char* tdk_last_error(void);           /* thread-local, valid until the next failing call */
const char* tdk_version(void);

/* Cache geometry.  Supported: dtype TDK_BF16; head_dim 128; 1 <= num_kv_heads <= 8;
 * page_tokens 16 or 32; both rope styles. */
typedef struct {
  int32_t num_layers;
  int32_t num_kv_heads;   /* H */
  int32_t head_dim;       /* D */
  int32_t page_tokens;    /* T: tokens per page = granularity of the diff (Sec. 4.3) */
  int32_t dtype;          /* TDK_BF16 */
  int32_t rope_style;     /* TDK_ROPE_* */
  double  rope_theta;
} tdk_model;

/* One shared span = one master. */
typedef struct {
  int32_t span_tokens;    /* S >= 0 */
  int64_t master_pos0;    /* absolute position the master's token 0 is rotated for */
} tdk_session;

/* One run of consecutive master tokens in an agent's prompt: master tokens src_tok .. src_tok+len-1
 * land at absolute positions dst_pos .. dst_pos+len-1.  diff_pos is the position the run started at
 * when the diff that will be restored was encoded (the per-segment form of tdk_agent::diff_pos0):
 * equal to dst_pos for a diff of this round; otherwise the K values of the run's payload rows are
 * re-rotated by dst_pos - diff_pos on restore.  Ignored by encode. */
typedef struct {
  int32_t src_tok;
  int32_t len;
  int64_t dst_pos;
  int64_t diff_pos;
} tdk_segment;

/* One agent sub-request (a mirror of its session's master). */
typedef struct {
  int32_t        session;          /* index into sessions[]                                        */
  int64_t        dst_pos0;         /* absolute position of its first shared token (history length) */
  const int32_t* block_table;      /* HOST: logical page -> physical page of the agent's sequence  */
  int32_t        block_table_len;  /* >= ceil((dst_pos0 + S) / T)                                  */
  int64_t        diff_pos0;        /* position of its first shared token when the diff that will be
                                      given to tdk_diff_decode / tdk_restore_layers was encoded: equal
                                      to dst_pos0 for a diff of this round; for a mirror stored in an
                                      earlier round its K values are re-rotated by dst_pos0 - diff_pos0
                                      on restore (Alg. 1, RoPERecover(P_old, P_new)).  Ignored by encode. */
  int32_t        n_segments;       /* 0: identity layout (the shared span sits at dst_pos0 .. dst_pos0+S-1).
                                      > 0: the scheduler-defined layout of the shared blocks for this agent
                                      (Sec. 2.1, Eq. 2): segments sorted by src_tok, covering [0, S) exactly
                                      once, destinations disjoint, every master page meeting at most two
                                      segments (true whenever blocks are at least a page long); dst_pos0 and
                                      diff_pos0 are then unused (each segment carries its own diff_pos). */
  const tdk_segment* segments;     /* HOST */
} tdk_agent;

typedef struct tdk_round tdk_round;   /* opaque: tables, descriptors, scratch on the current device */

/* Builds the plan of a round on the current HIP device: rotation tables per agent, the slices of
 * the block tables that cover the shared spans, the work list.  Copies everything it needs; the
 * arguments may be freed on return.  Errors: INVALID_ARG (NULL, negative sizes or positions, bad
 * session index, block table too short, negative page number, position beyond 2^31), UNSUPPORTED
 * (geometry), NOMEM, HIP. */
tdk_status tdk_round_create(const tdk_model* model,
                            const tdk_session* sessions, int32_t n_sessions,
                            const tdk_agent* agents, int32_t n_agents,
                            tdk_round** out);
void       tdk_round_destroy(tdk_round* r);             /* NULL-safe */
size_t     tdk_scratch_bytes(const tdk_round* r);       /* device bytes the round owns */

/* Launch shape and cache policy.  agents_per_group: agents of one session that share one read of a
 * master page (1..32), 0 = automatic.  flags: which accesses carry the non-temporal hint (streamed
 * through L2 and written back early instead of lingering as dirty lines that the next kernel has to
 * flush); the default was measured best for the whole rerotate / decode / encode sequence.
 * Synchronises the device (the work list it replaces may still be in use).  Results never depend on
 * these settings. */
#define TDK_TUNE_NT_REROTATE_STORES 1
#define TDK_TUNE_NT_DECODE_STORES   2
#define TDK_TUNE_NT_COMPARE_LOADS   4
#define TDK_TUNE_NT_SCATTER         8
#define TDK_TUNE_NT_GATHER          16
#define TDK_TUNE_PREFETCH_MASTER    32   /* rerotate: the first workgroups sweep the masters into the
                                            memory-side cache before anything is written           */
#define TDK_TUNE_PREFETCH_MASTER_DECODE 64 /* the same in decode: worth 5 % when its masters were not just
                                            read by another kernel, costs 0.6 % when they were    */
#define TDK_TUNE_XCD_QUEUES         128  /* the page kernels that write: two looping workgroups per compute unit take work
                                            items from one queue per XCD and, when theirs is empty, from the others' (the
                                            XCDs do not write at the same rate); off: one workgroup per item, fixed to an
                                            XCD by its number */
#define TDK_TUNE_TAPER              256  /* work list: smaller agent groups for the last pages, so that a launch does not
                                            end with a few long items on an otherwise idle chip                      */
#define TDK_TUNE_QUEUES_ANY_SIZE    512  /* queues also for rounds with fewer than four items per resident workgroup
                                            (by default such launches stay static: it is faster there)             */
#define TDK_TUNE_SCATTER_IN_DECODE  1024 /* small rounds (static launches): the workgroups that copy the listed pages ride
                                            behind the page items of decode's launch instead of a launch of their own */
#define TDK_TUNE_SHARED_TAIL        2048 /* static launches of the kernels that write: the last fifth of the work items goes
                                            to whichever of the launch's last workgroups start first (an XCD that writes
                                            faster takes more of it) instead of to fixed workgroups                     */
#define TDK_TUNE_ALL                4095
#define TDK_TUNE_DEFAULT            (191 + 1024 + 2048)
tdk_status tdk_round_tune(tdk_round* r, int32_t agents_per_group, int32_t flags);
int32_t    tdk_round_agents_per_group(const tdk_round* r);   /* the value in use (resolved if automatic); 0 for NULL */

/* Per-layer views, all DEV.
 *   master_k/v  [sum_s S_s][H][D] bf16, sessions concatenated in order (token-major rows)
 *   pool_k/v    [pool_pages][T][H][D] bf16, the paged KV memory of this layer */
typedef struct {
  const void* master_k;
  const void* master_v;
  void*       pool_k;
  void*       pool_v;
  int64_t     pool_pages;
} tdk_layer_io;

/* The mirrors of one layer (block-sparse diff of every agent), all DEV, caller-owned.
 *   count[n_agents]        pages in each agent's diff
 *   offset[n_agents + 1]   exclusive prefix of count
 *   idx[capacity_pages]    master-page numbers, ascending within an agent, agents in order
 *   payload[capacity_pages][2][T][H][D]  the agent's own K rows then V rows of each listed page
 *                          (values as they sit in the agent's cache; rows past the span are zero)
 *   overflow[1]            set to 1 by encode when sum(count) > capacity_pages, else 0; count and
 *                          offset are complete either way and nothing is written past capacity. */
typedef struct {
  int32_t* count;
  int64_t* offset;
  int32_t* idx;
  void*    payload;
  int64_t  capacity_pages;
  int32_t* overflow;
} tdk_diff;

/* pool_k[slot_i(m)] = bf16(R(dst_pos0_i - master_pos0) master_k[m]), pool_v[slot_i(m)] = master_v[m]
 * for every agent i and master token m, slot_i(m) = block_table_i[(dst_pos0_i+m)/T]*T + (dst_pos0_i+m)%T.
 * No other pool row is written.  Errors: INVALID_ARG (NULL, layer out of range, pool_pages smaller
 * than the largest mapped page + 1), HIP. */
tdk_status tdk_rerotate_round(tdk_round* r, int32_t layer, const tdk_layer_io* io, void* hip_stream);

/* Page p of agent i is in the diff iff some valid element of its K or V rows has
 * !(|a - ref| <= eps) in fp32, ref = what tdk_rerotate_round would write.  eps >= 0, not NaN.
 * Reads the pool, writes *out.  Errors as above plus INVALID_ARG for eps or NULL diff members. */
tdk_status tdk_diff_encode(tdk_round* r, int32_t layer, const tdk_layer_io* io, float eps,
                           const tdk_diff* out, void* hip_stream);

/* tdk_diff_encode for callers that cannot let the library own device allocations of its own choosing at
 * call time: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and bit-identical results, but the per-(agent, page) flag bytes live in a static
 * device array inside the library (TDK_STATIC_SCRATCH_BYTES per GPU, held until the process ends) instead of
 * the round's allocation.  Calls no hipMalloc / hipFree and takes no timing events.  A round with more than
 * TDK_STATIC_SCRATCH_BYTES (agent, page) pairs is refused with TDK_ERR_CAPACITY before anything is enqueued.
 * All calls on one GPU share the array (the compare kernel rewrites every flag of its round, so earlier
 * contents never matter): calls that overlap in time on one GPU race, whatever their rounds or streams. */
#define TDK_STATIC_SCRATCH_BYTES (4u << 20)
tdk_status tdk_diff_encode_static(tdk_round* r, int32_t layer, const tdk_layer_io* io, float eps,
                                  const tdk_diff* out, void* hip_stream);

/* Writes every agent's shared span: pages listed in the diff from the payload, all others from the
 * re-rotated master.  `in` must hold what tdk_diff_encode produced for this round (ascending
 * indices); entries at or past capacity_pages are ignored (those pages come from the master). */
tdk_status tdk_diff_decode(tdk_round* r, int32_t layer, const tdk_layer_io* io, const tdk_diff* in,
                           void* hip_stream);

/* Single-plane diffs (Sec. 5: K and V keep separate block-index lists unless both touch the same
 * blocks; the single-plane kernel of "Fused Sparse Restore").  plane = TDK_PLANE_K or TDK_PLANE_V.
 * Same as tdk_diff_encode / tdk_diff_decode restricted to one plane: only that plane is compared,
 * listed, stored and restored; payload is [capacity_pages][T][H][D] (one plane per slot). */
#define TDK_PLANE_K 1
#define TDK_PLANE_V 2
tdk_status tdk_diff_encode_plane(tdk_round* r, int32_t layer, const tdk_layer_io* io, float eps, int32_t plane,
                                 const tdk_diff* out, void* hip_stream);
tdk_status tdk_diff_decode_plane(tdk_round* r, int32_t layer, const tdk_layer_io* io, int32_t plane,
                                 const tdk_diff* in, void* hip_stream);

/* Reuse plan of the check layer (Sec. 4.2 "Layerwise Collective Reuse" and "Reuse Plan Output"), all DEV,
 * caller-owned.
 *   score[sum_i S_i]              per-token deviation of agent i at master token m, agents in order:
 *                                 sum over the K row of (fresh - rotated cached)^2 in fp32, where fresh
 *                                 is the agent's K row in the pool and rotated cached is what
 *                                 tdk_rerotate_round would write there
 *   important[n_agents][k_stride] the agent's important positions (master token numbers), ascending
 *   n_important[n_agents]         how many there are: min(ceil(ratio * S), #tokens with !(score <= min_score))
 *   total[n_agents]               the agent's accumulated deviation (sum of its scores)
 *   master[n_sessions]            agent with the lowest total in each session (first one on ties, NaN
 *                                 totals count as +inf, -1 for a session without agents) */
typedef struct {
  float*   score;
  int32_t* important;
  int32_t  k_stride;      /* >= ceil(ratio * S) of every session that has agents */
  int32_t* n_important;
  float*   total;
  int32_t* master;
} tdk_reuse_plan;

/* One batched key-difference pass over the whole group on the check layer, selection of the
 * important positions of every request (the ceil(ratio * S) largest scores among tokens with
 * !(score <= min_score); ties go to the lower token number) and the choice of each session's master.
 * Reads pool_k and master_k only.  0 < ratio <= 1, min_score finite and >= 0. */
tdk_status tdk_check_layer(tdk_round* r, int32_t layer, const tdk_layer_io* io, float ratio, float min_score,
                           const tdk_reuse_plan* out, void* hip_stream);

/* Attention of new query tokens over the shared span of every mirror, from master + diff, with no
 * restored copy (Sec. 4.4, last paragraphs: applying the diff as attention tiles are loaded; Fig. 9:
 * identical blocks go straight to attention, blocks with a diff are corrected first).  All DEV.
 *   q          bf16 [n_agents][n_q][n_q_heads][D], rotated for the queries' own positions (all of them
 *              after the shared span: no causal mask inside it); n_q_heads a multiple of H, query head
 *              hq reads KV head hq / (n_q_heads / H)
 *   out        fp32 [n_agents][n_q][n_q_heads][D]: softmax(scale * q . K_i) V_i over the S tokens of the
 *              span, where (K_i, V_i) is the agent's mirror: payload rows on the pages its diff lists,
 *              the master's K rotated to the agent's offset and the master's V everywhere else
 *   lse        fp32 [n_agents][n_q][n_q_heads]: log of the softmax denominator, so that the caller can
 *              merge `out` with attention over the agent's private tokens (-inf, out 0 for an empty span)
 *   workspace  tdk_attend_workspace_bytes(r, n_q, n_q_heads) bytes, 256-byte aligned, contents undefined
 * Arithmetic: each query row is rotated back by the agent's offset (fp32, rounded to bf16) so that all
 * agents of a session multiply the same un-rotated master tiles (bf16 MFMA, fp32 accumulation, softmax
 * weights rounded to bf16 for the second product); the listed pages go through the same products
 * from the payload.  The result agrees with the exact definition to about 1e-2 of the largest |V| at
 * scale = 1 / sqrt(128), in proportion for larger scales (not bit for bit).  Any finite scale is taken:
 * the kernels work with its magnitude and the query copies carry its sign; zero gives uniform weights. */
typedef struct {
  const void* q;
  int32_t     n_q;
  int32_t     n_q_heads;
  float       scale;
  float*      out;
  float*      lse;
  void*       workspace;
  size_t      workspace_bytes;
} tdk_attend_io;

size_t tdk_attend_workspace_bytes(const tdk_round* r, int32_t n_q, int32_t n_q_heads);   /* 0 on bad arguments */

/* io: master_k / master_v of the layer (the pool is not touched and may be NULL); in: the mirrors'
 * paired diff as tdk_diff_encode wrote it.  All layouts: identity or per-agent segments (one rotated copy
 * of a query row per segment), diffs stored at the current or at other positions (diff_pos0 / diff_pos).
 * Master values must be finite.
 * Shaped for decode-like calls (a few query tokens per agent): every block of 128 query rows of a
 * session and KV head reads the tiles again and owns its partial results in the workspace.
 * Allocates nothing, enqueues two to four kernels, does not synchronise.  Errors: INVALID_ARG (NULL,
 * misaligned, n_q < 1, n_q_heads not a multiple of H, scale not finite, workspace too small). */
tdk_status tdk_attend_shared(tdk_round* r, int32_t layer, const tdk_layer_io* io, const tdk_diff* in,
                             const tdk_attend_io* a, void* hip_stream);

/* Round-aware prompt interface (Sec. 4.1) and segment-based index (Sec. 5), HOST only.  Prompts are
 * split at a reserved separator token; a block is identified by its content (64-bit hash index,
 * every hit confirmed by comparison), so a shared update is recognised at whatever position it sits.
 * A content held by at least two prompts is shared; prompts that hold the same set of shared contents
 * (at least two prompts) form a session, numbered by first prompt; the session's master lists the
 * shared blocks in the order of its first prompt (span = their total length); each member gets the
 * segment list tdk_agent takes (src_tok in that master, dst_pos = position in the member's prompt,
 * diff_pos = dst_pos).  Other prompts get session -1 (the single-request path).  Empty blocks are
 * ignored; of a content repeated inside one prompt the first occurrence counts.  Token arrays are
 * borrowed during the call only. */
typedef struct {
  const int32_t* tokens;   /* HOST */
  int32_t        n_tokens;
} tdk_prompt;
typedef struct tdk_prompt_plan tdk_prompt_plan;   /* opaque, host memory */
tdk_status tdk_prompt_plan_create(const tdk_prompt* prompts, int32_t n_prompts, int32_t separator,
                                  tdk_prompt_plan** out);   /* INVALID_ARG, NOMEM, UNSUPPORTED (span >= 2^31) */
void       tdk_prompt_plan_destroy(tdk_prompt_plan* p);     /* NULL-safe */
int32_t    tdk_prompt_plan_n_sessions(const tdk_prompt_plan* p);
int32_t    tdk_prompt_plan_span(const tdk_prompt_plan* p, int32_t session);         /* -1 if out of range */
int32_t    tdk_prompt_plan_session_of(const tdk_prompt_plan* p, int32_t prompt);    /* -1: none */
/* number of segments of a prompt (0 if it has no session, -1 if out of range); *out points into the
 * plan and stays valid until the plan is destroyed */
int32_t    tdk_prompt_plan_segments(const tdk_prompt_plan* p, int32_t prompt, const tdk_segment** out);

/* Ping-pong staging buffers of the layerwise restore, DEV, caller-owned: two K and two V buffers of
 * stage_bytes each, stage_bytes >= (sum_s S_s) * H * D * 2 (one layer of masters). */
typedef struct {
  void*  stage_k[2];
  void*  stage_v[2];
  size_t stage_bytes;
} tdk_pingpong;

/* Algorithm 1 (Sec. 4.4) for layers first_layer .. first_layer + n_layers - 1 of every mirror of the
 * round: the masters of layer k are copied from HOST memory (host_master_k[k], host_master_v[k];
 * pinned memory, layout as tdk_layer_io.master_k) into one staging buffer on copy_stream while the
 * previous layer, staged in the other buffer, is restored on compute_stream exactly as
 * tdk_diff_decode does (io[k].pool_*, diffs[k]; io[k].master_* are ignored).  Returns after
 * enqueueing; the result is complete when compute_stream has drained.  Uses events owned by the
 * round, so calls on one round must not be issued concurrently from several threads.  Errors: as
 * tdk_diff_decode for every layer (all checked before anything is enqueued), INVALID_ARG for NULL or
 * undersized staging. */
tdk_status tdk_restore_layers(tdk_round* r, int32_t first_layer, int32_t n_layers,
                              const void* const* host_master_k, const void* const* host_master_v,
                              const tdk_layer_io* io, const tdk_diff* diffs, const tdk_pingpong* pp,
                              void* compute_stream, void* copy_stream);

/* Storage arithmetic of Sec. 6.4 (host only). */
double tdk_dense_bytes(const tdk_model* m, int64_t span_tokens);   /* one layer of one cache      */
double tdk_diff_bytes(const tdk_model* m, int64_t diff_pages);     /* values + idx + count/offset */
double tdk_family_cost(int64_t n_agents, double ratio);            /* 1 + (N-1)/R full caches     */

#ifdef __cplusplus
}
#endif
#endif
