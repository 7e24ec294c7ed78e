/*
 * segattn.h -- C ABI of libsegattn: segment-level causal attention for AMD MI355X (gfx950).
 *
 * The library implements the attention step of segmented execution (Sec. 3.1, Eq. 1: the
 * same forward operator F(x_i, C_{i-1}, R_{i-1}) at training and inference time) for one
 * attention layer:
 *
 *   - Eq. 12 (Appendix C): O = softmax(Q K^T * scale + M) V, where the mask M lets a
 *     segment query see every prefix row and the rows of its own segment up to itself;
 *   - Eq. 13 (Appendix C): the prefix a head sees -- the carried KV tail C_{i-1} (last T
 *     key/value rows of the previous segment; Sec. 3.4 "Local Continuity Channel"), the
 *     forward-only past KV (Sec. 3.4 "Long-Range Channel"), or nothing;
 *   - the cross-segment state itself: tail hand-off and append-only past pool
 *     (Sec. 3.4, Appendix D "Memory layout"; the paper applies no eviction, the evict call
 *     here is an extension).
 *
 * Conventions that hold for every entry point
 *   Pointers   Every q/k/v/out/lse/cache pointer is a DEVICE pointer unless the comment says
 *              "host".  All of them are borrowed for the duration of the enqueued work; the
 *              library never allocates or frees device memory.  The caller allocates one
 *              cache arena of segattn_cache_bytes() bytes (256-byte aligned) and keeps it
 *              alive until segattn_destroy().
 *   Streams    `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *              only enqueued; no entry point synchronises with the device.  All calls on one
 *              context must be issued on one stream or be ordered by the caller.
 *   Layouts    Dense, token-major:  q, out [B, rows, Hq, D];  k, v [B, rows, Hkv, D];
 *              lse [B, Hq, rows].  q/k/v are bf16.  out is bf16, or fp32 when the
 *              configuration sets out_fp32 or fp32_check.  lse is fp32, the natural logarithm of
 *              sum_j exp(scale * q.k_j) over the visible keys.  Query head h reads KV head
 *              h / (Hq / Hkv).
 *   Errors     Every call validates its arguments and the context state before it enqueues
 *              anything and returns a segattn_status; nothing aborts or throws.  After EINVAL,
 *              ECAPACITY or ESTATE nothing was enqueued and the context is unchanged.  EHIP means
 *              the HIP runtime refused a launch or a copy, possibly after earlier kernels of the
 *              same call had entered the stream: the device counters of the cache may then be
 *              ahead of the context's bookkeeping, so the context is marked not ready and every
 *              stateful call returns ESTATE until segattn_reset() or seg_kv_set_lengths().
 *   Threads    A context is not thread-safe; distinct contexts are independent.
 */
#ifndef SEGATTN_H
#define SEGATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct segattn_ctx segattn_ctx; /* opaque; host-side bookkeeping only */

typedef enum {
  SEGATTN_OK = 0,
  SEGATTN_EINVAL = 1,    /* bad argument or unsupported configuration               */
  SEGATTN_ECAPACITY = 2, /* a PAST head would hold more than past_capacity rows      */
  SEGATTN_ESTATE = 3,    /* call not valid in the current cache state                */
  SEGATTN_EHIP = 4,      /* the HIP runtime reported an error on launch / copy       */
  SEGATTN_ESCRATCH = 5   /* the problem does not fit the library's built-in scratch   */
} segattn_status;

/* Per-KV-head access policy (Eq. 13), a bit mask.  SEG: own segment only (a long-range head
 * outside a long-range layer).  TAIL: plus the carried tail (a local head).  PAST: plus every
 * row the head's past pool holds (a long-range head in a long-range layer; here the whole
 * history rather than a retrieved top-k subset).  TAIL|PAST sees the union of positions. */
enum { SEGATTN_SEG = 0, SEGATTN_TAIL = 1, SEGATTN_PAST = 2 };

typedef struct {
  int32_t batch;           /* B >= 1                                                      */
  int32_t n_q_heads;       /* Hq, a multiple of n_kv_heads                                */
  int32_t n_kv_heads;      /* Hkv, 1..128                                                 */
  int32_t head_dim;        /* D, 64 or 128                                                */
  int32_t seg_len;         /* S >= 1: segments start at multiples of S (Sec. 3.5)         */
  int32_t tail_len;        /* T, 0 <= T <= S: rows of the carried tail (the paper's M)    */
  int64_t past_capacity;   /* rows a PAST head's pool can hold (history + open segment);
                              must be >= S when any head is PAST; < 2^31                  */
  const uint8_t *kv_policy;/* host, [Hkv] policy bit masks; copied                        */
  float scale;             /* score scale; 0 means 1/sqrt(D) (Eq. 12)                     */
  int32_t fp32_check;      /* 1: fp32 FMA arithmetic and fp32 `out` (validation mode)     */
  int32_t out_fp32;        /* 1: `out` is fp32 (the unrounded accumulator) also in bf16
                              MFMA mode; implied by fp32_check                            */
  int32_t retrieved_capacity; /* 0: a PAST head attends to its whole pool.  R_max > 0:
                              retrieval mode (Sec. 3.4 "Long-Range Channel"): a PAST head
                              attends to [retrieved prefix ; own segment] (Eq. 13, second case),
                              the prefix being the rows seg_kv_past_select() gathered, at most
                              R_max of them; no head may then have both TAIL and PAST       */
  float rope_theta;        /* 0: positions are not the library's business.  > 0: base of the
                              rotary embedding (Appendix E): seg_rope_apply() rotates by it, and
                              in retrieval mode the gathered K rows are re-rotated (see
                              seg_kv_past_select)                                              */
  /* Launch-shape overrides for tests and A/B timing; 0 everywhere = the library chooses.  Results
   * do not depend on them beyond rounding order. */
  int32_t prefill_waves;   /* 4 or 8: waves per workgroup of the head_dim-128 bf16 forward kernel
                              (a forced shape also keeps seg_attn_fwd from cutting prefixes)     */
  int32_t item_queues;     /* forward and dQ kernels as a resident grid that takes its work items
                              from per-XCD queues: 1 never, 2 whenever a launch has more than one
                              item, 3 the same with a grid a third of the items (so that small
                              inputs loop and take over items of other queues too)               */
} segattn_config;

/* ---- context --------------------------------------------------------------------------- */

/* Bytes of device memory the cache arena needs for this configuration (0 if invalid).
 * Per TAIL/SEG head: (T + S) rows of K and of V; per PAST head: past_capacity rows (in
 * retrieval mode also retrieved_capacity + S rows: retrieved prefix and a copy of the open
 * segment); plus per-(sequence, head) counters, the split-K workspace of the decode path and,
 * where one segment alone cannot fill the chip with the query blocks of its PAST heads (few
 * sequences, few PAST heads) and the pool can hold 2048 rows or more, at most 34 MB of workspace
 * in which seg_attn_fwd merges the pieces it cuts such a head's prefix into. */
size_t segattn_cache_bytes(const segattn_config *cfg);

/* Create a context over a caller-allocated arena (device, >= segattn_cache_bytes(), aligned
 * to 256 bytes).  The cache starts empty (C_0 = R_0 = empty) once segattn_reset() has been
 * enqueued; create itself touches no device memory.  EINVAL on a bad configuration. */
segattn_status segattn_create(const segattn_config *cfg, void *cache_dev, size_t cache_bytes,
                              segattn_ctx **out_ctx);
void segattn_destroy(segattn_ctx *ctx); /* frees host bookkeeping only, never the arena */

/* Empty the cache of every sequence: no tail, no past, no open segment. */
segattn_status segattn_reset(segattn_ctx *ctx, void *stream);

/* ---- prefill ---------------------------------------------------------------------------- */

/* Attention for the next m rows of the open segment of every sequence (Eq. 12 / Eq. 13).
 * q [B,m,Hq,D], k,v [B,m,Hkv,D]; out [B,m,Hq,D]; lse [B,Hq,m].  Row t of the call sits at
 * in-segment offset fill+t, where fill is the number of rows already committed to the open
 * segment; it sees the head's prefix held in the cache, those fill rows, and rows 0..t of k/v.
 * Requires 1 <= m and fill + m <= S for every sequence (ESTATE otherwise).  Reads the cache,
 * does not change it: follow with seg_kv_commit() on the same stream.
 * (All prefill entry points, head_dim 128: the library runs workgroups of eight or of four waves
 * depending on how much work the launch has; segattn_config.prefill_waves forces one of them.) */
segattn_status seg_attn_fwd(segattn_ctx *ctx, const void *q, const void *k, const void *v,
                            int32_t m, void *out, float *lse, void *stream);

/* Stateless whole-sequence form: one launch over all ceil(n/S) segments of q [B,n,Hq,D],
 * k,v [B,n,Hkv,D] by absolute position; only the last segment may be short.  Needs no
 * context and no cache: each segment's prefix is read from k/v directly (the tail is rows
 * [s-T, s) and the past rows [0, s) of a segment starting at s).  out [B,n,Hq,D] (bf16, or
 * fp32 if cfg->out_fp32 or cfg->fp32_check), lse [B,Hq,n].  cfg->past_capacity is ignored. */
segattn_status seg_attn_fwd_seq(const segattn_config *cfg, const void *q, const void *k,
                                const void *v, int64_t n, void *out, float *lse, void *stream);

/* Packed ragged batch (sequences of different lengths, no padding): q [total,Hq,D], k,v
 * [total,Hkv,D], out [total,Hq,D], lse [Hq,total]; sequence b = rows cu_seqlens[b] ..
 * cu_seqlens[b+1]-1 with its own segment grid (segments start at multiples of S inside the
 * sequence).  cu_seqlens: DEVICE int32 [cfg->batch + 1], ascending, cu_seqlens[0] = 0; total and
 * max_seqlen (the longest sequence, which sizes the launch) are host values.  An empty sequence
 * is allowed.  Otherwise as seg_attn_fwd_seq. */
segattn_status seg_attn_fwd_varlen(const segattn_config *cfg, const void *q, const void *k,
                                   const void *v, const int32_t *cu_seqlens, int64_t total,
                                   int64_t max_seqlen, void *out, float *lse, void *stream);

/* Policy array of one layer from the paper's head/layer sets (Sec. 3.4): KV heads in
 * long_heads are long-range heads, the others local (TAIL); a long-range head is PAST in a layer
 * of L_long and within-segment only (SEG) elsewhere.  Host only: long_heads [n_long] KV-head
 * indices, policy_out [n_kv_heads].  EINVAL on a bad index. */
segattn_status segattn_layer_policy(int32_t n_kv_heads, const int32_t *long_heads, int32_t n_long,
                                    int32_t layer_in_l_long, uint8_t *policy_out);

/* ---- positions --------------------------------------------------------------------------- */

/* RoPE re-indexing for prefix concatenation (Sec. 3.4, Appendix E).  Rotates q [B,rows,Hq,D] and
 * k [B,rows,Hkv,D] in place: row t of sequence b by the position pos0[b] + t, channel pair
 * (i, i + D/2) by position * theta^(-2i/D), theta = cfg->rope_theta (> 0).  pos0: device int64 [B]
 * or NULL (all zero).  Rotating every token by its absolute position before seg_attn_fwd* /
 * seg_kv_commit / seg_attn_decode reproduces the paper's re-indexed positions (prefix 0..P-1,
 * segment P..P+m-1) exactly for the carried tail and for a whole-history prefix, because RoPE
 * scores depend on position differences only; a retrieved prefix is turned to the positions
 * just before its segment by seg_kv_past_select.  Values are never rotated. */
segattn_status seg_rope_apply(const segattn_config *cfg, void *q, void *k, int64_t rows,
                              const int64_t *pos0, void *stream);

/* ---- backward (training) ---------------------------------------------------------------- */

/* Gradients of seg_attn_fwd_seq for truncated backpropagation over segments (Sec. 3.2,
 * Definition "K-truncated consistent objective"): given dout = dL/dout [B,n,Hq,D] (bf16) and
 * the forward's out and lse, writes dq [B,n,Hq,D] and dk, dv [B,n,Hkv,D] (bf16, or fp32 if
 * cfg->out_fp32 or cfg->fp32_check; `out` has that same type).  Every visible key contributes to
 * dq.  dk and dv collect the pairs inside a query's own segment and, for a head with the TAIL
 * bit, its carried tail -- the differentiable interface state; rows a query reaches only through
 * the PAST bit are forward-only and receive nothing (no-gradient lemma, Appendix B).  A window
 * of K+1 segments passed as one sequence is therefore exactly the graph truncation depth K
 * backpropagates through.  The g query heads of a group add up in dk, dv.  workspace: device,
 * at least seg_attn_bwd_workspace_bytes(cfg, n) bytes, 256-byte aligned, overwritten. */
size_t seg_attn_bwd_workspace_bytes(const segattn_config *cfg, int64_t n);
segattn_status seg_attn_bwd_seq(const segattn_config *cfg, const void *q, const void *k,
                                const void *v, const void *out, const float *lse,
                                const void *dout, int64_t n, void *dq, void *dk, void *dv,
                                void *workspace, size_t workspace_bytes, void *stream);

/* seg_attn_bwd_seq for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving or training loops, harnesses that forbid hipMalloc.
 * Same arguments without the workspace, same kernels, same results bit for bit; the two [B,Hq,n]
 * fp32 row statistics that the backward kernels hand to each other live in an array inside the
 * library's device image instead (SEGATTN_BWD_STATIC_SCRATCH_BYTES per GPU, held from the moment
 * the library is loaded until the process ends).  The call allocates and frees nothing.
 * SEGATTN_ESCRATCH, before anything is enqueued, if the two statistics -- 2 * B * Hq * n * 4
 * bytes -- exceed the array (8 MiB: e.g. four 8192-token training windows of 32 query heads).  All calls on one GPU share that
 * GPU's array: calls whose kernels may overlap (different streams, several host threads) race on
 * it and must be ordered by the caller; the array keeps the last call's contents and nothing in
 * it needs clearing, since every call overwrites what it reads. */
#define SEGATTN_BWD_STATIC_SCRATCH_BYTES (8u << 20)
segattn_status seg_attn_bwd_seq_static(const segattn_config *cfg, const void *q, const void *k,
                                       const void *v, const void *out, const float *lse,
                                       const void *dout, int64_t n, void *dq, void *dk, void *dv,
                                       void *stream);

/* The same backward pass for a packed ragged batch (layout and cu_seqlens as for
 * seg_attn_fwd_varlen: q, out, dout, dq [total,Hq,D]; k, v, dk, dv [total,Hkv,D]; lse [Hq,total]);
 * every sequence is differentiated on its own, as one window of consecutive segments.
 * workspace: device, >= seg_attn_bwd_varlen_workspace_bytes(cfg, total), 256-byte aligned. */
size_t seg_attn_bwd_varlen_workspace_bytes(const segattn_config *cfg, int64_t total);
segattn_status seg_attn_bwd_varlen(const segattn_config *cfg, const void *q, const void *k,
                                   const void *v, const void *out, const float *lse,
                                   const void *dout, const int32_t *cu_seqlens, int64_t total,
                                   int64_t max_seqlen, void *dq, void *dk, void *dv,
                                   void *workspace, size_t workspace_bytes, void *stream);

/* ---- cache operations -------------------------------------------------------------------- */

/* Append m rows k,v [B,m,Hkv,D] to the open segment of every sequence.  When that makes the
 * segment complete (S rows) it is closed: the tail of every non-PAST head becomes the
 * segment's last T rows and the rest is dropped (this is what bounds memory, Sec. 3.5
 * "Memory Complexity"); a PAST head keeps all rows (append-only pool).  ESTATE if
 * fill + m > S for some sequence, ECAPACITY if a PAST pool would overflow. */
segattn_status seg_kv_commit(segattn_ctx *ctx, const void *k, const void *v, int32_t m,
                             void *stream);

/* The same for a whole prompt handed over at once: k,v [B,n,Hkv,D], every sequence's open segment
 * empty (ESTATE otherwise).  Leaves exactly the state that n/S calls of seg_kv_commit with S rows
 * and one with the remaining n%S rows would leave (pools of the PAST heads grown by the whole
 * segments, the tail of the last whole segment, the open rows), in two launches.  It is the
 * companion of seg_attn_fwd_seq: prefill in one launch, commit in one call, then decode.
 * ECAPACITY if a pool cannot take n more rows. */
segattn_status seg_kv_commit_seq(segattn_ctx *ctx, const void *k, const void *v, int64_t n,
                                 void *stream);

/* Append `rows` explicit rows k,v [B,rows,D] (e.g. rows gathered by a retrieval step,
 * Appendix D "Output") to the past pool of one PAST head, for every sequence.  Only valid
 * between segments (no open segment: ESTATE otherwise); EINVAL if the head is not PAST. */
segattn_status seg_kv_past_append(segattn_ctx *ctx, int32_t kv_head, const void *k,
                                  const void *v, int64_t rows, void *stream);

/* Retrieval mode only.  Retrieved prefix for the next segment (Appendix D "Output"): for every
 * sequence and every PAST head gather the R pool rows idx names into the head's retrieved
 * prefix.  idx: device int32 [B, n_past, R], n_past = the PAST heads in ascending KV-head
 * order; entries are pool row numbers (absolute positions, or the order of
 * seg_kv_past_append), distinct, each below the head's pool size and not evicted.  The
 * prefix rows take the order of the list (softmax does not depend on it).  The prefix serves
 * the segment that starts next (prefill calls and decode steps alike) and is dropped when
 * that segment closes; without a call the prefix is empty.  R = 0 empties it.  Valid between
 * segments only (ESTATE with an open segment); EINVAL if the context is not in retrieval
 * mode or R > retrieved_capacity; ECAPACITY if R exceeds the visible pool rows of some
 * sequence and head.  The lists are not read on the host: an out-of-range entry is clamped
 * into the pool (never an out-of-bounds access), a repeated entry counts twice.
 * With rope_theta > 0 the pool is taken to hold keys rotated by their absolute position (pool
 * row number = position, as seg_rope_apply + seg_kv_commit leave them) and list entry r is
 * re-rotated to position s - R + r, s the position at which the next segment starts: the
 * positions 0..R-1 / R..R+m-1 of Appendix E up to a common shift. */
segattn_status seg_kv_past_select(segattn_ctx *ctx, const int32_t *idx, int32_t R, void *stream);

/* Sizes of the top-k retrieval operator (Appendix D).  The paper names the steps and gives
 * L_q in [24, 64] and R = 512 (Appendix F); every other size is the caller's choice. */
typedef struct {
  int32_t n_queries;   /* L_q >= 1: the last L_q query rows of the previous segment are used     */
  int32_t pool_window; /* >= 1: sliding-window mean pooling, window = stride = this many rows     */
  int32_t tail_avg;    /* >= 1: one more summary, the mean of the last tail_avg rows              */
  int32_t n_anchors;   /* 1..32: rows with the highest scores                                      */
  int32_t win_before;  /* >= 0: an anchor a contributes rows a - win_before .. a + win_after       */
  int32_t win_after;   /* >= 0                                                                     */
} segattn_retrieval;

/* Bytes of device workspace seg_kv_retrieve needs for this context (0 if the sizes are invalid:
 * the summaries of one KV group, ceil(L_q / pool_window) + 1 per query head, must not exceed 64). */
size_t seg_kv_retrieve_workspace_bytes(const segattn_ctx *ctx, const segattn_retrieval *r);

/* Top-k retrieval operator (Appendix D): choose, for every sequence and every PAST head, the R
 * pool rows that form the retrieved prefix, and write them to idx_out (device int32
 * [B, n_past, R], ascending) in the form seg_kv_past_select takes.  q_prev: device bf16
 * [B, m, Hq, D], the queries of the previous segment (m >= 1).  Steps, as read here: query
 * summaries = means of consecutive pool_window-row windows of the last L_q rows plus the mean of
 * the last tail_avg rows, for every query head of the group, rounded to bf16; score of a pool
 * row = its best dot product with a summary over the visible pool (one bandwidth-bound pass over
 * the head's K rows); anchors = the n_anchors best rows (ties: lower row), which is what
 * per-summary top-k, de-duplication and anchor choice yield for any k >= n_anchors; anchors in
 * descending score order add their windows (clipped, rows already in skipped) until R rows are
 * in; the earliest visible rows pad to R.  ECAPACITY if some pool holds fewer than R visible
 * rows; EINVAL on bad sizes, a context without PAST heads, or a pool capacity above 2^20 rows.
 * workspace: device, >= seg_kv_retrieve_workspace_bytes(), 256-byte aligned, overwritten. */
segattn_status seg_kv_retrieve(segattn_ctx *ctx, const segattn_retrieval *r, const void *q_prev,
                               int32_t m, int32_t R, int32_t *idx_out, void *workspace,
                               size_t workspace_bytes, void *stream);

/* ---- retrieval mode for a whole prompt, stateless ------------------------------------------------
 * During prefill every segment's queries and every earlier key are present at once, so the
 * per-segment chain retrieve -> select -> attend -> commit (the calls above; they remain the form
 * for decoding) collapses into two calls with no context and no cache:
 *
 * seg_kv_retrieve_seq: the top-k retrieval operator (Appendix D, same reading and sizes as
 * seg_kv_retrieve) for every segment i >= 1 of q [B,n,Hq,D], k [B,n,Hkv,D] at once: the queries
 * are the last L_q rows of segment i-1, the pool of a PAST head is its keys [0, i S).  idx_out:
 * device int32 [B, n_seg, n_past, R], n_seg = ceil(n / S), PAST heads in ascending KV-head order;
 * the lists of segment 0 (no history) are not meaningful.  Requires 1 <= R <= S, at least one PAST
 * head and none with TAIL as well (Eq. 13), n <= 2^20; workspace: device, 256-byte aligned,
 * >= seg_kv_retrieve_seq_workspace_bytes() (0 if the sizes are invalid).
 *
 * seg_attn_fwd_seq_retrieved: seg_attn_fwd_seq in which a PAST head attends to [the R rows idx
 * names for its segment ; own segment] (Eq. 13, second case) instead of its whole history; the
 * first segment has no prefix.  idx as above (from seg_kv_retrieve_seq or the caller's own):
 * positions before the segment's start, distinct; an out-of-range entry is clamped into the
 * history, never read out of bounds.  The rows are first gathered into the workspace (device,
 * 256-byte aligned, >= seg_attn_fwd_seq_retrieved_workspace_bytes(): 2 R D bf16 per (sequence,
 * segment, PAST head)), with cfg->rope_theta > 0 re-rotated from their absolute positions to the
 * R positions just before the segment as seg_kv_past_select does; then one attention launch. */
size_t seg_kv_retrieve_seq_workspace_bytes(const segattn_config *cfg, const segattn_retrieval *r,
                                           int64_t n);
segattn_status seg_kv_retrieve_seq(const segattn_config *cfg, const segattn_retrieval *r,
                                   const void *q, const void *k, int64_t n, int32_t R,
                                   int32_t *idx_out, void *workspace, size_t workspace_bytes,
                                   void *stream);
size_t seg_attn_fwd_seq_retrieved_workspace_bytes(const segattn_config *cfg, int64_t n, int32_t R);
segattn_status seg_attn_fwd_seq_retrieved(const segattn_config *cfg, const void *q, const void *k,
                                          const void *v, int64_t n, const int32_t *idx, int32_t R,
                                          void *workspace, size_t workspace_bytes, void *out,
                                          float *lse, void *stream);

/* Hide the n_oldest oldest rows of one PAST head's pool from now on (all sequences).  Pure
 * bookkeeping: nothing is copied and the rows' storage is not reused.  If the head also has
 * the TAIL bit, rows inside the current tail window stay visible.  Evicting more rows than
 * the pool holds hides all of them. */
segattn_status seg_kv_past_evict(segattn_ctx *ctx, int32_t kv_head, int64_t n_oldest,
                                 void *stream);

/* Budget form of the same eviction (an extension: the paper's pool grows without eviction,
 * Sec. 3.4): per sequence, hide the oldest rows of the head's pool until at most max_rows
 * remain visible (a sequence holding fewer is left alone).  Called after each commit it keeps
 * a sliding budget of the most recent max_rows rows.  Rows of the current tail window of a
 * TAIL|PAST head stay visible even if max_rows is smaller. */
segattn_status seg_kv_past_keep_recent(segattn_ctx *ctx, int32_t kv_head, int64_t max_rows,
                                       void *stream);

/* Host copies of the cache counters (any pointer may be NULL): past [B,Hkv] = visible pool
 * rows of PAST heads (closed segments only; 0 for other heads), tail [B] = rows in the
 * carried tail, seg_fill [B] = rows in the open segment. */
segattn_status seg_kv_lengths(const segattn_ctx *ctx, int64_t *past, int32_t *tail,
                              int32_t *seg_fill);

/* Declare the cache contents after the caller has written K/V rows into the arena itself
 * (restore from a snapshot, benchmark set-up): host arrays closed_rows [B] = rows in closed
 * segments (a multiple of S), tail [B] (<= min(T, closed_rows)), seg_fill [B] (< S; 0 in
 * retrieval mode).  Row placement is given by segattn_cache_span().  The retrieved prefix
 * starts empty. */
segattn_status seg_kv_set_lengths(segattn_ctx *ctx, const int64_t *closed_rows,
                                  const int32_t *tail, const int32_t *seg_fill, void *stream);

/* Where the rows of (sequence b, KV head h) live inside the arena: K row r is the D bf16
 * values at byte offset *k_off + r*D*2, V likewise from *v_off; *cap_rows rows exist.
 * PAST head: row index = absolute position of the token (history, then the open segment).
 * Other heads: rows [T - tail, T) hold the tail, rows [T, T + seg_fill) the open segment. */
segattn_status segattn_cache_span(const segattn_ctx *ctx, int32_t b, int32_t kv_head,
                                  size_t *k_off, size_t *v_off, int64_t *cap_rows);

/* Bytes of K/V rows currently held (visible or not yet dropped) over all sequences and
 * heads: the quantity Sec. 3.5 bounds by S + T per local head plus the pool of PAST heads
 * (in retrieval mode plus the retrieved prefix and the segment mirror of those heads). */
size_t segattn_resident_bytes(const segattn_ctx *ctx);

/* ---- decode ----------------------------------------------------------------------------- */

/* One decoding step for every sequence (Eq. 2's conditioning on x_<t, C_{i-1}, R_{i-1}):
 * q [B,Hq,D], k_new,v_new [B,Hkv,D] belong to the newest token.  Appends the row to the open
 * segment, attends over [prefix | open segment] with a split-K kernel and a combine pass,
 * writes out [B,Hq,D] and lse [B,Hq], and closes the segment when it reaches S rows (same
 * rule as seg_kv_commit).  ECAPACITY if a PAST pool would overflow. */
segattn_status seg_attn_decode(segattn_ctx *ctx, const void *q, const void *k_new,
                               const void *v_new, void *out, float *lse, void *stream);

/* ---- misc ------------------------------------------------------------------------------- */
/* Diagnostic for benchmarks: stream `bytes` of device memory at buf (16-byte aligned) with one of
 * the two access patterns of the library's HBM-bound kernels and nothing else.  mode 0: every
 * 16-byte piece read once, non-temporal (the decode and retrieval scans); sink: device, >= 4
 * bytes, practically never written.  mode 1: every piece read and written back in place with two
 * sign bits flipped (the in-place rotation of seg_rope_apply); two calls restore the buffer.
 * Timing it gives the rate the part sustains for the pattern. */
segattn_status segattn_bandwidth_probe(void *buf, size_t bytes, int32_t mode, void *sink, void *stream);

/* Diagnostic for benchmarks: the shader clock the part holds while other work runs.  Launches
 * SEGATTN_CLOCK_PROBE_WAVES single-wave workgroups (one per XCD) on `stream`; each sleeps until
 * `microseconds` (1 .. 10,000,000, else EINVAL) of the device's constant-rate wall clock have
 * passed, then stores two uint64 into counts (device, 2 x SEGATTN_CLOCK_PROBE_WAVES uint64,
 * 8-byte aligned): the shader clocks and the wall-clock ticks it saw.  *wall_clock_khz (host,
 * required) receives the wall clock's rate: clock [MHz] = clocks / ticks * wall_clock_khz / 1000.
 * Launch it on a stream of its own just before the work to be observed; it occupies one wave
 * slot with a handful of registers on eight compute units and ends by itself. */
#define SEGATTN_CLOCK_PROBE_WAVES 8
segattn_status segattn_clock_probe(uint32_t microseconds, uint64_t *counts, int32_t *wall_clock_khz, void *stream);

/* Diagnostic for benchmarks: the dense bf16 rate of the matrix pipes with nothing else busy.
 * Launches two 256-thread workgroups per compute unit on `stream`; every wave runs `iterations`
 * (1 .. 10,000,000, else EINVAL) rounds of eight independent 32x32x16 bf16 products from
 * registers, no memory access in the loop.  operands = 0: pseudo-random values in [-1, 1), a
 * different one in every lane and register (the switching activity of real data); 1: one constant
 * everywhere (almost no switching: the part draws less power and holds a higher clock).  *flops
 * (host, required) receives the floating-point operations of the launch; sink: device, >= 4
 * bytes, practically never written.  Timing the launch gives the rate; with segattn_clock_probe
 * beside it, the clock the part holds for it. */
segattn_status segattn_mfma_probe(int32_t iterations, int32_t operands, void *sink, int64_t *flops, void *stream);

const char *segattn_strerror(segattn_status st);
/* Name and average device time bookkeeping are not kept by the library; the version string
 * names the kernels' target ISA, e.g. "segattn 0.1 gfx950". */
const char *segattn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SEGATTN_H */
