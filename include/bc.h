/*
 * bc.h - C ABI of the MI355X (gfx950) decode / compress / masked-prefill path of
 * Breadcrumbs Reasoning (arXiv 2510.13797), with the gradients of the masked attention and
 * the distillation loss of its training recipe.
 *
 * Problem statement (paper, Alg. 1 and Sec. 3.1): while a model generates, every c
 * generated tokens a beacon token is encoded; the beacon's K/V entry is kept and the
 * entries of the c tokens before it are dropped.  Per sequence the cache therefore
 * holds  [ prompt | one beacon per finished window | current window (<= c) ]  (Fig. 1).
 * Attention itself is the standard softmax attention (Sec. 2) over whatever is
 * resident.  Training does not evict; it masks (Fig. 2, Sec. 3.2).
 *
 * General conventions
 *  - Every pointer is a DEVICE pointer owned by the caller unless the argument is
 *    documented as "host".  The library allocates no device memory and keeps no state
 *    between calls: everything that steers a call travels in its arguments.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every
 *    call except bc_tables_to_host() only enqueues work on that stream and returns.
 *  - Return value: host-detectable errors only (bad argument, unsupported shape,
 *    workspace too small, launch failure).  Violations only the device can see
 *    (window already full, slab full, empty cache) set bits in *cache->err (sticky,
 *    never cleared by the library) and leave the offending sequence untouched.
 *  - `active` is an optional [B] byte mask (NULL = all active).  Inactive sequences
 *    are never read or written; their output rows are left as they were.
 *  - Step numbering: decode step t (t = 1, 2, ...) appends the K/V of the t-th generated
 *    token, then attends; compression is due after step t when t mod c == 0
 *    (iteration i = t of Alg. 1, whose x_i has been sampled but not yet encoded, so the
 *    window holds exactly c entries).
 *
 * Cache layout in HBM
 *  Sequence s owns cap[s] rows per KV head.  With E = Hkv * d elements per entry, its
 *  part of a slab starts at element base[s] * E and is head-major:
 *      element(s, kvh, j, x) = base[s]*E + (kvh*cap[s] + j)*d + x,   0 <= j < cap[s]
 *  so the rows one (sequence, KV head) pair streams through are contiguous.  Rows
 *  [0, P) are the prompt, [P, P+nb) the beacons, [P+nb, P+nb+w) the window; rows at and
 *  beyond L = P + nb + w are unspecified (stale data may remain after an eviction).
 *  Slabs and base[s]*E*elem_size must be 16-byte aligned.
 */
#ifndef BC_H
#define BC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  BC_OK = 0,
  BC_ERR_ARG = -1,        /* null / misaligned pointer, bad flag                 */
  BC_ERR_SHAPE = -2,      /* unsupported B, Hq, Hkv, d or dtype                   */
  BC_ERR_CAPACITY = -3,   /* (status string for the device error bit)            */
  BC_ERR_STATE = -4,      /* (status string for the device error bit)            */
  BC_ERR_WORKSPACE = -5,  /* workspace missing or smaller than required          */
  BC_ERR_HIP = -6         /* a HIP call or kernel launch failed                  */
} bc_status;

typedef enum { BC_F32 = 0, BC_BF16 = 1 } bc_dtype;

/* bits of *cache->err */
#define BC_ERRBIT_STATE 1     /* operation not allowed in the sequence's state   */
#define BC_ERRBIT_CAPACITY 2  /* the sequence's slab is full                     */

/* kinds of row bc_append_kv() appends */
#define BC_ROW_TOKEN 0
#define BC_ROW_BEACON 1

typedef struct {
  int32_t B;         /* sequences                                                 */
  int32_t Hq;        /* query heads                                               */
  int32_t Hkv;       /* KV heads; Hq % Hkv == 0, group g = Hq/Hkv <= 8            */
  int32_t d;         /* head dim: 64 or 128                                       */
  int32_t kv_dtype;  /* bc_dtype of q, k, v and the slabs; outputs are fp32       */
  float scale;       /* softmax scale; the paper is silent, callers pass 1/sqrt(d).
                      * Attention calls need a finite scale >= 0 (prefill: > 0), else BC_ERR_ARG */
} bc_shape;

typedef struct {
  void *k_slab, *v_slab; /* sum_s cap[s]*Hkv*d elements each                      */
  const int64_t *base;   /* [B] first entry of sequence s (in entries of Hkv*d)   */
  const int32_t *cap;    /* [B] rows per KV head (see the note on strides below)  */
  int32_t *P;            /* [B] prompt length         (rewritten by bc_cache_admit) */
  int32_t *c;            /* [B] compression ratio; <= 0: never compress (bc_set_ratio) */
  int32_t *nb;           /* [B] beacons so far           (updated by the library) */
  int32_t *w;            /* [B] rows after the beacons   (updated by the library) */
  int32_t *err;          /* [1] sticky error bits                                 */
  int32_t max_cap;       /* HOST value: max_s cap[s]; sizes grids and workspace   */
  const int32_t *order;  /* [B] optional dispatch order, see bc_sort_by_length(); or NULL */
  int32_t uniform_P;     /* HOST values, optional promise about the layout, 0 = none: see below */
  int32_t uniform_cap;
  int32_t rows_per_workgroup; /* HOST value, 0 = automatic: see "Plan of the decode calls" below */
  int32_t plan;               /* HOST value, 0 = automatic: BC_PLAN_* bits                      */
} bc_cache;

/* Plan of the decode calls (bc_decode_attn and the step calls).  Left at zero, the library picks
 * kernel, workgroup shape and chunking from the shape and max_cap.  Tests and measurements can
 * narrow that choice per call; no choice changes a result beyond the order of fp32 additions.
 *  rows_per_workgroup > 0: rows of one (sequence, KV head) stream handled by one workgroup (rounded
 *      up to the kernel's pass size and so that a sequence has at most 64 chunks); partial results
 *      are folded by a second launch.  On a batch with 128 or more (sequence, KV head) pairs the
 *      workspace of bc_decode_workspace_bytes() covers at most four chunks per sequence, beyond
 *      that the calls return BC_ERR_WORKSPACE.  < 0 is BC_ERR_ARG.
 *  plan: OR of the bits below; an unknown bit is BC_ERR_ARG. */
#define BC_PLAN_PLAIN_ALU 1               /* bf16 shapes on the register/FMA kernel as well        */
#define BC_PLAN_NEED_MATRIX_KERNEL 2      /* BC_ERR_SHAPE unless the LDS/MFMA kernel serves the shape */
#define BC_PLAN_IGNORE_ORDER 4            /* dispatch in index order although cache->order is set  */
#define BC_PLAN_CACHEABLE_LOADS 8         /* default cache policy for K/V loads of large launches  */
#define BC_PLAN_ONE_WORKGROUP_PER_PAIR 16 /* never two workgroups (V column halves) per pair       */
#define BC_PLAN_IGNORE_PROMISE 32         /* do not use uniform_P / uniform_cap                    */
#define BC_PLAN_NO_SMALL_WORKGROUPS 64    /* never the four-wave workgroups of large, short batches */
#define BC_PLAN_GENERAL_LOOP 128          /* short caches on the general tile loop as well         */
#define BC_PLAN_ALL_BITS 255

/* Promise of a uniform layout (not in the paper: a latency aid for batches of equal prompt length,
 * the shape of its evaluation rollouts).  With uniform_P > 0 the caller states that the slabs hold
 * B * Hkv * uniform_cap rows, that uniform_cap == max_cap, and that (normally) every sequence has
 * P[s] == uniform_P, cap[s] == uniform_cap and base[s] == s * uniform_cap.  The bf16 decode calls
 * then request the prompt rows - which never change and are always resident - from those addresses
 * while the tables are still on their way, about half a microsecond earlier.  Every sequence's
 * tables are compared with the promise afterwards; where they differ (say after bc_cache_admit
 * gave a slot another prompt length) the rows are simply requested again from the right place, so
 * results never depend on the promise - only the addresses it implies must lie inside the slabs.
 * uniform_P > 0 with uniform_cap != max_cap or uniform_P > uniform_cap is BC_ERR_ARG. */

/* Note on strides: all sequences are streamed at once, each KV head from base + kvh * cap rows.
 * When cap * d * (bytes per element) is close to a multiple of 512 KiB the concurrent streams
 * fall on the same memory channels (measured: cap = 2065 rows of 256 bytes, 516 KiB apart, runs
 * 15-20 % slower than cap = 2100 or 2200); pad cap by a few dozen rows in that case. */
const char *bc_status_str(int32_t status);
int32_t bc_version(void);

/* Fill a freshly allocated cache from prompt K/V (Alg. 1, "Initialize: encode the
 * prompt").  k_prompt / v_prompt: [total_rows, Hkv, d], token-major, sequences
 * concatenated; prompt_offsets: device [B+1] int64, row of each sequence's first
 * token.  total_rows is the host copy of prompt_offsets[B].  Sets nb = w = 0.  A
 * sequence whose P[s] differs from its offset span, or exceeds cap[s], sets the
 * state / capacity bit and is left unfilled. */
int32_t bc_cache_init(const bc_shape *shape, const bc_cache *cache, const void *k_prompt,
                      const void *v_prompt, const int64_t *prompt_offsets,
                      int64_t total_rows, void *stream);

/* Admission of new sequences into the slots of finished ones (the evaluation rule of Sec. 4 ends
 * generations at different times; a slot's slab can then serve the next request).  For every s
 * with admit[s] != 0, slot s starts over as Alg. 1 initialises a cache: the rows
 * [prompt_offsets[s], prompt_offsets[s+1]) of k_prompt / v_prompt become its prompt,
 * P[s] = that span, nb = w = 0, c[s] = new_c[s] when new_c is given, live[s] = 1 when live is
 * given.  base[s] and cap[s] stay: a prompt longer than cap[s] sets the capacity bit and leaves
 * the slot (and live[s]) as it was.  Slots with admit[s] == 0 are not touched and their spans are
 * ignored (normally empty).  prompt_offsets: device [B+1] int64; total_rows: host copy of
 * prompt_offsets[B]; new_c: device [B] int32 or NULL; admit: device [B] bytes; live: device [B]
 * bytes or NULL (the mask of bc_decode_step_budget).  There is no block table: compaction keeps
 * every sequence contiguous and bounded by P + G/c + c + 1 rows, so a slot is one fixed slab. */
int32_t bc_cache_admit(const bc_shape *shape, const bc_cache *cache, const void *k_prompt,
                       const void *v_prompt, const int64_t *prompt_offsets, int64_t total_rows,
                       const int32_t *new_c, const uint8_t *admit, uint8_t *live, void *stream);

/* Append one row per active sequence (Alg. 1: "KV is updated internally" for a token;
 * "encode b" for a beacon).  k, v: [B, Hkv, d].
 *  kind = BC_ROW_TOKEN : row goes to slot L; w += 1.  Needs w < c when c > 0 (else the
 *                        state bit) and L < cap (else the capacity bit).
 *  kind = BC_ROW_BEACON: acts only on sequences with c > 0 and w == c (others are
 *                        skipped silently, so one call serves a batch with
 *                        per-sequence c); the beacon joins at the tail, w = c + 1,
 *                        to be attended by its own query and then compacted by
 *                        bc_compress_evict(beacon_k = NULL). */
int32_t bc_append_kv(const bc_shape *shape, const bc_cache *cache, const void *k,
                     const void *v, const uint8_t *active, int32_t kind, void *stream);

/* Bytes of workspace bc_decode_attn() and the step calls need for this shape and max_cap
 * (enough for the automatic plan; for a forced chunk size see bc_cache::rows_per_workgroup). */
size_t bc_decode_workspace_bytes(const bc_shape *shape, int32_t max_cap);

/* Zero a freshly allocated workspace (it holds per-sequence counters that the library
 * expects to find at zero and leaves at zero).  Call once after allocating it; a workspace
 * allocated zero-filled needs no call.  Enqueues a fill kernel, no memset node. */
int32_t bc_workspace_init(void *workspace, size_t workspace_bytes, void *stream);

/* Which kernel, grid and chunking the decode calls use for this shape and cache (HOST fields of
 * `cache` only: max_cap, order, the layout promise, rows_per_workgroup, plan; nothing on the
 * device is read).  Writes a NUL-terminated line to text[text_bytes] (HOST memory), cut short if
 * it does not fit; the kernel's name is spelled as profilers print it.  For logs and for
 * benchmarks that report which kernel they timed.  Same status codes as bc_decode_attn for a bad
 * shape, cache or plan; text == NULL or text_bytes == 0 is BC_ERR_ARG. */
int32_t bc_decode_plan_describe(const bc_shape *shape, const bc_cache *cache, char *text,
                                size_t text_bytes);

/* Single-token grouped-query attention over the resident entries (Sec. 2, Sec. 3.1:
 * generation proceeds as in a vanilla Transformer over what is in the cache):
 *   out[s,h,:] = sum_j softmax_j(scale * q[s,h,:] . K_j[kvh,:]) V_j[kvh,:],
 *   j over all L_s = P+nb+w rows, kvh = floor(h / (Hq/Hkv)).
 * q: [B, Hq, d] in kv_dtype; out: [B, Hq, d] fp32 (fp32 accumulation throughout).
 * A sequence with L_s == 0 sets the state bit and its output is left untouched.
 * The result is deterministic: partial results are combined in a fixed order (no atomics).
 * Calls sharing one workspace must not overlap in time. */
int32_t bc_decode_attn(const bc_shape *shape, const bc_cache *cache, const void *q,
                       float *out, const uint8_t *active, void *workspace,
                       size_t workspace_bytes, void *stream);

/* Beacon append + window eviction + in-place compaction (Alg. 1, the two eviction
 * lines: drop the c entries before the beacon, keep the beacon).
 *  beacon_k/v = [B, Hkv, d]: the beacon row is written to slot P+nb (the first window
 *      slot); acts on active sequences with c > 0 and w == c, or 1 <= w <= c when
 *      require_full_window == 0 (an extension; the paper never compresses a partial
 *      window).  A sequence with w == c+1 (a beacon already at the tail) sets the state bit.
 *  beacon_k = beacon_v = NULL: the beacon is already the tail entry (appended with
 *      BC_ROW_BEACON); acts on sequences with w == c+1: row P+nb+c moves to P+nb.
 *      require_full_window must be 1.
 *  Afterwards nb += 1, w = 0.  Sequences that are not due are skipped silently. */
int32_t bc_compress_evict(const bc_shape *shape, const bc_cache *cache, const void *beacon_k,
                          const void *beacon_v, const uint8_t *active,
                          int32_t require_full_window, void *stream);

/* One decode step: append the token rows, attend, then evict where due (supplied-beacon
 * form); a single launch for every supported shape (a second one merges partial results when
 * a small batch's sequences are split into chunks).  Same semantics as bc_append_kv(TOKEN) +
 * bc_decode_attn + bc_compress_evict(beacon_k, beacon_v, require_full_window = 1) in that order.
 * beacon_k/v may be NULL: then no eviction is attempted. */
int32_t bc_decode_step(const bc_shape *shape, const bc_cache *cache, const void *k,
                       const void *v, const void *q, float *out, const void *beacon_k,
                       const void *beacon_v, const uint8_t *active, void *workspace,
                       size_t workspace_bytes, void *stream);

/* bc_decode_step for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * and semantics as bc_decode_step without the workspace: the counters and partial results live in
 * a fixed array of BC_NOALLOC_SCRATCH_BYTES in device memory that belongs to the library (one copy
 * per GPU it runs on, held until the process ends).  The call allocates and frees nothing.  Its
 * plan must fit the array: B * 128 bytes of counters, plus - only for batches of fewer than 128
 * (sequence, KV head) pairs whose sequences are split into chunks, or a forced chunk size - the
 * partial results of bc_decode_workspace_bytes(); a call that needs more returns BC_ERR_WORKSPACE
 * and launches nothing.  Every call on one GPU uses the same array (the counters are cleared at
 * the start of each call): calls that overlap in time on one GPU, on whatever streams, race -
 * serialise them, or give the overlapping ones a workspace of their own through bc_decode_step. */
#define BC_NOALLOC_SCRATCH_BYTES (4u << 20)
int32_t bc_decode_step_noalloc(const bc_shape *shape, const bc_cache *cache, const void *k,
                               const void *v, const void *q, float *out, const void *beacon_k,
                               const void *beacon_v, const uint8_t *active, void *stream);

/* The beacon's own step in one launch (Alg. 1: encode the beacon, then drop the window; Sec. 3.1):
 * the same as bc_append_kv(kind = BC_ROW_BEACON) + bc_decode_attn + bc_compress_evict(NULL, NULL)
 * on the sequences whose window is full.  k, v: the beacon token's K/V rows [B, Hkv, d]; q: its
 * query [B, Hq, d]; out [B, Hq, d]: its attention over prompt, earlier beacons, the full window
 * and itself.  Afterwards the beacon sits behind the earlier beacons, nb is one larger and w = 0.
 * Takes part: active sequences with c > 0 and w == c.  Other sequences are left alone and their
 * rows of `out` are unspecified (pass an `active` mask of the due sequences to have every written
 * row defined).  A due sequence without room for one more entry (L == cap) gets the capacity bit
 * and is left alone. */
int32_t bc_beacon_step(const bc_shape *shape, const bc_cache *cache, const void *k, const void *v,
                       const void *q, float *out, const uint8_t *active, void *workspace,
                       size_t workspace_bytes, void *stream);

/* bc_decode_step under the evaluation rule of the paper (Sec. 4, Evaluation: the cache size is
 * capped - 1,000 entries there - and generation is interrupted when the cap is reached).
 * budget: device [B] int32, cap on the generation entries nb + w (prompt rows not counted);
 * live: device [B] bytes, read as the `active` mask and updated: a sequence whose attention in
 * this step saw nb + w >= budget[s] entries is finished, live[s] becomes 0 and later calls skip
 * it - no host round trip.  The step in which the cap is reached is still carried out in full. */
int32_t bc_decode_step_budget(const bc_shape *shape, const bc_cache *cache, const void *k,
                              const void *v, const void *q, float *out, const void *beacon_k,
                              const void *beacon_v, const int32_t *budget, uint8_t *live,
                              void *workspace, size_t workspace_bytes, void *stream);

/* Change the compression ratio of active sequences in the middle of a generation (the paper
 * fixes c per generation and names dynamic ratios as future work, Sec. 6).  new_c: device [B]
 * int32.  Allowed when the current window fits the new ratio (w < new_c, or new_c <= 0, or a
 * window boundary w == 0); otherwise the state bit is set and c[s] is left unchanged.  From the
 * next append on, windows close at the new ratio; beacons already written are unaffected.
 * Capacity is the caller's business: cap[s] must cover the longest window still to come. */
int32_t bc_set_ratio(const bc_shape *shape, const bc_cache *cache, const int32_t *new_c,
                     const uint8_t *active, void *stream);

/* Training-time forward (Fig. 2, Sec. 3.2): attention over beacon-interleaved
 * trajectories where eviction is simulated by the mask.  Rows of trajectory b are
 * [row_offsets[b], row_offsets[b+1]); the first P[b] rows are the prompt (plain causal
 * mask, no beacons), then c[b] response tokens, one beacon row, c[b] tokens, one beacon
 * row, ...  A response row sees the prompt, every earlier beacon, the earlier rows of its
 * own window and itself.  c[b] <= 0: plain causal attention.
 * q: [total_rows, Hq, d]; k, v: [total_rows, Hkv, d] (kv_dtype must be BC_BF16);
 * out: [total_rows, Hq, d] fp32; lse (nullable): [total_rows, Hq] fp32, natural log of
 * the softmax denominator.  row_offsets: device [B+1] int64; P, c: device [B] int32;
 * max_rows: HOST value >= the longest trajectory (sizes the grid), < 2^26.  scale must be > 0 and finite (else BC_ERR_ARG).
 * Supported: kv_dtype BC_BF16 with d = 128 or 64; fp32 inputs are BC_ERR_SHAPE. */
int32_t bc_prefill_attn(const bc_shape *shape, const void *q, const void *k, const void *v,
                        const int64_t *row_offsets, const int32_t *P, const int32_t *c,
                        int32_t max_rows, float *out, float *lse, void *stream);

/* bc_prefill_attn with a workspace (Fig. 2, Sec. 3.2; same operation, same tensors, same
 * tolerance).  The workspace (device memory, bc_prefill_workspace_bytes() bytes, 16-byte aligned,
 * no initialisation, contents unspecified afterwards) receives a copy of V in half precision.
 * When every finite entry of V is below 65520 in magnitude - which a conversion pass checks on the
 * device - the softmax weights enter the value product as one half-precision part (11 bits)
 * against that copy instead of two bf16 parts against V: about a sixth less time.  The copy is exact
 * for entries of magnitude 2^-14 and above (smaller ones keep an absolute error below 2^-25).
 * Otherwise the call computes exactly what bc_prefill_attn computes.  The half-precision form stays
 * inside the forward tolerance (2e-3) but lies further from the exact result than the two-part
 * form (about 4e-4 against 6e-6 on N(0,1) inputs); gradients computed from its `out` inherit that
 * error scaled by the size of dO and K, so where bc_prefill_attn_bwd must meet the same absolute
 * bound whatever the data, take `out` and `lse` from bc_prefill_attn.  total_rows: HOST copy of
 * row_offsets[B].  Workspace missing or too small: BC_ERR_WORKSPACE. */
size_t bc_prefill_workspace_bytes(const bc_shape *shape, int64_t total_rows);
int32_t bc_prefill_attn_ws(const bc_shape *shape, const void *q, const void *k, const void *v,
                           const int64_t *row_offsets, const int32_t *P, const int32_t *c,
                           int32_t max_rows, int64_t total_rows, float *out, float *lse,
                           void *workspace, size_t workspace_bytes, void *stream);

/* Gradients of bc_prefill_attn (Sec. 3.2: the student is trained through the masked forward;
 * gradients flow to its parameters only).  Same tensors and tables as the forward, plus
 * out / lse as the forward wrote them and dout: [total_rows, Hq, d] in bf16.  Results, fp32:
 * dq [total_rows, Hq, d], dk and dv [total_rows, Hkv, d] (summed over the query heads of a
 * group); every element is written, nothing needs zeroing.  total_rows: HOST copy of
 * row_offsets[B].  workspace: bc_prefill_bwd_workspace_bytes() bytes, no initialisation.
 * No atomics: results are reproducible.  scale must be > 0 and finite (else BC_ERR_ARG). */
size_t bc_prefill_bwd_workspace_bytes(const bc_shape *shape, int64_t total_rows);
int32_t bc_prefill_attn_bwd(const bc_shape *shape, const void *q, const void *k, const void *v,
                            const float *out, const float *lse, const void *dout,
                            const int64_t *row_offsets, const int32_t *P, const int32_t *c,
                            int32_t max_rows, int64_t total_rows, float *dq, float *dk, float *dv,
                            void *workspace, size_t workspace_bytes, void *stream);

/* Token-level distillation loss of the training recipe (Eq. 1, Sec. 3.2) with the teacher given
 * by its stored top-k logits per token (App. A; k = 100 there).  The teacher distribution is the
 * softmax over its k stored logits; the student's log-probabilities are its full-vocabulary
 * log-softmax at the same token ids:  loss[t] = sum_i p_T(i) * (log p_T(i) - log p_S(idx[t,i])).
 * student_logits: device [T, V] row-major, logits_dtype BC_BF16 or BC_F32, finite values;
 * teacher_logits: device [T, k] fp32; teacher_idx: device [T, k] int32, distinct ids in [0, V)
 * per row (an id outside the range makes loss[t] NaN; nothing is read out of bounds).
 * loss_per_token: device [T] fp32.  lse (nullable): device [T] fp32, natural-log partition
 * function of the student row, the input of the backward call.  loss_mean (nullable): device
 * [1] fp32, the mean of loss_per_token (trajectories of equal weight per token), summed in a
 * fixed order.  1 <= k <= min(V, 1024).  Rows are read with 16-byte loads when V * element size
 * is a multiple of 16 and the pointer is aligned, element by element otherwise. */
int32_t bc_topk_kl_loss(int64_t T, int32_t V, int32_t k, const void *student_logits,
                        int32_t logits_dtype, const float *teacher_logits,
                        const int32_t *teacher_idx, float *loss_per_token, float *lse,
                        float *loss_mean, void *stream);

/* Gradient of grad_scale * sum_t loss[t] with respect to the student's logits (the teacher is
 * fixed, Sec. 3.2): dlogits[t, v] = grad_scale * (softmax(student)[t, v] - p_T at v, if v is one
 * of the teacher's ids).  lse: as written by bc_topk_kl_loss.  dlogits: device [T, V] of the
 * logits' dtype, every element written; must not alias student_logits.  For the mean loss pass
 * grad_scale = 1 / T. */
int32_t bc_topk_kl_loss_bwd(int64_t T, int32_t V, int32_t k, const void *student_logits,
                            int32_t logits_dtype, const float *teacher_logits,
                            const int32_t *teacher_idx, const float *lse, float grad_scale,
                            void *dlogits, void *stream);

/* Copy nb[B], w[B] and err[1] to HOST arrays (any may be NULL) and wait for the stream. */
int32_t bc_tables_to_host(const bc_shape *shape, const bc_cache *cache, int32_t *nb_host,
                          int32_t *w_host, int32_t *err_host, void *stream);

/* Dispatch order for large ragged batches (not in the paper: a scheduling aid for its ragged
 * caches).  Writes to order[B] (device) the sequence indices by decreasing resident length
 * P + nb + w, inactive sequences last.  While cache->order points to such an array, decode calls
 * (bc_decode_attn and all step calls) on batches with more than 256 (sequence, KV head) pairs -
 * more workgroups than the chip runs at once - let workgroup i serve sequence order[i], so the
 * longest sequences start first and the tail of the launch is short.  The array is only read by
 * those calls and may be stale: any permutation of 0..B-1 gives the same results as no array
 * (refreshing it once per window is enough; a uniform batch needs none).  An entry outside
 * 0..B-1 sets the state bit and its workgroups do nothing.  B <= 4096, else BC_ERR_SHAPE. */
int32_t bc_sort_by_length(const bc_shape *shape, const bc_cache *cache, const uint8_t *active,
                          int32_t *order, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BC_H */
