/*
 * hack.h -- C ABI of the MI355X (gfx950) library for head-aware KV-cache
 * compression in next-scale visual autoregressive generation
 * (arXiv 2504.09261).
 *
 * One "unit" is one (batch, head) pair, u = b*H + h.  At every scale step each
 * unit (i) scores its cache against a few of the current scale's queries,
 * (ii) selects a budget-limited subset under its head class's policy,
 * (iii) compacts the kept K/V rows, and (iv) lets the current scale's queries
 * attend over the compacted cache.  Units are independent.
 *
 * Conventions
 *  - Every call returns a hack_status (0 = OK, negative = error).  No C++
 *    exception crosses the ABI; hack_last_error() gives the message.
 *  - Pointers marked DEVICE point to GPU memory owned by the caller; pointers
 *    marked HOST are ordinary host arrays, read (or written) during the call
 *    and not retained.
 *  - Calls are asynchronous on the given HIP stream (a hipStream_t passed as
 *    void*).  They never synchronise the device and never read device memory
 *    from the host: every length is host-computable (len_out = min(budget, T_in)).
 *  - Element type and head_dim are fixed per context.  Tensors are row-major;
 *    a cache row is head_dim elements.  q/k_new/v_new/out are [B, H, N_k, head_dim].
 *  - Arguments are validated on the host before anything is launched; on error
 *    nothing has been launched.
 *  - A context serves one stream at a time (its workspace is shared by calls).
 *    It owns a second stream and two events, used only by hack_step when the
 *    two-group overlap is switched on (environment HACK_STEP_OVERLAP=1 when the
 *    context is created; off by default): the side work is forked from and
 *    joined back into the caller's stream inside the call, so callers, and
 *    stream captures, see one stream either way.
 *  - Small per-call launch tables (offsets, lengths, work lists) are uploaded
 *    the first time a particular table is seen and reused afterwards, so a
 *    repeated schedule issues kernel launches only and can be captured in a
 *    HIP graph after one eager warm-up pass.
 */
#ifndef HACK_MI355X_H
#define HACK_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hack_ctx hack_ctx;
typedef struct hack_kvcache hack_kvcache;
typedef void* hack_stream; /* hipStream_t */

typedef enum {
  HACK_OK = 0,
  HACK_EINVAL = -1,       /* bad argument (shape, range, alignment, NULL) */
  HACK_ECAPACITY = -2,    /* exceeds what the context / cache was sized for */
  HACK_EUNSUPPORTED = -3, /* valid request this build does not implement */
  HACK_EHIP = -4          /* a HIP runtime call failed */
} hack_status;

typedef enum { HACK_BF16 = 0, HACK_F32 = 1 } hack_dtype;

enum { HACK_CONTEXTUAL = 0, HACK_STRUCTURAL = 1 };

typedef struct {
  int32_t device;        /* HIP device ordinal */
  int32_t heads;         /* H */
  int32_t head_dim;      /* 64 or 128 */
  int32_t dtype;         /* hack_dtype of q/k/v/out and of the cache */
  int32_t max_units;     /* largest B*H of any call */
  int32_t max_cache_len; /* largest T_in (cache rows + current scale) of any unit */
  int32_t max_queries;   /* largest N_k */
  int32_t n_obs;         /* observation queries N_obs, 1..32 (paper: 32) */
} hack_config;

/* Ragged per-unit cache: rows of unit u are [off[u], off[u] + len[u]) of k and v. */
typedef struct {
  void* k;            /* DEVICE [rows, head_dim] */
  void* v;            /* DEVICE [rows, head_dim] */
  int32_t* pos;       /* DEVICE [rows] global token id of every row, or NULL */
  int64_t rows;       /* rows allocated in k, v (and pos) */
  const int64_t* off; /* HOST [B*H] first row of each unit; multiples of 8 */
  const int32_t* len; /* HOST [B*H] valid rows of each unit */
} hack_cache;

/* ---- life cycle ------------------------------------------------------- */

/* Creates a context on cfg->device and allocates its workspace (importance,
 * kept indices, softmax partials, launch tables; for bf16 contexts also the
 * merge workspace and the partial-result slots of cut attention work items:
 * 2 x resident work-groups x 128 x head_dim floats, 64 MiB at head_dim 128 on
 * MI355X).  Returns HACK_EINVAL for an
 * unsupported head_dim/dtype/n_obs or non-positive sizes, HACK_EHIP if the
 * device cannot be used. */
hack_status hack_create(hack_ctx** out, const hack_config* cfg);
void hack_destroy(hack_ctx* ctx);
const char* hack_strerror(hack_status s);
/* Message of the last failing call on ctx (valid until the next call). */
const char* hack_last_error(const hack_ctx* ctx);
/* Reports what kernels of earlier calls on ctx found while they ran (the calls
 * themselves are asynchronous and had already returned HACK_OK).  Meaningful
 * once the caller has synchronised the streams it used; every other entry
 * point performs the same check first and fails the same way.
 *   HACK_EUNSUPPORTED  a bf16 hack_score / hack_step met a logit
 *                      |scale * q.k| > 354: its importance was formed with that
 *                      logit clamped and may differ from the definition.
 *                      Reported once, the context stays usable.
 *   HACK_EHIP          a fused score launch gave up its bounded wait for the
 *                      other work-groups of a unit (the device did not keep
 *                      the launch resident as a whole, e.g. other work held
 *                      compute units).  Importance, kept indices, caches and
 *                      outputs produced by the calls since the last successful
 *                      check are incomplete: reset the managed cache and issue
 *                      those calls again.  Fused score launches queued after
 *                      the failing one have not run at all (they find a flag
 *                      in device memory and leave before reading anything).
 *                      The call that reports this drains the device, re-arms
 *                      the workspace and switches the context to
 *                      HACK_SCORE_TWO_PASS; the context stays usable.  HIP
 *                      graphs captured before keep their fused launches. */
hack_status hack_check(hack_ctx* ctx);

/* How a bf16 context forms the importance of hack_score / hack_step.
 *   HACK_SCORE_FUSED     one launch that reads K once; the work-groups of a unit
 *                        exchange their row sums inside the launch, which needs
 *                        the whole launch resident on the device at once (the
 *                        library sizes launches for an otherwise idle device).
 *                        Default.
 *   HACK_SCORE_TWO_PASS  two launches (row sums, then importance) that read K
 *                        twice and never wait inside a kernel: safe when other
 *                        streams or processes share the device.  Same results
 *                        bit for bit.
 * Switching drains the device (it re-arms the exchange workspace); do it
 * outside stream captures.  fp32 contexts always score in two passes. */
enum { HACK_SCORE_FUSED = 0, HACK_SCORE_TWO_PASS = 1 };
hack_status hack_set_score_mode(hack_ctx* ctx, int32_t mode);
int32_t hack_get_score_mode(const hack_ctx* ctx);

/* ---- a1: importance estimation by subset attention --------------------
 * Sec. 4.4, "Importance Estimation via Efficient Subset Attention":
 *   A~ = Softmax(scale * Q~ K^T) over the uncompressed keys of this step,
 *   importance[j] = sum_i A~[i, j].
 * The keys of unit u are its cache rows followed, if k_new != NULL, by the
 * N_k rows k_new[b, h] (the concatenation of the cache-update equation,
 * without materialising it): T_in[u] = in->len[u] + (k_new ? N_k : 0).
 *   q        DEVICE [B, H, N_k, d]
 *   q_idx    HOST [n_obs] rows of q that observe, or NULL for the evenly
 *            strided rows floor(i*N_k/n_obs); n_obs <= min(ctx n_obs, N_k)
 *   active   HOST [B*H] nonzero = score this unit, or NULL = all units
 *   importance DEVICE float [B*H, imp_stride]; row u receives T_in[u] values
 *            (rows of inactive units are left untouched)
 * Accuracy (bf16): importance is within 1e-6 relative of the exact value while
 * |scale * q.k| stays below ~40, and within 2.5e-8 * max|scale * q.k| beyond.
 * Logits are supported up to |scale * q.k| <= 354 (far beyond what a float32
 * importance can resolve); larger ones are clamped and reported by hack_check /
 * the next call.  Results are reproducible bit for bit from call to call: every
 * sum is formed in a fixed order (no floating-point atomics).
 * Errors: HACK_EINVAL (NULL/misaligned pointers, n_obs out of range, a q_idx
 * outside [0, N_k), offsets outside the cache), HACK_ECAPACITY (B*H, N_k or a
 * T_in above the context's limits, imp_stride < max T_in). */
hack_status hack_score(hack_ctx* ctx, int32_t B, int32_t N_k, const void* q,
                       const int32_t* q_idx, int32_t n_obs, float scale,
                       const hack_cache* in, const void* k_new,
                       const uint8_t* active, float* importance,
                       int64_t imp_stride, hack_stream stream);

/* hack_score for callers that cannot allocate: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * importance bit for bit (the two-pass form: no in-kernel waits), but every
 * scratch buffer of the kernels (work items, q-row table, row-sum exchange
 * slots) lives in a fixed device array of the library (about 1.6 MB per GPU, held
 * until the process ends) and the work items are planned by a kernel from by-value
 * arguments, so the call performs no allocation of any kind and no host-to-device
 * copy.  Limits: bf16 contexts (HACK_EUNSUPPORTED otherwise); at most 64
 * scored units per call (HACK_ECAPACITY beyond; use `active` to score a
 * larger batch in slices).  The array keeps no state between calls (every word
 * a call reads it has written itself), but all calls on one GPU share it:
 * calls that overlap in time on the same GPU, on whatever stream or context,
 * race on it; issue them on one stream or order them with events.
 * Other errors as hack_score. */
hack_status hack_score_static(hack_ctx* ctx, int32_t B, int32_t N_k, const void* q,
                              const int32_t* q_idx, int32_t n_obs, float scale,
                              const hack_cache* in, const void* k_new,
                              const uint8_t* active, float* importance,
                              int64_t imp_stride, hack_stream stream);

/* ---- a2: budgeted selection per head class -----------------------------
 * Sec. 4.4, f_C and f_S.  For unit u with T = t_in[u], b = min(budget[u], T):
 *   contextual: the b keys of largest importance;
 *   structural: the first n0 = min(n_init, T - n_recent) rows, the last
 *     n_recent rows, and the M = b - n0 - n_recent most important rows in
 *     between; if M < 0, the first min(n0, b) rows and the most important
 *     rows of the last n_recent.
 * Equal importance is resolved towards the lower index; indices are written
 * in ascending order.  Importance is compared as float32 bit patterns of
 * non-negative, non-NaN numbers.
 *   importance DEVICE float [B*H, imp_stride]
 *   head_type  HOST [H], HACK_CONTEXTUAL / HACK_STRUCTURAL
 *   kept_idx   DEVICE int32 [B*H, idx_stride]; row u receives b indices
 *   len_out    HOST [B*H] receives b (may be NULL)
 * budget[u] >= T writes the identity selection 0..T-1.
 * Errors: HACK_EINVAL (budget < 1, n_recent > T, bad head_type),
 * HACK_ECAPACITY (T above the context's max_cache_len, strides too small). */
hack_status hack_select(hack_ctx* ctx, int32_t B, const float* importance,
                        int64_t imp_stride, const int32_t* t_in,
                        const uint8_t* head_type, const int32_t* budget,
                        int32_t n_init, int32_t n_recent, int32_t* kept_idx,
                        int64_t idx_stride, int32_t* len_out,
                        hack_stream stream);

/* ---- a3: compaction ------------------------------------------------------
 * Sec. 4.4: K^ = K[I, :], V^ = V[I, :].  Row i of unit u in `out` becomes row
 * kept_idx[u, i] of the virtual concatenation (in rows, then k_new/v_new rows)
 * for i < out->len[u].  Bit-exact copy.  `pos` is gathered too when both
 * caches carry it (rows from k_new get pos_new + their row number).  `out` must
 * not overlap the rows of `in` that are read.
 * Errors: HACK_EINVAL (NULL, overlapping ranges, out rows outside out->rows). */
hack_status hack_compact(hack_ctx* ctx, int32_t B, int32_t N_k,
                         const hack_cache* in, const void* k_new,
                         const void* v_new, int32_t pos_new,
                         const int32_t* kept_idx, int64_t idx_stride,
                         const hack_cache* out, hack_stream stream);

/* ---- final-step merge of contextual heads ---------------------------------
 * Sec. 4.4, paragraph after the f_C equation ("discarded KV tokens in the last
 * generation step are softly integrated into their nearest retained counterparts
 * through similarity-weighted averaging"); supplementary "Compression Setting":
 * only f_C, only the final generation step.  The paper refers to another work
 * for the definition; this library's reading: with k_j the key rows of the
 * uncompressed cache of the step, I the kept rows and E the others,
 *   n(e) = argmax_{r in I} cos(k_e, k_r)        (ties: lower row index)
 *   w_e  = max(cos(k_e, k_n(e)), 0)
 *   K^_r = (k_r + sum_{e in E: n(e) = r} w_e k_e) / (1 + sum w_e),  V^_r likewise
 * (cosine similarity of key rows; a row of zero norm has similarity 0).
 * Call it after hack_compact with the same in / k_new / v_new / kept_idx / out:
 * the rows of `out` are rewritten in place; a kept row nothing was merged into
 * stays bit for bit as hack_compact wrote it.  Row order and `pos` are unchanged.
 *   active  HOST [B*H] nonzero = merge this unit (the contextual heads), or NULL = all
 * Units with out->len[u] == T_in[u] (nothing evicted) are left alone.
 * Similarities are formed in float32 (bf16 products are exact; dots accumulate in
 * float32 on the matrix core), the averages in float32 in ascending row order, so
 * results are reproducible bit for bit.  bf16 contexts only (HACK_EUNSUPPORTED).
 * Errors: HACK_EINVAL (NULL, a unit that keeps no row or more rows than it has,
 * output rows overlapping the unit's input rows), HACK_ECAPACITY. */
hack_status hack_merge(hack_ctx* ctx, int32_t B, int32_t N_k, const hack_cache* in,
                       const void* k_new, const void* v_new, const int32_t* kept_idx,
                       int64_t idx_stride, const uint8_t* active, const hack_cache* out,
                       hack_stream stream);

/* ---- a4: attention of the current scale over the ragged cache -----------
 * Preliminaries, attention equation: O = Softmax(scale * Q K^T) V for every
 * unit over its own kv->len[u] rows, no mask.  out has the layout and element
 * type of q.  Every unit must have at least one row.
 * Errors: HACK_EINVAL, HACK_ECAPACITY as above. */
hack_status hack_attn(hack_ctx* ctx, int32_t B, int32_t N_k, const void* q,
                      const hack_cache* kv, float scale, void* out,
                      hack_stream stream);
/* Which kernel hack_attn / hack_step use for the attention of a launch with B
 * batch elements and N_k queries per unit (same attention equation, same
 * tolerances; reported so that measurements can be attributed to a kernel):
 *   0  work items of 128 queries that share every K/V block (large steps; fp32
 *      contexts always); in a bf16 launch with no more work items than the
 *      device holds work-groups, a few work items may be served by two
 *      work-groups each (half of the keys each, the partial results added up
 *      in float32 in a fixed order) where that shortens the launch,
 *   1  work items of 32 queries whose four waves split the keys and merge their
 *      partial softmax results at the end (bf16, early scale steps: few
 *      queries); in hack_step this kernel also performs the append when no unit
 *      of the step compresses.
 * The choice depends only on B * H, N_k and the context's head_dim.
 * Returns a negative hack_status for a NULL context or B, N_k < 1. */
int32_t hack_attn_variant(const hack_ctx* ctx, int32_t B, int32_t N_k);

/* ---- offline head classification: attention variance --------------------
 * Sec. 4.2, "Offline Head Classification via Attention Variance": for every
 * unit, A = Softmax(scale * Q K^T) over ALL keys of kv (the uncompressed cache
 * of the final step) and all N_k queries, and
 *   sigma[u] = sum_j Var_i(A[i, j])     (population variance across queries).
 * The caller averages sigma over a validation set, ranks all (layer, head)
 * pairs and calls the lowest alpha * L * H of them contextual; that ranking is
 * host arithmetic on L * H numbers and is not part of this library.
 *   q      DEVICE [B, H, N_k, d]
 *   kv     the cache to attend over (kv->v may be NULL: values are not used)
 *   sigma  DEVICE double [B*H], overwritten
 * bf16 contexts only (HACK_EUNSUPPORTED otherwise).  Accuracy: probabilities
 * are formed in float32 from chained MFMA scores (relative error ~1e-5 at most),
 * the moments are accumulated in fp64.
 * Errors: HACK_EINVAL (NULL/misaligned pointers, empty unit, bad scale),
 * HACK_ECAPACITY (B*H or N_k above the context's limits). */
hack_status hack_head_variance(hack_ctx* ctx, int32_t B, int32_t N_k, const void* q,
                               const hack_cache* kv, float scale, double* sigma,
                               hack_stream stream);

/* ---- a5: the whole step on a library-managed cache -----------------------
 * The managed cache gives every unit two slabs of cap[u] rows inside memory
 * the caller provides (compaction writes from one slab to the other; a unit
 * that does not compress appends in place).  cap[u] must cover the longest
 * cache the unit ever holds after a step (normally its budget).
 *
 * hack_kvcache_rows_required: rows k_mem/v_mem/pos_mem must hold. */
hack_status hack_kvcache_rows_required(int32_t n_units, const int32_t* cap,
                                       int64_t* rows);
/* k_mem, v_mem: DEVICE [mem_rows, head_dim]; pos_mem: DEVICE int32 [mem_rows] or NULL. */
hack_status hack_kvcache_create(hack_ctx* ctx, int32_t n_units,
                                const int32_t* cap, void* k_mem, void* v_mem,
                                int32_t* pos_mem, int64_t mem_rows,
                                hack_kvcache** out);
void hack_kvcache_destroy(hack_kvcache* c);
/* Forget all rows (start of a new image). */
hack_status hack_kvcache_reset(hack_kvcache* c);
/* Current state as a hack_cache; view->off/len point into c and stay valid
 * until the next hack_step / reset / destroy on c. */
hack_status hack_kvcache_view(const hack_kvcache* c, hack_cache* view);

/* One scale step for all units of a layer (Sec. 4.3: compression is applied
 * prior to the attention computation whenever a unit's cache exceeds its
 * budget): append k_new/v_new, and for every unit with budget[u] < T_in[u]
 * score -> select -> compact; then attention over the resulting cache.
 * Observation rows are the evenly strided n_obs = min(cfg n_obs, N_k).
 *   head_type HOST [H]; budget HOST [B*H]; n_init as in hack_select
 *   out DEVICE [B, H, N_k, d]
 *   kept_idx_opt DEVICE int32 [B*H, idx_stride] or NULL: receives the kept
 *     indices of compressing units (rows of other units untouched).
 * Errors: as the individual calls; HACK_ECAPACITY if a unit would outgrow its slab. */
hack_status hack_step(hack_ctx* ctx, hack_kvcache* cache, int32_t B,
                      int32_t N_k, const void* q, const void* k_new,
                      const void* v_new, const uint8_t* head_type,
                      const int32_t* budget, int32_t n_init, float scale,
                      void* out, int32_t* kept_idx_opt, int64_t idx_stride,
                      hack_stream stream);

/* The last scale step of an image: hack_step, and every contextual unit that
 * compresses at this step merges the rows it discards into the rows it keeps
 * (hack_merge) before the attention of the step runs over them (Sec. 4.4,
 * paragraph after the f_C equation; supplementary "Compression Setting").
 * Structural units and units that do not compress behave as in hack_step.
 * bf16 contexts only.  Arguments and errors as hack_step. */
hack_status hack_step_final(hack_ctx* ctx, hack_kvcache* cache, int32_t B,
                            int32_t N_k, const void* q, const void* k_new,
                            const void* v_new, const uint8_t* head_type,
                            const int32_t* budget, int32_t n_init, float scale,
                            void* out, int32_t* kept_idx_opt, int64_t idx_stride,
                            hack_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* HACK_MI355X_H */
