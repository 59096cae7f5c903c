/*
 * ifkv.h -- C ABI of the InfoFlow KV per-layer selective-recompute path for
 * AMD MI355X (gfx950).
 *
 * Given independently prefilled chunk KV caches, a chunk order, prompt queries
 * and a recompute ratio, one layer of the path is five calls:
 *
 *   ifkv_reposition_keys      assemble the chunks in order and advance each key's
 *                             rotary phase from its chunk-local to its global
 *                             position
 *   ifkv_score_tokens         prompt-conditioned attention-norm score per token
 *   ifkv_select_topk          the k = floor(ratio * N) best tokens
 *   ifkv_recompute_attention  causal attention of the selected rows over the
 *                             full prefix
 *   ifkv_splice_kv            write the recomputed K/V rows back into the cache
 *
 * and, where the chunks are exchangeable, ifkv_chunk_counts + ifkv_reorder_chunks
 * derive a better chunk order from a first-stage selection.
 *
 * General conventions
 * -------------------
 * - Every tensor is dense, row-major, [tokens, heads, head_dim], in the dtype of
 *   the layer descriptor (IFKV_F32: IEEE binary32; IFKV_BF16: bfloat16).
 * - "device" pointers are HIP device memory of the GPU that is current when the
 *   call is made; "host" pointers are ordinary host memory, read before the
 *   call returns.  The caller owns every buffer passed in; the library never
 *   frees, reallocates or keeps a caller pointer after the call's kernels end.
 *   The context owns only its own scratch memory: one allocation (and a 1 KiB
 *   block of counters beside it), sized from the layer descriptor (max_ctx,
 *   max_prompt, head counts), made by the first stage call that needs scratch
 *   and freed by ifkv_destroy.  No later call allocates, frees or synchronises
 *   (except under IFKV_FLAG_VALIDATE, which synchronises by design).
 * - All device work is enqueued on the context's HIP stream and the calls
 *   return without waiting for it.  Host outputs (chunk starts, N, k) are
 *   computed on the host from host inputs and are valid on return.
 * - Return value: IFKV_OK (0) or a negative ifkv_status.  Nothing throws or
 *   aborts.  After a failure ifkv_last_error() describes it.  Arguments are
 *   validated before any GPU call, so invalid arguments are reported even on a
 *   machine without a GPU.
 * - Preconditions on device-resident data that cannot be checked without a
 *   host sync (row_pos strictly ascending, idx unique) are the caller's
 *   responsibility; indices outside [0, n_kv) are skipped by the kernels, never
 *   dereferenced.  A context created with IFKV_FLAG_VALIDATE checks both on
 *   the device before the stage runs, at the price of a host sync per call.
 * - Tensor layouts: chunk caches, queries, outputs and freshly projected rows
 *   are packed row-major as stated per argument; the concatenated caches
 *   follow the descriptor's token_stride / head_stride.
 * - A context is not thread-safe; use one per host thread / stream.
 */
#ifndef IFKV_H
#define IFKV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ifkv_ctx ifkv_ctx;

typedef enum {
  IFKV_OK = 0,
  IFKV_EINVAL = -1, /* null pointer, value out of range, not a permutation ... */
  IFKV_ESHAPE = -2, /* sizes inconsistent with the layer descriptor or its maxima */
  IFKV_EDTYPE = -3, /* unknown dtype / pairing */
  IFKV_ENOMEM = -4, /* scratch allocation failed */
  IFKV_EHIP = -5    /* a HIP runtime call or kernel launch failed */
} ifkv_status;

typedef enum { IFKV_F32 = 0, IFKV_BF16 = 1 } ifkv_dtype;

/* Which two coordinates are rotated together as one plane (Preliminary, "Rotary
 * Positional Embedding", Eq. (3)).  HALF couples (x_i, x_{i+d/2}); INTERLEAVED
 * couples (x_{2i}, x_{2i+1}). */
typedef enum { IFKV_ROPE_HALF = 0, IFKV_ROPE_INTERLEAVED = 1 } ifkv_rope_pairing;

/* Route every stage through the plain fp32 ALU kernels even where a bf16 MFMA
 * kernel exists (cross-checking and debugging). */
#define IFKV_FLAG_FORCE_GENERIC 1u
/* Debug mode: check on the device the preconditions that host code cannot see
 * -- row_pos of ifkv_recompute_attention strictly ascending, idx of
 * ifkv_splice_kv free of duplicates -- before the stage runs.  With this flag
 * the two calls wait for the stream (the answer has to reach the host) and
 * return IFKV_EINVAL, with the offending position in the message, instead of
 * computing on bad input.  Without it such input is undefined behaviour. */
#define IFKV_FLAG_VALIDATE 2u

typedef struct {
  int32_t dtype;      /* ifkv_dtype of K, V, Q and attention outputs */
  int32_t n_q_heads;  /* H_q; must be a multiple of n_kv_heads */
  int32_t n_kv_heads; /* H_kv; query head h reads kv head h / (H_q / H_kv) */
  int32_t head_dim;   /* d: 64 or 128 */
  double rope_theta;  /* base of Eq. (4): theta_i = base^(-2 i / d) */
  const double *inv_freq; /* host, d/2 entries, or NULL to use rope_theta; copied by ifkv_create */
  int32_t pairing;    /* ifkv_rope_pairing */
  float sm_scale;     /* logit scale; 0 selects 1/sqrt(d) */
  int64_t max_ctx;    /* largest number of cache rows (context + prompt rows) any call will pass */
  int32_t max_prompt; /* largest m_prompt */
  uint32_t flags;     /* IFKV_FLAG_* */
  /* Layout of the concatenated caches (k_out / v_out of stage 1, k_global of
   * stage 2, k_cache / v_cache of stages 4 and 5), in elements: element c of kv
   * head h of cache row t sits at t * token_stride + h * head_stride + c.  Both
   * 0 selects the packed [T, H_kv, d] layout (token_stride = H_kv * d,
   * head_stride = d).  [H_kv, T_cap, d] is token_stride = d, head_stride =
   * T_cap * d.  Both must be multiples of 16 bytes' worth of elements, at least
   * d, and the heads of a row / the rows of a head must not overlap: either
   * token_stride >= (H_kv - 1) * head_stride + d or head_stride >= (max_ctx - 1)
   * * token_stride + d.  Chunk caches, query tensors and freshly projected rows
   * (k_new, v_new, k_prompt, x of ifkv_rope_rows) are always packed. */
  int64_t token_stride;
  int64_t head_stride;
} ifkv_layer_desc;

/* Creates a context for one layer shape bound to `hip_stream` (a hipStream_t;
 * NULL = the default stream).  Makes no GPU call.  On success *out is a
 * context to be released with ifkv_destroy.  On failure *out is NULL and the
 * message is available through ifkv_last_error(NULL). */
int ifkv_create(ifkv_ctx **out, const ifkv_layer_desc *desc, void *hip_stream);

/* Frees the context and its scratch memory.  The caller must have synchronised
 * the stream.  NULL is ignored. */
void ifkv_destroy(ifkv_ctx *ctx);

/* Message of the last failed call on `ctx` (or of the last failed ifkv_create
 * on this thread when ctx is NULL).  Never NULL; valid until the next call. */
const char *ifkv_last_error(const ifkv_ctx *ctx);

/* Library version, "major.minor". */
const char *ifkv_version(void);

/*
 * Stage 1 -- Method, "Token Selection and Recomputation", Eq. (5) with the
 * rotation of Eq. (3)-(4).
 *
 * The chunk in slot s of the concatenation starts at row
 *   Delta = sum_{s' < s} chunk_len[chunk_order[s']]
 * and its token with chunk-local index p gets global position g = Delta + p.
 * Each cached key carries the rotary phase of the position it was prefilled at
 * (cached_pos0[i] + p); the kernel advances every 2-D pair j of every key of
 * chunk i by the angle (Delta_i - cached_pos0[i]) * theta_j, which is exactly
 * the rotary embedding at g because rotations about the same axis add, and
 * writes it to row g of k_out.  Values have no rotary phase; v rows are copied
 * to the same rows of v_out.  Angles are formed in fp64 on the device, the
 * rotation itself runs in fp32, and the result is rounded once to the storage
 * dtype.
 *
 *   n_chunks       number of chunks (>= 0)
 *   k_chunks       host array of n_chunks DEVICE pointers, chunk i is
 *                  [chunk_len[i], H_kv, d]; an entry may be NULL iff its length is 0
 *   v_chunks       same for values, or NULL to process keys only (then v_out is ignored)
 *   chunk_len      host, n_chunks entries, each >= 0
 *   chunk_order    host, permutation of 0..n_chunks-1, slot -> chunk id; NULL = identity
 *   cached_pos0    host, rotary position of each chunk's first cached row; NULL = all 0
 *   delta_override host, per chunk: use this phase advance instead of
 *                  Delta_i - cached_pos0[i] (the other RoPE geometries of the
 *                  "RoPE Geometry" paragraph); NULL = GLOBAL geometry
 *   k_out, v_out   device [N, H_kv, d], N = sum of chunk_len; must not overlap any chunk
 *   chunk_start_out host, n_chunks entries: Delta_i by chunk id; may be NULL
 *   n_ctx_out      host: N; may be NULL
 *
 * Errors: IFKV_EINVAL for NULL required pointers, negative lengths, a
 * chunk_order that is not a permutation; IFKV_ESHAPE if N > max_ctx.
 */
int ifkv_reposition_keys(ifkv_ctx *ctx, int32_t n_chunks,
                         const void *const *k_chunks, const void *const *v_chunks,
                         const int32_t *chunk_len, const int32_t *chunk_order,
                         const int32_t *cached_pos0, const int64_t *delta_override,
                         void *k_out, void *v_out,
                         int64_t *chunk_start_out, int64_t *n_ctx_out);

/*
 * Stage 2 -- Eq. (7): s_j = sum_i A_ij, the attention mass context token j
 * receives from all prompt tokens, A being the prompt-to-context attention.
 *
 * For query head h (kv head h / G), prompt row i and context token j the logit
 * is sm_scale * q_{i,h} . k_{j,h/G}; A is its softmax over the n_ctx context
 * columns.  If k_prompt is given the softmax of row i additionally runs over
 * prompt keys 0..i (what a real forward pass would normalise over); those
 * columns are not part of the output.  Scores are averaged over the H_q query
 * heads, so without k_prompt they sum to m_prompt.  Logits, exponentials and
 * sums are fp32.
 *
 *   k_global   device [n_ctx, H_kv, d], keys in the global rotary frame
 *   q_prompt   device [m_prompt, H_q, d], queries with their rotary embedding
 *              (positions n_ctx .. n_ctx + m_prompt - 1 in the GLOBAL geometry)
 *              already applied by the caller
 *   k_prompt   device [m_prompt, H_kv, d] or NULL
 *   accumulate 0: scores[j] = s_j; 1: scores[j] += s_j (summing several layers)
 *   scores     device float [n_ctx]
 *
 * n_ctx == 0 or m_prompt == 0 with accumulate == 0 writes zeros (nothing for
 * n_ctx == 0).  Errors: IFKV_EINVAL (NULL pointers, negative sizes),
 * IFKV_ESHAPE (n_ctx > max_ctx, m_prompt > max_prompt).
 */
int ifkv_score_tokens(ifkv_ctx *ctx, const void *k_global, int64_t n_ctx,
                      const void *q_prompt, int32_t m_prompt,
                      const void *k_prompt, int32_t accumulate, float *scores);

/*
 * Stages 1 and 2 in one call -- Eq. (5) and Eq. (7): ifkv_reposition_keys followed
 * by ifkv_score_tokens on its k_out, with the same arguments, the same outputs
 * (k_out, v_out, chunk_start_out, n_ctx_out, scores) and the same error
 * behaviour as the two calls.  The scores need every re-rotated key twice (once
 * for the softmax statistics of each prompt row, once for the column sums); given
 * both stages at once the library may take the first of these sweeps straight
 * from the chunk caches: a key is read once, advanced to its global rotary phase
 * in registers, stored to k_out and multiplied with the prompt queries in the
 * same kernel.  Either way k_out and v_out hold bit for bit what
 * ifkv_reposition_keys writes and the scores are those of ifkv_score_tokens on
 * that k_out.  Which way is taken is the library's choice (on the MI355X the two
 * stages one after the other are faster at every measured shape, so that is the
 * default; include/ifkv_debug.h has the knob).  Layer shapes the fused kernel
 * does not serve (fp32, head_dim 64, IFKV_FLAG_FORCE_GENERIC, more than 512
 * non-empty chunks, m_prompt = 0) always run the two stages.
 */
int ifkv_reposition_score(ifkv_ctx *ctx, int32_t n_chunks, const void *const *k_chunks,
                          const void *const *v_chunks, const int32_t *chunk_len,
                          const int32_t *chunk_order, const int32_t *cached_pos0,
                          const int64_t *delta_override, void *k_out, void *v_out,
                          int64_t *chunk_start_out, int64_t *n_ctx_out,
                          const void *q_prompt, int32_t m_prompt, const void *k_prompt,
                          int32_t accumulate, float *scores);

/*
 * Stage 3 -- Eq. (8) with the budget k = floor(rho * N) of "Chunk Reordering":
 * one global top-k set, no per-chunk quota.
 *
 * Selects the k largest scores; equal scores are resolved in favour of the
 * smaller index (-0 and +0 compare equal); the selected indices are written in
 * ascending order.  NaN scores are not supported.  Integer work only: the
 * result is exact for the fp32 values given.
 *
 *   scores      device float [n_ctx]
 *   ratio       rho in [0, 1]; used when k_override < 0: k = floor(ratio * n_ctx)
 *               evaluated in double precision
 *   k_override  >= 0: use this k (must be <= n_ctx)
 *   idx_out     device int32 [k]; NULL: nothing is selected, the call only
 *               reports k (to size idx_out for a second call), no GPU work
 *   k_out       host: k (known without a device sync); may be NULL
 *
 * Errors: IFKV_EINVAL (ratio outside [0,1], k > n_ctx, NULL pointers),
 * IFKV_ESHAPE (n_ctx > max_ctx or >= 2^31).
 */
int ifkv_select_topk(ifkv_ctx *ctx, const float *scores, int64_t n_ctx,
                     double ratio, int64_t k_override,
                     int32_t *idx_out, int64_t *k_out);

/*
 * ifkv_select_topk for callers that cannot allocate device memory: code under
 * HIP graph capture before the context's scratch exists, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same result bit for bit.
 * The call allocates nothing on host or device: the histograms and counts its
 * kernels need live in a static device array inside the library
 * (24 KiB + 8 bytes per 4096 scores, 32 KiB in all; every GPU the library runs
 * on holds it until the process ends), which limits n_ctx to 2^22 = 4194304.
 * All calls on one GPU share that array, whatever their context: calls that
 * overlap on one GPU (different streams) race; calls on one stream do not.
 * What must start at zero is cleared by a kernel of the call itself.
 *
 * Errors: as ifkv_select_topk, and IFKV_ESHAPE for n_ctx above the limit.
 */
int ifkv_select_topk_noalloc(ifkv_ctx *ctx, const float *scores, int64_t n_ctx,
                             double ratio, int64_t k_override, int32_t *idx_out,
                             int64_t *k_out);

/*
 * Stage 4 -- "KV Recomputation" paragraph: every selected token runs an
 * ordinary causal forward pass at its global position over the concatenated
 * sequence.  This call is the attention of that pass.
 *
 * For row r with global position p = row_pos[r] and query head h:
 *   out[r,h,:] = sum_{j <= p} softmax_j(sm_scale * q[r,h] . k[j,h/G]) * v[j,h/G,:]
 * over cache rows 0..p inclusive.  bf16 inputs use bf16 MFMA with fp32
 * accumulation and an fp32 online softmax (probabilities are rounded to bf16
 * for the second product); fp32 inputs are computed in fp32 throughout.
 *
 *   q_sel     device [n_rows, H_q, d], rotary embedding at row_pos already applied
 *   row_pos   device int32 [n_rows], strictly ascending, each in [0, n_kv);
 *             rows with a position outside that range produce zeros
 *   k_cache, v_cache  device [n_kv, H_kv, d]
 *   out       device [n_rows, H_q, d]
 *   lse_out   device float [n_rows, H_q]: natural-log sum-exp of the scaled
 *             logits of each row; may be NULL
 *
 * Errors: IFKV_EINVAL, IFKV_ESHAPE (n_kv > max_ctx).
 */
int ifkv_recompute_attention(ifkv_ctx *ctx, const void *q_sel,
                             const int32_t *row_pos, int64_t n_rows,
                             const void *k_cache, const void *v_cache, int64_t n_kv,
                             void *out, float *lse_out);

/*
 * Stage 5 -- "KV Recomputation" paragraph, last sentence: the recomputed K/V
 * rows replace the cached rows of the selected tokens; all other rows are
 * reused unchanged.
 *
 *   k_cache[idx[r]] = k_new[r];  v_cache[idx[r]] = v_new[r]   (bit-exact copy)
 *
 *   k_new, v_new  device [n_rows, H_kv, d]; v_new/v_cache may both be NULL (keys only)
 *   idx           device int32 [n_rows], unique, in [0, n_kv); out-of-range rows are skipped
 *   k_cache, v_cache  device [n_kv, H_kv, d], updated in place
 */
int ifkv_splice_kv(ifkv_ctx *ctx, const void *k_new, const void *v_new,
                   const int32_t *idx, int64_t n_rows,
                   void *k_cache, void *v_cache, int64_t n_kv);

/*
 * Glue between the model's projections and stages 4/5 -- "KV Recomputation":
 * the forward pass of a selected token runs at the token's position in the
 * concatenated sequence, so its freshly projected query and key rows carry the
 * rotary embedding of Eq. (3)-(4) at that position.  Row r of x is turned, in every
 * 2-D pair j, by pos[r] * theta_j; angles are formed in fp64, the rotation runs
 * in fp32 and is rounded once to the storage dtype.  In place.  (The
 * projections themselves need the model's weights and are not part of this
 * library.)
 *
 *   x        device [n_rows, n_heads, d], 16-byte aligned, updated in place
 *   pos      device int32 [n_rows], the rows' global positions (e.g. the index
 *            list of ifkv_select_topk for context rows)
 *   n_heads  H_q for query rows, H_kv for key rows (any value > 0)
 * Errors: IFKV_EINVAL for NULL pointers, negative sizes, misaligned x.
 */
int ifkv_rope_rows(ifkv_ctx *ctx, void *x, const int32_t *pos, int64_t n_rows, int32_t n_heads);

/*
 * Optional step before the path -- Method, "Chunk Reordering", Eq. (9).
 *
 * After a first-stage selection (stages 1-3 run with the local-context
 * geometry: delta_override all 0, prompt queries at their global positions),
 * chunk i's importance is the density r_i = |S ∩ C_i| / |C_i| of selected
 * tokens in it.  ifkv_chunk_counts computes the numerators on the device from
 * the selected set; ifkv_reorder_chunks (host only, no GPU call) turns them
 * into the new order: ascending r_i, so the densest chunk ends up next to the
 * prompt, and chunks with equal r_i keep their relative order.  Densities are
 * compared exactly (count_a * len_b against count_b * len_a); an empty chunk
 * has density 0.  The caller then runs the path again with the new order.
 *
 *   idx          device int32 [k], ascending (as ifkv_select_topk writes it)
 *   n_slots      number of chunk slots in the concatenation idx refers to
 *   slot_start   host, n_slots entries: first row of each slot, ascending
 *                (chunk_start_out of stage 1 gathered by chunk_order)
 *   n_ctx        total rows; slot s covers [slot_start[s], slot_start[s+1]) and
 *                the last slot ends at n_ctx
 *   counts_out   device int32 [n_slots]: selected rows per slot
 * Errors: IFKV_EINVAL for NULL pointers, negative sizes, slot_start not
 * ascending within [0, n_ctx].
 */
int ifkv_chunk_counts(ifkv_ctx *ctx, const int32_t *idx, int64_t k, int32_t n_slots,
                      const int64_t *slot_start, int64_t n_ctx, int32_t *counts_out);

/*
 *   n_chunks     number of chunks
 *   order_in     host, slot -> chunk id of the order the counts refer to; NULL = identity
 *   slot_counts  host, n_chunks entries: selected rows per SLOT (ifkv_chunk_counts copied back)
 *   chunk_len    host, n_chunks entries indexed by chunk id
 *   order_out    host, n_chunks entries: the new slot -> chunk id order
 * Errors: IFKV_EINVAL for NULL pointers, order_in not a permutation, a count
 * that is negative or exceeds its chunk's length.  ctx may be NULL.
 */
int ifkv_reorder_chunks(ifkv_ctx *ctx, int32_t n_chunks, const int32_t *order_in, const int32_t *slot_counts,
                        const int32_t *chunk_len, int32_t *order_out);

#ifdef __cplusplus
}
#endif
#endif /* IFKV_H */
