/*
 * ifkv_debug.h -- tuning and testing aids of libifkv (not part of the method).
 */
#ifndef IFKV_DEBUG_H
#define IFKV_DEBUG_H

#include "ifkv.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Overrides one of the library's own launch choices for this context.  The
 * results of every stage are the same to the stage's tolerance whatever the
 * values; the tests use the knobs to reach code paths (several launches over
 * row ranges, launches cut along the kv axis into many parts) on inputs small
 * enough for the CPU oracle, and the benchmark uses them for sweeps.
 *
 *   key                     value
 *   "attn_split_parts"      stage 4: cut the kv axis of every launch into this
 *                           many equal parts, 1 .. 65535 (1 = never cut); 0
 *                           restores the library's own choice
 *   "attn_part_tiles"       stage 4: cut the kv axis into parts of this many
 *                           64-row tiles (row blocks shorter than a part are
 *                           not cut); takes precedence over attn_split_parts;
 *                           0 restores the library's own choice
 *   "attn_max_row_blocks"   stage 4: row blocks (128 query columns each) per
 *                           launch, 1 .. 65535; more rows take several
 *                           launches; 0 restores the default (65535)
 *   "attn_exact_sweep"      stage 4 (bf16 MFMA kernel): 1 = every workgroup sweeps
 *                           its keys with the running maximum right away; 0
 *                           (default) = first with the logit of the sweep's
 *                           first key as the fixed reference exponent, and
 *                           again with the running maximum only if a column's
 *                           sum shows that some key outweighs that first key
 *                           by more than 4096 times the number of keys
 *   "fused_repo_score"      ifkv_reposition_score: 1 = take the first scoring
 *                           sweep straight from the chunk caches (one kernel
 *                           re-rotates, stores and scores) where the layer
 *                           shape allows; 0 (default) = the two stages one
 *                           after the other, which is the faster of the two
 *                           at every measured shape
 * A cut whose partial results would not fit the context's scratch (sized for
 * the largest launch the library cuts by itself) is not made.
 *
 * Host only, no GPU call.  Errors: IFKV_EINVAL for a NULL context or key, an
 * unknown key or a value out of range.
 */
int ifkv_set_tuning(ifkv_ctx *ctx, const char *key, int64_t value);

/*
 * Reports how ifkv_recompute_attention would serve a call of n_rows rows against
 * n_kv keys under the context's descriptor and tuning, without launching
 * anything: plan[0] = launches (more than 65535 row blocks take several),
 * plan[1] = the largest number of kv parts any launch is cut into (1 = not
 * cut), plan[2] = the shortest part, in 64-row tiles, plan[3] = the most bytes
 * of partial results any launch keeps in scratch, plan[4] = the bytes of the
 * context's scratch (as allocated, or as the first stage call will allocate
 * it).  The library never makes a cut with plan[3] > plan[4]; the host tests
 * check that over sweeps of shapes and knobs.
 *
 * Host only, no GPU call.  plan: host, 5 entries.  Errors: IFKV_EINVAL for a
 * NULL context or plan, n_rows < 0, n_kv < 1 or beyond max_ctx.
 */
int ifkv_attention_plan(ifkv_ctx *ctx, int64_t n_rows, int64_t n_kv, int64_t *plan);

#ifdef __cplusplus
}
#endif
#endif /* IFKV_DEBUG_H */
