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
 * row ranges, row blocks cut between many workgroups) on inputs small enough
 * for the CPU oracle, and the benchmark uses them for sweeps.
 *
 *   key                     value
 *   "attn_wg_per_head"      stage 4: workgroups per kv head, 1 .. the default
 *                           (512 / H_kv, at least 1); 0 restores the default
 *   "attn_min_share_tiles"  stage 4: a workgroup is only used if its share of
 *                           the launch is at least this many 64-row kv tiles
 *                           (default 8); 0 restores the default
 *   "attn_max_row_blocks"   stage 4: row blocks (128 query columns each) per
 *                           launch, 1 .. 3072; more rows take several launches;
 *                           0 restores the default
 *
 * Host only, no GPU call.  Errors: IFKV_EINVAL for a NULL context or key, an
 * unknown key or a value out of range.
 */
int ifkv_set_tuning(ifkv_ctx *ctx, const char *key, int64_t value);

#ifdef __cplusplus
}
#endif
#endif /* IFKV_DEBUG_H */
