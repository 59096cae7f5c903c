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
 *   "attn_tail_div"         stage 4: the units of the last stretch of a launch
 *                           are 1/value of a kv range long, a power of two,
 *                           1 .. 8 and at most the range (default 8); 0
 *                           restores the default
 *   "attn_max_row_blocks"   stage 4: row blocks (128 query columns each) per
 *                           launch, 1 .. 1024 (the default may be lower: it
 *                           follows from the partial-result slots the layer's
 *                           max_ctx allows); more rows take several launches;
 *                           0 restores the default
 *   "attn_range_tiles"      stage 4: shortest kv range of the work plan in
 *                           64-row tiles, a power of two, 1 .. 4096 (default
 *                           64); 0 restores the default
 *
 * Host only, no GPU call.  Errors: IFKV_EINVAL for a NULL context or key, an
 * unknown key or a value out of range.
 */
int ifkv_set_tuning(ifkv_ctx *ctx, const char *key, int64_t value);

/*
 * Host only, no GPU call: the stage-4 work plan of one kv head for a launch
 * whose row blocks (128 query columns each, longest first) span the given
 * numbers of 64-row kv tiles.  It runs the same walk and slot functions as the
 * kernel, so that tests can check on the CPU that every (row block, kv tile)
 * pair is processed exactly once, that no two pieces share a partial-result
 * slot and that the merge of a row block finds exactly the pieces written.
 *   block_tiles   host, [n_rb], non-increasing, each >= 1; n_rb 1 .. 1024
 *   wg_per_head, tail_div, range_tiles (a power of two), slot_cap: as the
 *                 launch would pass them
 *   segments      host, nullable, [max_segments][6]: unit, row block, first
 *                 tile, end tile, slot, 1 if the piece is a whole row block
 *                 (written directly, the slot is unused) else 0 -- in the
 *                 order of the line; workgroup w starts with unit w and takes
 *                 its next unit from a shared counter whenever it starts one
 *   pieces        host, nullable, [max_pieces][2]: row block, slot -- what
 *                 the merge of each row block reads, in merge order
 *   n_pieces_out  host, nullable: number of (row block, slot) pairs
 *   range_out     host, nullable: the range length the plan settled on
 * Returns the number of segments (which may exceed max_segments: then only
 * the first max_segments were stored), IFKV_EINVAL for bad arguments,
 * IFKV_ESHAPE if no range length fits slot_cap.
 */
int64_t ifkv_attention_plan(const int32_t *block_tiles, int32_t n_rb, int32_t wg_per_head, int32_t tail_div,
                            int32_t range_tiles, int32_t slot_cap, int32_t *segments, int64_t max_segments,
                            int32_t *pieces, int64_t max_pieces, int64_t *n_pieces_out, int32_t *range_out);

#ifdef __cplusplus
}
#endif
#endif /* IFKV_DEBUG_H */
