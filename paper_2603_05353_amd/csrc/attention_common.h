// Declarations shared by the two attention translation units.
#pragma once

#include "ifkv_internal.h"

namespace ifkv {

bool attention_mfma_supported(const ifkv_ctx *ctx);
// Scratch the MFMA path needs for the partial results of row blocks shared between workgroups, and
// for their arrival counters: fixed for a layer shape.
size_t attention_mfma_scratch_bytes(const ifkv_ctx *ctx);
size_t attention_mfma_counter_bytes(const ifkv_ctx *ctx);
int attention_mfma_slot_cap(const ifkv_ctx *ctx);
int attention_mfma_max_row_blocks(const ifkv_ctx *ctx);
// Host-side bounds check of one launch against the allocated scratch and the plan's capacity.
bool attention_mfma_launch_fits(const ifkv_ctx *ctx, int wg_per_head, int64_t n_row_blocks, int64_t n_kv, int r_min, int tail_div);
hipError_t launch_attention_mfma(ifkv_ctx *ctx, const void *q_sel, const int32_t *row_pos, int64_t n_rows,
                                 const void *k_cache, const void *v_cache, int64_t n_kv, void *out,
                                 float *lse_out);

}  // namespace ifkv
