// Declarations shared by the two attention translation units.
#pragma once

#include "ifkv_internal.h"

namespace ifkv {

bool attention_mfma_supported(const ifkv_ctx *ctx);
// Scratch the MFMA path needs for the partial results of launches cut along the kv axis: fixed for
// a layer shape.
size_t attention_mfma_scratch_bytes(const ifkv_ctx *ctx);
hipError_t launch_attention_mfma(ifkv_ctx *ctx, const void *q_sel, const int32_t *row_pos, int64_t n_rows,
                                 const void *k_cache, const void *v_cache, int64_t n_kv, void *out,
                                 float *lse_out);

}  // namespace ifkv
