// Declarations shared by the two attention translation units.
#pragma once

#include "ifkv_internal.h"

namespace ifkv {

bool attention_mfma_supported(const ifkv_ctx *ctx);
// Scratch the MFMA path needs for the partial results of launches cut along the kv axis: fixed for
// a layer shape.
size_t attention_mfma_scratch_bytes(const ifkv_ctx *ctx);
// The launches launch_attention_mfma would make (see the definition); out = {launches, most kv parts,
// shortest part in tiles, most bytes of partial results}.
void attention_mfma_plan(const ifkv_ctx *ctx, int64_t n_rows, int64_t n_kv, size_t scratch_bytes, int64_t out[4]);
hipError_t launch_attention_mfma(ifkv_ctx *ctx, const void *q_sel, const int32_t *row_pos, int64_t n_rows,
                                 const void *k_cache, const void *v_cache, int64_t n_kv, void *out,
                                 float *lse_out);

}  // namespace ifkv
