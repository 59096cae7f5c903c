// Internal declarations shared by the host-side C ABI and the per-stage HIP
// translation units.  Not installed; the public interface is include/ifkv.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>

#include "ifkv.h"

// Tuning and testing knobs (include/ifkv_debug.h); 0 = the library's own choice.
struct ifkv_tuning {
  int attn_split_parts = 0;      // stage 4: cut the kv axis into this many equal parts
  int attn_part_tiles = 0;       // stage 4: cut the kv axis into parts of this many tiles (takes precedence)
  int attn_max_row_blocks = 0;   // stage 4: row blocks per launch (can only lower the default)
  int attn_exact_sweep = 0;      // stage 4: 1 = always sweep with the running maximum (skip the fixed-reference sweep)
  int fused_repo_score = 0;      // stages 1+2 in one call: 1 = take the first scoring sweep from the chunk caches
};

struct ifkv_ctx {
  ifkv_layer_desc desc;
  ifkv_tuning tune;
  hipStream_t stream = nullptr;
  float sm_scale = 0.f;
  int64_t token_stride = 0;     // concatenated caches: elements between rows / between kv heads (resolved, never 0)
  int64_t head_stride = 0;
  bool packed = true;           // token_stride == H_kv * d and head_stride == d
  double inv_freq[128];         // d/2 entries, host copy
  double *d_inv_freq = nullptr; // device copy, uploaded on first use
  void *scratch = nullptr;      // device scratch shared by the stages, allocated once
  size_t scratch_bytes = 0;
  int *score_arrived = nullptr; // stage 2: blocks of a key range that have finished; zero between launches
  std::string err;
};

namespace ifkv {

constexpr int kMaxHeadDim = 256;

// Where the concatenated caches keep element c of kv head h of row t (elements).
struct CacheLayout {
  int64_t token_stride, head_stride;
  __host__ __device__ __forceinline__ int64_t at(int64_t t, int h) const { return t * token_stride + h * head_stride; }
};
inline CacheLayout cache_layout(const ifkv_ctx *ctx) { return CacheLayout{ctx->token_stride, ctx->head_stride}; }

inline size_t dtype_size(int dtype) { return dtype == IFKV_BF16 ? 2 : 4; }

// ---- stage launchers (each returns a hipError_t from launch checking) ------

// Stage 1.  One launch handles up to kRepoMaxChunks chunks; descriptors travel
// by value in the kernel arguments so no staging copy or host sync is needed.
constexpr int kRepoMaxChunks = 64;
struct RepoChunk {
  const void *k;    // device, [len, H_kv, d]
  const void *v;    // device or null
  int64_t dst_row;  // first row in the concatenated cache
  double advance;   // rotary phase advance in positions
  int32_t len;
  int32_t tile0;    // first tile index of this chunk within the launch
};
struct RepoBatch {
  RepoChunk c[kRepoMaxChunks];
  int32_t n;
  int32_t total_tiles;
};
hipError_t launch_reposition(ifkv_ctx *ctx, const RepoBatch &batch, void *k_out, void *v_out);
int reposition_rows_per_tile();

// Stage 2.
size_t score_scratch_bytes(const ifkv_ctx *ctx, int64_t n_ctx, int m_prompt);
struct FusedRepo;  // score_common.h: stage 1 folded into the first scoring sweep
hipError_t launch_score(ifkv_ctx *ctx, const void *k_global, int64_t n_ctx, const void *q_prompt,
                        int m_prompt, const void *k_prompt, int accumulate, float *scores,
                        const FusedRepo *fused = nullptr);

// Stage 3.
size_t topk_scratch_bytes(const ifkv_ctx *ctx, int64_t n_ctx);
hipError_t launch_topk(ifkv_ctx *ctx, const float *scores, int64_t n_ctx, int64_t k, int32_t *idx_out, void *work);
// the entry point that allocates nothing: its static device scratch and the largest n_ctx it serves
hipError_t topk_static_scratch(void **out);
int64_t topk_static_max_ctx();

// Stage 4.
size_t attention_scratch_bytes(const ifkv_ctx *ctx);
// {launches, most kv parts, shortest part in tiles, most bytes of partial results} of a stage-4 call
void attention_plan(const ifkv_ctx *ctx, int64_t n_rows, int64_t n_kv, size_t scratch_bytes, int64_t out[4]);
hipError_t launch_attention(ifkv_ctx *ctx, const void *q_sel, const int32_t *row_pos, int64_t n_rows,
                            const void *k_cache, const void *v_cache, int64_t n_kv, void *out,
                            float *lse_out);

// Chunk reordering: selected rows per slot.  At most kRepoMaxChunks boundaries per launch.
struct SlotBounds {
  int32_t bound[kRepoMaxChunks + 1];  // bound[s] .. bound[s+1]: rows of slot s
  int32_t n;                          // slots in this launch
};
hipError_t launch_chunk_counts(ifkv_ctx *ctx, const int32_t *idx, int64_t k, const SlotBounds &b, int32_t *counts_out);

// Stage 5.
hipError_t launch_splice(ifkv_ctx *ctx, const void *k_new, const void *v_new, const int32_t *idx,
                         int64_t n_rows, void *k_cache, void *v_cache, int64_t n_kv);

// Debug-mode checks of device-resident preconditions (validate.hip); *bad_out = offending index or -1.
// They wait for the stream.
size_t validate_scratch_bytes(const ifkv_ctx *ctx);
hipError_t validate_ascending(ifkv_ctx *ctx, const int32_t *v, int64_t n, int64_t *bad_out);
hipError_t validate_unique(ifkv_ctx *ctx, const int32_t *idx, int64_t n, int64_t n_kv, int64_t *bad_out);

// Calibration copy.
hipError_t launch_copy(ifkv_ctx *ctx, void *dst, const void *src, int64_t n_bytes);
// matrix-pipe calibration loop (calibrate.hip)
size_t mfma_probe_sink_floats();
double mfma_probe_flops(int iters);
hipError_t launch_mfma_probe(ifkv_ctx *ctx, int pattern, int iters, float *sink);

// Rotary embedding of recomputed rows at given positions, in place.
hipError_t launch_rope_rows(ifkv_ctx *ctx, void *x, const int32_t *pos, int64_t n_rows, int n_heads);

}  // namespace ifkv
