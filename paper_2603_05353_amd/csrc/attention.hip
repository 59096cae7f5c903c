// Stage 4 -- "KV Recomputation": causal attention of the selected rows over
// the full prefix of the concatenated cache.
//
// This file holds the dispatcher and the plain fp32 ALU kernel (any dtype;
// used for fp32 layers and for cross-checking).  The bf16 MFMA kernel lives in
// attention_mfma.hip.
#include "attention_common.h"
#include "ifkv_device.h"
#include "ifkv_internal.h"

namespace ifkv {

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float block_reduce_max(float v, float *red) {
  v = wave_max(v);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int w = 1; w < kThreads / 64; ++w) r = fmaxf(r, red[w]);
  return r;
}
__device__ __forceinline__ float block_reduce_sum(float v, float *red) {
  v = wave_sum(v);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int w = 1; w < kThreads / 64; ++w) r += red[w];
  return r;
}

// One block per (selected row, query head).  Keys are taken 256 at a time:
// every thread forms one logit, the block agrees on the running max and sum,
// and then thread t accumulates output column t % D over a 1/PARTS share of the
// tile's keys (coalesced reads of V across columns).
template <typename Tag, int D>
__global__ __launch_bounds__(kThreads) void attn_generic_kernel(const void *__restrict__ q_sel,
                                                                const int32_t *__restrict__ row_pos,
                                                                const void *__restrict__ k_cache,
                                                                const void *__restrict__ v_cache, int64_t n_kv,
                                                                int n_q_heads, int n_kv_heads, float sm_scale,
                                                                CacheLayout lay, void *__restrict__ out,
                                                                float *__restrict__ lse_out) {
  using E = Elem<Tag>;
  constexpr int VE = E::kVec;
  constexpr int PARTS = kThreads / D;
  __shared__ float qs[D];
  __shared__ float ps[kThreads];
  __shared__ float red[kThreads / 64];
  __shared__ float comb[kThreads];

  const int r = blockIdx.x;
  const int h = blockIdx.y;
  const int g = h / (n_q_heads / n_kv_heads);
  const int tid = threadIdx.x;
  const int64_t obase = (static_cast<int64_t>(r) * n_q_heads + h) * D;
  const int64_t p = row_pos[r];
  if (p < 0 || p >= n_kv) {
    if (tid < D) E::store1(out, obase + tid, 0.f);
    if (lse_out != nullptr && tid == 0) lse_out[static_cast<int64_t>(r) * n_q_heads + h] = 0.f;
    return;
  }
  if (tid < D) qs[tid] = E::load1(q_sel, obase + tid) * sm_scale;
  __syncthreads();

  const int c = tid % D;
  const int part = tid / D;
  float acc = 0.f, m_run = -INFINITY, l_run = 0.f;
  for (int64_t j0 = 0; j0 <= p; j0 += kThreads) {
    const int64_t j = j0 + tid;
    const bool valid = j <= p;
    float logit = -INFINITY;
    if (valid) {
      const v4u *kr = reinterpret_cast<const v4u *>(static_cast<const char *>(k_cache) + lay.at(j, g) * E::kBytes);
      float dot = 0.f;
#pragma unroll
      for (int v = 0; v < D / VE; ++v) {
        float f[VE];
        E::unpack(kr[v], f);
#pragma unroll
        for (int e = 0; e < VE; ++e) dot = fmaf(qs[v * VE + e], f[e], dot);
      }
      logit = dot;
    }
    const float m_new = fmaxf(m_run, block_reduce_max(logit, red));
    const float alpha = expf(m_run - m_new);  // 0 on the first tile
    const float pj = valid ? expf(logit - m_new) : 0.f;
    ps[tid] = pj;
    const float tile_sum = block_reduce_sum(pj, red);  // its barriers also publish ps
    l_run = l_run * alpha + tile_sum;
    m_run = m_new;
    const int nt = static_cast<int>(min<int64_t>(kThreads, p + 1 - j0));
    acc *= alpha;
    for (int jj = part; jj < nt; jj += PARTS)
      acc = fmaf(ps[jj], E::load1(v_cache, lay.at(j0 + jj, g) + c), acc);
    __syncthreads();
  }
  comb[tid] = acc;
  __syncthreads();
  if (tid < D) {
    float o = 0.f;
#pragma unroll
    for (int q = 0; q < PARTS; ++q) o += comb[q * D + tid];
    E::store1(out, obase + tid, o / l_run);
  }
  if (lse_out != nullptr && tid == 0) lse_out[static_cast<int64_t>(r) * n_q_heads + h] = m_run + logf(l_run);
}

template <typename Tag, int D>
hipError_t run_generic(ifkv_ctx *ctx, const void *q_sel, const int32_t *row_pos, int64_t n_rows, const void *k_cache,
                       const void *v_cache, int64_t n_kv, void *out, float *lse_out) {
  const auto &d = ctx->desc;
  // grid.x carries the rows; split very large row counts over several launches
  const int64_t kMaxRows = 1 << 20;
  for (int64_t r0 = 0; r0 < n_rows; r0 += kMaxRows) {
    const int64_t nr = n_rows - r0 < kMaxRows ? n_rows - r0 : kMaxRows;
    const int64_t qoff = r0 * d.n_q_heads * D * Elem<Tag>::kBytes;
    hipLaunchKernelGGL((attn_generic_kernel<Tag, D>), dim3(static_cast<unsigned>(nr), d.n_q_heads), dim3(kThreads), 0,
                       ctx->stream, static_cast<const char *>(q_sel) + qoff, row_pos + r0, k_cache, v_cache, n_kv,
                       d.n_q_heads, d.n_kv_heads, ctx->sm_scale, cache_layout(ctx), static_cast<char *>(out) + qoff,
                       lse_out ? lse_out + r0 * d.n_q_heads : nullptr);
  }
  return hipGetLastError();
}

}  // namespace

void attention_plan(const ifkv_ctx *ctx, int64_t n_rows, int64_t n_kv, size_t scratch_bytes, int64_t out[4]) {
  const bool generic = (ctx->desc.flags & IFKV_FLAG_FORCE_GENERIC) || !attention_mfma_supported(ctx);
  if (generic) {  // one launch of the ALU kernel, never cut
    out[0] = n_rows > 0 ? 1 : 0;
    out[1] = 1;
    out[2] = (n_kv + 63) / 64;
    out[3] = 0;
    return;
  }
  attention_mfma_plan(ctx, n_rows, n_kv, scratch_bytes, out);
}

size_t attention_scratch_bytes(const ifkv_ctx *ctx) {
  const bool generic = (ctx->desc.flags & IFKV_FLAG_FORCE_GENERIC) || !attention_mfma_supported(ctx);
  return generic ? 0 : attention_mfma_scratch_bytes(ctx);
}

hipError_t launch_attention(ifkv_ctx *ctx, const void *q_sel, const int32_t *row_pos, int64_t n_rows,
                            const void *k_cache, const void *v_cache, int64_t n_kv, void *out, float *lse_out) {
  if (n_rows <= 0) return hipSuccess;
  const auto &d = ctx->desc;
  const bool generic = (d.flags & IFKV_FLAG_FORCE_GENERIC) || !attention_mfma_supported(ctx);
  if (!generic) return launch_attention_mfma(ctx, q_sel, row_pos, n_rows, k_cache, v_cache, n_kv, out, lse_out);
  if (d.dtype == IFKV_BF16) {
    if (d.head_dim == 128) return run_generic<BF16Tag, 128>(ctx, q_sel, row_pos, n_rows, k_cache, v_cache, n_kv, out, lse_out);
    return run_generic<BF16Tag, 64>(ctx, q_sel, row_pos, n_rows, k_cache, v_cache, n_kv, out, lse_out);
  }
  if (d.head_dim == 128) return run_generic<F32Tag, 128>(ctx, q_sel, row_pos, n_rows, k_cache, v_cache, n_kv, out, lse_out);
  return run_generic<F32Tag, 64>(ctx, q_sel, row_pos, n_rows, k_cache, v_cache, n_kv, out, lse_out);
}

}  // namespace ifkv
