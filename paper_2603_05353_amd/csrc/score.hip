// Stage 2 -- Eq. (7): s_j = sum_i A_ij, the attention mass each context token
// receives from the prompt, averaged over query heads.
//
// A (M x N per head) is never stored.  The softmax normaliser of every prompt
// row is global over the context, so the stage is two sweeps over the keys:
//   pass A: per (head, prompt row) running max m and sum Z = sum_j exp(l - m),
//           computed per slice of the context and merged;
//   pass B: s_j = (1/H_q) sum_h sum_i exp(l_hij - m_hi) / Z_hi.
// All arithmetic on logits, exponentials and sums is fp32.
//
// This file holds the plain fp32 ALU kernels (any dtype; used for fp32 layers
// and for cross-checking).  The bf16 MFMA kernels live in score_mfma.hip.
#include <algorithm>

#include "ifkv_device.h"
#include "ifkv_internal.h"
#include "score_common.h"

namespace ifkv {

namespace {

constexpr int kStatThreads = 64;   // one prompt row per thread
constexpr int kStatTile = 32;      // context tokens staged in LDS per step

// Pass A: partial (m, Z) of one slice of the context for 64 prompt rows of one head.
template <typename Tag, int D>
__global__ __launch_bounds__(kStatThreads) void score_stats_generic(const void *__restrict__ k_global, int64_t n_ctx,
                                                                    const void *__restrict__ q_prompt, int m_prompt,
                                                                    int n_q_heads, int n_kv_heads, float sm_scale,
                                                                    CacheLayout lay, int slice_len,
                                                                    float2 *__restrict__ partial) {
  using E = Elem<Tag>;
  __shared__ float ks[kStatTile][D];
  const int slice = blockIdx.x;
  const int h = blockIdx.y;
  const int r = blockIdx.z * kStatThreads + threadIdx.x;
  const int g = h / (n_q_heads / n_kv_heads);
  const bool active = r < m_prompt;

  float q[D];
  if (active) {
    const int64_t qoff = (static_cast<int64_t>(r) * n_q_heads + h) * D;
#pragma unroll
    for (int c = 0; c < D; ++c) q[c] = E::load1(q_prompt, qoff + c) * sm_scale;
  } else {
#pragma unroll
    for (int c = 0; c < D; ++c) q[c] = 0.f;
  }

  const int64_t j_begin = static_cast<int64_t>(slice) * slice_len;
  const int64_t j_end = min(n_ctx, j_begin + slice_len);
  float m = -INFINITY, z = 0.f;
  for (int64_t j0 = j_begin; j0 < j_end; j0 += kStatTile) {
    const int nt = static_cast<int>(min<int64_t>(kStatTile, j_end - j0));
    __syncthreads();
    for (int e = threadIdx.x; e < nt * D; e += kStatThreads) {
      const int jj = e / D, c = e - jj * D;
      ks[jj][c] = E::load1(k_global, lay.at(j0 + jj, g) + c);
    }
    __syncthreads();
    for (int jj = 0; jj < nt; ++jj) {
      float dot = 0.f;
#pragma unroll
      for (int c = 0; c < D; ++c) dot = fmaf(q[c], ks[jj][c], dot);
      const float mn = fmaxf(m, dot);
      z = z * expf(m - mn) + expf(dot - mn);
      m = mn;
    }
  }
  if (active) partial[(static_cast<int64_t>(slice) * n_q_heads + h) * m_prompt + r] = make_float2(m, z);
}

// Merge the per-slice partials of each (head, row); optionally extend the
// normaliser over the prompt keys the row sees causally (rows 0..r).  Writes
// (m, 1/Z).
template <typename Tag, int D>
__global__ __launch_bounds__(64) void score_merge_kernel(const float2 *__restrict__ partial, int n_slices,
                                                          const void *__restrict__ q_prompt,
                                                          const void *__restrict__ k_prompt, int m_prompt,
                                                          int n_q_heads, int n_kv_heads, float sm_scale,
                                                          float2 *__restrict__ stats) {
  using E = Elem<Tag>;
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_q_heads * m_prompt) return;
  const int h = t / m_prompt, r = t - h * m_prompt;
  // Slices are merged eight at a time: the eight loads are independent, so their latencies overlap.
  float m = -INFINITY, z = 0.f;
  for (int s0 = 0; s0 < n_slices; s0 += 8) {
    float2 p[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      p[u] = make_float2(-INFINITY, 0.f);
      if (s0 + u < n_slices) p[u] = partial[(static_cast<int64_t>(s0 + u) * n_q_heads + h) * m_prompt + r];
    }
    float mn = m;
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (p[u].y > 0.f) mn = fmaxf(mn, p[u].x);
    if (mn > -INFINITY) {
      float acc = z * expf(m - mn);
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (p[u].y > 0.f) acc += p[u].y * expf(p[u].x - mn);
      z = acc;
      m = mn;
    }
  }
  if (k_prompt != nullptr) {
    const int g = h / (n_q_heads / n_kv_heads);
    const int64_t qoff = (static_cast<int64_t>(r) * n_q_heads + h) * D;
    for (int tt = 0; tt <= r; ++tt) {
      const int64_t koff = (static_cast<int64_t>(tt) * n_kv_heads + g) * D;
      float dot = 0.f;
      for (int c = 0; c < D; ++c) dot = fmaf(E::load1(q_prompt, qoff + c) * sm_scale, E::load1(k_prompt, koff + c), dot);
      const float mn = fmaxf(m, dot);
      z = z * expf(m - mn) + expf(dot - mn);
      m = mn;
    }
  }
  stats[h * m_prompt + r] = make_float2(m, z > 0.f ? 1.f / z : 0.f);
}

constexpr int kColThreads = 128;  // one context token per thread
constexpr int kColRows = 32;      // prompt rows staged in LDS per step

// Pass B: column sums with the final (m, 1/Z).  A block owns 128 context tokens of ONE kv head (its
// key rows stay in registers) and sums over that head's G query heads and all prompt rows; the
// per-kv-head partial sums are added up by score_colsum_reduce (no float atomics: the result does not
// depend on the order in which blocks finish).
template <typename Tag, int D>
__global__ __launch_bounds__(kColThreads) void score_colsum_generic(const void *__restrict__ k_global, int64_t n_ctx,
                                                                    const void *__restrict__ q_prompt, int m_prompt,
                                                                    int n_q_heads, int n_kv_heads, float sm_scale,
                                                                    CacheLayout lay, const float2 *__restrict__ stats,
                                                                    float *__restrict__ colpart) {
  using E = Elem<Tag>;
  __shared__ float qs[kColRows][D];
  __shared__ float2 st[kColRows];
  const int64_t j = static_cast<int64_t>(blockIdx.x) * kColThreads + threadIdx.x;
  const bool active = j < n_ctx;
  const int G = n_q_heads / n_kv_heads;
  const int g = blockIdx.y;
  float acc = 0.f;
  float kreg[D];
  if (active) {
    const int64_t koff = lay.at(j, g);
#pragma unroll
    for (int c = 0; c < D; ++c) kreg[c] = E::load1(k_global, koff + c);
  } else {
#pragma unroll
    for (int c = 0; c < D; ++c) kreg[c] = 0.f;
  }
  for (int hh = 0; hh < G; ++hh) {
    const int h = g * G + hh;
    for (int r0 = 0; r0 < m_prompt; r0 += kColRows) {
      const int nr = min(kColRows, m_prompt - r0);
      __syncthreads();
      for (int e = threadIdx.x; e < nr * D; e += kColThreads) {
        const int rr = e / D, c = e - rr * D;
        qs[rr][c] = E::load1(q_prompt, (static_cast<int64_t>(r0 + rr) * n_q_heads + h) * D + c) * sm_scale;
      }
      if (threadIdx.x < nr) st[threadIdx.x] = stats[h * m_prompt + r0 + threadIdx.x];
      __syncthreads();
      for (int rr = 0; rr < nr; ++rr) {
        float dot = 0.f;
#pragma unroll
        for (int c = 0; c < D; ++c) dot = fmaf(qs[rr][c], kreg[c], dot);
        acc += expf(dot - st[rr].x) * st[rr].y;
      }
    }
  }
  if (active) colpart[static_cast<int64_t>(g) * n_ctx + j] = acc;
}

// scores[j] = (accumulate ? scores[j] : 0) + (1 / H_q) * sum over kv heads of the partial column sums
__global__ void score_colsum_reduce(const float *__restrict__ colpart, int n_parts, int64_t n_ctx, float inv_heads,
                                    int accumulate, float *__restrict__ scores) {
  const int64_t j = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (j >= n_ctx) return;
  float s = 0.f;
  for (int p = 0; p < n_parts; ++p) s += colpart[static_cast<int64_t>(p) * n_ctx + j];
  s *= inv_heads;
  scores[j] = accumulate ? scores[j] + s : s;
}

__global__ void fill_zero_kernel(float *p, int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

int slice_len_for(int64_t n_ctx) {
  // at most 64 slices, each a multiple of the LDS tile
  int64_t sl = (n_ctx + 63) / 64;
  sl = ((sl + kStatTile - 1) / kStatTile) * kStatTile;
  if (sl < 64) sl = 64;
  return static_cast<int>(sl);
}

template <typename Tag, int D>
hipError_t run_generic(ifkv_ctx *ctx, const void *k_global, int64_t n_ctx, const void *q_prompt, int m_prompt,
                       const void *k_prompt, int accumulate, float *scores) {
  const auto &d = ctx->desc;
  const int sl = slice_len_for(n_ctx);
  const int n_slices = static_cast<int>((n_ctx + sl - 1) / sl);
  ScoreScratch sc = score_scratch_layout(ctx, n_ctx, m_prompt);
  float2 *partial = reinterpret_cast<float2 *>(static_cast<char *>(ctx->scratch) + sc.partial_off);
  float2 *stats = reinterpret_cast<float2 *>(static_cast<char *>(ctx->scratch) + sc.stats_off);
  hipStream_t st = ctx->stream;
  dim3 ga(n_slices, d.n_q_heads, (m_prompt + kStatThreads - 1) / kStatThreads);
  hipLaunchKernelGGL((score_stats_generic<Tag, D>), ga, dim3(kStatThreads), 0, st, k_global, n_ctx, q_prompt,
                     m_prompt, d.n_q_heads, d.n_kv_heads, ctx->sm_scale, cache_layout(ctx), sl, partial);
  const int rows = d.n_q_heads * m_prompt;
  hipLaunchKernelGGL((score_merge_kernel<Tag, D>), dim3((rows + 63) / 64), dim3(64), 0, st, partial, n_slices,
                     q_prompt, k_prompt, m_prompt, d.n_q_heads, d.n_kv_heads, ctx->sm_scale, stats);
  float *colpart = reinterpret_cast<float *>(static_cast<char *>(ctx->scratch) + sc.colpart_off);
  hipLaunchKernelGGL((score_colsum_generic<Tag, D>),
                     dim3(static_cast<unsigned>((n_ctx + kColThreads - 1) / kColThreads), d.n_kv_heads),
                     dim3(kColThreads), 0, st, k_global, n_ctx, q_prompt, m_prompt, d.n_q_heads, d.n_kv_heads,
                     ctx->sm_scale, cache_layout(ctx), stats, colpart);
  hipLaunchKernelGGL(score_colsum_reduce, dim3(static_cast<unsigned>((n_ctx + 255) / 256)), dim3(256), 0, st, colpart,
                     d.n_kv_heads, n_ctx, 1.0f / d.n_q_heads, accumulate, scores);
  return hipGetLastError();
}

}  // namespace

ScoreScratch score_scratch_layout(const ifkv_ctx *ctx, int64_t n_ctx, int m_prompt) {
  const auto &d = ctx->desc;
  ScoreScratch s;
  const int64_t rows = static_cast<int64_t>(d.n_q_heads) * (m_prompt > 0 ? m_prompt : 1);
  const int64_t max_slices = 256;  // upper bound for both the ALU and the MFMA partition
  s.stats_off = 0;
  s.partial_off = ((rows * sizeof(float2) + 255) / 256) * 256;
  // the MFMA sweeps without a merge kernel keep them per block: at most max(256, kv heads x query
  // chunks) blocks of at most 512 rows
  const int64_t mfma_blocks = std::max<int64_t>(256, static_cast<int64_t>(d.n_kv_heads) * kMaxQChunks);
  const int64_t partial_entries = std::max<int64_t>(max_slices * rows, mfma_blocks * 512);
  s.fused_off = s.partial_off + ((partial_entries * sizeof(float2) + 255) / 256) * 256;
  s.colpart_off = s.fused_off + ((kFusedTableBytes + 255) / 256) * 256;
  // per-(kv head, query chunk) partial column sums of the MFMA pass B
  const int64_t parts = static_cast<int64_t>(d.n_kv_heads) * kMaxQChunks;
  s.total = s.colpart_off + static_cast<size_t>(parts) * static_cast<size_t>(n_ctx > 0 ? n_ctx : 1) * sizeof(float);
  return s;
}

size_t score_scratch_bytes(const ifkv_ctx *ctx, int64_t n_ctx, int m_prompt) {
  return score_scratch_layout(ctx, n_ctx, m_prompt).total;
}

hipError_t launch_score(ifkv_ctx *ctx, const void *k_global, int64_t n_ctx, const void *q_prompt, int m_prompt,
                        const void *k_prompt, int accumulate, float *scores, const FusedRepo *fused) {
  if (n_ctx <= 0) return hipSuccess;
  const auto &d = ctx->desc;
  if (m_prompt <= 0) {
    if (!accumulate)
      hipLaunchKernelGGL(fill_zero_kernel, dim3(static_cast<unsigned>((n_ctx + 255) / 256)), dim3(256), 0, ctx->stream,
                         scores, n_ctx);
    return hipGetLastError();
  }
  const bool generic = (d.flags & IFKV_FLAG_FORCE_GENERIC) || d.dtype != IFKV_BF16 || d.head_dim != 128 ||
                       !score_mfma_supported(ctx, m_prompt);
  if (!generic) {
    // MFMA sweeps around the same merge kernel (which also folds in the prompt keys)
    int n_slices = 0;
    hipError_t e = launch_score_mfma_passes(ctx, k_global, n_ctx, q_prompt, m_prompt, &n_slices, false, 0, nullptr, fused,
                                            k_prompt != nullptr);
    if (e != hipSuccess) return e;
    ScoreScratch sc = score_scratch_layout(ctx, n_ctx, m_prompt);
    float2 *partial = reinterpret_cast<float2 *>(static_cast<char *>(ctx->scratch) + sc.partial_off);
    float2 *stats = reinterpret_cast<float2 *>(static_cast<char *>(ctx->scratch) + sc.stats_off);
    const int rows = d.n_q_heads * m_prompt;
    if (k_prompt != nullptr)  // the normaliser also runs over the prompt keys: the merge kernel folds them in
      hipLaunchKernelGGL((score_merge_kernel<BF16Tag, 128>), dim3((rows + 63) / 64), dim3(64), 0, ctx->stream, partial,
                         n_slices, q_prompt, k_prompt, m_prompt, d.n_q_heads, d.n_kv_heads, ctx->sm_scale, stats);
    return launch_score_mfma_passes(ctx, k_global, n_ctx, q_prompt, m_prompt, &n_slices, true, accumulate, scores, nullptr,
                                    k_prompt != nullptr);
  }
  if (d.dtype == IFKV_BF16) {
    if (d.head_dim == 128) return run_generic<BF16Tag, 128>(ctx, k_global, n_ctx, q_prompt, m_prompt, k_prompt, accumulate, scores);
    return run_generic<BF16Tag, 64>(ctx, k_global, n_ctx, q_prompt, m_prompt, k_prompt, accumulate, scores);
  }
  if (d.head_dim == 128) return run_generic<F32Tag, 128>(ctx, k_global, n_ctx, q_prompt, m_prompt, k_prompt, accumulate, scores);
  return run_generic<F32Tag, 64>(ctx, k_global, n_ctx, q_prompt, m_prompt, k_prompt, accumulate, scores);
}

}  // namespace ifkv
