// Debug mode (IFKV_FLAG_VALIDATE): checks of the preconditions that only the device can see --
// row positions of the attention stage strictly ascending (its causal tiling relies on it), indices
// of the splice stage free of duplicates (two rows written to one place would make the result depend
// on timing).  The answer travels to the host, so these calls wait for the stream.
#include <limits.h>

#include "ifkv_internal.h"

namespace ifkv {

namespace {

__global__ void fill_words_kernel(uint32_t *p, int64_t n, uint32_t value) {
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n;
       i += static_cast<int64_t>(gridDim.x) * blockDim.x)
    p[i] = value;
}

// first_bad: smallest i with v[i] <= v[i-1]
__global__ void check_ascending_kernel(const int32_t *__restrict__ v, int64_t n, int *first_bad) {
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x + 1; i < n;
       i += static_cast<int64_t>(gridDim.x) * blockDim.x)
    if (v[i] <= v[i - 1]) atomicMin(first_bad, static_cast<int>(i));
}

// first_bad: smallest i whose row was also named by another entry (the later of the two in the
// order the hardware happened to process them, so "a" duplicate, not "the first" one);
// rows outside [0, n_kv) are skipped, as the splice skips them
__global__ void check_unique_kernel(const int32_t *__restrict__ idx, int64_t n, int64_t n_kv, uint32_t *bitmap,
                                    int *first_bad) {
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n;
       i += static_cast<int64_t>(gridDim.x) * blockDim.x) {
    const int64_t row = idx[i];
    if (row < 0 || row >= n_kv) continue;
    const uint32_t bit = 1u << (row & 31);
    if (atomicOr(&bitmap[row >> 5], bit) & bit) atomicMin(first_bad, static_cast<int>(i));
  }
}

unsigned blocks_for(int64_t n) {
  const int64_t b = (n + 255) / 256;
  return static_cast<unsigned>(b < 1 ? 1 : (b > 2048 ? 2048 : b));
}

hipError_t read_flag(ifkv_ctx *ctx, const int *d_flag, int64_t *bad_out) {
  int h = INT_MAX;
  hipError_t e = hipMemcpyAsync(&h, d_flag, sizeof(int), hipMemcpyDeviceToHost, ctx->stream);
  if (e != hipSuccess) return e;
  e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return e;
  *bad_out = h == INT_MAX ? -1 : h;
  return hipSuccess;
}

}  // namespace

// one flag word, then one bit per cache row
size_t validate_scratch_bytes(const ifkv_ctx *ctx) {
  if (!(ctx->desc.flags & IFKV_FLAG_VALIDATE)) return 0;
  return 256 + static_cast<size_t>((ctx->desc.max_ctx + 31) / 32) * sizeof(uint32_t);
}

hipError_t validate_ascending(ifkv_ctx *ctx, const int32_t *v, int64_t n, int64_t *bad_out) {
  *bad_out = -1;
  if (n < 2) return hipSuccess;
  int *flag = static_cast<int *>(ctx->scratch);
  hipLaunchKernelGGL(fill_words_kernel, dim3(1), dim3(64), 0, ctx->stream, reinterpret_cast<uint32_t *>(flag), int64_t(1),
                     static_cast<uint32_t>(INT_MAX));
  hipLaunchKernelGGL(check_ascending_kernel, dim3(blocks_for(n)), dim3(256), 0, ctx->stream, v, n, flag);
  hipError_t e = hipGetLastError();
  return e != hipSuccess ? e : read_flag(ctx, flag, bad_out);
}

hipError_t validate_unique(ifkv_ctx *ctx, const int32_t *idx, int64_t n, int64_t n_kv, int64_t *bad_out) {
  *bad_out = -1;
  if (n < 2 || n_kv < 1) return hipSuccess;
  int *flag = static_cast<int *>(ctx->scratch);
  uint32_t *bitmap = reinterpret_cast<uint32_t *>(static_cast<char *>(ctx->scratch) + 256);
  const int64_t words = (n_kv + 31) / 32;
  hipLaunchKernelGGL(fill_words_kernel, dim3(1), dim3(64), 0, ctx->stream, reinterpret_cast<uint32_t *>(flag), int64_t(1),
                     static_cast<uint32_t>(INT_MAX));
  hipLaunchKernelGGL(fill_words_kernel, dim3(blocks_for(words)), dim3(256), 0, ctx->stream, bitmap, words, 0u);
  hipLaunchKernelGGL(check_unique_kernel, dim3(blocks_for(n)), dim3(256), 0, ctx->stream, idx, n, n_kv, bitmap, flag);
  hipError_t e = hipGetLastError();
  return e != hipSuccess ? e : read_flag(ctx, flag, bad_out);
}

}  // namespace ifkv
