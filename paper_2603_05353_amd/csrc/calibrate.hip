// Calibration kernel: a loop of independent 32x32x16 bf16 MFMAs with register-resident operands.
// Nothing of the method runs here.  The benchmark times it to state, next to the published
// matrix peak, what the machine sustains (a) with constant operands, where the shader clock
// holds, and (b) with operands that switch like real activations (random sign and mantissa,
// exponent near 1), where the board power limit lowers the clock.
#include "ifkv_internal.h"

namespace ifkv {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

constexpr int kProbeBlocks = 256 * 2;   // two workgroups of 4 waves per compute unit: 2 waves per SIMD
constexpr int kProbeThreads = 256;
constexpr int kMfmaPerIter = 32;        // 8 operand pairs x 4 accumulators

__device__ __forceinline__ v4u operand_bits(uint32_t seed, int pattern) {
  if (pattern == 0) return v4u{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};  // 1.0 everywhere
  const uint32_t h = seed * 2654435761u;
  v4u r{h, h * 31u, h * 17u, h * 5u};
  // keep sign and mantissa bits, force the exponent field to 0x7e or 0x7f: magnitudes in [0.5, 2)
  for (int i = 0; i < 4; ++i) r[i] = (r[i] & 0x807F807Fu) | 0x3F003F00u | ((r[i] >> 3) & 0x00800080u);
  return r;
}

__global__ __launch_bounds__(kProbeThreads) void mfma_probe_kernel(int iters, int pattern, float *__restrict__ sink) {
  const int lane = threadIdx.x & 63;
  v4u a[8], b[8];
  for (int i = 0; i < 8; ++i) {
    a[i] = operand_bits(lane * 97 + i * 13 + 1, pattern);
    b[i] = operand_bits(lane * 31 + i * 7 + 5, pattern);
  }
  f32x16 acc[4];
  for (int c = 0; c < 4; ++c)
    for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int c = 0; c < 4; ++c)
        acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]),
                                                         __builtin_bit_cast(bf16x8, b[(i + c) & 7]), acc[c], 0, 0, 0);
  }
  float r = 0.f;
  for (int c = 0; c < 4; ++c)
    for (int q = 0; q < 16; ++q) r += acc[c][q];
  sink[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = r;
}

}  // namespace

size_t mfma_probe_sink_floats() { return (size_t)kProbeBlocks * kProbeThreads; }

double mfma_probe_flops(int iters) {
  // each wave issues kMfmaPerIter MFMAs of 2*32*32*16 flop per iteration
  return (double)kProbeBlocks * (kProbeThreads / 64) * (double)iters * kMfmaPerIter * 32768.0;
}

hipError_t launch_mfma_probe(ifkv_ctx *ctx, int pattern, int iters, float *sink) {
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(kProbeBlocks), dim3(kProbeThreads), 0, ctx->stream, iters, pattern, sink);
  return hipGetLastError();
}

}  // namespace ifkv
