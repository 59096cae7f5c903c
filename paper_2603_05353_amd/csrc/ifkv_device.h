// Device-side helpers: storage dtype packing and small wavefront utilities.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ifkv {

typedef uint32_t v4u __attribute__((ext_vector_type(4)));  // one 16-byte access

struct F32Tag {};
struct BF16Tag {};

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// Round-to-nearest-even float -> bfloat16 bit pattern (inputs are finite).
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

template <typename Tag>
struct Elem;

template <>
struct Elem<F32Tag> {
  static constexpr int kBytes = 4;
  static constexpr int kVec = 4;  // elements per 16-byte vector
  static __device__ __forceinline__ void unpack(const v4u &v, float *f) {
    f[0] = __uint_as_float(v.x);
    f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z);
    f[3] = __uint_as_float(v.w);
  }
  static __device__ __forceinline__ v4u pack(const float *f) {
    v4u v;
    v.x = __float_as_uint(f[0]);
    v.y = __float_as_uint(f[1]);
    v.z = __float_as_uint(f[2]);
    v.w = __float_as_uint(f[3]);
    return v;
  }
  static __device__ __forceinline__ float load1(const void *p, int64_t i) {
    return reinterpret_cast<const float *>(p)[i];
  }
  static __device__ __forceinline__ void store1(void *p, int64_t i, float v) {
    reinterpret_cast<float *>(p)[i] = v;
  }
};

template <>
struct Elem<BF16Tag> {
  static constexpr int kBytes = 2;
  static constexpr int kVec = 8;
  static __device__ __forceinline__ void unpack(const v4u &v, float *f) {
    f[0] = __uint_as_float(v.x << 16);
    f[1] = __uint_as_float(v.x & 0xFFFF0000u);
    f[2] = __uint_as_float(v.y << 16);
    f[3] = __uint_as_float(v.y & 0xFFFF0000u);
    f[4] = __uint_as_float(v.z << 16);
    f[5] = __uint_as_float(v.z & 0xFFFF0000u);
    f[6] = __uint_as_float(v.w << 16);
    f[7] = __uint_as_float(v.w & 0xFFFF0000u);
  }
  static __device__ __forceinline__ v4u pack(const float *f) {
    v4u v;
    v.x = float_to_bf16_bits(f[0]) | (float_to_bf16_bits(f[1]) << 16);
    v.y = float_to_bf16_bits(f[2]) | (float_to_bf16_bits(f[3]) << 16);
    v.z = float_to_bf16_bits(f[4]) | (float_to_bf16_bits(f[5]) << 16);
    v.w = float_to_bf16_bits(f[6]) | (float_to_bf16_bits(f[7]) << 16);
    return v;
  }
  static __device__ __forceinline__ float load1(const void *p, int64_t i) {
    return bf16_bits_to_float(reinterpret_cast<const uint16_t *>(p)[i]);
  }
  static __device__ __forceinline__ void store1(void *p, int64_t i, float v) {
    reinterpret_cast<uint16_t *>(p)[i] = static_cast<uint16_t>(float_to_bf16_bits(v));
  }
};

// Butterfly reductions over the 64 lanes of a wavefront.
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

}  // namespace ifkv
