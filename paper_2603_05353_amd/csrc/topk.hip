// Stage 3 -- Eq. (8): the k context tokens with the largest scores, k = floor(rho N).
//
// The score vector is small (128 KiB at 32K context), so the stage is bound by
// launch latency and dependent steps, not by bandwidth.  It therefore runs as
// ONE workgroup in ONE launch: the scores are turned into order-preserving
// 32-bit keys, bit-transposed into per-thread bit planes held in registers,
// and the k-th largest key is found by a radix descent of two bits per step
// whose counting is a handful of AND + popcount operations per thread.  There
// are no atomics, so the cost does not depend on how the scores are
// distributed (near-uniform attention puts almost every score into the same
// high-order digits, the worst case for histogram-based selection).
//
// Ties are resolved towards the smaller index and the result is emitted in
// ascending index order by a block-wide prefix sum over (greater, tie) counts.
#include "ifkv_device.h"
#include "ifkv_internal.h"

namespace ifkv {

namespace {

// Monotone map float -> uint32: larger float <=> larger key; -0 and +0 coincide.
// Every real (non-NaN) score maps to a key > 0, so key 0 can pad the tail.
__device__ __forceinline__ uint32_t score_key(float f) {
  uint32_t u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Sum within each row of 16 lanes (data-parallel primitives; every lane of a
// row ends up with the row total).
__device__ __forceinline__ int row16_sum(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
  v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true);   // quad_perm [2,3,0,1]
  v += __builtin_amdgcn_update_dpp(0, v, 0x124, 0xF, 0xF, true);  // row_ror:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x128, 0xF, 0xF, true);  // row_ror:8
  return v;
}
__device__ __forceinline__ int wave64_sum(int v) {
  v = row16_sum(v);
  return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) +
         __builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48);
}

// In-register 32x32 bit-matrix transpose: afterwards word b, bit i == bit b of
// the original word i.
__device__ __forceinline__ void transpose32(uint32_t (&a)[32]) {
  uint32_t m = 0x0000FFFFu;
#pragma unroll
  for (int j = 16; j != 0; j >>= 1) {
#pragma unroll
    for (int k = 0; k < 32; k = (k + j + 1) & ~j) {
      const uint32_t t = ((a[k] >> j) ^ a[k + j]) & m;
      a[k] ^= t << j;
      a[k + j] ^= t;
    }
    m ^= m << (j >> 1);
  }
}

constexpr int kStageThreads = 256;                 // threads served per staging round
constexpr int kStageElems = kStageThreads * 32;    // 8192 scores per staging round

// THREADS x WORDS x 32 keys held in registers as bit planes.
template <int THREADS, int WORDS>
__global__ __launch_bounds__(THREADS) void topk_resident_kernel(const float *__restrict__ scores, int n, int k,
                                                                int32_t *__restrict__ idx_out) {
  constexpr int NW = THREADS / 64;
  constexpr int SUB = THREADS / kStageThreads;
  constexpr int PER = kStageElems / THREADS;  // scores loaded per thread per staging round
  __shared__ uint32_t stage[kStageThreads * 33];  // 32 keys per owner thread, padded to 33 words
  __shared__ uint32_t red[2][16][2];
  __shared__ uint32_t wave_tot[16];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const bool vec_ok = (reinterpret_cast<uintptr_t>(scores) & 15u) == 0;

  uint32_t plane[WORDS][32];
#pragma unroll
  for (int w = 0; w < WORDS; ++w) {
#pragma unroll
    for (int q = 0; q < SUB; ++q) {
      const int base = (w * THREADS + q * kStageThreads) * 32;
#pragma unroll
      for (int i = 0; i < PER / 4; ++i) {
        const int e = (i * THREADS + tid) * 4;
        const int gi = base + e;
        uint32_t k0 = 0, k1 = 0, k2 = 0, k3 = 0;
        if (vec_ok && gi + 3 < n) {
          const float4 f = *reinterpret_cast<const float4 *>(scores + gi);
          k0 = score_key(f.x);
          k1 = score_key(f.y);
          k2 = score_key(f.z);
          k3 = score_key(f.w);
        } else {
          if (gi < n) k0 = score_key(scores[gi]);
          if (gi + 1 < n) k1 = score_key(scores[gi + 1]);
          if (gi + 2 < n) k2 = score_key(scores[gi + 2]);
          if (gi + 3 < n) k3 = score_key(scores[gi + 3]);
        }
        uint32_t *dst = stage + e + (e >> 5);
        dst[0] = k0;
        dst[1] = k1;
        dst[2] = k2;
        dst[3] = k3;
      }
      __syncthreads();
      if ((tid / kStageThreads) == q) {
        const int t = tid % kStageThreads;
#pragma unroll
        for (int i = 0; i < 32; ++i) plane[w][i] = stage[t * 33 + i];
      }
      __syncthreads();
    }
    transpose32(plane[w]);
  }

  // ---- radix descent, two bits per step ------------------------------------
  uint32_t alive[WORDS], greater[WORDS];
#pragma unroll
  for (int w = 0; w < WORDS; ++w) {
    alive[w] = 0xFFFFFFFFu;
    greater[w] = 0u;
  }
  int need = k;
#pragma unroll
  for (int step = 0; step < 16; ++step) {
    const int hi = 31 - 2 * step;
    const int lo = hi - 1;
    int c3 = 0, c2 = 0, c1 = 0;
#pragma unroll
    for (int w = 0; w < WORDS; ++w) {
      const uint32_t ah = alive[w] & plane[w][hi];
      const uint32_t pl = plane[w][lo];
      c3 += __popc(ah & pl);
      c2 += __popc(ah & ~pl);
      c1 += __popc(alive[w] & ~plane[w][hi] & pl);
    }
    // per-thread counts <= 32*WORDS, per-wave totals < 2^16: c3 and c2 share a word
    const int w32 = wave64_sum(c3 | (c2 << 16));
    const int w1 = wave64_sum(c1);
    const int p = step & 1;
    if (lane == 0) {
      red[p][wave][0] = static_cast<uint32_t>(w32);
      red[p][wave][1] = static_cast<uint32_t>(w1);
    }
    __syncthreads();
    int t3 = 0, t2 = 0, t1 = 0;
    if (lane < NW) {
      const uint32_t a = red[p][lane][0];
      t3 = static_cast<int>(a & 0xFFFFu);
      t2 = static_cast<int>(a >> 16);
      t1 = static_cast<int>(red[p][lane][1]);
    }
    t3 = __builtin_amdgcn_readlane(row16_sum(t3), 0);
    t2 = __builtin_amdgcn_readlane(row16_sum(t2), 0);
    t1 = __builtin_amdgcn_readlane(row16_sum(t1), 0);

    int digit;
    if (need <= t3) {
      digit = 3;
    } else if (need <= t3 + t2) {
      digit = 2;
      need -= t3;
    } else if (need <= t3 + t2 + t1) {
      digit = 1;
      need -= t3 + t2;
    } else {
      digit = 0;
      need -= t3 + t2 + t1;
    }
#pragma unroll
    for (int w = 0; w < WORDS; ++w) {
      const uint32_t ph = plane[w][hi], pl = plane[w][lo], a = alive[w];
      if (digit == 3) {
        alive[w] = a & ph & pl;
      } else if (digit == 2) {
        greater[w] |= a & ph & pl;
        alive[w] = a & ph & ~pl;
      } else if (digit == 1) {
        greater[w] |= a & ph;
        alive[w] = a & ~ph & pl;
      } else {
        greater[w] |= a & (ph | pl);
        alive[w] = a & ~ph & ~pl;
      }
    }
  }
  // alive = keys equal to the k-th largest; `need` of them (lowest indices) are taken.

  // ---- ordered compaction ----------------------------------------------------
  int carry_g = 0, carry_t = 0;
#pragma unroll
  for (int w = 0; w < WORDS; ++w) {
    const int g = __popc(greater[w]);
    const int t = __popc(alive[w]);
    // greater count in the low half, tie count in the high half; block totals
    // are <= 32768 each, so unsigned sums never carry between the halves
    const uint32_t v = static_cast<uint32_t>(g) | (static_cast<uint32_t>(t) << 16);
    uint32_t incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t up = __shfl_up(incl, o, 64);
      if (lane >= o) incl += up;
    }
    __syncthreads();  // wave_tot reuse
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t wave_before = 0, block_total = 0;
#pragma unroll
    for (int x = 0; x < NW; ++x) {
      const uint32_t wt = wave_tot[x];
      if (x < wave) wave_before += wt;
      block_total += wt;
    }
    const uint32_t excl = wave_before + incl - v;
    const int g_before = carry_g + static_cast<int>(excl & 0xFFFFu);
    int t_seen = carry_t + static_cast<int>(excl >> 16);
    int pos = g_before + min(t_seen, need);
    const int base_index = (w * THREADS + tid) * 32;
    const uint32_t gm = greater[w];
    uint32_t m = gm | alive[w];
    while (m) {
      const int i = __ffs(m) - 1;
      m &= m - 1;
      bool take = (gm >> i) & 1u;
      if (!take) take = (t_seen++ < need);
      if (take) {
        if (pos < k) idx_out[pos] = base_index + i;  // pos < k always holds; the guard keeps a logic slip in bounds
        ++pos;
      }
    }
    carry_g += static_cast<int>(block_total & 0xFFFFu);
    carry_t += static_cast<int>(block_total >> 16);
  }
}

// ---------------------------------------------------------------------------
// Fallback for score vectors beyond the register-resident capacity: the same
// selection by bitwise descent, re-reading the scores from L2/HBM at every
// step.  Correct for any n < 2^31, linear in n per step.
// ---------------------------------------------------------------------------
constexpr int kStreamThreads = 1024;

template <bool STRICT>
__device__ __forceinline__ int block_count_above(const float *__restrict__ scores, int n, uint32_t cand,
                                                 uint32_t *red, int slot) {
  int c = 0;
  for (int i = threadIdx.x; i < n; i += kStreamThreads) {
    const uint32_t key = score_key(scores[i]);
    c += STRICT ? (key > cand) : (key >= cand);
  }
  c = wave64_sum(c);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (lane == 0) red[slot * 16 + wave] = static_cast<uint32_t>(c);
  __syncthreads();
  int t = (lane < kStreamThreads / 64) ? static_cast<int>(red[slot * 16 + lane]) : 0;
  return __builtin_amdgcn_readlane(row16_sum(t), 0);
}

__global__ __launch_bounds__(kStreamThreads) void topk_streaming_kernel(const float *__restrict__ scores, int n,
                                                                        int k, int32_t *__restrict__ idx_out) {
  __shared__ uint32_t red[2 * 16];
  __shared__ uint32_t wave_tot[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  uint32_t T = 0;
  for (int b = 31; b >= 0; --b) {
    const uint32_t cand = T | (1u << b);
    const int cnt = block_count_above<false>(scores, n, cand, red, b & 1);
    if (cnt >= k) T = cand;
  }
  const int n_greater = block_count_above<true>(scores, n, T, red, 1);  // slot 0 may still be read
  const int need = k - n_greater;

  constexpr int PER = 8;
  int carry_g = 0, carry_t = 0;
  for (int base = 0; base < n; base += kStreamThreads * PER) {
    const int i0 = base + tid * PER;
    uint32_t gm = 0, tm = 0;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      if (i0 + e < n) {
        const uint32_t key = score_key(scores[i0 + e]);
        gm |= (key > T ? 1u : 0u) << e;
        tm |= (key == T ? 1u : 0u) << e;
      }
    }
    const uint32_t v = static_cast<uint32_t>(__popc(gm)) | (static_cast<uint32_t>(__popc(tm)) << 16);
    uint32_t incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t up = __shfl_up(incl, o, 64);
      if (lane >= o) incl += up;
    }
    __syncthreads();
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t wave_before = 0, block_total = 0;
#pragma unroll
    for (int x = 0; x < kStreamThreads / 64; ++x) {
      const uint32_t wt = wave_tot[x];
      if (x < wave) wave_before += wt;
      block_total += wt;
    }
    const uint32_t excl = wave_before + incl - v;
    int t_seen = carry_t + static_cast<int>(excl >> 16);
    int pos = carry_g + static_cast<int>(excl & 0xFFFFu) + min(t_seen, need);
    uint32_t m = gm | tm;
    while (m) {
      const int i = __ffs(m) - 1;
      m &= m - 1;
      bool take = (gm >> i) & 1u;
      if (!take) take = (t_seen++ < need);
      if (take) {
        if (pos < k) idx_out[pos] = i0 + i;
        ++pos;
      }
    }
    carry_g += static_cast<int>(block_total & 0xFFFFu);
    carry_t += static_cast<int>(block_total >> 16);
  }
}

// "Chunk Reordering", Eq. (9), numerator: idx is ascending, so the rows of slot s are the
// index range [lower_bound(bound[s]), lower_bound(bound[s+1])).  One thread per boundary.
__global__ __launch_bounds__(128) void chunk_counts_kernel(const int32_t *__restrict__ idx, int k, SlotBounds b,
                                                           int32_t *__restrict__ counts_out) {
  __shared__ int pos[kRepoMaxChunks + 1];
  const int t = threadIdx.x;
  if (t <= b.n) {
    const int target = b.bound[t];
    int lo = 0, hi = k;  // first position whose index is >= target
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (idx[mid] < target)
        lo = mid + 1;
      else
        hi = mid;
    }
    pos[t] = lo;
  }
  __syncthreads();
  if (t < b.n) counts_out[t] = pos[t + 1] - pos[t];
}

}  // namespace

hipError_t launch_chunk_counts(ifkv_ctx *ctx, const int32_t *idx, int64_t k, const SlotBounds &b,
                               int32_t *counts_out) {
  if (b.n <= 0) return hipSuccess;
  hipLaunchKernelGGL(chunk_counts_kernel, dim3(1), dim3(128), 0, ctx->stream, idx, static_cast<int>(k), b, counts_out);
  return hipGetLastError();
}

size_t topk_scratch_bytes(const ifkv_ctx *, int64_t) { return 0; }

hipError_t launch_topk(ifkv_ctx *ctx, const float *scores, int64_t n_ctx, int64_t k, int32_t *idx_out) {
  if (k <= 0 || n_ctx <= 0) return hipSuccess;
  const int n = static_cast<int>(n_ctx);
  const int kk = static_cast<int>(k);
  hipStream_t st = ctx->stream;
  if (n <= 256 * 32) {
    hipLaunchKernelGGL((topk_resident_kernel<256, 1>), dim3(1), dim3(256), 0, st, scores, n, kk, idx_out);
  } else if (n <= 1024 * 32) {
    hipLaunchKernelGGL((topk_resident_kernel<1024, 1>), dim3(1), dim3(1024), 0, st, scores, n, kk, idx_out);
  } else {
    hipLaunchKernelGGL(topk_streaming_kernel, dim3(1), dim3(kStreamThreads), 0, st, scores, n, kk, idx_out);
  }
  return hipGetLastError();
}

}  // namespace ifkv
