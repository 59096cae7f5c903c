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
//
// Vectors of more than 32768 scores do not fit one workgroup's registers; they take the
// multi-workgroup radix select further down (six short launches).
#include <mutex>

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

// THREADS x WORDS x 32 keys held in registers as bit planes.
template <int THREADS, int WORDS>
__global__ __launch_bounds__(THREADS) void topk_resident_kernel(const float *__restrict__ scores, int n, int k,
                                                                int32_t *__restrict__ idx_out) {
  constexpr int NW = THREADS / 64;
  // Thread t owns keys 32 t .. 32 t + 31 of a word.  They are loaded with coalesced 16-byte reads (all
  // of a thread's eight requests are issued before anything waits: one memory latency for the whole
  // vector), handed over through LDS (33 words per owner: conflict-free both ways) in one round with
  // one barrier, and transposed into bit planes.
  __shared__ uint32_t stage[THREADS * 33];
  __shared__ uint32_t red[2][16][2];
  __shared__ uint32_t wave_tot[16];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const bool vec_ok = (reinterpret_cast<uintptr_t>(scores) & 15u) == 0;

  uint32_t plane[WORDS][32];
#pragma unroll
  for (int w = 0; w < WORDS; ++w) {
    const int base = w * THREADS * 32;
    float4 f[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int gi = base + (i * THREADS + tid) * 4;
      f[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (vec_ok && gi + 3 < n) {
        f[i] = *reinterpret_cast<const float4 *>(scores + gi);
      } else {
        if (gi < n) f[i].x = scores[gi];
        if (gi + 1 < n) f[i].y = scores[gi + 1];
        if (gi + 2 < n) f[i].z = scores[gi + 2];
        if (gi + 3 < n) f[i].w = scores[gi + 3];
      }
    }
    if (w > 0) __syncthreads();  // the previous word's keys have been taken out of the stage
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int e = (i * THREADS + tid) * 4;
      const int gi = base + e;
      uint32_t *dst = stage + e + (e >> 5);
      // key 0 pads the tail: every real score maps to a key > 0
      dst[0] = gi < n ? score_key(f[i].x) : 0u;
      dst[1] = gi + 1 < n ? score_key(f[i].y) : 0u;
      dst[2] = gi + 2 < n ? score_key(f[i].z) : 0u;
      dst[3] = gi + 3 < n ? score_key(f[i].w) : 0u;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 32; ++i) plane[w][i] = stage[tid * 33 + i];
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
// Score vectors beyond the register-resident capacity: radix select over many workgroups.
// The key's 32 bits are resolved in three digits (11 + 11 + 10 bits).  Pass p counts, per digit
// value, the keys that match the prefix found so far (LDS histogram per workgroup, then one global
// atomic add per non-empty bin: integer counts, so the result does not depend on the order); the
// next kernel starts by locating the digit that holds the k-th largest key in that histogram (every
// workgroup redoes this small scan, which saves a launch per pass).  After the third digit the
// threshold key T is exact; the last two kernels count (greater, tie) elements per workgroup and
// write the indices in ascending order, taking ties by ascending index.
// Near-uniform attention puts most keys into one bin of the first digit; the cost is LDS atomics on
// one address (a few hundred cycles per workgroup), not correctness.
// ---------------------------------------------------------------------------
constexpr int kSelThreads = 256;
constexpr int kSelPer = 16;                       // keys per thread
constexpr int kSelChunk = kSelThreads * kSelPer;  // keys per workgroup
constexpr int kSelBins = 2048;

struct SelectState {  // lives in scratch
  uint32_t hist[3][kSelBins];
};
__device__ __forceinline__ int digit_shift(int pass) { return pass == 0 ? 21 : (pass == 1 ? 10 : 0); }
__device__ __forceinline__ uint32_t digit_mask(int pass) { return pass == 2 ? 0x3FFu : 0x7FFu; }

// Locates, in the histogram of pass `pass`, the digit that holds the need-th largest key among
// the keys matching `prefix`; returns it and lowers `need` by the keys in higher digits.
// Called by every thread of a 256-thread workgroup with the same arguments; `red` holds 257 ints.
__device__ __forceinline__ uint32_t locate_digit(const uint32_t *__restrict__ hist, int pass, int &need, int *red) {
  const int nb = pass == 2 ? 1024 : kSelBins;
  const int per = nb / kSelThreads;  // consecutive bins per thread (8 or 4)
  const int tid = threadIdx.x;
  // thread t owns bins [nb - (t+1)*per, nb - t*per): thread 0 the highest digits
  int mine = 0;
  for (int e = 0; e < per; ++e) mine += static_cast<int>(hist[nb - 1 - (tid * per + e)]);
  red[tid] = mine;
  __syncthreads();
  if (tid == 0) {  // 256-entry exclusive scan: short, and only here
    int acc = 0;
    for (int t = 0; t < kSelThreads; ++t) {
      const int v = red[t];
      red[t] = acc;
      acc += v;
    }
    red[kSelThreads] = acc;
  }
  __syncthreads();
  const int before = red[tid];  // keys in digits above this thread's bins
  __syncthreads();
  if (before < need && need <= before + mine) {  // exactly one thread
    int acc = before;
    for (int e = 0; e < per; ++e) {
      const int bin = nb - 1 - (tid * per + e);
      const int c = static_cast<int>(hist[bin]);
      if (need <= acc + c) {
        red[0] = bin;
        red[1] = need - acc;
        break;
      }
      acc += c;
    }
  }
  __syncthreads();
  const uint32_t digit = static_cast<uint32_t>(red[0]);
  need = red[1];
  __syncthreads();
  return digit;
}

// Replays the digits found so far: prefix of the threshold key and the remaining rank.
__device__ __forceinline__ uint32_t replay_prefix(const SelectState *st, int passes_done, int k, int &need, int *red) {
  uint32_t prefix = 0;
  need = k;
  for (int p = 0; p < passes_done; ++p) prefix |= locate_digit(st->hist[p], p, need, red) << digit_shift(p);
  return prefix;
}

__global__ __launch_bounds__(kSelThreads) void select_hist_kernel(const float *__restrict__ scores, int n, int k,
                                                                  int pass, SelectState *__restrict__ st) {
  __shared__ uint32_t lh[kSelBins];
  __shared__ int red[kSelThreads + 1];
  for (int b = threadIdx.x; b < kSelBins; b += kSelThreads) lh[b] = 0u;
  __syncthreads();
  int need;
  const uint32_t prefix = replay_prefix(st, pass, k, need, red);
  const uint32_t hi_mask = pass == 0 ? 0u : (pass == 1 ? 0xFFE00000u : 0xFFFFFC00u);
  const int sh = digit_shift(pass);
  const uint32_t dm = digit_mask(pass);
  const int base = blockIdx.x * kSelChunk;
#pragma unroll 4
  for (int e = 0; e < kSelPer; ++e) {
    const int i = base + e * kSelThreads + threadIdx.x;
    if (i < n) {
      const uint32_t key = score_key(scores[i]);
      if ((key & hi_mask) == prefix) atomicAdd(&lh[(key >> sh) & dm], 1u);
    }
  }
  __syncthreads();
  for (int b = threadIdx.x; b < kSelBins; b += kSelThreads)
    if (lh[b] != 0u) atomicAdd(&st->hist[pass][b], lh[b]);
}

// Per workgroup: how many keys are above the threshold and how many equal it.
__global__ __launch_bounds__(kSelThreads) void select_count_kernel(const float *__restrict__ scores, int n, int k,
                                                                   const SelectState *__restrict__ st,
                                                                   uint2 *__restrict__ block_counts) {
  __shared__ int red[kSelThreads + 1];
  __shared__ uint32_t wsum[2][kSelThreads / 64];
  int need;
  const uint32_t T = replay_prefix(st, 3, k, need, red);
  const int base = blockIdx.x * kSelChunk + threadIdx.x * kSelPer;
  int g = 0, t = 0;
#pragma unroll 4
  for (int e = 0; e < kSelPer; ++e)
    if (base + e < n) {
      const uint32_t key = score_key(scores[base + e]);
      g += key > T;
      t += key == T;
    }
  g = wave64_sum(g);
  t = wave64_sum(t);
  if ((threadIdx.x & 63) == 0) {
    wsum[0][threadIdx.x >> 6] = g;
    wsum[1][threadIdx.x >> 6] = t;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t gs = 0, ts = 0;
    for (int w = 0; w < kSelThreads / 64; ++w) {
      gs += wsum[0][w];
      ts += wsum[1][w];
    }
    block_counts[blockIdx.x] = make_uint2(gs, ts);
  }
}

// Ordered output.  Thread t of workgroup b owns keys [b*chunk + t*16, +16): a contiguous run, so
// ascending index order is (workgroup, thread, element).
__global__ __launch_bounds__(kSelThreads) void select_write_kernel(const float *__restrict__ scores, int n, int k,
                                                                   const SelectState *__restrict__ st,
                                                                   const uint2 *__restrict__ block_counts,
                                                                   int32_t *__restrict__ idx_out) {
  __shared__ int red[kSelThreads + 1];
  __shared__ uint32_t wave_tot[kSelThreads / 64];
  int need;
  const uint32_t T = replay_prefix(st, 3, k, need, red);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // elements taken by the workgroups before this one
  uint32_t g_before = 0, t_before = 0;
  for (int b = tid; b < static_cast<int>(blockIdx.x); b += kSelThreads) {
    const uint2 c = block_counts[b];
    g_before += c.x;
    t_before += c.y;
  }
  g_before = static_cast<uint32_t>(wave64_sum(static_cast<int>(g_before)));
  t_before = static_cast<uint32_t>(wave64_sum(static_cast<int>(t_before)));
  __shared__ uint32_t pre[2][kSelThreads / 64];
  if (lane == 0) {
    pre[0][wave] = g_before;
    pre[1][wave] = t_before;
  }
  __syncthreads();
  g_before = 0;
  t_before = 0;
  for (int w = 0; w < kSelThreads / 64; ++w) {
    g_before += pre[0][w];
    t_before += pre[1][w];
  }
  const int base = blockIdx.x * kSelChunk + tid * kSelPer;
  uint32_t gm = 0, tm = 0;
#pragma unroll 4
  for (int e = 0; e < kSelPer; ++e)
    if (base + e < n) {
      const uint32_t key = score_key(scores[base + e]);
      gm |= (key > T ? 1u : 0u) << e;
      tm |= (key == T ? 1u : 0u) << e;
    }
  // (greater, tie) counts packed in one word: a workgroup holds 4096 keys, so 16 bits each suffice
  const uint32_t v = static_cast<uint32_t>(__popc(gm)) | (static_cast<uint32_t>(__popc(tm)) << 16);
  uint32_t incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t up = __shfl_up(incl, o, 64);
    if (lane >= o) incl += up;
  }
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  uint32_t wave_before = 0;
  for (int x = 0; x < wave; ++x) wave_before += wave_tot[x];
  const uint32_t excl = wave_before + incl - v;
  int t_seen = static_cast<int>(t_before + (excl >> 16));
  int pos = static_cast<int>(g_before + (excl & 0xFFFFu)) + min(t_seen, need);
  uint32_t m = gm | tm;
  while (m) {
    const int i = __ffs(m) - 1;
    m &= m - 1;
    bool take = (gm >> i) & 1u;
    if (!take) take = (t_seen++ < need);
    if (take) {
      if (pos < k) idx_out[pos] = base + i;  // pos < k always holds; the guard keeps a logic slip in bounds
      ++pos;
    }
  }
}

__global__ void select_zero_kernel(SelectState *st) {
  uint32_t *p = &st->hist[0][0];
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < 3 * kSelBins; i += gridDim.x * blockDim.x) p[i] = 0u;
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

namespace {

constexpr size_t kSelStateBytes = (sizeof(SelectState) + 255) & ~static_cast<size_t>(255);

// Device memory of the entry point that allocates nothing: the histograms and the per-workgroup
// counts of the largest score vector it accepts.  Every GPU the library runs on holds its own copy
// of the array at its own address; in host code the array's name is only a handle for looking that
// address up, never a pointer to pass on.
constexpr int64_t kStaticMaxCtx = int64_t(1) << 22;
constexpr size_t kStaticScratchBytes = kSelStateBytes + static_cast<size_t>(kStaticMaxCtx / kSelChunk) * sizeof(uint2);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
void *g_static_ptr[kMaxDevices] = {};

}  // namespace

int64_t topk_static_max_ctx() { return kStaticMaxCtx; }

// Address of the static scratch on the device that is current; looked up once per device.
hipError_t topk_static_scratch(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (g_static_ptr[dev] == nullptr) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    g_static_ptr[dev] = p;
  }
  *out = g_static_ptr[dev];
  return hipSuccess;
}

size_t topk_scratch_bytes(const ifkv_ctx *, int64_t n_ctx) {
  if (n_ctx <= 1024 * 32) return 0;
  const size_t blocks = static_cast<size_t>((n_ctx + kSelChunk - 1) / kSelChunk);
  return kSelStateBytes + blocks * sizeof(uint2);
}

// `work`: device memory of at least topk_scratch_bytes(n_ctx) bytes (may be null when that is 0)
hipError_t launch_topk(ifkv_ctx *ctx, const float *scores, int64_t n_ctx, int64_t k, int32_t *idx_out, void *work) {
  if (k <= 0 || n_ctx <= 0) return hipSuccess;
  const int n = static_cast<int>(n_ctx);
  const int kk = static_cast<int>(k);
  hipStream_t st = ctx->stream;
  if (n <= 256 * 32) {
    hipLaunchKernelGGL((topk_resident_kernel<256, 1>), dim3(1), dim3(256), 0, st, scores, n, kk, idx_out);
  } else if (n <= 1024 * 32) {
    hipLaunchKernelGGL((topk_resident_kernel<1024, 1>), dim3(1), dim3(1024), 0, st, scores, n, kk, idx_out);
  } else {
    if (work == nullptr) return hipErrorInvalidValue;
    SelectState *state = static_cast<SelectState *>(work);
    uint2 *counts = reinterpret_cast<uint2 *>(static_cast<char *>(work) + kSelStateBytes);
    const unsigned blocks = static_cast<unsigned>((n + kSelChunk - 1) / kSelChunk);
    hipLaunchKernelGGL(select_zero_kernel, dim3(6), dim3(1024), 0, st, state);
    for (int pass = 0; pass < 3; ++pass)
      hipLaunchKernelGGL(select_hist_kernel, dim3(blocks), dim3(kSelThreads), 0, st, scores, n, kk, pass, state);
    hipLaunchKernelGGL(select_count_kernel, dim3(blocks), dim3(kSelThreads), 0, st, scores, n, kk, state, counts);
    hipLaunchKernelGGL(select_write_kernel, dim3(blocks), dim3(kSelThreads), 0, st, scores, n, kk, state, counts,
                       idx_out);
  }
  return hipGetLastError();
}

}  // namespace ifkv
