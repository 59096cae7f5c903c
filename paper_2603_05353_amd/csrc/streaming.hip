// Streaming stages: key re-rotation + cache assembly (stage 1), row splice
// (stage 5) and the calibration copy.  All three are HBM-bound: every element
// is read once and written once with 16-byte accesses, and each wavefront keeps
// several independent loads in flight.
#include "ifkv_device.h"
#include "ifkv_internal.h"


namespace ifkv {

namespace {

constexpr int kThreads = 256;
constexpr int kBatch = 4;      // independent 16-byte loads in flight per thread and stream
// Stage 1 tile shape; the two macros exist so that a build can sweep them (-DIFKV_REPO_ROWS=..).
#ifndef IFKV_REPO_ROWS
#define IFKV_REPO_ROWS 8
#endif
#ifndef IFKV_REPO_BATCH
#define IFKV_REPO_BATCH 4
#endif
constexpr int kRepoRows = IFKV_REPO_ROWS;    // stage 1: rows per tile (16 KiB of keys and of values at 8 x 128 bf16)
constexpr int kRepoBatch = IFKV_REPO_BATCH;  // stage 1: work items per thread and batch, four 16-byte loads each

// ---------------------------------------------------------------------------
// Stage 1.  Method, Eq. (5): global position = chunk start + local index; a
// key cached at its local position reaches its global rotary phase when every
// 2-D pair j is turned by advance * theta_j (Eq. 3-4; rotations add).
// The advance is per chunk, so a block needs d/2 (cos, sin) values only; they
// are formed in fp64 by the first d/2 threads and shared through LDS.
//
// A block owns kRepoRows rows of one chunk.  It requests its key vectors and
// the matching value vectors before anything else, forms the (cos, sin) table
// while those loads are in flight, and then rotates and stores.
// ---------------------------------------------------------------------------

// Row copy of `total` 16-byte vectors, kBatch loads in flight per thread.
__device__ __forceinline__ void copy_vectors(const v4u *__restrict__ src, v4u *__restrict__ dst, int total,
                                             int tid) {
  for (int base = tid; base < total; base += kThreads * kBatch) {
    v4u x[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int it = base + u * kThreads;
      if (it < total) x[u] = __builtin_nontemporal_load(src + it);
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int it = base + u * kThreads;
      if (it < total) __builtin_nontemporal_store(x[u], dst + it);
    }
  }
}

// The chunk caches are packed; the concatenated caches may be strided (PACKED false): then the
// destination of a 16-byte vector follows from its (row, head, vector within the head).
template <typename Tag, int PAIRING, int RB, bool PACKED>
__global__ __launch_bounds__(kThreads) void reposition_kernel(RepoBatch b, const double *__restrict__ inv_freq,
                                                              int rows_per_tile, int n_kv_heads, int head_dim,
                                                              CacheLayout lay, v4u *__restrict__ k_out,
                                                              v4u *__restrict__ v_out) {
  using E = Elem<Tag>;
  constexpr int VE = E::kVec;
  __shared__ float s_cos[kMaxHeadDim / 2];
  __shared__ float s_sin[kMaxHeadDim / 2];

  // Chunk of this tile: first-tile indices ascend, so the chunk is the number of entries not above
  // the tile index, minus one.  One lane per entry, one ballot.
  const int tile = blockIdx.x;
  const int lane = threadIdx.x & 63;
  const int first = lane < b.n ? b.c[lane].tile0 : 0x7fffffff;
  const int ci = __builtin_amdgcn_readfirstlane(__popcll(__ballot(tile >= first)) - 1);
  const RepoChunk c = b.c[ci];
  const int row0 = (tile - c.tile0) * rows_per_tile;
  const int nrows = min(rows_per_tile, c.len - row0);
  if (nrows <= 0) return;

  const int tid = threadIdx.x;
  const int half = head_dim / 2;
  const int row_vecs = n_kv_heads * head_dim / VE;  // 16-byte vectors per row
  const int total_vecs = nrows * row_vecs;          // rows are contiguous: the tile is one flat range
  const v4u *k_src = reinterpret_cast<const v4u *>(c.k) + static_cast<int64_t>(row0) * row_vecs;
  const bool has_v = c.v != nullptr && v_out != nullptr;
  const v4u *v_src = has_v ? reinterpret_cast<const v4u *>(c.v) + static_cast<int64_t>(row0) * row_vecs : nullptr;
  // where vector o of the tile (o counts the tile's source vectors) goes in the concatenated cache
  const int head_vecs_log2 = __builtin_ctz(head_dim / VE);
  auto dst_of = [&](int o) -> int64_t {
    if (PACKED) return (c.dst_row + row0) * row_vecs + o;
    const int r = o / row_vecs, rem = o - r * row_vecs;
    return lay.at(c.dst_row + row0 + r, rem >> head_vecs_log2) / VE + (rem & ((1 << head_vecs_log2) - 1));
  };

  if (c.advance == 0.0) {  // already at its global phase: both tensors are plain row copies
    if (PACKED) {
      copy_vectors(k_src, k_out + dst_of(0), total_vecs, tid);
      if (has_v) copy_vectors(v_src, v_out + dst_of(0), total_vecs, tid);
    } else {
      for (int it = tid; it < total_vecs; it += kThreads) {
        const int64_t dd = dst_of(it);
        __builtin_nontemporal_store(__builtin_nontemporal_load(k_src + it), k_out + dd);
        if (has_v) __builtin_nontemporal_store(__builtin_nontemporal_load(v_src + it), v_out + dd);
      }
    }
    return;
  }

  // Every thread walks the same number of batches, so the barrier after the first load phase is
  // reached by all of them.
  bool table_ready = false;
  auto build_table = [&]() {
    if (table_ready) return;
    if (tid < half) {
      double sn, cs;
      sincos(c.advance * inv_freq[tid], &sn, &cs);
      s_cos[tid] = static_cast<float>(cs);
      s_sin[tid] = static_cast<float>(sn);
    }
    __syncthreads();
    table_ready = true;
  };

  if (PAIRING == IFKV_ROPE_HALF) {
    // Work item = vector cc of the low half of one (row, head) slice plus its partner in the high
    // half.  The slices of a tile are contiguous, so slice = item / hv and hv is a power of two.
    const int hv = half / VE;  // vectors per half head: 4, 8 or 16
    const int hv_shift = __builtin_ctz(hv);
    const int total = total_vecs >> 1;
    for (int base0 = 0; base0 < total; base0 += kThreads * RB) {
      v4u lo[RB], hi[RB], vlo[RB], vhi[RB];
      int off[RB], cc[RB];
#pragma unroll
      for (int u = 0; u < RB; ++u) {
        const int it = base0 + tid + u * kThreads;
        cc[u] = it & (hv - 1);
        off[u] = ((it >> hv_shift) << (hv_shift + 1)) + cc[u];
        if (it < total) {
          lo[u] = __builtin_nontemporal_load(k_src + off[u]);
          hi[u] = __builtin_nontemporal_load(k_src + off[u] + hv);
        }
      }
      if (has_v) {
#pragma unroll
        for (int u = 0; u < RB; ++u) {
          const int it = base0 + tid + u * kThreads;
          if (it < total) {
            vlo[u] = __builtin_nontemporal_load(v_src + off[u]);
            vhi[u] = __builtin_nontemporal_load(v_src + off[u] + hv);
          }
        }
      }
      build_table();
#pragma unroll
      for (int u = 0; u < RB; ++u) {
        const int it = base0 + tid + u * kThreads;
        if (it < total) {
          float a[VE], bb[VE], ra[VE], rb[VE];
          E::unpack(lo[u], a);
          E::unpack(hi[u], bb);
#pragma unroll
          for (int e = 0; e < VE; ++e) {
            const float cs = s_cos[cc[u] * VE + e];
            const float sn = s_sin[cc[u] * VE + e];
            ra[e] = fmaf(a[e], cs, -(bb[e] * sn));
            rb[e] = fmaf(a[e], sn, bb[e] * cs);
          }
          const int64_t dd = dst_of(off[u]);
          __builtin_nontemporal_store(E::pack(ra), k_out + dd);
          __builtin_nontemporal_store(E::pack(rb), k_out + dd + hv);
        }
      }
      if (has_v) {
#pragma unroll
        for (int u = 0; u < RB; ++u) {
          const int it = base0 + tid + u * kThreads;
          if (it < total) {
            const int64_t dd = dst_of(off[u]);
            __builtin_nontemporal_store(vlo[u], v_out + dd);
            __builtin_nontemporal_store(vhi[u], v_out + dd + hv);
          }
        }
      }
    }
  } else {  // interleaved pairs (x_{2i}, x_{2i+1}): a vector holds VE/2 whole pairs
    const int head_vecs = head_dim / VE;  // power of two
    for (int base0 = 0; base0 < total_vecs; base0 += kThreads * RB) {
      v4u x[RB], y[RB];
#pragma unroll
      for (int u = 0; u < RB; ++u) {
        const int it = base0 + tid + u * kThreads;
        if (it < total_vecs) {
          x[u] = __builtin_nontemporal_load(k_src + it);
          if (has_v) y[u] = __builtin_nontemporal_load(v_src + it);
        }
      }
      build_table();
#pragma unroll
      for (int u = 0; u < RB; ++u) {
        const int it = base0 + tid + u * kThreads;
        if (it < total_vecs) {
          const int pair0 = (it & (head_vecs - 1)) * (VE / 2);
          float f[VE], r[VE];
          E::unpack(x[u], f);
#pragma unroll
          for (int e = 0; e < VE / 2; ++e) {
            const float cs = s_cos[pair0 + e];
            const float sn = s_sin[pair0 + e];
            r[2 * e] = fmaf(f[2 * e], cs, -(f[2 * e + 1] * sn));
            r[2 * e + 1] = fmaf(f[2 * e], sn, f[2 * e + 1] * cs);
          }
          const int64_t dd = dst_of(it);
          __builtin_nontemporal_store(E::pack(r), k_out + dd);
          if (has_v) __builtin_nontemporal_store(y[u], v_out + dd);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Stage 5.  "KV Recomputation": recomputed rows replace the cached rows of the
// selected tokens.  One work item moves one 16-byte vector of one row.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void splice_kernel(const v4u *__restrict__ k_new,
                                                          const v4u *__restrict__ v_new,
                                                          const int32_t *__restrict__ idx, int64_t n_rows,
                                                          int row_vecs, int head_vecs_log2, int64_t token_vecs,
                                                          int64_t head_stride_vecs, v4u *__restrict__ k_cache,
                                                          v4u *__restrict__ v_cache, int64_t n_kv) {
  const int64_t total = n_rows * row_vecs;
  const int64_t base0 = static_cast<int64_t>(blockIdx.x) * (kThreads * kBatch) + threadIdx.x;
  v4u xk[kBatch], xv[kBatch];
  int64_t dst[kBatch];
#pragma unroll
  for (int u = 0; u < kBatch; ++u) {
    const int64_t it = base0 + u * kThreads;
    dst[u] = -1;
    if (it < total) {
      const int64_t r = it / row_vecs;
      const int w = static_cast<int>(it - r * row_vecs);
      const int64_t row = idx[r];
      if (row >= 0 && row < n_kv) {
        dst[u] = row * token_vecs + (w >> head_vecs_log2) * head_stride_vecs + (w & ((1 << head_vecs_log2) - 1));
        xk[u] = __builtin_nontemporal_load(k_new + it);
        if (v_new != nullptr) xv[u] = __builtin_nontemporal_load(v_new + it);
      }
    }
  }
#pragma unroll
  for (int u = 0; u < kBatch; ++u) {
    if (dst[u] >= 0) {
      k_cache[dst[u]] = xk[u];
      if (v_new != nullptr) v_cache[dst[u]] = xv[u];
    }
  }
}

// ---------------------------------------------------------------------------
// Rotary embedding of recomputed rows -- "KV Recomputation": the forward pass of a selected token
// runs at the token's position in the concatenated sequence, so its freshly projected query/key
// row r is turned by pos[r] * theta_j in every pair j (Eq. 3-4).  One workgroup per row; the first d/2 threads form the row's cos/sin
// in fp64 (positions reach 1e5: an fp32 angle would be off by 1e-2 rad), the rotation itself is
// fp32 FMA, rounded once to the storage type.  In place.
// ---------------------------------------------------------------------------
template <typename Tag, int PAIRING>
__global__ __launch_bounds__(kThreads) void rope_rows_kernel(v4u *__restrict__ x, const int32_t *__restrict__ pos,
                                                             const double *__restrict__ inv_freq, int n_heads,
                                                             int head_dim) {
  using E = Elem<Tag>;
  constexpr int VE = E::kVec;
  __shared__ float s_cos[kMaxHeadDim / 2];
  __shared__ float s_sin[kMaxHeadDim / 2];
  const int tid = threadIdx.x;
  const int half = head_dim / 2;
  const int row_vecs = n_heads * head_dim / VE;
  v4u *row = x + static_cast<int64_t>(blockIdx.x) * row_vecs;
  if (tid < half) {
    double sn, cs;
    sincos(static_cast<double>(pos[blockIdx.x]) * inv_freq[tid], &sn, &cs);
    s_cos[tid] = static_cast<float>(cs);
    s_sin[tid] = static_cast<float>(sn);
  }
  __syncthreads();
  if (PAIRING == IFKV_ROPE_HALF) {
    const int hv = half / VE, hv_shift = __builtin_ctz(hv);
    for (int it = tid; it < row_vecs / 2; it += kThreads) {
      const int cc = it & (hv - 1);
      const int off = ((it >> hv_shift) << (hv_shift + 1)) + cc;
      float a[VE], b[VE], ra[VE], rb[VE];
      E::unpack(row[off], a);
      E::unpack(row[off + hv], b);
#pragma unroll
      for (int e = 0; e < VE; ++e) {
        const float cs = s_cos[cc * VE + e], sn = s_sin[cc * VE + e];
        ra[e] = fmaf(a[e], cs, -(b[e] * sn));
        rb[e] = fmaf(a[e], sn, b[e] * cs);
      }
      row[off] = E::pack(ra);
      row[off + hv] = E::pack(rb);
    }
  } else {
    const int head_vecs = head_dim / VE;
    for (int it = tid; it < row_vecs; it += kThreads) {
      const int pair0 = (it & (head_vecs - 1)) * (VE / 2);
      float f[VE], r[VE];
      E::unpack(row[it], f);
#pragma unroll
      for (int e = 0; e < VE / 2; ++e) {
        const float cs = s_cos[pair0 + e], sn = s_sin[pair0 + e];
        r[2 * e] = fmaf(f[2 * e], cs, -(f[2 * e + 1] * sn));
        r[2 * e + 1] = fmaf(f[2 * e], sn, f[2 * e + 1] * cs);
      }
      row[it] = E::pack(r);
    }
  }
}

// Plain streaming copy with the same access shape (calibration only).
__global__ __launch_bounds__(kThreads) void copy_kernel(v4u *__restrict__ dst, const v4u *__restrict__ src,
                                                        int64_t n_vecs) {
  const int64_t base0 = static_cast<int64_t>(blockIdx.x) * (kThreads * kBatch) + threadIdx.x;
  v4u x[kBatch];
#pragma unroll
  for (int u = 0; u < kBatch; ++u) {
    const int64_t it = base0 + u * kThreads;
    if (it < n_vecs) x[u] = __builtin_nontemporal_load(src + it);
  }
#pragma unroll
  for (int u = 0; u < kBatch; ++u) {
    const int64_t it = base0 + u * kThreads;
    if (it < n_vecs) __builtin_nontemporal_store(x[u], dst + it);
  }
}

}  // namespace

int reposition_rows_per_tile() { return kRepoRows; }

hipError_t launch_reposition(ifkv_ctx *ctx, const RepoBatch &batch, void *k_out, void *v_out) {
  if (batch.total_tiles <= 0) return hipSuccess;
  const auto &d = ctx->desc;
  dim3 grid(batch.total_tiles), block(kThreads);
  v4u *ko = reinterpret_cast<v4u *>(k_out);
  v4u *vo = reinterpret_cast<v4u *>(v_out);
  const CacheLayout lay = cache_layout(ctx);
#define IFKV_LAUNCH_REPO(TAG, PAIR)                                                                          \
  do {                                                                                                       \
    if (ctx->packed)                                                                                         \
      hipLaunchKernelGGL((reposition_kernel<TAG, PAIR, kRepoBatch, true>), grid, block, 0, ctx->stream,      \
                         batch, ctx->d_inv_freq, kRepoRows, d.n_kv_heads, d.head_dim, lay, ko, vo);          \
    else                                                                                                     \
      hipLaunchKernelGGL((reposition_kernel<TAG, PAIR, kRepoBatch, false>), grid, block, 0, ctx->stream,     \
                         batch, ctx->d_inv_freq, kRepoRows, d.n_kv_heads, d.head_dim, lay, ko, vo);          \
  } while (0)
  if (d.dtype == IFKV_BF16) {
    if (d.pairing == IFKV_ROPE_HALF)
      IFKV_LAUNCH_REPO(BF16Tag, IFKV_ROPE_HALF);
    else
      IFKV_LAUNCH_REPO(BF16Tag, IFKV_ROPE_INTERLEAVED);
  } else {
    if (d.pairing == IFKV_ROPE_HALF)
      IFKV_LAUNCH_REPO(F32Tag, IFKV_ROPE_HALF);
    else
      IFKV_LAUNCH_REPO(F32Tag, IFKV_ROPE_INTERLEAVED);
  }
#undef IFKV_LAUNCH_REPO
  return hipGetLastError();
}

hipError_t launch_splice(ifkv_ctx *ctx, const void *k_new, const void *v_new, const int32_t *idx,
                         int64_t n_rows, void *k_cache, void *v_cache, int64_t n_kv) {
  if (n_rows <= 0) return hipSuccess;
  const auto &d = ctx->desc;
  const int row_vecs = static_cast<int>(d.n_kv_heads * d.head_dim * dtype_size(d.dtype) / 16);
  const int64_t total = n_rows * row_vecs;
  const int64_t per_block = kThreads * kBatch;
  dim3 grid(static_cast<unsigned>((total + per_block - 1) / per_block)), block(kThreads);
  const int ve = static_cast<int>(16 / dtype_size(d.dtype));
  hipLaunchKernelGGL(splice_kernel, grid, block, 0, ctx->stream, reinterpret_cast<const v4u *>(k_new),
                     reinterpret_cast<const v4u *>(v_new), idx, n_rows, row_vecs, __builtin_ctz(d.head_dim / ve),
                     ctx->token_stride / ve, ctx->head_stride / ve, reinterpret_cast<v4u *>(k_cache),
                     reinterpret_cast<v4u *>(v_cache), n_kv);
  return hipGetLastError();
}

hipError_t launch_rope_rows(ifkv_ctx *ctx, void *x, const int32_t *pos, int64_t n_rows, int n_heads) {
  if (n_rows <= 0 || n_heads <= 0) return hipSuccess;
  const auto &d = ctx->desc;
  dim3 grid(static_cast<unsigned>(n_rows)), block(kThreads);
  v4u *xv = reinterpret_cast<v4u *>(x);
#define IFKV_LAUNCH_ROPE(TAG, PAIR) \
  hipLaunchKernelGGL((rope_rows_kernel<TAG, PAIR>), grid, block, 0, ctx->stream, xv, pos, ctx->d_inv_freq, n_heads, d.head_dim)
  if (d.dtype == IFKV_BF16) {
    if (d.pairing == IFKV_ROPE_HALF)
      IFKV_LAUNCH_ROPE(BF16Tag, IFKV_ROPE_HALF);
    else
      IFKV_LAUNCH_ROPE(BF16Tag, IFKV_ROPE_INTERLEAVED);
  } else {
    if (d.pairing == IFKV_ROPE_HALF)
      IFKV_LAUNCH_ROPE(F32Tag, IFKV_ROPE_HALF);
    else
      IFKV_LAUNCH_ROPE(F32Tag, IFKV_ROPE_INTERLEAVED);
  }
#undef IFKV_LAUNCH_ROPE
  return hipGetLastError();
}

hipError_t launch_copy(ifkv_ctx *ctx, void *dst, const void *src, int64_t n_bytes) {
  const int64_t n_vecs = n_bytes / 16;
  if (n_vecs <= 0) return hipSuccess;
  const int64_t per_block = kThreads * kBatch;
  dim3 grid(static_cast<unsigned>((n_vecs + per_block - 1) / per_block)), block(kThreads);
  hipLaunchKernelGGL(copy_kernel, grid, block, 0, ctx->stream, reinterpret_cast<v4u *>(dst),
                     reinterpret_cast<const v4u *>(src), n_vecs);
  return hipGetLastError();
}

}  // namespace ifkv
