// Stage 2, bf16 MFMA kernels -- Eq. (7): s_j = sum_i A_ij.
//
// Per kv head the work is a [M*G x d] x [d x N] product (all prompt rows of the
// G query heads that share the kv head against every context key) whose
// softmax is taken along N and then summed along M*G.  With M*G = 512 and
// d = 128 that is ~500 flop per byte of K: the stage is bound by the matrix
// and transcendental units, not by HBM, so both sweeps run on MFMA.
//
// Layout of one block (512 threads, 8 wavefronts): the query rows of one kv
// head (up to 512, 136 KB with padding) stay in LDS for the whole block; each
// wavefront streams its own 64-key tiles of K straight from global memory into
// MFMA operand registers (a key is used by exactly one wavefront, so there is
// nothing to share through LDS) and walks over the query rows in blocks of 32.
//   pass A: S^T = K.Q^T, a lane owns one query row -> running (max, sum) per
//           lane with no cross-lane traffic; merged over lanes, wavefronts and
//           blocks at the end.
//   pass B: S = Q.K^T, a lane owns one key -> sum over query rows of
//           exp2(S*c - b_q) with b_q = log2-domain max + log2 Z, in-lane.
#include "ifkv_device.h"
#include "score_common.h"

namespace ifkv {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128;
constexpr int QSTR = D + 8;        // LDS row stride in elements (272 B: conflict-free b128 reads)
constexpr int kQChunk = 512;       // query rows resident in LDS
constexpr int kQBlocks = kQChunk / 32;
constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kTile = 64;          // keys per wavefront step
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct ScoreGeom {
  int n_ctx, m_prompt, n_q_heads, n_kv_heads;
  int n_qchunks;   // query-row chunks per kv head
  int kv_per_block;
  float scale_log2;
};

// Query row `ql` of chunk `qc` for kv head g: rows are ordered (prompt row, head-in-group).
__device__ __forceinline__ bool q_row_address(const ScoreGeom &gm, int g, int qc, int ql, int64_t *off, int *h,
                                              int *r) {
  const int G = gm.n_q_heads / gm.n_kv_heads;
  const int qi = qc * kQChunk + ql;
  *r = qi / G;
  *h = g * G + (qi - *r * G);
  *off = (static_cast<int64_t>(*r) * gm.n_q_heads + *h) * D;
  return qi < gm.m_prompt * G;
}

__device__ __forceinline__ void load_q_chunk(uint16_t *q_lds, const uint16_t *__restrict__ q_prompt,
                                             const ScoreGeom &gm, int g, int qc, int rows) {
  for (int v = threadIdx.x; v < rows * (D / 8); v += kThreads) {
    const int ql = v >> 4, c = v & 15;
    int64_t off;
    int h, r;
    v4u x = {0u, 0u, 0u, 0u};
    if (q_row_address(gm, g, qc, ql, &off, &h, &r)) x = *reinterpret_cast<const v4u *>(q_prompt + off + 8 * c);
    *reinterpret_cast<v4u *>(&q_lds[ql * QSTR + 8 * c]) = x;
  }
}

// K fragments of one 64-key tile in MFMA operand layout: lane (row, hf) holds
// key j0 + 32 t + row, columns 16 s + 8 hf .. +7.
__device__ __forceinline__ void load_k_frags(bf16x8 (&kf)[2][8], const uint16_t *__restrict__ k_global,
                                             const ScoreGeom &gm, int g, int j0, int row, int hf) {
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int j = min(j0 + 32 * t + row, gm.n_ctx - 1);
    const uint16_t *p = k_global + (static_cast<int64_t>(j) * gm.n_kv_heads + g) * D + 8 * hf;
#pragma unroll
    for (int s = 0; s < 8; ++s) kf[t][s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const v4u *>(p + 16 * s));
  }
}

// ---------------------------------------------------------------------------
// pass A
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void score_stats_mfma(
    const uint16_t *__restrict__ k_global, const uint16_t *__restrict__ q_prompt, ScoreGeom gm,
    float2 *__restrict__ partial) {
  __shared__ __attribute__((aligned(16))) uint16_t q_lds[kQChunk * QSTR];
  const int G = gm.n_q_heads / gm.n_kv_heads;
  const int kb = blockIdx.x;
  const int g = blockIdx.y / gm.n_qchunks;
  const int qc = blockIdx.y - g * gm.n_qchunks;
  const int q_total = gm.m_prompt * G;
  const int q_rows = min(kQChunk, q_total - qc * kQChunk);
  const int nqb = (q_rows + 31) >> 5;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = lane & 31, hf = lane >> 5;

  load_q_chunk(q_lds, q_prompt, gm, g, qc, nqb * 32);
  __syncthreads();

  float m[kQBlocks], z[kQBlocks];
#pragma unroll
  for (int qb = 0; qb < kQBlocks; ++qb) {
    m[qb] = -INFINITY;
    z[qb] = 0.f;
  }
  const float c = gm.scale_log2;
  const int kv_begin = kb * gm.kv_per_block;
  const int kv_end = min(gm.n_ctx, kv_begin + gm.kv_per_block);
  for (int j0 = kv_begin + wave * kTile; j0 < kv_end; j0 += kWaves * kTile) {
    bf16x8 kf[2][8];
    load_k_frags(kf, k_global, gm, g, j0, row, hf);
    const bool tail = j0 + kTile > kv_end;
#pragma unroll
    for (int qb = 0; qb < kQBlocks; ++qb) {
      if (qb < nqb) {
        f32x16 S0, S1;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          S0[r] = 0.f;
          S1[r] = 0.f;
        }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          const bf16x8 qf = __builtin_bit_cast(
              bf16x8, *reinterpret_cast<const v4u *>(&q_lds[(qb * 32 + row) * QSTR + 16 * s + 8 * hf]));
          S0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0][s], qf, S0, 0, 0, 0);
          S1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[1][s], qf, S1, 0, 0, 0);
        }
        // register r of S_t: key j0 + 32 t + 8 (r/4) + 4 hf + r%4, query row qb*32 + (lane & 31)
        if (tail) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kv = j0 + 8 * (r >> 2) + 4 * hf + (r & 3);
            if (kv >= kv_end) S0[r] = -INFINITY;
            if (kv + 32 >= kv_end) S1[r] = -INFINITY;
          }
        }
        float mx = S0[0];
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, fmaxf(S0[r], S1[r]));
        const float m_new = fmaxf(m[qb], mx * c);
        const float m_use = fmaxf(m_new, -1e30f);  // a lane that has seen no valid key yet stays at (-inf, 0)
        float acc = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          acc += __builtin_amdgcn_exp2f(fmaf(S0[r], c, -m_use));
          acc += __builtin_amdgcn_exp2f(fmaf(S1[r], c, -m_use));
        }
        z[qb] = z[qb] * __builtin_amdgcn_exp2f(m[qb] - m_use) + acc;
        m[qb] = m_new;
      }
    }
  }

  // merge the two lane halves (same query row, disjoint keys), then the wavefronts
  __syncthreads();  // every wavefront is done with the query tile: LDS is reused below
  float2 *w_stats = reinterpret_cast<float2 *>(q_lds);  // [kWaves][kQChunk]
#pragma unroll
  for (int qb = 0; qb < kQBlocks; ++qb) {
    if (qb < nqb) {
      const float mo = __shfl_xor(m[qb], 32, 64);
      const float zo = __shfl_xor(z[qb], 32, 64);
      const float mm = fmaxf(m[qb], mo);
      const float mu = fmaxf(mm, -1e30f);
      const float zz = z[qb] * __builtin_amdgcn_exp2f(m[qb] - mu) + zo * __builtin_amdgcn_exp2f(mo - mu);
      if (hf == 0) w_stats[wave * kQChunk + qb * 32 + row] = make_float2(mm, zz);
    }
  }
  __syncthreads();
  for (int ql = threadIdx.x; ql < q_rows; ql += kThreads) {
    float mm = -INFINITY, zz = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float2 p = w_stats[w * kQChunk + ql];
      const float mn = fmaxf(mm, p.x);
      const float mu = fmaxf(mn, -1e30f);
      zz = zz * __builtin_amdgcn_exp2f(mm - mu) + p.y * __builtin_amdgcn_exp2f(p.x - mu);
      mm = mn;
    }
    int64_t off;
    int h, r;
    q_row_address(gm, g, qc, ql, &off, &h, &r);
    // natural-log domain, as the merge kernel expects
    partial[(static_cast<int64_t>(kb) * gm.n_q_heads + h) * gm.m_prompt + r] = make_float2(mm * kLn2, zz);
  }
}

// ---------------------------------------------------------------------------
// pass B
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) void score_colsum_mfma(
    const uint16_t *__restrict__ k_global, const uint16_t *__restrict__ q_prompt, ScoreGeom gm,
    const float2 *__restrict__ stats, float *__restrict__ colpart) {
  __shared__ __attribute__((aligned(16))) uint16_t q_lds[kQChunk * QSTR];
  __shared__ __attribute__((aligned(16))) float b_lds[kQChunk];
  const int G = gm.n_q_heads / gm.n_kv_heads;
  const int kb = blockIdx.x;
  const int g = blockIdx.y / gm.n_qchunks;
  const int qc = blockIdx.y - g * gm.n_qchunks;
  const int q_total = gm.m_prompt * G;
  const int q_rows = min(kQChunk, q_total - qc * kQChunk);
  const int nqb = (q_rows + 31) >> 5;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = lane & 31, hf = lane >> 5;

  load_q_chunk(q_lds, q_prompt, gm, g, qc, nqb * 32);
  for (int ql = threadIdx.x; ql < nqb * 32; ql += kThreads) {
    int64_t off;
    int h, r;
    float b = INFINITY;  // padded rows contribute exp2(-inf) = 0
    if (q_row_address(gm, g, qc, ql, &off, &h, &r)) {
      const float2 st = stats[h * gm.m_prompt + r];  // (max, 1/Z), natural-log domain
      b = st.y > 0.f ? st.x * kLog2e - __log2f(st.y) : INFINITY;
    }
    b_lds[ql] = b;
  }
  __syncthreads();

  const float c = gm.scale_log2;
  const int kv_begin = kb * gm.kv_per_block;
  const int kv_end = min(gm.n_ctx, kv_begin + gm.kv_per_block);
  float *dst = colpart + static_cast<int64_t>(blockIdx.y) * gm.n_ctx;
  for (int j0 = kv_begin + wave * kTile; j0 < kv_end; j0 += kWaves * kTile) {
    bf16x8 kf[2][8];
    load_k_frags(kf, k_global, gm, g, j0, row, hf);
    float col0 = 0.f, col1 = 0.f;
    for (int qb = 0; qb < nqb; ++qb) {
      f32x16 S0, S1;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        S0[r] = 0.f;
        S1[r] = 0.f;
      }
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const bf16x8 qf = __builtin_bit_cast(
            bf16x8, *reinterpret_cast<const v4u *>(&q_lds[(qb * 32 + row) * QSTR + 16 * s + 8 * hf]));
        S0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[0][s], S0, 0, 0, 0);
        S1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[1][s], S1, 0, 0, 0);
      }
      // register r: query row qb*32 + 8 (r/4) + 4 hf + r%4, key j0 + 32 t + (lane & 31)
#pragma unroll
      for (int ri = 0; ri < 4; ++ri) {
        const f32x4 b = *reinterpret_cast<const f32x4 *>(&b_lds[qb * 32 + 8 * ri + 4 * hf]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          col0 += __builtin_amdgcn_exp2f(fmaf(S0[4 * ri + e], c, -b[e]));
          col1 += __builtin_amdgcn_exp2f(fmaf(S1[4 * ri + e], c, -b[e]));
        }
      }
    }
    col0 += __shfl_xor(col0, 32, 64);
    col1 += __shfl_xor(col1, 32, 64);
    if (hf == 0) {
      if (j0 + row < kv_end) dst[j0 + row] = col0;
      if (j0 + 32 + row < kv_end) dst[j0 + 32 + row] = col1;
    }
  }
}

// scores[j] = (accumulate ? scores[j] : 0) + (1 / H_q) * sum over (kv head, chunk) partials
__global__ void score_reduce_kernel(const float *__restrict__ colpart, int n_parts, int n_ctx, float inv_heads,
                                    int accumulate, float *__restrict__ scores) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n_ctx) return;
  float s = 0.f;
  for (int p = 0; p < n_parts; ++p) s += colpart[static_cast<int64_t>(p) * n_ctx + j];
  s *= inv_heads;
  scores[j] = accumulate ? scores[j] + s : s;
}

}  // namespace

bool score_mfma_supported(const ifkv_ctx *ctx, int m_prompt) {
  const auto &d = ctx->desc;
  const int G = d.n_q_heads / d.n_kv_heads;
  return d.dtype == IFKV_BF16 && d.head_dim == D && m_prompt > 0 &&
         static_cast<int64_t>(m_prompt) * G <= static_cast<int64_t>(kMaxQChunks) * kQChunk;
}

hipError_t launch_score_mfma_passes(ifkv_ctx *ctx, const void *k_global, int64_t n_ctx, const void *q_prompt,
                                    int m_prompt, int *n_slices_out, bool pass_b, int accumulate, float *scores) {
  const auto &d = ctx->desc;
  const int G = d.n_q_heads / d.n_kv_heads;
  ScoreGeom gm;
  gm.n_ctx = static_cast<int>(n_ctx);
  gm.m_prompt = m_prompt;
  gm.n_q_heads = d.n_q_heads;
  gm.n_kv_heads = d.n_kv_heads;
  gm.n_qchunks = (m_prompt * G + kQChunk - 1) / kQChunk;
  gm.scale_log2 = ctx->sm_scale * kLog2e;
  // one block per CU when the context is long enough; a block owns whole 64-key tiles
  const int per_head = d.n_kv_heads * gm.n_qchunks;
  int kv_blocks = 256 / per_head;
  if (kv_blocks < 1) kv_blocks = 1;
  const int max_blocks = static_cast<int>((n_ctx + kTile - 1) / kTile);
  if (kv_blocks > max_blocks) kv_blocks = max_blocks;
  int kvpb = static_cast<int>((n_ctx + kv_blocks - 1) / kv_blocks);
  kvpb = ((kvpb + kTile - 1) / kTile) * kTile;
  kv_blocks = static_cast<int>((n_ctx + kvpb - 1) / kvpb);
  gm.kv_per_block = kvpb;
  *n_slices_out = kv_blocks;

  ScoreScratch sc = score_scratch_layout(ctx, n_ctx, m_prompt);
  char *base = static_cast<char *>(ctx->scratch);
  float2 *partial = reinterpret_cast<float2 *>(base + sc.partial_off);
  float2 *stats = reinterpret_cast<float2 *>(base + sc.stats_off);
  float *colpart = reinterpret_cast<float *>(base + sc.colpart_off);
  dim3 grid(kv_blocks, per_head);
  if (!pass_b) {
    hipLaunchKernelGGL(score_stats_mfma, grid, dim3(kThreads), 0, ctx->stream,
                       static_cast<const uint16_t *>(k_global), static_cast<const uint16_t *>(q_prompt), gm, partial);
  } else {
    hipLaunchKernelGGL(score_colsum_mfma, grid, dim3(kThreads), 0, ctx->stream,
                       static_cast<const uint16_t *>(k_global), static_cast<const uint16_t *>(q_prompt), gm, stats,
                       colpart);
    hipLaunchKernelGGL(score_reduce_kernel, dim3(static_cast<unsigned>((n_ctx + 255) / 256)), dim3(256), 0,
                       ctx->stream, colpart, per_head, static_cast<int>(n_ctx), 1.0f / d.n_q_heads, accumulate,
                       scores);
  }
  return hipGetLastError();
}

}  // namespace ifkv
