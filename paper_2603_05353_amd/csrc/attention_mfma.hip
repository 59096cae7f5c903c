// Stage 4, bf16 MFMA kernel -- "KV Recomputation": each selected row attends
// causally to cache rows 0..p_r of the concatenated sequence.
//
// Shape of the problem: few, scattered query rows (k = rho N of them) against a
// long, dense K/V prefix.  The kernel therefore packs the G query heads that
// share a kv head together with a block of consecutive selected rows into one
// tile of NWAVES*32 "query columns", so that every K/V tile fetched from HBM/L2
// is used by all of them, and walks the kv axis in tiles of 64 rows with an
// online softmax (flash-attention style).  Rows are sorted by position, so only
// the last one or two kv tiles of a wavefront need the causal mask.
//
// Per wavefront (32 query columns), per kv tile, with 32x32x16 bf16 MFMAs:
//   S^T [64 kv x 32 q]  = K_tile . Q^T         (A = K rows from LDS, B = Q in registers)
//   P^T = exp2(S^T * c - m)                     (fp32, per-lane statistics: a lane owns one query column)
//   O^T [128 d x 32 q] += V_tile^T . P^T       (A = V^T from LDS, B = P^T straight from the S^T registers)
// Computing the transposed products keeps each query column in one lane (two
// lanes, one per half-wave), so row max / row sum need a single cross-lane
// exchange per tile, and the S^T accumulator layout is exactly the B-operand
// layout of the second product once the K rows are fed in a fixed permuted
// order (sigma below): no LDS round trip for P.
// V is transposed on its way into LDS (8x8 register transposes) because the
// second product contracts over kv, which is the strided axis of the cache.
#include <cstdlib>

#include "attention_common.h"
#include "ifkv_device.h"

namespace ifkv {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int D = 128;        // head_dim served by this kernel
constexpr int TK = 64;        // kv rows per tile
constexpr int KSTR = D + 8;   // LDS row stride of the K tile in elements (272 B: conflict-free b128 reads)
constexpr int VSTR = TK + 8;  // LDS row stride of the V^T tile in elements (144 B)

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);  // round-to-nearest-even
  return __builtin_bit_cast(uint32_t, r);
}

// Order in which K rows are fed as MFMA A-rows.  A 32x32 accumulator gives lane
// half hf, register r the A-row 8*(r/4) + 4*hf + r%4; feeding row sigma(i) as
// A-row i makes registers 0..7 of a lane hold kv rows 8*hf + 0..7 and registers
// 8..15 hold kv rows 16 + 8*hf + 0..7, i.e. eight consecutive kv rows per
// 16-row contraction step, which is what the B operand of V^T.P^T needs.
__device__ __forceinline__ int sigma(int i) { return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1); }

template <int NWAVES>
__global__ __launch_bounds__(NWAVES * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_mfma_kernel(
    const uint16_t *__restrict__ q_sel, const int32_t *__restrict__ row_pos, int n_rows,
    const uint16_t *__restrict__ k_cache, const uint16_t *__restrict__ v_cache, int n_kv,
    uint16_t *__restrict__ out, float *__restrict__ lse_out, int n_q_heads, int n_kv_heads,
    float scale_log2, int rows_per_block) {
  constexpr int NT = NWAVES * 64;
  constexpr int KTHREADS = NT - 128;                         // threads that stage K (the first 128 stage V)
  constexpr int KPT = (TK * D / 8 + KTHREADS - 1) / KTHREADS;  // 16-byte K vectors per staging thread
  static_assert(KPT <= 8, "prefetch registers");

  // two stages of (K tile, V^T tile): a tile is written while the previous one is read
  __shared__ __attribute__((aligned(16))) uint16_t k_lds[2][TK * KSTR];
  __shared__ __attribute__((aligned(16))) uint16_t vt_lds[2][D * VSTR];
  __shared__ int s_pmax[NWAVES];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int col = lane & 31;
  const int hf = lane >> 5;
  const int G = n_q_heads / n_kv_heads;
  const int g = blockIdx.x;
  const int rb = gridDim.y - 1 - blockIdx.y;  // longest prefixes are dispatched first
  const int row0 = rb * rows_per_block;

  // ---- this lane's query column -------------------------------------------------
  const int qc = wave * 32 + col;
  const int rr = qc / G;
  const int hh = qc - rr * G;
  const int row = row0 + rr;
  const bool col_valid = (rr < rows_per_block) && (row < n_rows);
  int p_q = 0;
  bool in_range = false;
  if (col_valid) {
    const int p = row_pos[row];
    in_range = (p >= 0) && (p < n_kv);
    p_q = in_range ? p : 0;
  }
  const int64_t q_off = (static_cast<int64_t>(row) * n_q_heads + g * G + hh) * D;

  bf16x8 qf[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    v4u x = {0u, 0u, 0u, 0u};
    if (col_valid) x = *reinterpret_cast<const v4u *>(q_sel + q_off + 16 * s + 8 * hf);
    qf[s] = __builtin_bit_cast(bf16x8, x);
  }

  // wavefront and block extents of the causal prefix
  int p_wmax = p_q, p_wmin = col_valid ? p_q : 0x7FFFFFFF;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    p_wmax = max(p_wmax, __shfl_xor(p_wmax, o, 64));
    p_wmin = min(p_wmin, __shfl_xor(p_wmin, o, 64));
  }
  if (lane == 0) s_pmax[wave] = p_wmax;
  __syncthreads();
  int p_bmax = 0;
#pragma unroll
  for (int w = 0; w < NWAVES; ++w) p_bmax = max(p_bmax, s_pmax[w]);
  const int n_tiles = p_bmax / TK + 1;

  // ---- staging roles -----------------------------------------------------------
  // V: thread (q8, dg) owns kv rows 8*q8..+7 x d columns 8*dg..+7 of the tile.  q8 varies fastest
  // over the lanes so that the eight transposed 16-byte rows a wavefront writes per
  // instruction land in distinct LDS banks; the global loads still cover whole 128-byte lines.
  const int v_q8 = lane & 7;
  const int v_dg = 8 * wave + (lane >> 3);
  const int64_t kv_row_elems = static_cast<int64_t>(n_kv_heads) * D;
  const uint16_t *k_base = k_cache + static_cast<int64_t>(g) * D;
  const uint16_t *v_base = v_cache + static_cast<int64_t>(g) * D;

  v4u pre[8];
  auto issue_loads = [&](int j0) {
    if (wave < 2) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int jr = min(j0 + 8 * v_q8 + i, n_kv - 1);
        pre[i] = *reinterpret_cast<const v4u *>(v_base + jr * kv_row_elems + 8 * v_dg);
      }
    } else {
#pragma unroll
      for (int i = 0; i < KPT; ++i) {
        const int vi = (tid - 128) + i * KTHREADS;
        if (vi < TK * D / 8) {
          const int jr = min(j0 + (vi >> 4), n_kv - 1);
          pre[i] = *reinterpret_cast<const v4u *>(k_base + jr * kv_row_elems + 8 * (vi & 15));
        }
      }
    }
  };
  auto store_tile = [&](int stage) {
    if (wave < 2) {
      // 8x8 transpose in registers: word w of output row di pairs kv rows 2w, 2w+1 at d column di
#pragma unroll
      for (int di = 0; di < 8; ++di) {
        v4u o;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const uint32_t a = pre[2 * w][di >> 1];
          const uint32_t b = pre[2 * w + 1][di >> 1];
          o[w] = (di & 1) ? ((a >> 16) | (b & 0xFFFF0000u)) : ((a & 0xFFFFu) | (b << 16));
        }
        *reinterpret_cast<v4u *>(&vt_lds[stage][(8 * v_dg + di) * VSTR + 8 * v_q8]) = o;
      }
    } else {
#pragma unroll
      for (int i = 0; i < KPT; ++i) {
        const int vi = (tid - 128) + i * KTHREADS;
        // kv row j is stored at LDS row sigma(j): MFMA A-row i then reads LDS row i
        if (vi < TK * D / 8) *reinterpret_cast<v4u *>(&k_lds[stage][sigma(vi >> 4) * KSTR + 8 * (vi & 15)]) = pre[i];
      }
    }
  };

  // ---- main loop ---------------------------------------------------------------
  f32x16 O[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) O[dt][r] = 0.f;
  float m_run = -INFINITY;  // running max of the scaled logits, log2 domain
  float l_run = 0.f;        // this lane's share of the running sum

  issue_loads(0);
  store_tile(0);
  if (n_tiles > 1) issue_loads(TK);
  __syncthreads();
  for (int tile = 0; tile < n_tiles; ++tile) {
    const int j0 = tile * TK;
    const int cur = tile & 1;
    if (j0 <= p_wmax) {  // otherwise this wavefront's rows end before the tile (it still stages and syncs)
    f32x16 S[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
      for (int r = 0; r < 16; ++r) S[t][r] = 0.f;
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const v4u x = *reinterpret_cast<const v4u *>(&k_lds[cur][(32 * t + col) * KSTR + 16 * s + 8 * hf]);
        S[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, x), qf[s], S[t], 0, 0, 0);
      }
    }
    // register r of S[t] is kv row j0 + 32 t + 16 (r / 8) + 8 hf + r % 8
    if (j0 + TK - 1 > p_wmin) {
      const int base = j0 + 8 * hf - p_q;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (base + 32 * t + 16 * (r >> 3) + (r & 7) > 0) S[t][r] = -INFINITY;
    }
    float mx = S[0][0];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[t][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx * scale_log2);
    if (__any(m_new > m_run)) {
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) O[dt][r] *= alpha;
      m_run = m_new;
    }
    float psum[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        S[t][r] = __builtin_amdgcn_exp2f(fmaf(S[t][r], scale_log2, -m_run));
        psum[r & 3] += S[t][r];  // four independent chains; fp32 sum of the unrounded probabilities
      }
    l_run += (psum[0] + psum[1]) + (psum[2] + psum[3]);

#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int t = u >> 1, r0 = 8 * (u & 1);
      v4u pb;
      pb[0] = pack_bf16x2(S[t][r0 + 0], S[t][r0 + 1]);
      pb[1] = pack_bf16x2(S[t][r0 + 2], S[t][r0 + 3]);
      pb[2] = pack_bf16x2(S[t][r0 + 4], S[t][r0 + 5]);
      pb[3] = pack_bf16x2(S[t][r0 + 6], S[t][r0 + 7]);
      const bf16x8 pfrag = __builtin_bit_cast(bf16x8, pb);
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        const v4u x = *reinterpret_cast<const v4u *>(&vt_lds[cur][(32 * dt + col) * VSTR + 16 * u + 8 * hf]);
        O[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, x), pfrag, O[dt], 0, 0, 0);
      }
    }
    }  // compute
    // stage the next tile into the other buffer (last read one iteration ago, before the
    // previous barrier) and start fetching the one after it
    if (tile + 1 < n_tiles) {
      store_tile(cur ^ 1);
      if (tile + 2 < n_tiles) issue_loads(j0 + 2 * TK);
    }
    __syncthreads();
  }

  // ---- epilogue ------------------------------------------------------------------
  if (!col_valid) return;
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = in_range ? 1.f / l_tot : 0.f;
  uint16_t *orow = out + q_off;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int ri = 0; ri < 4; ++ri) {
      uint2 w;
      w.x = pack_bf16x2(O[dt][4 * ri + 0] * inv, O[dt][4 * ri + 1] * inv);
      w.y = pack_bf16x2(O[dt][4 * ri + 2] * inv, O[dt][4 * ri + 3] * inv);
      *reinterpret_cast<uint2 *>(orow + 32 * dt + 8 * ri + 4 * hf) = w;
    }
  if (lse_out != nullptr && hf == 0)
    lse_out[static_cast<int64_t>(row) * n_q_heads + g * G + hh] =
        in_range ? 0.6931471805599453f * (m_run + __log2f(l_tot)) : 0.f;
}

}  // namespace

bool attention_mfma_supported(const ifkv_ctx *ctx) {
  const auto &d = ctx->desc;
  const int G = d.n_q_heads / d.n_kv_heads;
  return d.dtype == IFKV_BF16 && d.head_dim == D && G <= 32;
}

hipError_t launch_attention_mfma(ifkv_ctx *ctx, const void *q_sel, const int32_t *row_pos, int64_t n_rows,
                                 const void *k_cache, const void *v_cache, int64_t n_kv, void *out,
                                 float *lse_out) {
  const auto &d = ctx->desc;
  const int G = d.n_q_heads / d.n_kv_heads;
  const float scale_log2 = ctx->sm_scale * 1.4426950408889634f;
  // 256 query columns (8 wavefronts) per block halve the K/V traffic per flop; fall back to 128
  // when that would leave too few blocks to fill the chip.  IFKV_ATTN_WAVES=4|8 overrides.
  const int rpb8 = 256 / G;
  const int64_t blocks8 = ((n_rows + rpb8 - 1) / rpb8) * d.n_kv_heads;
  bool big = blocks8 >= 512;
  if (const char *env = getenv("IFKV_ATTN_WAVES")) big = atoi(env) == 8;
  const int rpb = big ? rpb8 : 128 / G;
  const unsigned n_rb = static_cast<unsigned>((n_rows + rpb - 1) / rpb);
  dim3 grid(d.n_kv_heads, n_rb);
  if (big) {
    hipLaunchKernelGGL((attn_mfma_kernel<8>), grid, dim3(512), 0, ctx->stream,
                       static_cast<const uint16_t *>(q_sel), row_pos, static_cast<int>(n_rows),
                       static_cast<const uint16_t *>(k_cache), static_cast<const uint16_t *>(v_cache),
                       static_cast<int>(n_kv), static_cast<uint16_t *>(out), lse_out, d.n_q_heads, d.n_kv_heads,
                       scale_log2, rpb);
  } else {
    hipLaunchKernelGGL((attn_mfma_kernel<4>), grid, dim3(256), 0, ctx->stream,
                       static_cast<const uint16_t *>(q_sel), row_pos, static_cast<int>(n_rows),
                       static_cast<const uint16_t *>(k_cache), static_cast<const uint16_t *>(v_cache),
                       static_cast<int>(n_kv), static_cast<uint16_t *>(out), lse_out, d.n_q_heads, d.n_kv_heads,
                       scale_log2, rpb);
  }
  return hipGetLastError();
}

}  // namespace ifkv
