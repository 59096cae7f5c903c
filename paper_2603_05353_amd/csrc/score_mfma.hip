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
//   pass A: S^T = K.Q^T, a lane owns one query row -> (reference exponent,
//           sum) per lane with no cross-lane traffic; merged over lanes,
//           wavefronts and blocks at the end.
//   pass B: S = Q.K^T, a lane owns one key -> sum over query rows of
//           exp2(S*c - b_q) with b_q = log2-domain reference + log2 Z, in-lane.
#include <algorithm>
#include <type_traits>

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
constexpr int kWpe = kThreads / 256;  // wavefronts per SIMD
constexpr int kWaves = kThreads / 64;
constexpr int kTile = 64;          // keys per wavefront step
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct ScoreGeom {
  int n_ctx, m_prompt, n_q_heads, n_kv_heads;
  int n_qchunks;   // query-row chunks per kv head
  int q_chunk_rows;  // rows per chunk (multiple of 128, <= kQChunk); the last chunk may hold fewer
  int kv_per_block;
  // Layout of the per-slice partials.  0: [slice][query head][prompt row], what the merge kernel
  // reads.  1: [slice][kv head, query chunk][row of the chunk], the order in which a block of the
  // second sweep holds its rows, so that its own merge reads whole lines.
  int partial_by_block;
  float scale_log2;
  int64_t token_stride, head_stride;  // layout of k_global, in elements
};

// Query row `ql` of chunk `qc` for kv head g: rows are ordered (prompt row, head-in-group).
__device__ __forceinline__ bool q_row_address(const ScoreGeom &gm, int g, int qc, int ql, int64_t *off, int *h,
                                              int *r) {
  const int G = gm.n_q_heads / gm.n_kv_heads;
  const int qi = qc * gm.q_chunk_rows + ql;
  *r = qi / G;
  *h = g * G + (qi - *r * G);
  *off = (static_cast<int64_t>(*r) * gm.n_q_heads + *h) * D;
  return qi < gm.m_prompt * G;
}

// Staging of a kv head's query tile (NV * 32 rows, NV = 4, 8, 12 or 16; rows past the real ones are
// zero) in two halves, so that the caller can put other requests between them: q_tile_request issues
// all of a thread's 16-byte loads (NV of them, rows 32 apart: the row -> (prompt row, head) split
// needs one division, the rest is incremental), q_tile_store writes them to LDS.
template <int NV>
__device__ __forceinline__ void q_tile_request(v4u (&x)[NV], const uint16_t *__restrict__ q_prompt,
                                               const ScoreGeom &gm, int g, int qc) {
  const int G = gm.n_q_heads / gm.n_kv_heads;
  const int total = gm.m_prompt * G;
  const int c = threadIdx.x & 15;
  int qi = qc * gm.q_chunk_rows + (threadIdx.x >> 4);
  int r = qi / G, hg = qi - r * G;
  const int dr = 32 / G, dh = 32 - dr * G;
#pragma unroll
  for (int u = 0; u < NV; ++u) {
    x[u] = v4u{0u, 0u, 0u, 0u};
    if (qi < total)
      x[u] = *reinterpret_cast<const v4u *>(q_prompt + (static_cast<int64_t>(r) * gm.n_q_heads + g * G + hg) * D +
                                            8 * c);
    qi += 32;
    r += dr;
    hg += dh;
    if (hg >= G) {
      hg -= G;
      ++r;
    }
  }
}
template <int NV>
__device__ __forceinline__ void q_tile_store(uint16_t *q_lds, const v4u (&x)[NV]) {
  const int c = threadIdx.x & 15, ql = threadIdx.x >> 4;
#pragma unroll
  for (int u = 0; u < NV; ++u) *reinterpret_cast<v4u *>(&q_lds[(ql + 32 * u) * QSTR + 8 * c]) = x[u];
}

// K fragments of one 64-key tile in MFMA operand layout: lane (row, hf) holds
// key j0 + 32 t + row, columns 16 s + 8 hf .. +7.
__device__ __forceinline__ void load_k_frags(bf16x8 (&kf)[2][8], const uint16_t *__restrict__ k_global,
                                             const ScoreGeom &gm, int g, int j0, int row, int hf) {
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int j = min(j0 + 32 * t + row, gm.n_ctx - 1);
    const uint16_t *p = k_global + static_cast<int64_t>(j) * gm.token_stride + g * gm.head_stride + 8 * hf;
#pragma unroll
    for (int s = 0; s < 8; ++s) kf[t][s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const v4u *>(p + 16 * s));
  }
}

// ---------------------------------------------------------------------------
// Fused stage 1 + pass A -- Eq. (5) and Eq. (7) in one sweep: the key fragments come from the chunk
// caches instead of the concatenated cache, are advanced to their global rotary phase in
// registers, rounded to bf16 once (exactly the values stage 1 stores), written to the
// concatenated cache by the blocks of query chunk 0, and fed to the MFMAs.  A lane holds, for each
// of its two keys, columns 16 s + 8 hf .. +7 (s = 0..7): both halves of every (x_i, x_{i+64}) pair
// and every (x_{2i}, x_{2i+1}) pair it touches, so the rotation needs no other lane.  The value
// rows of the same keys are copied along (stage 1 moves them too).
// Measured at 32K context (64 chunks of 512 rows, prompt lengths 1 .. 256): the fused sweep is 20 to
// 50 us slower than the two stages one after the other.  A kernel shaped for the matrix pipes (eight
// wavefronts per compute unit, a few dozen loads in flight each, two key tiles per wavefront) keeps
// about 0.5 MB in flight over the whole chip, where streaming 256 MB at the rate of stage 1's own
// kernel takes some 10 MB; the streaming does not hide under the matrix work, it stretches it.  The
// library therefore runs the two stages separately unless the fused sweep is asked for by the
// tuning knob "fused_repo_score" (which the tests use to keep this path checked).
// ---------------------------------------------------------------------------
struct FusedChunk {      // one non-empty chunk, in the order of the concatenation
  const uint16_t *k;     // [len, H_kv, 128] packed
  const uint16_t *v;     // same shape, or null
  int32_t dst_row;       // first row in the concatenated cache
  int32_t rotate;        // 0: phase advance is zero, the rows are copied bit for bit
};
struct FusedArgs {
  const FusedChunk *chunks;  // device, [n_chunks]
  const int32_t *starts;     // device, [n_chunks]: dst_row of every chunk, ascending
  const float *rot;          // device, [n_chunks][128]: per half-wave 64 floats, see fused_table_kernel
  uint16_t *k_out, *v_out;   // concatenated caches (v_out may be null)
  int32_t n_chunks;
  int32_t pairing;
};
constexpr int kMaxFusedChunks = 512;

// (cos, sin) of a chunk's phase advance in the order a lane consumes them: for lane half hf the 64
// floats at rot[c * 128 + hf * 64 ..].  Half-split pairs: [s = 0..3][cos of frequencies
// 16 s + 8 hf + 0..7, then their sines].  Interleaved pairs: [s = 0..7][cos of pairs
// 8 s + 4 hf + 0..3, then their sines].  Angles in fp64 (positions reach 1e5), stored as fp32: the
// same values stage 1's own kernel uses.
struct FusedTableBatch {
  FusedChunk c[64];
  double advance[64];
  int32_t n, base;
};
__global__ __launch_bounds__(64) void fused_table_kernel(FusedTableBatch b, const double *__restrict__ inv_freq,
                                                         FusedChunk *__restrict__ chunks, int32_t *__restrict__ starts,
                                                         float *__restrict__ rot, int pairing) {
  const int i = blockIdx.x, f = threadIdx.x;
  const int c = b.base + i;
  if (f == 0) {
    chunks[c] = b.c[i];
    starts[c] = b.c[i].dst_row;
  }
  double sn, cs;
  sincos(b.advance[i] * inv_freq[f], &sn, &cs);
  int at;
  if (pairing == IFKV_ROPE_HALF)
    at = ((f >> 3) & 1) * 64 + (f >> 4) * 16 + (f & 7);
  else
    at = ((f >> 2) & 1) * 64 + (f >> 3) * 8 + (f & 3);
  const int to_sin = pairing == IFKV_ROPE_HALF ? 8 : 4;
  rot[c * 128 + at] = static_cast<float>(cs);
  rot[c * 128 + at + to_sin] = static_cast<float>(sn);
}

__device__ __forceinline__ uint32_t pack_bf16_rne(float a, float b) {
  return float_to_bf16_bits(a) | (float_to_bf16_bits(b) << 16);
}

// The fused counterpart of load_k_frags for keys j0 .. j0+63 (lane (row, hf): keys j0 + row and
// j0 + 32 + row); s_starts: the chunks' first rows in LDS.
__device__ __forceinline__ void fused_k_frags(bf16x8 (&kf)[2][8], const FusedArgs &fa, const int32_t *s_starts,
                                              const ScoreGeom &gm, int g, int j0, int row, int hf, bool store) {
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int j_real = j0 + 32 * t + row;
    const int j = min(j_real, gm.n_ctx - 1);
    int lo = 0, hi = fa.n_chunks;  // s_starts[lo] <= j < s_starts[hi]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (s_starts[mid] <= j) lo = mid; else hi = mid;
    }
    const FusedChunk ch = fa.chunks[lo];
    const int64_t src = (static_cast<int64_t>(j - ch.dst_row) * gm.n_kv_heads + g) * D + 8 * hf;
    const int64_t dst = static_cast<int64_t>(j) * gm.token_stride + g * gm.head_stride + 8 * hf;
    const bool write = store && j_real < gm.n_ctx;
    v4u x[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) x[s] = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(ch.k + src + 16 * s));
    if (ch.v != nullptr && fa.v_out != nullptr && write) {
      v4u y[8];
#pragma unroll
      for (int s = 0; s < 8; ++s) y[s] = __builtin_nontemporal_load(reinterpret_cast<const v4u *>(ch.v + src + 16 * s));
#pragma unroll
      for (int s = 0; s < 8; ++s) __builtin_nontemporal_store(y[s], reinterpret_cast<v4u *>(fa.v_out + dst + 16 * s));
    }
    if (ch.rotate != 0) {
      const float4 *tb = reinterpret_cast<const float4 *>(fa.rot + lo * 128 + hf * 64);
      if (fa.pairing == IFKV_ROPE_HALF) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const float4 c0 = tb[4 * s], c1 = tb[4 * s + 1], s0 = tb[4 * s + 2], s1 = tb[4 * s + 3];
          const float cs[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
          const float sn[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
          float a[8], b[8], ra[8], rb[8];
          Elem<BF16Tag>::unpack(x[s], a);
          Elem<BF16Tag>::unpack(x[s + 4], b);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            ra[e] = fmaf(a[e], cs[e], -(b[e] * sn[e]));
            rb[e] = fmaf(a[e], sn[e], b[e] * cs[e]);
          }
          x[s] = Elem<BF16Tag>::pack(ra);
          x[s + 4] = Elem<BF16Tag>::pack(rb);
        }
      } else {
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          const float4 c0 = tb[2 * s], s0 = tb[2 * s + 1];
          const float cs[4] = {c0.x, c0.y, c0.z, c0.w};
          const float sn[4] = {s0.x, s0.y, s0.z, s0.w};
          float f[8], r[8];
          Elem<BF16Tag>::unpack(x[s], f);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            r[2 * e] = fmaf(f[2 * e], cs[e], -(f[2 * e + 1] * sn[e]));
            r[2 * e + 1] = fmaf(f[2 * e], sn[e], f[2 * e + 1] * cs[e]);
          }
          x[s] = Elem<BF16Tag>::pack(r);
        }
      }
    }
    if (write) {
#pragma unroll
      for (int s = 0; s < 8; ++s) __builtin_nontemporal_store(x[s], reinterpret_cast<v4u *>(fa.k_out + dst + 16 * s));
    }
#pragma unroll
    for (int s = 0; s < 8; ++s) kf[t][s] = __builtin_bit_cast(bf16x8, x[s]);
  }
}

// Query fragment s of 32-row block qb: lane (row, hf) holds columns 16 s + 8 hf .. +7 of row qb*32 + row.
__device__ __forceinline__ bf16x8 q_frag(const uint16_t *q_lds, int qb, int s, int row, int hf) {
  return __builtin_bit_cast(bf16x8,
                            *reinterpret_cast<const v4u *>(&q_lds[(qb * 32 + row) * QSTR + 16 * s + 8 * hf]));
}

// Contraction step s of one 32-query block against the 64-key tile in `kf`.
// KEYS_AS_ROWS selects the operand order: S^T = K.Q^T (pass A) or S = Q.K^T (pass B).
template <bool KEYS_AS_ROWS>
__device__ __forceinline__ void qk_step(f32x16 &S0, f32x16 &S1, const bf16x8 (&kf)[2][8], bf16x8 qf, int s) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (KEYS_AS_ROWS) {
    S0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0][s], qf, s == 0 ? zero : S0, 0, 0, 0);
    S1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[1][s], qf, s == 0 ? zero : S1, 0, 0, 0);
  } else {
    S0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[0][s], s == 0 ? zero : S0, 0, 0, 0);
    S1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[1][s], s == 0 ? zero : S1, 0, 0, 0);
  }
}

// The same, one MFMA at a time (t = 0: keys 0..31 of the tile, t = 1: keys 32..63).
template <bool KEYS_AS_ROWS>
__device__ __forceinline__ void qk_half_step(f32x16 &S, const bf16x8 (&kf)[2][8], bf16x8 qf, int s, int t) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (KEYS_AS_ROWS)
    S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t][s], qf, s == 0 ? zero : S, 0, 0, 0);
  else
    S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[t][s], s == 0 ? zero : S, 0, 0, 0);
}

// A whole block with nothing interleaved (pipeline prologue).
template <bool KEYS_AS_ROWS>
__device__ __forceinline__ void qk_block(f32x16 &S0, f32x16 &S1, const bf16x8 (&kf)[2][8], const uint16_t *q_lds,
                                         int qb, int row, int hf) {
#pragma unroll
  for (int s = 0; s < 8; ++s) qk_step<KEYS_AS_ROWS>(S0, S1, kf, q_frag(q_lds, qb, s, row, hf), s);
}

// ---------------------------------------------------------------------------
// pass A
// ---------------------------------------------------------------------------
// Pass A for blocks whose query rows fill NQB 32-row blocks (NQB even; rows past the real ones are
// zero in LDS and their statistics are never written).  NQB is a compile-time constant so that a
// tile is one straight run of code: the software pipeline below relies on scheduling fences, which
// order instructions only within a basic block.  With a run-time block count the compiler hoisted
// all MFMAs of a tile above the vector work of its first block and moved the vector work of one
// step behind the MFMAs of the next.
// FUSED: the keys come from the chunk caches through fused_k_frags (k_global is not read).
template <int NQB, bool FUSED>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(kWpe, kWpe))) void score_stats_mfma(
    const uint16_t *__restrict__ k_global, const uint16_t *__restrict__ q_prompt, ScoreGeom gm,
    float2 *__restrict__ partial, FusedArgs fa) {
  __shared__ __attribute__((aligned(16))) uint16_t q_lds[NQB * 32 * QSTR];
  __shared__ int32_t s_starts[FUSED ? kMaxFusedChunks : 1];
  const int kb = blockIdx.x;
  const int g = blockIdx.y / gm.n_qchunks;
  const int qc = blockIdx.y - g * gm.n_qchunks;
  const int G = gm.n_q_heads / gm.n_kv_heads;
  const int q_rows = min(gm.q_chunk_rows, gm.m_prompt * G - qc * gm.q_chunk_rows);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = lane & 31, hf = lane >> 5;

  const float c = gm.scale_log2;
  const int kv_begin = kb * gm.kv_per_block;
  const int kv_end = min(gm.n_ctx, kv_begin + gm.kv_per_block);
  if (FUSED) {  // the chunks' first rows, searched by every lane for its keys
    for (int i = threadIdx.x; i < fa.n_chunks; i += kThreads) s_starts[i] = fa.starts[i];
    __syncthreads();
  }
  auto next_keys = [&](bf16x8 (&dst)[2][8], int j) __attribute__((always_inline)) {
    if (FUSED)
      fused_k_frags(dst, fa, s_starts, gm, g, j, row, hf, qc == 0);
    else
      load_k_frags(dst, k_global, gm, g, j, row, hf);
  };
  // the query tile and the first key tile are requested together, before anything waits
  bf16x8 kf[2][8];
  int j0 = kv_begin + wave * kTile;
  {
    v4u qx[NQB];
    q_tile_request<NQB>(qx, q_prompt, gm, g, qc);
    if (j0 < kv_end) next_keys(kf, j0);
    q_tile_store<NQB>(q_lds, qx);
  }
  __syncthreads();

  // This lane's row in the lower and in the upper eight query blocks.  From one base the byte offsets
  // of the far blocks exceed the 16-bit immediate of an LDS read, and the compiler then keeps a
  // separate address register per fragment (22 of them, spilled); the empty asm hides that the
  // second base is a constant away from the first.
  typedef __attribute__((address_space(3))) const v4u lds_v4u;
  lds_v4u *q_lo = (lds_v4u *)(q_lds + row * QSTR + 8 * hf);
  lds_v4u *q_hi = (lds_v4u *)(q_lds + ((NQB > 8 ? 8 * 32 : 0) + row) * QSTR + 8 * hf);
  asm volatile("" : "+v"(q_hi));
  auto q_frag_a = [&](int qb, int s) {
    lds_v4u *base = qb < 8 ? q_lo : q_hi;
    return __builtin_bit_cast(bf16x8, base[((qb & 7) * 32 * QSTR + 16 * s) / 8]);
  };

  float m[NQB], z[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    m[qb] = -INFINITY;
    z[qb] = 0.f;
  }
  // register r of S_t: key j0 + 32 t + 8 (r/4) + 4 hf + r%4, query row qb*32 + (lane & 31)
  //
  // Software pipeline over the query blocks.  pipe_step issues the sixteen MFMAs of block qn into
  // (N0, N1) in eight slices of two; each slice is followed by a share of the vector work on the
  // finished block (C0, C1).  The fences keep the slices in this order, so the matrix pipe works
  // underneath the vector instructions of the same wavefront.  The last step of a tile issues one
  // block whose products are not used.  tail_tag (a compile-time tag, for the same reason as NQB)
  // selects the variant for a ragged last tile, which masks the keys past the end.
  //
  // Two variants of the vector work (exact_tag).  The sums only need SOME reference exponent per row
  // that keeps them inside the fp32 range, not the row maximum: the fast variant takes the logit of
  // the first key a lane sees for the row (always the logit of a real key, because the key loads
  // are clamped to the last key of the context) and keeps it for the whole sweep, which saves the
  // maximum over every tile and the rescaling: slice s handles four of the 32 values.  Sums that
  // leave [0, 2^60] (a logit more than 60 above the reference: attention far more peaked than
  // anything a model produces) make the block repeat its sweep with the exact variant, which keeps
  // a running maximum: slice 0 takes the maximum, slices 1..7 the exponentials and the sum.
  auto pipe_step = [&](auto tail_tag, auto exact_tag, f32x16 &N0, f32x16 &N1, int qn, f32x16 &C0, f32x16 &C1,
                       float &mq, float &zq, int j0, bool first) __attribute__((always_inline)) {
    constexpr bool kExact = decltype(exact_tag)::value;
    const float first_logit = C0[0];  // taken before the mask
    if (decltype(tail_tag)::value) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int kv = j0 + 8 * (r >> 2) + 4 * hf + (r & 3);
        if (kv >= kv_end) C0[r] = -INFINITY;
        if (kv + 32 >= kv_end) C1[r] = -INFINITY;
      }
    }
    float m_use = 0.f, m_new = 0.f, acc = 0.f;
    bf16x8 qf = q_frag_a(qn, 0);
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      bf16x8 qf_next = qf;
      if (s < 7) qf_next = q_frag_a(qn, s + 1);
      // The empty asm statements tie the vector work to its slice: they are ordered against the
      // fences, the values that pass through them cannot be formed earlier or used later, so the
      // instruction selector cannot collect the vector work of all slices behind the last MFMA.
      if (kExact) {
        qk_step<true>(N0, N1, kf, qf, s);
        if (s == 0) {
          float mx = C0[0];
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(fmaxf(mx, C0[r]), C1[r]);  // chain form: one v_max3 per pair
          m_new = fmaxf(mq, mx * c);
          m_use = fmaxf(m_new, -1e30f);  // a lane that has seen no valid key yet stays at (-inf, 0)
          asm volatile("" : "+v"(m_use));
        } else {
          // 32 values over seven slices: registers [lo, hi) of both halves
          const int lo = ((s - 1) * 16) / 7, hi = (s * 16) / 7;
          asm volatile("" : "+v"(m_use));
#pragma unroll
          for (int r = lo; r < hi; ++r) {
            acc += __builtin_amdgcn_exp2f(fmaf(C0[r], c, -m_use));
            acc += __builtin_amdgcn_exp2f(fmaf(C1[r], c, -m_use));
          }
          asm volatile("" : "+v"(acc));
        }
      } else {
        qk_step<true>(N0, N1, kf, qf, s);
        if (s == 0) m_use = first ? first_logit * c : mq;
        asm volatile("" : "+v"(m_use));
#pragma unroll
        for (int r = 2 * s; r < 2 * s + 2; ++r) {
          acc += __builtin_amdgcn_exp2f(fmaf(C0[r], c, -m_use));
          acc += __builtin_amdgcn_exp2f(fmaf(C1[r], c, -m_use));
        }
        asm volatile("" : "+v"(acc));
      }
      __builtin_amdgcn_sched_barrier(0);
      qf = qf_next;
    }
    if (kExact) {
      zq = zq * __builtin_amdgcn_exp2f(mq - m_use) + acc;
      mq = m_new;
    } else {
      zq += acc;
      mq = m_use;
    }
  };
  auto tile = [&](auto tail_tag, auto exact_tag, int j0, bool first) __attribute__((always_inline)) {
    f32x16 A0, A1, B0, B1;
#pragma unroll
    for (int s = 0; s < 8; ++s) qk_step<true>(A0, A1, kf, q_frag_a(0, s), s);  // block 0, nothing interleaved
#pragma unroll
    for (int qb = 0; qb < NQB; qb += 2) {
      pipe_step(tail_tag, exact_tag, B0, B1, qb + 1, A0, A1, m[qb], z[qb], j0, first);
      pipe_step(tail_tag, exact_tag, A0, A1, qb + 2 < NQB ? qb + 2 : NQB - 1, B0, B1, m[qb + 1], z[qb + 1], j0, first);
    }
  };
  const int j_first = j0;
  auto sweep = [&](auto exact_tag) __attribute__((always_inline)) {
    for (; j0 < kv_end; j0 += kWaves * kTile) {
      if (j0 + kTile > kv_end)
        tile(std::true_type{}, exact_tag, j0, j0 == j_first);
      else
        tile(std::false_type{}, exact_tag, j0, j0 == j_first);
      const int j_next = j0 + kWaves * kTile;
      if (j_next < kv_end) next_keys(kf, j_next);
    }
  };
  sweep(std::false_type{});
  {
    bool out_of_range = false;
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) out_of_range |= !(z[qb] <= 0x1p60f);  // also true for NaN
    if (__syncthreads_or(out_of_range ? 1 : 0)) {  // uniform over the block
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        m[qb] = -INFINITY;
        z[qb] = 0.f;
      }
      j0 = j_first;
      if (j0 < kv_end) next_keys(kf, j0);
      sweep(std::true_type{});
    }
  }
  // a lane half that saw no valid key, or whose terms all vanished against its reference, takes no part
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb)
    if (!(z[qb] > 0.f)) m[qb] = -INFINITY;

  // merge the two lane halves (same query row, disjoint keys), then the wavefronts
  __syncthreads();
  // every wavefront is done with the query tile: LDS is reused below
  float2 *w_stats = reinterpret_cast<float2 *>(q_lds);  // [kWaves][NQB * 32]
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const float mo = __shfl_xor(m[qb], 32, 64);
    const float zo = __shfl_xor(z[qb], 32, 64);
    const float mm = fmaxf(m[qb], mo);
    const float mu = fmaxf(mm, -1e30f);
    const float zz = z[qb] * __builtin_amdgcn_exp2f(m[qb] - mu) + zo * __builtin_amdgcn_exp2f(mo - mu);
    if (hf == 0) w_stats[wave * (NQB * 32) + qb * 32 + row] = make_float2(mm, zz);
  }
  __syncthreads();
  for (int ql = threadIdx.x; ql < q_rows; ql += kThreads) {
    float mm = -INFINITY, zz = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float2 p = w_stats[w * (NQB * 32) + ql];
      const float mn = fmaxf(mm, p.x);
      const float mu = fmaxf(mn, -1e30f);
      zz = zz * __builtin_amdgcn_exp2f(mm - mu) + p.y * __builtin_amdgcn_exp2f(p.x - mu);
      mm = mn;
    }
    int64_t off;
    int h, r;
    q_row_address(gm, g, qc, ql, &off, &h, &r);
    // natural-log domain, as the merge kernel expects
    const int64_t at = gm.partial_by_block
                           ? (static_cast<int64_t>(kb) * gridDim.y + blockIdx.y) * gm.q_chunk_rows + ql
                           : (static_cast<int64_t>(kb) * gm.n_q_heads + h) * gm.m_prompt + r;
    partial[at] = make_float2(mm * kLn2, zz);
  }
}

// ---------------------------------------------------------------------------
// pass B
// ---------------------------------------------------------------------------
// What pass B needs besides the keys and queries.  Either `stats` (final (max, 1/Z) per (head, prompt
// row), written by the merge kernel, which also folds in the prompt keys) or, when it is null, the
// per-slice partials of pass A, which every block merges for its own query rows while its first
// operands are on their way: one launch less.  The per-(kv head, query chunk) column sums go to
// `colpart`; the block that is the last of a key range to finish (counted in `arrived`, which reads
// zero between launches) adds them up in a fixed order and writes the scores: another launch less.
struct ColsumIo {
  const float2 *stats;
  const float2 *partial;
  int n_slices;
  float *colpart;
  int *arrived;     // [key ranges]
  float *scores;
  float inv_heads;
  int accumulate;
};

// The column sums travel between blocks that sit on different XCDs, whose L2s are not coherent with
// each other: they are written and read with device-scope relaxed atomics (write-through stores,
// loads that do not hit a stale line) instead of cache-wide write-backs and invalidations.
__device__ __forceinline__ void store_coherent(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_coherent(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Slices s0 .. s0 + kMergeBatch - 1 of one query row's partials (independent loads; a slice past the
// last one reads the last one again and is ignored by merge_partials).
constexpr int kMergeBatch = 32;
__device__ __forceinline__ void load_partials(float2 (&p)[kMergeBatch], const float2 *row, int slice_stride, int s0,
                                              int n_slices) {
#pragma unroll
  for (int u = 0; u < kMergeBatch; ++u) p[u] = row[min(s0 + u, n_slices - 1) * slice_stride];
}
// What the merge kernel computes, kMergeBatch slices at a time, with the hardware exponential (one
// instruction instead of a library call: 32 of those per row held every block up for 3 us).
__device__ __forceinline__ void merge_partials(const float2 (&p)[kMergeBatch], int s0, int n_slices, float &m, float &z) {
  float mn = m;
#pragma unroll
  for (int u = 0; u < kMergeBatch; ++u)
    if (s0 + u < n_slices && p[u].y > 0.f) mn = fmaxf(mn, p[u].x);
  if (mn > -INFINITY) {
    float acc = z * __builtin_amdgcn_exp2f((m - mn) * kLog2e);
#pragma unroll
    for (int u = 0; u < kMergeBatch; ++u) {
      const float w = s0 + u < n_slices && p[u].y > 0.f ? p[u].y : 0.f;
      acc += w * __builtin_amdgcn_exp2f(fminf(p[u].x - mn, 0.f) * kLog2e);
    }
    z = acc;
    m = mn;
  }
}

__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(kWpe, kWpe))) void score_colsum_mfma(
    const uint16_t *__restrict__ k_global, const uint16_t *__restrict__ q_prompt, ScoreGeom gm, ColsumIo io) {
  __shared__ __attribute__((aligned(16))) uint16_t q_lds[kQChunk * QSTR];
  __shared__ __attribute__((aligned(16))) float b_lds[kQChunk];
  __shared__ int s_last;
  float *const colpart = io.colpart;
  const int G = gm.n_q_heads / gm.n_kv_heads;
  const int kb = blockIdx.x;
  const int g = blockIdx.y / gm.n_qchunks;
  const int qc = blockIdx.y - g * gm.n_qchunks;
  const int q_total = gm.m_prompt * G;
  const int q_rows = min(gm.q_chunk_rows, q_total - qc * gm.q_chunk_rows);
  const int nqb = ((q_rows + 63) >> 6) << 1;  // 32-row query blocks, padded to an even count
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = lane & 31, hf = lane >> 5;
  const float c = gm.scale_log2;
  const int kv_begin = kb * gm.kv_per_block;
  const int kv_end = min(gm.n_ctx, kv_begin + gm.kv_per_block);
  // the query tile and the first key tile are requested together, before anything waits
  bf16x8 kf[2][8];
  int j0 = kv_begin + wave * kTile;
  // This thread's query row (a chunk holds at most kThreads rows).  When the block merges the
  // per-slice partials itself, the first kMergeBatch of them are requested first (they come from
  // memory: other blocks wrote them in the previous launch), then the query tile and the first key
  // tile, and the merge arithmetic runs while the key tile is on its way.
  static_assert(kQChunk <= kThreads, "one query row per thread");
  const int ql = threadIdx.x;
  const bool merge_here = io.stats == nullptr;
  auto my_partials = [&]() __attribute__((always_inline)) {
    return io.partial + blockIdx.y * gm.q_chunk_rows + min(ql, gm.q_chunk_rows - 1);
  };
  const int slice_stride = static_cast<int>(gridDim.y) * gm.q_chunk_rows;  // at most 256 blocks of 512 rows
  auto softmax_offsets = [&](const float2 (&part)[kMergeBatch]) __attribute__((always_inline)) {
    if (ql < nqb * 32) {
      int64_t off;
      int h, r;
      float b = INFINITY;  // padded rows contribute exp2(-inf) = 0
      if (q_row_address(gm, g, qc, ql, &off, &h, &r)) {
        float2 st;  // (max, 1/Z), natural-log domain
        if (!merge_here) {
          st = io.stats[h * gm.m_prompt + r];
        } else {
          float m = -INFINITY, z = 0.f;
          merge_partials(part, 0, io.n_slices, m, z);
          for (int s0 = kMergeBatch; s0 < io.n_slices; s0 += kMergeBatch) {
            float2 more[kMergeBatch];
            load_partials(more, my_partials(), slice_stride, s0, io.n_slices);
            merge_partials(more, s0, io.n_slices, m, z);
          }
          st = make_float2(m, z > 0.f ? 1.f / z : 0.f);
        }
        b = st.y > 0.f ? st.x * kLog2e - __log2f(st.y) : INFINITY;
      }
      b_lds[ql] = b;
    }
  };
  auto stage_q = [&](auto nv_tag) __attribute__((always_inline)) {
    constexpr int NV = decltype(nv_tag)::value;
    float2 part[kMergeBatch];
    if (merge_here) load_partials(part, my_partials(), slice_stride, 0, io.n_slices);
    v4u qx[NV];
    q_tile_request<NV>(qx, q_prompt, gm, g, qc);
    if (j0 < kv_end) load_k_frags(kf, k_global, gm, g, j0, row, hf);
    q_tile_store<NV>(q_lds, qx);  // the query tile arrives before the key tile
    softmax_offsets(part);
  };
  switch (gm.q_chunk_rows >> 7) {  // uniform over the grid
    case 1: stage_q(std::integral_constant<int, 4>{}); break;
    case 2: stage_q(std::integral_constant<int, 8>{}); break;
    case 3: stage_q(std::integral_constant<int, 12>{}); break;
    default: stage_q(std::integral_constant<int, 16>{}); break;
  }
  __syncthreads();

  float *dst = colpart + static_cast<int64_t>(blockIdx.y) * gm.n_ctx;
  // register r of S_t: query row qb*32 + 8 (r/4) + 4 hf + r%4, key j0 + 32 t + (lane & 31)
  //
  // Software pipeline over the query blocks (their count is even).  pipe_step issues the sixteen
  // MFMAs of block qn into (N0, N1) in eight slices of two; each slice is followed by the
  // exponentials of four values of the finished block qc in (C0, C1).  The fences keep the slices
  // in this order, so the matrix pipe works underneath the vector instructions of the same
  // wavefront.  The last step of a tile issues one block whose products are not used.
  // qf is a ring of four query fragments: on entry it holds contraction steps 0..2 of block qn;
  // step s requests the fragment three steps ahead (of block qn, then of the block after it, qn2),
  // so an LDS read has three slices of work to hide behind.  bn receives the softmax offsets of
  // block qn, which the next call consumes as bc.
  auto pipe_step = [&](const bf16x8 (&kf)[2][8], bf16x8 (&qf)[4], f32x16 &N0, f32x16 &N1, int qn, int qn2,
                       const f32x16 &C0, const f32x16 &C1, const f32x4 (&bc)[4], f32x4 (&bn)[4], float &col0,
                       float &col1) __attribute__((always_inline)) {
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      qf[(s + 3) & 3] = s + 3 < 8 ? q_frag(q_lds, qn, s + 3, row, hf) : q_frag(q_lds, qn2, s + 3 - 8, row, hf);
      if ((s & 1) == 0) bn[s >> 1] = *reinterpret_cast<const f32x4 *>(&b_lds[qn * 32 + 8 * (s >> 1) + 4 * hf]);
      // MFMA, two values, MFMA, two values: each MFMA finds the matrix pipe free
      qk_half_step<false>(N0, kf, qf[s & 3], s, 0);
      __builtin_amdgcn_sched_barrier(0);
      {
        const int e = 2 * (s & 1);
        col0 += __builtin_amdgcn_exp2f(fmaf(C0[4 * (s >> 1) + e], c, -bc[s >> 1][e]));
        col1 += __builtin_amdgcn_exp2f(fmaf(C1[4 * (s >> 1) + e], c, -bc[s >> 1][e]));
      }
      __builtin_amdgcn_sched_barrier(0);
      qk_half_step<false>(N1, kf, qf[s & 3], s, 1);
      __builtin_amdgcn_sched_barrier(0);
      {
        const int e = 2 * (s & 1) + 1;
        col0 += __builtin_amdgcn_exp2f(fmaf(C0[4 * (s >> 1) + e], c, -bc[s >> 1][e]));
        col1 += __builtin_amdgcn_exp2f(fmaf(C1[4 * (s >> 1) + e], c, -bc[s >> 1][e]));
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  for (; j0 < kv_end; j0 += kWaves * kTile) {
    // the next tile's fragments travel while this one is processed
    bf16x8 kf_next[2][8];
    const int j_next = j0 + kWaves * kTile;
    if (j_next < kv_end) load_k_frags(kf_next, k_global, gm, g, j_next, row, hf);
    float col0 = 0.f, col1 = 0.f;
    f32x16 A0, A1, B0, B1;
    f32x4 ba[4], bb[4];
    bf16x8 qf[4];
    qk_block<false>(A0, A1, kf, q_lds, 0, row, hf);
#pragma unroll
    for (int ri = 0; ri < 4; ++ri) ba[ri] = *reinterpret_cast<const f32x4 *>(&b_lds[8 * ri + 4 * hf]);
#pragma unroll
    for (int s = 0; s < 3; ++s) qf[s] = q_frag(q_lds, 1, s, row, hf);
    for (int qb = 0; qb < nqb; qb += 2) {
      const int q2 = min(qb + 2, nqb - 1), q3 = min(qb + 3, nqb - 1);
      pipe_step(kf, qf, B0, B1, qb + 1, q2, A0, A1, ba, bb, col0, col1);
      pipe_step(kf, qf, A0, A1, q2, q3, B0, B1, bb, ba, col0, col1);
    }
    if (j_next < kv_end) {
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int s2 = 0; s2 < 8; ++s2) kf[t][s2] = kf_next[t][s2];
    }
    col0 += __shfl_xor(col0, 32, 64);
    col1 += __shfl_xor(col1, 32, 64);
    if (hf == 0) {
      if (j0 + row < kv_end) store_coherent(&dst[j0 + row], col0);
      if (j0 + 32 + row < kv_end) store_coherent(&dst[j0 + 32 + row], col1);
    }
  }
  // This block's column sums have reached memory when its stores have completed; the block that
  // completes the count of its key range adds up all partials of the range.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  if (threadIdx.x == 0) {
    const int n_parts = static_cast<int>(gridDim.y);
    const int done = __hip_atomic_fetch_add(&io.arrived[kb], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1;
    s_last = done == n_parts ? 1 : 0;
    if (done == n_parts) __hip_atomic_store(&io.arrived[kb], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  if (s_last != 0) {
    const int n_parts = static_cast<int>(gridDim.y);
    for (int j = kv_begin + threadIdx.x; j < kv_end; j += kThreads) {
      float sum = 0.f;
      for (int p = 0; p < n_parts; ++p) sum += load_coherent(&colpart[static_cast<int64_t>(p) * gm.n_ctx + j]);
      sum *= io.inv_heads;
      io.scores[j] = io.accumulate ? io.scores[j] + sum : sum;
    }
  }
}

}  // namespace

bool score_mfma_supported(const ifkv_ctx *ctx, int m_prompt) {
  const auto &d = ctx->desc;
  const int G = d.n_q_heads / d.n_kv_heads;
  return d.dtype == IFKV_BF16 && d.head_dim == D && m_prompt > 0 &&
         static_cast<int64_t>(m_prompt) * G <= static_cast<int64_t>(kMaxQChunks) * kQChunk;
}

bool fused_repo_score_supported(const ifkv_ctx *ctx, int m_prompt, int n_chunks) {
  return ctx->tune.fused_repo_score != 0 && !(ctx->desc.flags & IFKV_FLAG_FORCE_GENERIC) && score_mfma_supported(ctx, m_prompt) && n_chunks >= 1 &&
         n_chunks <= kFusedMaxChunks;
}

hipError_t launch_score_mfma_passes(ifkv_ctx *ctx, const void *k_global, int64_t n_ctx, const void *q_prompt,
                                    int m_prompt, int *n_slices_out, bool pass_b, int accumulate, float *scores,
                                    const FusedRepo *fused, bool merged_stats) {
  // merged_stats: the merge kernel runs between the sweeps (both calls of a pair pass the same value)
  static_assert(kMaxFusedChunks == kFusedMaxChunks, "one limit");
  static_assert(sizeof(FusedChunk) <= 32, "descriptor slot");
  const auto &d = ctx->desc;
  const int G = d.n_q_heads / d.n_kv_heads;
  ScoreGeom gm;
  gm.n_ctx = static_cast<int>(n_ctx);
  gm.m_prompt = m_prompt;
  gm.n_q_heads = d.n_q_heads;
  gm.n_kv_heads = d.n_kv_heads;
  gm.token_stride = ctx->token_stride;
  gm.head_stride = ctx->head_stride;
  // query rows of a kv head are cut into equal chunks of a multiple of 128 rows (pass A is compiled
  // for 4, 8, 12 and 16 blocks of 32 rows)
  gm.n_qchunks = (m_prompt * G + kQChunk - 1) / kQChunk;
  gm.q_chunk_rows = ((m_prompt * G + gm.n_qchunks - 1) / gm.n_qchunks + 127) / 128 * 128;
  gm.scale_log2 = ctx->sm_scale * kLog2e;
  gm.partial_by_block = merged_stats ? 0 : 1;
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
    const auto *kg = static_cast<const uint16_t *>(k_global);
    const auto *qp = static_cast<const uint16_t *>(q_prompt);
    FusedArgs fa = {};
    if (fused != nullptr) {
      // the chunk table, the first rows and the rotation table reach the device through the
      // arguments of small kernels (64 chunks each): no staging copy, no host sync
      char *fb = base + sc.fused_off;
      FusedChunk *d_chunks = reinterpret_cast<FusedChunk *>(fb);
      int32_t *d_starts = reinterpret_cast<int32_t *>(fb + kFusedMaxChunks * 32);
      float *d_rot = reinterpret_cast<float *>(fb + kFusedMaxChunks * 36);
      for (int b0 = 0; b0 < fused->n_chunks; b0 += 64) {
        FusedTableBatch tb;
        tb.n = std::min(64, fused->n_chunks - b0);
        tb.base = b0;
        for (int i = 0; i < tb.n; ++i) {
          const FusedHostChunk &hc = fused->chunks[b0 + i];
          tb.c[i].k = static_cast<const uint16_t *>(hc.k);
          tb.c[i].v = static_cast<const uint16_t *>(hc.v);
          tb.c[i].dst_row = static_cast<int32_t>(hc.dst_row);
          tb.c[i].rotate = hc.advance != 0.0 ? 1 : 0;
          tb.advance[i] = hc.advance;
        }
        hipLaunchKernelGGL(fused_table_kernel, dim3(tb.n), dim3(64), 0, ctx->stream, tb, ctx->d_inv_freq, d_chunks,
                           d_starts, d_rot, static_cast<int>(d.pairing));
      }
      fa.chunks = d_chunks;
      fa.starts = d_starts;
      fa.rot = d_rot;
      fa.k_out = static_cast<uint16_t *>(fused->k_out);
      fa.v_out = static_cast<uint16_t *>(fused->v_out);
      fa.n_chunks = fused->n_chunks;
      fa.pairing = d.pairing;
    }
#define IFKV_LAUNCH_STATS(NQB)                                                                                          \
  do {                                                                                                                  \
    if (fused != nullptr)                                                                                               \
      hipLaunchKernelGGL((score_stats_mfma<NQB, true>), grid, dim3(kThreads), 0, ctx->stream, kg, qp, gm, partial, fa); \
    else                                                                                                                \
      hipLaunchKernelGGL((score_stats_mfma<NQB, false>), grid, dim3(kThreads), 0, ctx->stream, kg, qp, gm, partial, fa); \
  } while (0)
    switch (gm.q_chunk_rows / 128) {
      case 1: IFKV_LAUNCH_STATS(4); break;
      case 2: IFKV_LAUNCH_STATS(8); break;
      case 3: IFKV_LAUNCH_STATS(12); break;
      default: IFKV_LAUNCH_STATS(16); break;
    }
#undef IFKV_LAUNCH_STATS
  } else {
    if (ctx->score_arrived == nullptr || kv_blocks > kScoreMaxKeyRanges) return hipErrorInvalidValue;
    ColsumIo io;
    io.stats = merged_stats ? stats : nullptr;
    io.partial = partial;
    io.n_slices = kv_blocks;
    io.colpart = colpart;
    io.arrived = ctx->score_arrived;
    io.scores = scores;
    io.inv_heads = 1.0f / d.n_q_heads;
    io.accumulate = accumulate;
    hipLaunchKernelGGL(score_colsum_mfma, grid, dim3(kThreads), 0, ctx->stream,
                       static_cast<const uint16_t *>(k_global), static_cast<const uint16_t *>(q_prompt), gm, io);
  }
  return hipGetLastError();
}

}  // namespace ifkv
