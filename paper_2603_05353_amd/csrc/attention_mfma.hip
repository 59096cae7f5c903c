// Stage 4, bf16 MFMA kernels -- "KV Recomputation": each selected row attends
// causally to cache rows 0..p_r of the concatenated sequence.
//
// Shape of the problem: few, scattered query rows (k = rho N of them) against a
// long, dense K/V prefix.  The kernels therefore pack the G query heads that
// share a kv head together with a block of consecutive selected rows into one
// tile of NWAVES*32 "query columns", so that every K/V tile fetched from HBM/L2
// is used by all of them, and walk the kv axis in tiles of 64 rows with an
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
// Staging uses the gfx950 direct global->LDS loads (16 bytes per lane, no registers, no VALU) and
// keeps NS tiles in an LDS ring.  K rows land in sigma order with their 16-byte chunks XOR-swizzled
// by the row index, so the A-operand reads (32 rows, one chunk) hit distinct banks.  V lands
// row-major, swizzled by the row within each group of four rows, and the A operand of the second
// product -- which needs eight kv values of one d column per lane, the strided axis -- is read
// with the LDS transpose loads (ds_read_b64_tr_b16), two per operand.
//
// attn_mfma_kernel<4, 2>: 128 query columns per block, two LDS stages (64 KiB), two blocks per CU --
// the default.  The two wavefronts that share a SIMD then belong to different blocks and are not
// tied together by barriers.  (An 8-wavefront, three-stage instantiation with 256 query columns and
// half the K/V traffic per flop measured within 2 % of it and is not built.)
#include <cstdlib>

#include "attention_common.h"
#include "ifkv_device.h"

namespace ifkv {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int D = 128;        // head_dim served by these kernels
constexpr int TK = 64;        // kv rows per tile
constexpr int TILE_ELEMS = TK * D;  // one K or V tile in LDS: 64 rows x 256 B, no padding (swizzled instead)
// The running max is only raised (and O, l rescaled) when a new tile exceeds it by more than
// this many powers of two, so probabilities stay <= 2^kSlack: exact in fp32 sums and harmless
// for the bf16 rounding, and the 64-register rescale becomes rare.
constexpr float kSlack = 8.f;

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);  // round-to-nearest-even
  return __builtin_bit_cast(uint32_t, r);
}

// Order in which K rows are fed as MFMA A-rows.  A 32x32 accumulator gives lane
// half hf, register r the A-row 8*(r/4) + 4*hf + r%4; feeding kv row sigma(i) as
// A-row i makes registers 0..7 of a lane hold kv rows 8*hf + 0..7 and registers
// 8..15 hold kv rows 16 + 8*hf + 0..7, i.e. eight consecutive kv rows per
// 16-row contraction step, which is what the B operand of V^T.P^T needs.
// sigma swaps bits 2 and 3 (an involution); K rows are stored in LDS at row
// sigma(j), so A-row i simply reads LDS row i.
__device__ __forceinline__ int sigma(int i) { return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1); }

// max of a value with the one held by the lane 32 positions away (the other half of the same
// query column): one lane-half swap in the vector ALU instead of a round trip through LDS.
__device__ __forceinline__ float half_swap_max(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Everything one wavefront carries through the kv loop.
struct WaveState {
  f32x16 O[4];   // O^T accumulator, 128 d x 32 q
  float m_run;   // reference max of the scaled logits (log2 domain); may lag the true max by <= kSlack
  float l_run;   // this lane's share of the running sum
};

// Per-lane LDS read offsets (in elements) that do not change from tile to tile.
struct ReadOffsets {
  int k[8];  // K A-operand, contraction step s: row (lane & 31), chunk (2 s + hf) ^ (row & 15)
  int v[4];  // V transpose read, d tile dt (see pv_tile)
};

__device__ __forceinline__ ReadOffsets make_read_offsets(int lane) {
  ReadOffsets o;
  const int col = lane & 31, hf = lane >> 5;
#pragma unroll
  for (int s = 0; s < 8; ++s) o.k[s] = col * D + (((2 * s + hf) ^ (col & 15)) << 3);
  // transpose read: in every group of 16 lanes, lane j supplies row j / 4, d columns 4 (j % 4)..+3
  // (8 bytes) and receives the four rows of d column j.  Group g covers d columns 16 (g & 1)..+15
  // of the 32-column d tile; hf = g / 2 selects kv rows +8.
  const int g = lane >> 4, j = lane & 15;
  const int r = j >> 2;
  const int low = 2 * (g & 1) + ((j & 3) >> 1);  // 16-byte chunk within the d tile's four chunks
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
    o.v[dt] = (2 * hf) * 512 + ((16 * r + ((4 * dt + low) ^ (4 * r))) << 3) + 4 * (j & 1);
  return o;
}

// S^T = K_tile . Q^T for one 64-row tile held in LDS stage `k_stage`.  An MFMA takes 32 cycles, an
// LDS read returns after a few hundred when eight wavefronts share the LDS, so the A operands are
// requested four contraction steps (eight reads) ahead of their use; the fences keep the
// compiler from sinking the reads back next to their consumers.
__device__ __forceinline__ void qk_tile(f32x16 (&S)[2], const uint16_t *k_stage, const bf16x8 (&qf)[8],
                                        const ReadOffsets &ro) {
  v4u ka[8], kb[8];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    ka[s] = *reinterpret_cast<const v4u *>(&k_stage[ro.k[s]]);
    kb[s] = *reinterpret_cast<const v4u *>(&k_stage[ro.k[s] + 32 * D]);
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    S[0][r] = 0.f;
    S[1][r] = 0.f;
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    S[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ka[s]), qf[s], S[0], 0, 0, 0);
    S[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kb[s]), qf[s], S[1], 0, 0, 0);
    if (s + 4 < 8) {
      ka[s + 4] = *reinterpret_cast<const v4u *>(&k_stage[ro.k[s + 4]]);
      kb[s + 4] = *reinterpret_cast<const v4u *>(&k_stage[ro.k[s + 4] + 32 * D]);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Causal mask (only on tiles that reach past the wavefront's smallest position), row max, and
// the lazy update of the reference max with the rescale of O and l it implies.
// Register r of S[t] is kv row j0 + 32 t + 16 (r / 8) + 8 hf + r % 8.
__device__ __forceinline__ void row_stats(f32x16 (&S)[2], WaveState &w, int j0, int p_q, int p_wmin, int hf,
                                          float scale_log2) {
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
  mx = half_swap_max(mx);
  const float m_new = fmaxf(w.m_run, mx * scale_log2);
  if (__any(m_new > w.m_run + kSlack)) {
    const float alpha = __builtin_amdgcn_exp2f(w.m_run - m_new);  // 0 on the first tile (m_run = -inf)
    w.l_run *= alpha;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) w.O[dt][r] *= alpha;
    w.m_run = m_new;
  }
}

// P^T of one tile, rounded to bf16 and packed as the four B operands of the second product.
struct PTile {
  v4u step[4];  // contraction step u: kv rows 16 u + 8 hf + 0..7 of this lane's query column
};

// P^T = exp2(S^T c - m) and l += sum P (fp32, before rounding).
__device__ __forceinline__ void exp_tile(f32x16 (&S)[2], WaveState &w, PTile &P, float scale_log2) {
  float psum[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      S[t][r] = __builtin_amdgcn_exp2f(fmaf(S[t][r], scale_log2, -w.m_run));
      psum[r & 3] += S[t][r];
    }
  w.l_run += (psum[0] + psum[1]) + (psum[2] + psum[3]);
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int t = u >> 1, r0 = 8 * (u & 1);
    P.step[u][0] = pack_bf16x2(S[t][r0 + 0], S[t][r0 + 1]);
    P.step[u][1] = pack_bf16x2(S[t][r0 + 2], S[t][r0 + 3]);
    P.step[u][2] = pack_bf16x2(S[t][r0 + 4], S[t][r0 + 5]);
    P.step[u][3] = pack_bf16x2(S[t][r0 + 6], S[t][r0 + 7]);
  }
}

// O^T += V_tile^T . P^T.  The A operand of contraction step u, d tile dt is lane (d = 32 dt + lane % 32)
// x kv rows 16 u + 8 hf + 0..7: two transpose reads of four rows each from the row-major V tile.
// The sixteen operands are numbered x = 4 u + dt and requested four ahead; the first four are
// requested by pv_preload, which the caller places before the exponentials (they do not depend on
// them), so that they arrive while the vector ALU is busy.
struct VFrags {
  s16x4 lo[4], hi[4];
};
__device__ __forceinline__ void v_read(s16x4 &lo, s16x4 &hi, const uint16_t *v_stage, const ReadOffsets &ro, int x) {
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  const uint16_t *p = v_stage + ro.v[x & 3] + (4 * (x >> 2)) * 512;  // 4-row groups 4 u + 2 hf (+1)
  lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
  hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 512));
}
__device__ __forceinline__ void pv_preload(VFrags &f, const uint16_t *v_stage, const ReadOffsets &ro) {
#pragma unroll
  for (int x = 0; x < 4; ++x) v_read(f.lo[x], f.hi[x], v_stage, ro, x);
}
__device__ __forceinline__ void pv_tile(const PTile &P, VFrags &f, WaveState &w, const uint16_t *v_stage,
                                        const ReadOffsets &ro) {
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int x = 0; x < 16; ++x) {
    const int u = x >> 2, dt = x & 3;
    const s16x8 a = __builtin_shufflevector(f.lo[x & 3], f.hi[x & 3], 0, 1, 2, 3, 4, 5, 6, 7);
    w.O[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                      __builtin_bit_cast(bf16x8, P.step[u]), w.O[dt], 0, 0, 0);
    if (x + 4 < 16) v_read(f.lo[x & 3], f.hi[x & 3], v_stage, ro, x + 4);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Direct global->LDS staging of one kv tile.  A load instruction moves 64 x 16 bytes: lane L's
// 16 bytes land at the instruction's LDS base + 16 L, whatever global address the lane names, so
// a "unit" of 1 KiB = four 256-byte tile rows is filled per instruction and the lanes choose which
// chunk goes where.  K unit q: LDS rows 4q..4q+3 hold kv rows sigma(4q..4q+3); position c of a row
// holds chunk c ^ (row & 15).  V unit q: kv rows 4q..4q+3; position c of row r holds chunk c ^ 4r.
//
// The load is emitted as inline assembly (M0 = LDS base of the instruction, then the load).  The
// compiler's own builtin works, but it cannot tell which LDS stage such a load writes and so
// waits for ALL outstanding loads before every later LDS read, which serialises the look-ahead.
// Ordering is done by hand instead: a vmcnt wait plus a barrier before a stage is read.
__device__ __forceinline__ uint32_t lds_address(const void *p) {
  return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const void *)p));
}
// per-lane 64-bit global address; lds_dst: wavefront-uniform LDS byte address of the instruction
__device__ __forceinline__ void dma16(const void *global_src, uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(global_src), "s"(lds_dst) : "memory");
}
// wavefront-uniform 64-bit base + per-lane 32-bit byte offset
__device__ __forceinline__ void dma16_base(const void *uniform_base, uint32_t lane_offset, uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_offset), "s"(uniform_base), "s"(lds_dst)
               : "memory");
}

template <int NWAVES>
struct Dma {
  static constexpr int UPW = 16 / NWAVES;   // units per wavefront and matrix (2 or 4)
  static constexpr int PER_TILE = 2 * UPW;  // load instructions a wavefront issues per tile
};

// What a lane fetches for each of its units, as byte offsets from the tile's first row: fixed for
// the whole kernel, so a tile that lies fully inside the cache costs one scalar base update and
// PER_TILE load instructions, no vector arithmetic.
template <int NWAVES>
struct DmaPlan {
  uint32_t k_off[Dma<NWAVES>::UPW];
  uint32_t v_off[Dma<NWAVES>::UPW];
};

template <int NWAVES>
__device__ __forceinline__ DmaPlan<NWAVES> make_dma_plan(int64_t kv_row_elems) {
  DmaPlan<NWAVES> pl;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane >> 4, cpos = lane & 15;
  const uint32_t row_bytes = static_cast<uint32_t>(kv_row_elems) * 2u;
#pragma unroll
  for (int x = 0; x < Dma<NWAVES>::UPW; ++x) {
    const int i = 4 * (wave * Dma<NWAVES>::UPW + x) + r;  // LDS row
    pl.k_off[x] = sigma(i) * row_bytes + 16u * (cpos ^ (i & 15));
    pl.v_off[x] = i * row_bytes + 16u * (cpos ^ (4 * r));
  }
  return pl;
}

// k_stage / v_stage: wavefront-uniform LDS byte addresses of the stage to fill (plain integers, so
// the per-instruction LDS base is scalar arithmetic and costs no vector instruction)
template <int NWAVES>
__device__ __forceinline__ void issue_tile_dma(const DmaPlan<NWAVES> &pl, uint32_t k_stage, uint32_t v_stage,
                                               const uint16_t *k_base, const uint16_t *v_base, int64_t kv_row_elems,
                                               int tile, int n_kv) {
  const uint32_t unit0 = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6) * Dma<NWAVES>::UPW;
  int j0 = tile * TK;
  const bool partial = (j0 < n_kv && j0 + TK > n_kv) || n_kv < TK;
  if (!partial) {
    if (j0 >= n_kv) j0 = 0;  // look-ahead past the end: fetch any valid tile, it is never read
    const uint16_t *kb = k_base + j0 * kv_row_elems;
    const uint16_t *vb = v_base + j0 * kv_row_elems;
#pragma unroll
    for (int x = 0; x < Dma<NWAVES>::UPW; ++x) {
      dma16_base(kb, pl.k_off[x], k_stage + (unit0 + x) * 1024u);
      dma16_base(vb, pl.v_off[x], v_stage + (unit0 + x) * 1024u);
    }
  } else {
    // the one tile that straddles the end of the cache: rows past the end are clamped (and masked later)
    const int lane = threadIdx.x & 63;
    const int r = lane >> 4, cpos = lane & 15;
#pragma unroll
    for (int x = 0; x < Dma<NWAVES>::UPW; ++x) {
      const uint32_t unit = unit0 + x;
      const int i = 4 * unit + r;
      const int jk = min(j0 + sigma(i), n_kv - 1);
      const int jv = min(j0 + i, n_kv - 1);
      dma16(k_base + jk * kv_row_elems + 8 * (cpos ^ (i & 15)), k_stage + unit * 1024u);
      dma16(v_base + jv * kv_row_elems + 8 * (cpos ^ (4 * r)), v_stage + unit * 1024u);
    }
  }
}

// Per-lane query column set-up shared by both kernels.
struct Column {
  int row, hh, p_q, p_wmax, p_wmin;
  bool col_valid, in_range;
  int64_t q_off;
};

// qc: this lane's query column within the block (columns are numbered row-major over (row, head in group)).
__device__ __forceinline__ Column setup_column(const int32_t *__restrict__ row_pos, int n_rows, int n_kv, int row0,
                                               int rows_per_block, int G, int g, int n_q_heads, int qc) {
  Column c;
  const int rr = qc / G;
  c.hh = qc - rr * G;
  c.row = row0 + rr;
  c.col_valid = (rr < rows_per_block) && (c.row < n_rows);
  // Loads are unconditional on a clamped row (then zeroed): no divergent control flow before
  // the main loop, so no memory operation is still pending on a side path when it is entered.
  const int row_c = min(c.row, n_rows - 1);
  const int p_ld = row_pos[row_c];
  c.in_range = c.col_valid && (p_ld >= 0) && (p_ld < n_kv);
  c.p_q = c.in_range ? p_ld : 0;
  c.q_off = (static_cast<int64_t>(row_c) * n_q_heads + g * G + c.hh) * D;
  int p_wmax = c.p_q, p_wmin = c.col_valid ? c.p_q : 0x7FFFFFFF;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    p_wmax = max(p_wmax, __shfl_xor(p_wmax, o, 64));
    p_wmin = min(p_wmin, __shfl_xor(p_wmin, o, 64));
  }
  c.p_wmax = __builtin_amdgcn_readfirstlane(p_wmax);
  c.p_wmin = __builtin_amdgcn_readfirstlane(p_wmin);
  return c;
}

__device__ __forceinline__ void load_q_frags(bf16x8 (&qf)[8], const uint16_t *__restrict__ q_sel, const Column &c,
                                             int hf) {
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    v4u x = *reinterpret_cast<const v4u *>(q_sel + c.q_off + 16 * s + 8 * hf);
    if (!c.col_valid) x = v4u{0u, 0u, 0u, 0u};
    qf[s] = __builtin_bit_cast(bf16x8, x);
  }
}

__device__ __forceinline__ void write_output(const WaveState &w, const Column &c, uint16_t *__restrict__ out,
                                             float *__restrict__ lse_out, int n_q_heads, int g, int G, int hf) {
  if (!c.col_valid) return;
  const float l_tot = w.l_run + __shfl_xor(w.l_run, 32, 64);
  const float inv = c.in_range ? 1.f / l_tot : 0.f;
  uint16_t *orow = out + c.q_off;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int ri = 0; ri < 4; ++ri) {
      uint2 x;
      x.x = pack_bf16x2(w.O[dt][4 * ri + 0] * inv, w.O[dt][4 * ri + 1] * inv);
      x.y = pack_bf16x2(w.O[dt][4 * ri + 2] * inv, w.O[dt][4 * ri + 3] * inv);
      *reinterpret_cast<uint2 *>(orow + 32 * dt + 8 * ri + 4 * hf) = x;
    }
  if (lse_out != nullptr && hf == 0)
    lse_out[static_cast<int64_t>(c.row) * n_q_heads + g * G + c.hh] =
        c.in_range ? 0.6931471805599453f * (w.m_run + __log2f(l_tot)) : 0.f;
}

template <int NWAVES>
__device__ __forceinline__ int block_tiles(int p_wmax, int *s_pmax) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) s_pmax[wave] = p_wmax;
  __syncthreads();
  int p_bmax = 0;
#pragma unroll
  for (int w = 0; w < NWAVES; ++w) p_bmax = max(p_bmax, s_pmax[w]);
  return p_bmax / TK + 1;
}

// ---------------------------------------------------------------------------
// Split over the kv axis.  Row blocks differ in length by two orders of magnitude (a row at
// position p costs p keys), and a launch has only a few blocks per CU, so the longest blocks set
// the finish time.  With `part_tiles` < the tile count of a row block, the block's kv range is
// divided into parts of part_tiles tiles, one workgroup each (blockIdx.z); each part keeps its own
// running (max, sum) and unnormalised O and writes them to scratch, and attn_combine_kernel merges
// the parts of every row that was split.  Row blocks that fit in one part write their output
// directly, as without the split.
// ---------------------------------------------------------------------------
struct SplitPlan {
  int part_tiles;     // kv tiles per part (>= number of tiles of the cache: no split)
  float *o_part;      // [parts][n_rows][H_q][D] unnormalised O
  float2 *ml_part;    // [parts][n_rows][H_q] (reference max in the log2 domain, sum)
  int *block_tiles;   // [row blocks] tile count of each row block (written by part 0)
};

__device__ __forceinline__ void write_partial(const WaveState &w, const Column &c, const SplitPlan &sp, int part,
                                              int n_rows, int n_q_heads, int g, int G, int hf) {
  if (!c.col_valid) return;
  const float l_tot = w.l_run + __shfl_xor(w.l_run, 32, 64);
  const int64_t slot = (static_cast<int64_t>(part) * n_rows + c.row) * n_q_heads + g * G + c.hh;
  float *orow = sp.o_part + slot * D;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int ri = 0; ri < 4; ++ri) {
      float4 x = make_float4(w.O[dt][4 * ri + 0], w.O[dt][4 * ri + 1], w.O[dt][4 * ri + 2], w.O[dt][4 * ri + 3]);
      *reinterpret_cast<float4 *>(orow + 32 * dt + 8 * ri + 4 * hf) = x;
    }
  if (hf == 0) sp.ml_part[slot] = make_float2(w.m_run, l_tot);
}

// One wavefront per (row, head) of a split row block: O = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.
__global__ __launch_bounds__(256) void attn_combine_kernel(SplitPlan sp, const int32_t *__restrict__ row_pos,
                                                           int n_rows, int n_kv, int n_q_heads, int rows_per_block,
                                                           uint16_t *__restrict__ out, float *__restrict__ lse_out) {
  const int lane = threadIdx.x & 63;
  const int64_t item = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  const int row = static_cast<int>(item / n_q_heads), head = static_cast<int>(item - static_cast<int64_t>(row) * n_q_heads);
  if (row >= n_rows) return;
  const int n_tiles = sp.block_tiles[row / rows_per_block];
  const int n_parts = (n_tiles + sp.part_tiles - 1) / sp.part_tiles;
  if (n_parts <= 1) return;  // written directly by the attention kernel
  const int p = row_pos[row];
  const bool in_range = p >= 0 && p < n_kv;
  float m_max = -INFINITY;
  for (int s = 0; s < n_parts; ++s)
    m_max = fmaxf(m_max, sp.ml_part[(static_cast<int64_t>(s) * n_rows + row) * n_q_heads + head].x);
  float l = 0.f, o0 = 0.f, o1 = 0.f;
  for (int s = 0; s < n_parts; ++s) {
    const int64_t slot = (static_cast<int64_t>(s) * n_rows + row) * n_q_heads + head;
    const float2 ml = sp.ml_part[slot];
    if (ml.y > 0.f) {  // a part whose keys all lie behind this row's position holds (-inf, 0)
      const float wgt = __builtin_amdgcn_exp2f(ml.x - m_max);
      const float2 o = *reinterpret_cast<const float2 *>(sp.o_part + slot * D + 2 * lane);
      l += ml.y * wgt;
      o0 += o.x * wgt;
      o1 += o.y * wgt;
    }
  }
  const float inv = in_range && l > 0.f ? 1.f / l : 0.f;
  const int64_t q = (static_cast<int64_t>(row) * n_q_heads + head);
  *reinterpret_cast<uint32_t *>(out + q * D + 2 * lane) = pack_bf16x2(o0 * inv, o1 * inv);
  if (lse_out != nullptr && lane == 0)
    lse_out[q] = in_range && l > 0.f ? 0.6931471805599453f * (m_max + __log2f(l)) : 0.f;
}

// ---------------------------------------------------------------------------
// NWAVES wavefronts, ring of NS LDS stages filled by direct global->LDS loads NS-1 tiles ahead.
// ---------------------------------------------------------------------------
template <int NWAVES, int NS>
__global__ __launch_bounds__(NWAVES * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_mfma_kernel(
    const uint16_t *__restrict__ q_sel, const int32_t *__restrict__ row_pos, int n_rows,
    const uint16_t *__restrict__ k_cache, const uint16_t *__restrict__ v_cache, int n_kv,
    uint16_t *__restrict__ out, float *__restrict__ lse_out, int n_q_heads, int n_kv_heads, float scale_log2,
    int rows_per_block, SplitPlan sp) {
  __shared__ __attribute__((aligned(1024))) uint16_t k_lds[NS][TILE_ELEMS];
  __shared__ __attribute__((aligned(1024))) uint16_t v_lds[NS][TILE_ELEMS];
  __shared__ int s_pmax[NWAVES];

  const int lane = threadIdx.x & 63;
  const int hf = lane >> 5;
  const int G = n_q_heads / n_kv_heads;
  const int g = blockIdx.x;
  const int rb = gridDim.y - 1 - blockIdx.y;  // longest prefixes are dispatched first
  const int part = blockIdx.z;
  const Column c = setup_column(row_pos, n_rows, n_kv, rb * rows_per_block, rows_per_block, G, g, n_q_heads,
                                (threadIdx.x >> 6) * 32 + (lane & 31));
  bf16x8 qf[8];
  load_q_frags(qf, q_sel, c, hf);
  const int n_tiles = block_tiles<NWAVES>(c.p_wmax, s_pmax);
  // this workgroup's share of the kv axis: tiles t0 .. t1-1 (the whole range unless the block is split)
  const int t0 = part * sp.part_tiles;
  const int t1 = min(n_tiles, t0 + sp.part_tiles);
  if (t0 >= n_tiles) return;  // nothing left for this part (uniform over the workgroup)
  const bool split = n_tiles > sp.part_tiles;
  if (part == 0 && g == 0 && threadIdx.x == 0 && sp.block_tiles != nullptr) sp.block_tiles[rb] = n_tiles;
  const ReadOffsets ro = make_read_offsets(lane);

  const int64_t kv_row_elems = static_cast<int64_t>(n_kv_heads) * D;
  const uint16_t *k_base = k_cache + static_cast<int64_t>(g) * D;
  const uint16_t *v_base = v_cache + static_cast<int64_t>(g) * D;
  const auto plan = make_dma_plan<NWAVES>(kv_row_elems);

  const uint32_t k_lds_addr = __builtin_amdgcn_readfirstlane(lds_address(&k_lds[0][0]));
  const uint32_t v_lds_addr = __builtin_amdgcn_readfirstlane(lds_address(&v_lds[0][0]));
  constexpr uint32_t kStageBytes = TILE_ELEMS * 2;

  WaveState w;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) w.O[dt][r] = 0.f;
  w.m_run = -INFINITY;
  w.l_run = 0.f;

  // Tiles t0 .. t0+NS-2 are requested up front; iteration i requests tile i + NS - 1 (rows past the
  // end are clamped, the data is never used), so exactly NS-1 tiles are in flight at every wait.
#pragma unroll
  for (int t = 0; t < NS - 1; ++t)
    issue_tile_dma<NWAVES>(plan, k_lds_addr + t * kStageBytes, v_lds_addr + t * kStageBytes, k_base, v_base,
                           kv_row_elems, t0 + t, n_kv);

  const int my_tiles = min(t1, c.p_wmax / TK + 1);
  // One tile.  `st` is a compile-time constant at every call (the loop below is unrolled over the
  // ring), so the LDS stage base folds into the immediate offset of every LDS read and the reads
  // cost no address arithmetic.
  auto tile_step = [&](int i, int st) {
    // this wavefront's share of tile i has landed when at most the NS-2 younger tiles are outstanding
    // (loads complete in order; the query loads issued before them are therefore complete too)
    __builtin_amdgcn_s_waitcnt(0x0F70 | ((NS - 2) * Dma<NWAVES>::PER_TILE));
    __syncthreads();  // everyone's share is visible, and everyone is done with tile i-1
    {
      const int wr = (st == 0) ? NS - 1 : st - 1;  // the stage tile i-1 occupied
      issue_tile_dma<NWAVES>(plan, k_lds_addr + wr * kStageBytes, v_lds_addr + wr * kStageBytes, k_base, v_base,
                             kv_row_elems, i + NS - 1, n_kv);
    }
    if (i < my_tiles) {  // otherwise this wavefront's rows end before the tile (it still stages and syncs)
      f32x16 S[2];
      qk_tile(S, k_lds[st], qf, ro);
      VFrags vf;
      pv_preload(vf, v_lds[st], ro);
      row_stats(S, w, i * TK, c.p_q, c.p_wmin, hf, scale_log2);
      PTile P;
      exp_tile(S, w, P, scale_log2);
      pv_tile(P, vf, w, v_lds[st], ro);
    }
  };
  for (int i0 = t0; i0 < t1; i0 += NS) {
#pragma unroll
    for (int st = 0; st < NS; ++st)
      if (i0 + st < t1) tile_step(i0 + st, st);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // drain the look-ahead loads before the LDS is released
  if (split)
    write_partial(w, c, sp, part, n_rows, n_q_heads, g, G, hf);
  else
    write_output(w, c, out, lse_out, n_q_heads, g, G, hf);
}


// ---------------------------------------------------------------------------
// Wide kernel: ONE wavefront per SIMD, 64 query columns per wavefront (two blocks, A and B, of
// 32), four wavefronts = 256 columns per block.
//
// The 128-column kernel above saturates the LDS read path: every K and V fragment read from LDS
// feeds a single MFMA.  Here each fragment feeds two (one per column block), which halves the LDS
// bytes per flop.  With one wavefront per SIMD nothing else hides the exponentials, so the kv loop
// is software-pipelined by hand over HALF tiles of 32 kv rows (which keeps the logits of two
// half tiles, for two column blocks, within the register file).  Step j issues, as one
// instruction stream of 32 slots,
//     slot  0..15   O^T += V(j-1)^T . P(j-1)^T   for A and B   (V fragment read once, used twice)
//     slot 16..31   S(j+1)^T = K(j+1) . Q^T      for A and B   (K fragment read once, used twice)
// and after the MFMA of slot n the n-th piece of the softmax of half tile j (block A in slots
// 0..15, block B in slots 16..31): running max, exponentials, row sums, bf16 packing.  The fences
// keep this order, so the matrix pipe runs underneath the vector work of the same wavefront.
// A rescale of O that half tile j asks for is applied after the last MFMA of half tile j-1 on
// that accumulator (it must scale those contributions too) and before step j+1 adds half tile j.
//
// LDS: ring of four 64-row stages; while tile i is being processed tiles i-1 (V), i and i+1 (K)
// are read and tile i+2 is being written by the direct loads.
// ---------------------------------------------------------------------------
constexpr int kWideStages = 4;
constexpr int kVAhead = 3;  // V operands requested ahead (two transpose reads each)
constexpr int kKAhead = 3;  // K operands requested ahead


// The first product of the wide kernel is emitted as inline assembly so that the register file
// split is explicit: query fragments (64 registers, read by nothing but these MFMAs) in the
// accumulation half of the register file, logits in the vector half where the softmax reads them.
// Left to itself the compiler chooses the opposite and pays 5 register copies per MFMA.  It cannot
// see what this statement is, so the wait states the ISA asks for between an MFMA and a vector
// instruction that reads its result are kept by construction in the pipelined step (the logits are
// read one step later) and by an explicit s_nop in the plain routine.
__device__ __forceinline__ void mfma_s(f32x16 &s_acc, v4u a, v4u q, bool first) {  // S (+)= a . q
  if (first)
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=v"(s_acc) : "v"(a), "a"(q));
  else
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s_acc) : "v"(a), "a"(q));
}

struct SoftmaxTmp {
  float mx, alpha, psum0, psum1;
  bool rescale;
};
struct PHalf {
  v4u step[2];  // contraction step u of the half tile: kv rows 16 u + 8 hf + 0..7
};

// Piece C (0..15) of the softmax of one half tile for one 32-column block.  Register r of S is kv
// row jbase + 16 (r / 8) + 8 hf + r % 8.  Only piece 0 may branch (wavefront-uniform, and it is the
// first piece of a step): the other pieces must stay in one basic block with the MFMAs they are
// interleaved with.
__device__ __forceinline__ void softmax_piece(int C, f32x16 &S, WaveState &w, PHalf &P, SoftmaxTmp &t, int jbase,
                                              int p_q, int p_wmin, int hf, float scale_log2) {
  if (C < 2) {  // running maximum over registers 8 C .. 8 C + 7; piece 0 applies the causal mask first
    if (C == 0 && jbase + 31 > p_wmin) {
      const int base = jbase + 8 * hf - p_q;
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (base + 16 * (r >> 3) + (r & 7) > 0) S[r] = -INFINITY;
    }
    // three-input maximum as one instruction (the logits come out of an assembly statement, so
    // fmaxf would first re-canonicalise every one of them)
    float mx = C == 0 ? S[0] : t.mx;
#pragma unroll
    for (int r = 0; r < 8; r += 2)
      asm("v_max3_f32 %0, %1, %2, %3" : "=v"(mx) : "v"(mx), "v"(S[8 * C + r]), "v"(S[8 * C + r + 1]));
    t.mx = mx;
  } else if (C == 2) {
    const float mx = half_swap_max(t.mx);
    const float m_new = fmaxf(w.m_run, mx * scale_log2);
    t.rescale = __any(m_new > w.m_run + kSlack);
    const float m_upd = t.rescale ? m_new : w.m_run;  // wavefront-uniform choice: a select, no branch
    // 1 when nothing changes, 0 on the first tile (m_run = -inf); a lane that has seen only masked
    // values keeps m_run = m_upd = -inf, where the difference is undefined: it has nothing to scale
    t.alpha = m_upd == w.m_run ? 1.f : __builtin_amdgcn_exp2f(w.m_run - m_upd);
    w.l_run *= t.alpha;
    w.m_run = m_upd;
    t.psum0 = 0.f;
    t.psum1 = 0.f;
  } else if (C < 11) {  // exponentials of two values
    const int r = 2 * (C - 3);
    S[r] = __builtin_amdgcn_exp2f(fmaf(S[r], scale_log2, -w.m_run));
    S[r + 1] = __builtin_amdgcn_exp2f(fmaf(S[r + 1], scale_log2, -w.m_run));
    t.psum0 += S[r];
    t.psum1 += S[r + 1];
  } else if (C < 15) {  // bf16 packing of half a contraction step
    const int q = C - 11, u = q >> 1, h = q & 1, r0 = 8 * u + 4 * h;
    P.step[u][2 * h + 0] = pack_bf16x2(S[r0 + 0], S[r0 + 1]);
    P.step[u][2 * h + 1] = pack_bf16x2(S[r0 + 2], S[r0 + 3]);
  } else {
    w.l_run += t.psum0 + t.psum1;
  }
}

__device__ __forceinline__ void apply_rescale(WaveState &w, const SoftmaxTmp &t) {
  if (t.rescale) {
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) w.O[dt][r] *= t.alpha;
  }
}

struct WideLane {
  int pA, pB, p_wminA, p_wminB, hf;  // p_wmin*: smallest position among the block's valid columns
  float scale_log2;
};

// One pipelined step (see the header above).  Pp*: P of half tile j-1 (consumed), Pc*: P of half
// tile j (produced), Sc*: S of half tile j (consumed), Sn*: S of half tile j+1 (produced).
// v_prev: V stage of half tile j-1, whose half is vh; k_next: K stage of half tile j+1, half kh.
__device__ __forceinline__ void wide_step(WaveState &wA, WaveState &wB, const v4u (&qA)[8], const v4u (&qB)[8],
                                          const PHalf &PpA, const PHalf &PpB, PHalf &PcA, PHalf &PcB, f32x16 &ScA,
                                          f32x16 &ScB, f32x16 &SnA, f32x16 &SnB, const uint16_t *v_prev, int vh,
                                          const uint16_t *k_next, int kh, const ReadOffsets &ro, const WideLane &ln,
                                          int jbase) {
  SoftmaxTmp tA, tB;
  s16x4 vlo[kVAhead], vhi[kVAhead];
  v4u kf[kKAhead];
  const uint16_t *kp = k_next + kh * (32 * D);
#pragma unroll
  for (int x = 0; x < kVAhead; ++x) v_read(vlo[x], vhi[x], v_prev, ro, 8 * vh + x);
  __builtin_amdgcn_sched_barrier(0);
  // slots 0..15: second product of half tile j-1, softmax of half tile j for block A
#pragma unroll
  for (int x = 0; x < 8; ++x) {
    const int u = x >> 2, dt = x & 3;
    const s16x8 a16 = __builtin_shufflevector(vlo[x % kVAhead], vhi[x % kVAhead], 0, 1, 2, 3, 4, 5, 6, 7);
    const bf16x8 a = __builtin_bit_cast(bf16x8, a16);
    wA.O[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, PpA.step[u]), wA.O[dt], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    softmax_piece(2 * x, ScA, wA, PcA, tA, jbase, ln.pA, ln.p_wminA, ln.hf, ln.scale_log2);
    __builtin_amdgcn_sched_barrier(0);
    wB.O[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, PpB.step[u]), wB.O[dt], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    softmax_piece(2 * x + 1, ScA, wA, PcA, tA, jbase, ln.pA, ln.p_wminA, ln.hf, ln.scale_log2);
    if (x + kVAhead < 8) v_read(vlo[x % kVAhead], vhi[x % kVAhead], v_prev, ro, 8 * vh + x + kVAhead);
    if (x >= 8 - kKAhead) {  // first K operands of the next phase
      const int s = x - (8 - kKAhead);
      kf[s] = *reinterpret_cast<const v4u *>(&kp[ro.k[s]]);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  // The results of the pieces are only needed by a later step; this empty statement "uses" them
  // here, so the compiler cannot sink the pieces out of the slots, past the branch below.
  asm volatile("" ::"v"(PcA.step[0]), "v"(PcA.step[1]), "v"(wA.l_run), "v"(wA.m_run));
  // the rescale half tile j asked for in block A: after the last MFMA of half tile j-1 on O_A
  apply_rescale(wA, tA);
  __builtin_amdgcn_sched_barrier(0);
  // slots 16..31: first product of half tile j+1, softmax of half tile j for block B
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const v4u a = kf[s % kKAhead];
    mfma_s(SnA, a, qA[s], s == 0);
    __builtin_amdgcn_sched_barrier(0);
    softmax_piece(2 * s, ScB, wB, PcB, tB, jbase, ln.pB, ln.p_wminB, ln.hf, ln.scale_log2);
    __builtin_amdgcn_sched_barrier(0);
    mfma_s(SnB, a, qB[s], s == 0);
    __builtin_amdgcn_sched_barrier(0);
    softmax_piece(2 * s + 1, ScB, wB, PcB, tB, jbase, ln.pB, ln.p_wminB, ln.hf, ln.scale_log2);
    if (s + kKAhead < 8) kf[s % kKAhead] = *reinterpret_cast<const v4u *>(&kp[ro.k[s + kKAhead]]);
    __builtin_amdgcn_sched_barrier(0);
  }
  asm volatile("" ::"v"(PcB.step[0]), "v"(PcB.step[1]), "v"(wB.l_run), "v"(wB.m_run));
  apply_rescale(wB, tB);
}

// Not pipelined: first product of one half tile for both blocks (prologue).
__device__ __forceinline__ void wide_qk(f32x16 &SA, f32x16 &SB, const v4u (&qA)[8], const v4u (&qB)[8],
                                        const uint16_t *k_stage, int kh, const ReadOffsets &ro) {
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const v4u a = *reinterpret_cast<const v4u *>(&k_stage[ro.k[s] + kh * (32 * D)]);
    mfma_s(SA, a, qA[s], s == 0);
    mfma_s(SB, a, qB[s], s == 0);
  }
  asm volatile("s_nop 15\n\ts_nop 15");  // the logits are read by vector instructions next
}

// Not pipelined: second product of one half tile for both blocks (epilogue).
__device__ __forceinline__ void wide_pv(WaveState &wA, WaveState &wB, const PHalf &PA, const PHalf &PB,
                                        const uint16_t *v_stage, int vh, const ReadOffsets &ro) {
#pragma unroll
  for (int x = 0; x < 8; ++x) {
    const int u = x >> 2, dt = x & 3;
    s16x4 lo, hi;
    v_read(lo, hi, v_stage, ro, 8 * vh + x);
    const bf16x8 a = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    wA.O[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, PA.step[u]), wA.O[dt], 0, 0, 0);
    wB.O[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, PB.step[u]), wB.O[dt], 0, 0, 0);
  }
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void attn_wide_kernel(
    const uint16_t *__restrict__ q_sel, const int32_t *__restrict__ row_pos, int n_rows,
    const uint16_t *__restrict__ k_cache, const uint16_t *__restrict__ v_cache, int n_kv,
    uint16_t *__restrict__ out, float *__restrict__ lse_out, int n_q_heads, int n_kv_heads, float scale_log2,
    int rows_per_block) {
  constexpr int NW = 4, NS = kWideStages;
  __shared__ __attribute__((aligned(1024))) uint16_t k_lds[NS][TILE_ELEMS];
  __shared__ __attribute__((aligned(1024))) uint16_t v_lds[NS][TILE_ELEMS];
  __shared__ int s_pmax[NW];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int hf = lane >> 5;
  const int G = n_q_heads / n_kv_heads;
  const int g = blockIdx.x;
  const int rb = gridDim.y - 1 - blockIdx.y;  // longest prefixes are dispatched first
  const int row0 = rb * rows_per_block;
  const Column cA = setup_column(row_pos, n_rows, n_kv, row0, rows_per_block, G, g, n_q_heads, wave * 64 + (lane & 31));
  const Column cB =
      setup_column(row_pos, n_rows, n_kv, row0, rows_per_block, G, g, n_q_heads, wave * 64 + 32 + (lane & 31));
  // Query fragments go from memory straight into the accumulation half of the register file.  The
  // compiler does not know that these statements are loads, so the wait for them is part of the same
  // dependency chain: the statement after the loop waits for all outstanding loads and names every
  // fragment as read and written, which keeps any later use (or register copy) behind the wait.
  // Columns without a row read a clamped (valid) row and are never written back.
  v4u qA[8], qB[8];
#pragma unroll
  for (int x = 0; x < 8; ++x) {
    asm volatile("global_load_dwordx4 %0, %1, off" : "=a"(qA[x]) : "v"(q_sel + cA.q_off + 16 * x + 8 * hf) : "memory");
    asm volatile("global_load_dwordx4 %0, %1, off" : "=a"(qB[x]) : "v"(q_sel + cB.q_off + 16 * x + 8 * hf) : "memory");
  }
  asm volatile("s_waitcnt vmcnt(0)"
               : "+a"(qA[0]), "+a"(qA[1]), "+a"(qA[2]), "+a"(qA[3]), "+a"(qA[4]), "+a"(qA[5]), "+a"(qA[6]), "+a"(qA[7]),
                 "+a"(qB[0]), "+a"(qB[1]), "+a"(qB[2]), "+a"(qB[3]), "+a"(qB[4]), "+a"(qB[5]), "+a"(qB[6]), "+a"(qB[7])
               :
               : "memory");
  const int n_tiles = block_tiles<NW>(max(cA.p_wmax, cB.p_wmax), s_pmax);
  const ReadOffsets ro = make_read_offsets(lane);
  WideLane ln;
  ln.pA = cA.p_q;
  ln.pB = cB.p_q;
  ln.p_wminA = cA.p_wmin;
  ln.p_wminB = cB.p_wmin;
  ln.hf = hf;
  ln.scale_log2 = scale_log2;

  const int64_t kv_row_elems = static_cast<int64_t>(n_kv_heads) * D;
  const uint16_t *k_base = k_cache + static_cast<int64_t>(g) * D;
  const uint16_t *v_base = v_cache + static_cast<int64_t>(g) * D;
  const auto plan = make_dma_plan<NW>(kv_row_elems);

  WaveState wA, wB;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      wA.O[dt][r] = 0.f;
      wB.O[dt][r] = 0.f;
    }
  wA.m_run = wB.m_run = -INFINITY;
  wA.l_run = wB.l_run = 0.f;

  // Prologue: tiles 0 and 1 staged; S and softmax of half tile 0 and S of half tile 1 without overlap.
  const uint32_t k_lds_addr = __builtin_amdgcn_readfirstlane(lds_address(&k_lds[0][0]));
  const uint32_t v_lds_addr = __builtin_amdgcn_readfirstlane(lds_address(&v_lds[0][0]));
  constexpr uint32_t kStageBytes = TILE_ELEMS * 2;
  issue_tile_dma<NW>(plan, k_lds_addr, v_lds_addr, k_base, v_base, kv_row_elems, 0, n_kv);
  issue_tile_dma<NW>(plan, k_lds_addr + kStageBytes, v_lds_addr + kStageBytes, k_base, v_base, kv_row_elems, 1, n_kv);
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();
  issue_tile_dma<NW>(plan, k_lds_addr + 2 * kStageBytes, v_lds_addr + 2 * kStageBytes, k_base, v_base, kv_row_elems, 2,
                     n_kv);

  // S0/P0 belong to the first half of a tile, S1/P1 to the second.
  f32x16 S0A, S0B, S1A, S1B;
  PHalf P0A, P0B, P1A, P1B;
  wide_qk(S0A, S0B, qA, qB, k_lds[0], 0, ro);
  {
    SoftmaxTmp tA, tB;
#pragma unroll
    for (int C = 0; C < 16; ++C) softmax_piece(C, S0A, wA, P0A, tA, 0, ln.pA, ln.p_wminA, hf, scale_log2);
#pragma unroll
    for (int C = 0; C < 16; ++C) softmax_piece(C, S0B, wB, P0B, tB, 0, ln.pB, ln.p_wminB, hf, scale_log2);
    // O is still zero: the rescale of the first half tile has nothing to scale
  }
  wide_qk(S1A, S1B, qA, qB, k_lds[0], 1, ro);
  // second half of tile 0: adds half 0, normalises half 1, multiplies the first half of tile 1
  wide_step(wA, wB, qA, qB, P0A, P0B, P1A, P1B, S1A, S1B, S0A, S0B, v_lds[0], 0, k_lds[1], 0, ro, ln, 32);

  for (int i = 1; i < n_tiles; ++i) {
    // tile i+1 must have landed (requested one iteration earlier); the stage that held tile i-2 is
    // free once every wavefront has passed the barrier
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    issue_tile_dma<NW>(plan, k_lds_addr + ((i + 2) & 3) * kStageBytes, v_lds_addr + ((i + 2) & 3) * kStageBytes, k_base,
                       v_base, kv_row_elems, i + 2, n_kv);
    // first half of tile i: adds the second half of tile i-1, multiplies the second half of tile i
    wide_step(wA, wB, qA, qB, P1A, P1B, P0A, P0B, S0A, S0B, S1A, S1B, v_lds[(i - 1) & 3], 1, k_lds[i & 3], 1, ro, ln,
              i * TK);
    // second half of tile i: adds the first half of tile i, multiplies the first half of tile i+1
    wide_step(wA, wB, qA, qB, P0A, P0B, P1A, P1B, S1A, S1B, S0A, S0B, v_lds[i & 3], 0, k_lds[(i + 1) & 3], 0, ro, ln,
              i * TK + 32);
  }
  // Epilogue: second product of the last half tile.
  wide_pv(wA, wB, P1A, P1B, v_lds[(n_tiles - 1) & 3], 1, ro);
  __builtin_amdgcn_s_waitcnt(0x0F70);  // drain the look-ahead loads before the LDS is released
  write_output(wA, cA, out, lse_out, n_q_heads, g, G, hf);
  write_output(wB, cB, out, lse_out, n_q_heads, g, G, hf);
}

}  // namespace

bool attention_mfma_supported(const ifkv_ctx *ctx) {
  const auto &d = ctx->desc;
  const int G = d.n_q_heads / d.n_kv_heads;
  return d.dtype == IFKV_BF16 && d.head_dim == D && G <= 32;
}

namespace {

// Whether and where the kv axis of the default kernel is cut.  The chip holds 512 of these workgroups
// at a time (two per CU) and a row block at position p costs p keys, so a launch is bound either by
// its total work (tiles per slot, if the jobs spread evenly) or by its longest row block alone.  With
// rows spread uniformly over the context a job averages half the tiles of the cache; when the longest
// job is clearly longer than the even share per slot, the kv axis is cut into parts of about that
// share: row blocks shorter than one part are not affected (they write their output directly), only
// the long ones run as several workgroups whose partial results are merged by the combine pass.
// Measured at 32K context: 5 % of the rows (416 jobs) 0.66 -> 0.48 ms; 8K context (312 jobs) 0.150 ->
// 0.125 ms.  Only launches with no more jobs than slots are cut: with more, every slot is busy for
// most of the launch anyway and the partial writes plus the combine pass cost more than the shorter
// tail gains (684 jobs: 0.469 -> 0.479 ms; 1232 jobs: 1.28 -> 1.37 ms).
// A part spans at least 32 tiles.  IFKV_ATTN_SPLIT=<parts> (equal parts) and
// IFKV_ATTN_PART_TILES=<tiles> override (tuning aids).
struct SplitChoice {
  int parts, part_tiles;
};
SplitChoice choose_split(const ifkv_ctx *ctx, int64_t n_rows, int64_t n_kv) {
  const auto &d = ctx->desc;
  const int G = d.n_q_heads / d.n_kv_heads;
  const int rpb = 128 / G;
  const int64_t jobs = ((n_rows + rpb - 1) / rpb) * d.n_kv_heads;
  const int n_kv_tiles = static_cast<int>((n_kv + TK - 1) / TK);
  constexpr int kSlots = 512, kMinPartTiles = 32, kMaxParts = 8;
  int part_tiles = n_kv_tiles;
  if (const char *env = getenv("IFKV_ATTN_PART_TILES")) {
    part_tiles = atoi(env);
  } else if (const char *env2 = getenv("IFKV_ATTN_SPLIT")) {
    const int parts = atoi(env2) > 0 ? atoi(env2) : 1;
    part_tiles = (n_kv_tiles + parts - 1) / parts;
  } else if (jobs > 0 && jobs <= kSlots) {
    const double even_share = static_cast<double>(jobs) * (0.5 * n_kv_tiles) / kSlots;
    if (even_share < 0.9 * n_kv_tiles) part_tiles = static_cast<int>(1.15 * even_share) + 1;
  }
  if (part_tiles < kMinPartTiles) part_tiles = kMinPartTiles;
  if (part_tiles * kMaxParts < n_kv_tiles) part_tiles = (n_kv_tiles + kMaxParts - 1) / kMaxParts;
  if (part_tiles > n_kv_tiles) part_tiles = n_kv_tiles > 0 ? n_kv_tiles : 1;
  SplitChoice c;
  c.part_tiles = part_tiles;
  c.parts = (n_kv_tiles + part_tiles - 1) / part_tiles;
  if (c.parts < 1) c.parts = 1;
  return c;
}

size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

}  // namespace

size_t attention_mfma_scratch_bytes(const ifkv_ctx *ctx, int64_t n_rows, int64_t n_kv) {
  const auto &d = ctx->desc;
  if ((d.flags & IFKV_FLAG_ATTN_WIDE) || n_rows <= 0) return 0;
  const SplitChoice c = choose_split(ctx, n_rows, n_kv);
  if (c.parts <= 1) return 0;
  const size_t slots = static_cast<size_t>(c.parts) * static_cast<size_t>(n_rows) * d.n_q_heads;
  const int G = d.n_q_heads / d.n_kv_heads;
  const size_t n_rb = static_cast<size_t>((n_rows + 128 / G - 1) / (128 / G));
  return align256(slots * D * sizeof(float)) + align256(slots * sizeof(float2)) + align256(n_rb * sizeof(int));
}

namespace {

// One launch covers at most 65535 row blocks (the y extent of a grid); more rows than that are
// served by several launches over consecutive row ranges (rows are independent).
constexpr int64_t kMaxRowBlocks = 65535;

hipError_t launch_attention_range(ifkv_ctx *ctx, const uint16_t *q_sel, const int32_t *row_pos, int64_t n_rows,
                                  const uint16_t *k_cache, const uint16_t *v_cache, int64_t n_kv, uint16_t *out,
                                  float *lse_out, bool wide) {
  const auto &d = ctx->desc;
  const int G = d.n_q_heads / d.n_kv_heads;
  const float scale_log2 = ctx->sm_scale * 1.4426950408889634f;
  if (wide) {
    const int rpbw = 256 / G;
    dim3 gridw(d.n_kv_heads, static_cast<unsigned>((n_rows + rpbw - 1) / rpbw));
    hipLaunchKernelGGL(attn_wide_kernel, gridw, dim3(256), 0, ctx->stream, q_sel, row_pos, static_cast<int>(n_rows),
                       k_cache, v_cache, static_cast<int>(n_kv), out, lse_out, d.n_q_heads, d.n_kv_heads, scale_log2,
                       rpbw);
    return hipGetLastError();
  }
  const int rpb = 128 / G;
  const unsigned n_rb = static_cast<unsigned>((n_rows + rpb - 1) / rpb);
  const SplitChoice sc = choose_split(ctx, n_rows, n_kv);
  SplitPlan sp;
  sp.part_tiles = sc.part_tiles;
  sp.o_part = nullptr;
  sp.ml_part = nullptr;
  sp.block_tiles = nullptr;
  if (sc.parts > 1) {
    const size_t slots = static_cast<size_t>(sc.parts) * static_cast<size_t>(n_rows) * d.n_q_heads;
    char *base = static_cast<char *>(ctx->scratch);
    sp.o_part = reinterpret_cast<float *>(base);
    sp.ml_part = reinterpret_cast<float2 *>(base + align256(slots * D * sizeof(float)));
    sp.block_tiles = reinterpret_cast<int *>(base + align256(slots * D * sizeof(float)) + align256(slots * sizeof(float2)));
  }
  dim3 grid(d.n_kv_heads, n_rb, sc.parts);
  hipLaunchKernelGGL((attn_mfma_kernel<4, 2>), grid, dim3(256), 0, ctx->stream, q_sel, row_pos, static_cast<int>(n_rows),
                     k_cache, v_cache, static_cast<int>(n_kv), out, lse_out, d.n_q_heads, d.n_kv_heads, scale_log2, rpb,
                     sp);
  if (sc.parts > 1) {
    const int64_t items = n_rows * d.n_q_heads;
    hipLaunchKernelGGL(attn_combine_kernel, dim3(static_cast<unsigned>((items + 3) / 4)), dim3(256), 0, ctx->stream, sp,
                       row_pos, static_cast<int>(n_rows), static_cast<int>(n_kv), d.n_q_heads, rpb, out, lse_out);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attention_mfma(ifkv_ctx *ctx, const void *q_sel, const int32_t *row_pos, int64_t n_rows,
                                 const void *k_cache, const void *v_cache, int64_t n_kv, void *out,
                                 float *lse_out) {
  const auto &d = ctx->desc;
  const int G = d.n_q_heads / d.n_kv_heads;
  const char *env = getenv("IFKV_ATTN_WIDE");  // tuning aid: same as the layer flag
  const bool wide = (d.flags & IFKV_FLAG_ATTN_WIDE) || (env != nullptr && atoi(env) == 1);
  int64_t max_rb = kMaxRowBlocks;
  if (const char *env_rb = getenv("IFKV_ATTN_MAX_ROW_BLOCKS")) {  // testing aid: exercise the range loop
    const int64_t v = atoll(env_rb);
    if (v >= 1 && v < max_rb) max_rb = v;
  }
  const int64_t rows_per_launch = max_rb * ((wide ? 256 : 128) / G);
  const int64_t row_elems = static_cast<int64_t>(d.n_q_heads) * D;
  for (int64_t r0 = 0; r0 < n_rows; r0 += rows_per_launch) {
    const int64_t nr = n_rows - r0 < rows_per_launch ? n_rows - r0 : rows_per_launch;
    hipError_t e = launch_attention_range(ctx, static_cast<const uint16_t *>(q_sel) + r0 * row_elems, row_pos + r0, nr,
                                          static_cast<const uint16_t *>(k_cache), static_cast<const uint16_t *>(v_cache),
                                          n_kv, static_cast<uint16_t *>(out) + r0 * row_elems,
                                          lse_out != nullptr ? lse_out + r0 * d.n_q_heads : nullptr, wide);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace ifkv
