// Stage 4, bf16 MFMA kernels -- "KV Recomputation": each selected row attends
// causally to cache rows 0..p_r of the concatenated sequence.
//
// Shape of the problem: few, scattered query rows (k = rho N of them) against a
// long, dense K/V prefix.  The kernel therefore packs the G query heads that
// share a kv head together with a block of consecutive selected rows into one
// "row block" of 128 query columns, so that every K/V tile fetched from HBM/L2
// is used by all of them, and walks the kv axis in tiles of 64 rows with an
// online softmax (flash-attention style).  Rows are sorted by position, so only
// the last one or two kv tiles of a wavefront need the causal mask.
//
// Per wavefront (32 query columns), per kv tile, with 32x32x16 bf16 MFMAs:
//   S^T [64 kv x 32 q]  = K_tile . Q^T         (A = K rows from LDS, B = Q in registers)
//   P^T = exp2(S^T * c - m)                     (fp32, per-lane statistics: a lane owns one query column)
//   O^T [128 d x 32 q] += V_tile^T . P^T       (A = V^T from LDS, B = P^T straight from the S^T registers)
// Computing the transposed products keeps each query column in one lane (two
// lanes, one per half-wave), so a column's statistics need at most one
// cross-lane exchange per tile, and the S^T accumulator layout is exactly the
// B-operand layout of the second product once the K rows are fed in a fixed
// permuted order (sigma below): no LDS round trip for P.  The reference
// exponent m is, in the first sweep, the logit of the sweep's first key (kept
// for the whole sweep: no maximum, no exchange, no rescaling); a second sweep
// with a running maximum follows where the first is not accepted (see the kernel).
// Staging uses the gfx950 direct global->LDS loads (16 bytes per lane, no registers, no VALU) and
// keeps NS tiles in an LDS ring.  K rows land in sigma order with their 16-byte chunks XOR-swizzled
// by the row index, so the A-operand reads (32 rows, one chunk) hit distinct banks.  V lands
// row-major, swizzled by the row within each group of four rows, and the A operand of the second
// product -- which needs eight kv values of one d column per lane, the strided axis -- is read
// with the LDS transpose loads (ds_read_b64_tr_b16), two per operand.
//
// Work distribution.  One workgroup per (kv head, row block), dispatched longest row block first,
// so that the short ones fill the end of the launch; all workgroups of a head start at tile 0 and
// walk the kv axis together, which lets the L2 serve most tile fetches (0.8 GB reach the fabric per
// launch at 32K context; cutting the blocks' tiles into equal contiguous shares per workgroup
// instead, which balances the launch perfectly on paper, sends 6.8 GB through the fabric and is
// slower).  Launches with fewer row blocks than the chip has workgroup slots are cut along the kv
// axis: each part leaves its unnormalised O, reference max and sum in scratch and
// attn_combine_kernel merges them.
#include <algorithm>
#include <type_traits>

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
// Reference max of a column that has seen no key yet.  Finite on purpose: differences of two such
// values are 0 (not NaN), a masked logit (-inf) minus it is still -inf, and 2^(kNoMax - m) is 0.
constexpr float kNoMax = -1.0e30f;

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

// Causal mask (only on tiles that reach past the wavefront's smallest position) and, in the exact
// variant, the row max with the lazy update of the reference max and the rescale of O and l it
// implies.  The fast variant keeps the reference it was given (see the kernel): nothing but the mask.
// Register r of S[t] is kv row j0 + 32 t + 16 (r / 8) + 8 hf + r % 8.
template <bool EXACT>
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
  if (!EXACT) return;
  float mx = S[0][0];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[t][r]);
  mx = half_swap_max(mx);
  const float m_new = fmaxf(w.m_run, mx * scale_log2);
  if (__any(m_new > w.m_run + kSlack)) {
    const float alpha = __builtin_amdgcn_exp2f(w.m_run - m_new);  // 0 when m_run is still kNoMax, 1 when neither moved
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

// Normalised output of one query column: out = O / l (bf16), lse = ln 2 (m + log2 l).
__device__ __forceinline__ void store_output(const f32x16 (&O)[4], float m_ref, float l_tot, const Column &c,
                                             uint16_t *__restrict__ out, float *__restrict__ lse_out, int n_q_heads,
                                             int g, int G, int hf) {
  if (!c.col_valid) return;
  const bool ok = c.in_range && l_tot > 0.f;
  const float inv = ok ? 1.f / l_tot : 0.f;
  uint16_t *orow = out + c.q_off;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int ri = 0; ri < 4; ++ri) {
      uint2 x;
      x.x = pack_bf16x2(O[dt][4 * ri + 0] * inv, O[dt][4 * ri + 1] * inv);
      x.y = pack_bf16x2(O[dt][4 * ri + 2] * inv, O[dt][4 * ri + 3] * inv);
      *reinterpret_cast<uint2 *>(orow + 32 * dt + 8 * ri + 4 * hf) = x;
    }
  if (lse_out != nullptr && hf == 0)
    lse_out[static_cast<int64_t>(c.row) * n_q_heads + g * G + c.hh] =
        ok ? 0.6931471805599453f * (m_ref + __log2f(l_tot)) : 0.f;
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
  int exact_only;     // 1: skip the fixed-reference sweep
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

// The merge of a split row block, per (row, head): O = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.
// Measured: the pass is bound by the bytes of the partial results (8K context, 1228 rows in three parts:
// 34 MB, 16 us); several pairs per wavefront change nothing there, and eight parts per step are what
// the launches with many parts (a few rows against a long context) gain from: 134 -> 102 us.
constexpr int kCombineItems = 1;  // (row, head) pairs per wavefront of the combine pass
constexpr int kCombineBatch = 8;  // parts of each that are loaded together
__global__ __launch_bounds__(256) void attn_combine_kernel(SplitPlan sp, const int32_t *__restrict__ row_pos,
                                                           int n_rows, int n_kv, int n_q_heads, int rows_per_block,
                                                           uint16_t *__restrict__ out, float *__restrict__ lse_out) {
  const int lane = threadIdx.x & 63;
  const int64_t n_items = static_cast<int64_t>(n_rows) * n_q_heads;
  const int64_t first = (static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6)) * kCombineItems;
  if (first >= n_items) return;
  // A wavefront merges kCombineItems (row, head) pairs, kCombineBatch parts of each at a time: all loads
  // of a step are independent, so a wavefront waits for memory once per step (the partial results come
  // from memory: other workgroups wrote them in the previous launch) instead of twice per part.
  // Between steps the running (max, sum, O) are rescaled as in the attention kernel itself.
  int row[kCombineItems], head[kCombineItems], n_parts[kCombineItems], pos[kCombineItems];
#pragma unroll
  for (int j = 0; j < kCombineItems; ++j) {
    const int64_t item = min(first + j, n_items - 1);  // past the end: the last item again, not stored
    row[j] = static_cast<int>(item / n_q_heads);
    head[j] = static_cast<int>(item - static_cast<int64_t>(row[j]) * n_q_heads);
    n_parts[j] = sp.block_tiles[row[j] / rows_per_block];
    pos[j] = row_pos[row[j]];
  }
  int max_parts = 0;
#pragma unroll
  for (int j = 0; j < kCombineItems; ++j) {
    n_parts[j] = (n_parts[j] + sp.part_tiles - 1) / sp.part_tiles;
    if (first + j >= n_items || n_parts[j] <= 1) n_parts[j] = 0;  // written directly by the attention kernel
    max_parts = max(max_parts, n_parts[j]);
  }
  if (max_parts == 0) return;  // uniform over the wavefront
  float m_max[kCombineItems], l[kCombineItems], o0[kCombineItems], o1[kCombineItems];
#pragma unroll
  for (int j = 0; j < kCombineItems; ++j) {
    m_max[j] = -INFINITY;
    l[j] = o0[j] = o1[j] = 0.f;
  }
  for (int s0 = 0; s0 < max_parts; s0 += kCombineBatch) {
    float2 ml[kCombineItems][kCombineBatch], o[kCombineItems][kCombineBatch];
#pragma unroll
    for (int j = 0; j < kCombineItems; ++j)
#pragma unroll
      for (int u = 0; u < kCombineBatch; ++u) {
        const int s = max(min(s0 + u, n_parts[j] - 1), 0);  // past the last part: a valid slot, masked below
        const int64_t slot = (static_cast<int64_t>(s) * n_rows + row[j]) * n_q_heads + head[j];
        ml[j][u] = sp.ml_part[slot];
        o[j][u] = *reinterpret_cast<const float2 *>(sp.o_part + slot * D + 2 * lane);
      }
#pragma unroll
    for (int j = 0; j < kCombineItems; ++j) {
      float m_new = m_max[j];
#pragma unroll
      for (int u = 0; u < kCombineBatch; ++u) {
        // a part whose keys all lie behind this row's position holds a zero sum
        if (s0 + u >= n_parts[j] || !(ml[j][u].y > 0.f)) {
          ml[j][u] = make_float2(-INFINITY, 0.f);
          o[j][u] = make_float2(0.f, 0.f);  // whatever the slot holds
        }
        m_new = fmaxf(m_new, ml[j][u].x);
      }
      if (m_new > -INFINITY) {
        const float keep = __builtin_amdgcn_exp2f(m_max[j] - m_new);  // 0 for the first step that holds anything
        l[j] *= keep;
        o0[j] *= keep;
        o1[j] *= keep;
#pragma unroll
        for (int u = 0; u < kCombineBatch; ++u) {
          const float wgt = __builtin_amdgcn_exp2f(ml[j][u].x - m_new);  // 0 for a masked part
          l[j] += ml[j][u].y * wgt;
          o0[j] += o[j][u].x * wgt;
          o1[j] += o[j][u].y * wgt;
        }
        m_max[j] = m_new;
      }
    }
  }
#pragma unroll
  for (int j = 0; j < kCombineItems; ++j) {
    if (n_parts[j] == 0) continue;
    const bool in_range = pos[j] >= 0 && pos[j] < n_kv;
    const float inv = in_range && l[j] > 0.f ? 1.f / l[j] : 0.f;
    const int64_t q = (static_cast<int64_t>(row[j]) * n_q_heads + head[j]);
    *reinterpret_cast<uint32_t *>(out + q * D + 2 * lane) = pack_bf16x2(o0[j] * inv, o1[j] * inv);
    if (lse_out != nullptr && lane == 0)
      lse_out[q] = in_range && l[j] > 0.f ? 0.6931471805599453f * (m_max[j] + __log2f(l[j])) : 0.f;
  }
}

// ---------------------------------------------------------------------------
// NWAVES wavefronts, ring of NS LDS stages filled by direct global->LDS loads NS-1 tiles ahead.
// ---------------------------------------------------------------------------
template <int NWAVES, int NS>
__global__ __launch_bounds__(NWAVES * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_mfma_kernel(
    const uint16_t *__restrict__ q_sel, const int32_t *__restrict__ row_pos, int n_rows,
    const uint16_t *__restrict__ k_cache, const uint16_t *__restrict__ v_cache, int n_kv,
    uint16_t *__restrict__ out, float *__restrict__ lse_out, int n_q_heads, int n_kv_heads, float scale_log2,
    int rows_per_block, CacheLayout lay, SplitPlan sp) {
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

  const int64_t kv_row_elems = lay.token_stride;
  const uint16_t *k_base = k_cache + g * lay.head_stride;
  const uint16_t *v_base = v_cache + g * lay.head_stride;
  const auto plan = make_dma_plan<NWAVES>(kv_row_elems);

  const uint32_t k_lds_addr = __builtin_amdgcn_readfirstlane(lds_address(&k_lds[0][0]));
  const uint32_t v_lds_addr = __builtin_amdgcn_readfirstlane(lds_address(&v_lds[0][0]));
  constexpr uint32_t kStageBytes = TILE_ELEMS * 2;

  WaveState w;
  const int my_tiles = min(t1, c.p_wmax / TK + 1);
  // The sweep over this workgroup's kv tiles, in two variants.  The softmax only needs SOME reference
  // exponent per query column that keeps exp2(logit - reference) inside the fp32 / bf16 range, not the
  // column maximum.  The fast variant takes the logit of the first key of the sweep (key t0 * 64: the
  // reference of both lane halves of a column, which feed one product) and keeps it: no maximum over
  // the tile, no lane-half exchange, no rescaling of O, ever (2.3 % of the launch at 32K context).
  // It is accepted when every column's sum stays below 4096 x the keys of the sweep, i.e. when no key
  // outweighs the first one by more than that: flat and moderately peaked attention.  Otherwise --
  // sharply peaked columns, where the running maximum makes the dominant probability exactly 1 and
  // thereby free of rounding error, and sums on their way out of the fp32 range -- the whole
  // workgroup repeats the sweep in the exact variant, which tracks the running maximum (lazily: O is
  // rescaled only when a tile exceeds the reference by more than 2^8).
  auto sweep = [&](auto exact_tag) __attribute__((always_inline)) {
    constexpr bool kExact = decltype(exact_tag)::value;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) w.O[dt][r] = 0.f;
    w.m_run = kNoMax;
    w.l_run = 0.f;

    // Tiles t0 .. t0+NS-2 are requested up front; iteration i requests tile i + NS - 1 (rows past the
    // end are clamped, the data is never used), so exactly NS-1 tiles are in flight at every wait.
#pragma unroll
    for (int t = 0; t < NS - 1; ++t)
      issue_tile_dma<NWAVES>(plan, k_lds_addr + t * kStageBytes, v_lds_addr + t * kStageBytes, k_base, v_base,
                             kv_row_elems, t0 + t, n_kv);

    // One tile.  `st` is a compile-time constant at every call (the loop below is unrolled over the
    // ring), so the LDS stage base folds into the immediate offset of every LDS read and the reads
    // cost no address arithmetic.
    auto tile_step = [&](int i, int st) __attribute__((always_inline)) {
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
        if (!kExact && i == t0) {
          // register 0 of the lower lane half is key t0 * 64 (before the mask: a real key's logit even
          // for a column that does not see it); the upper half takes it from its partner lane
          w.m_run = __shfl(S[0][0], lane & 31, 64) * scale_log2;
        }
        row_stats<kExact>(S, w, i * TK, c.p_q, c.p_wmin, hf, scale_log2);
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
    __builtin_amdgcn_s_waitcnt(0x0F70);  // drain the look-ahead loads before the LDS is reused or released
  };
  bool redo = sp.exact_only != 0;
  if (!redo) {
    sweep(std::false_type{});
    const float limit = 4096.f * TK * static_cast<float>(t1 - t0);
    redo = __syncthreads_or(!(w.l_run <= limit) ? 1 : 0) != 0;  // also true for NaN; uniform over the workgroup
    // every wavefront has passed that barrier, so nobody still reads the LDS ring
  }
  if (redo) sweep(std::true_type{});
  if (split) {
    write_partial(w, c, sp, part, n_rows, n_q_heads, g, G, hf);
  } else {
    const float l_tot = w.l_run + __shfl_xor(w.l_run, 32, 64);
    store_output(w.O, w.m_run, l_tot, c, out, lse_out, n_q_heads, g, G, hf);
  }
}


}  // namespace

bool attention_mfma_supported(const ifkv_ctx *ctx) {
  const auto &d = ctx->desc;
  const int G = d.n_q_heads / d.n_kv_heads;
  return d.dtype == IFKV_BF16 && d.head_dim == D && G <= 32;
}

namespace {

constexpr int kSlots = 512;       // workgroups the chip holds at a time (256 CUs, two each)
constexpr int kMinPartTiles = 32;
constexpr int kMaxParts = 8;      // parts of a launch that fills the slots (the scratch is sized for this)
constexpr int kMaxPartsFew = 64;  // launches with a handful of row blocks: as many parts as slots stay free

size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

// bytes of partial results for a launch of n_rows rows cut into `parts`
size_t partial_bytes(const ifkv_ctx *ctx, int64_t n_rows, int parts) {
  const auto &d = ctx->desc;
  const size_t slots = static_cast<size_t>(parts) * static_cast<size_t>(n_rows) * d.n_q_heads;
  const int G = d.n_q_heads / d.n_kv_heads;
  const size_t n_rb = static_cast<size_t>((n_rows + 128 / G - 1) / (128 / G));
  return align256(slots * D * sizeof(float)) + align256(slots * sizeof(float2)) + align256(n_rb * sizeof(int));
}

// Whether and where the kv axis is cut.  The chip holds 512 of these workgroups at a time and a row
// block at position p costs p keys, so a launch is bound either by its total work (tiles per slot, if
// the jobs spread evenly) or by its longest row block alone.  With rows spread uniformly over the
// context a job averages half the tiles of the cache; when the longest job is clearly longer than the
// even share per slot, the kv axis is cut into parts of about that share: row blocks shorter than one
// part are not affected (they write their output directly), only the long ones run as several
// workgroups whose partial results are merged by the combine pass.  Measured at 32K context: 5 % of
// the rows (416 jobs) 0.66 -> 0.48 ms; 8K context (312 jobs) 0.150 -> 0.125 ms.  Only launches with
// no more jobs than slots are cut: with more, every slot is busy for most of the launch anyway and
// the partial writes plus the combine pass cost more than the shorter tail gains (684 jobs: 0.469 ->
// 0.479 ms; 1232 jobs: 1.28 -> 1.37 ms; cutting only the longest row blocks of such a launch: 1.23
// -> 1.26 .. 1.33 ms).  A part spans at least 32 tiles and there are at most 8 parts -- with so few
// row blocks that 8 parts each would leave slots empty (a few dozen rows against a long context), up
// to 64, as long as jobs x parts stays within the slots, which also keeps the partial results within
// the scratch -- unless the tuning knobs say otherwise; a cut whose partial results would not fit
// the scratch is not made.
struct SplitChoice {
  int parts, part_tiles;
};
SplitChoice choose_split(const ifkv_ctx *ctx, int64_t n_rows, int64_t n_kv, size_t scratch_bytes) {
  const auto &d = ctx->desc;
  const int G = d.n_q_heads / d.n_kv_heads;
  const int rpb = 128 / G;
  const int64_t jobs = ((n_rows + rpb - 1) / rpb) * d.n_kv_heads;
  const int n_kv_tiles = static_cast<int>((n_kv + TK - 1) / TK);
  int part_tiles = n_kv_tiles;
  bool forced = false;
  if (ctx->tune.attn_part_tiles > 0) {
    part_tiles = ctx->tune.attn_part_tiles;
    forced = true;
  } else if (ctx->tune.attn_split_parts > 0) {
    part_tiles = (n_kv_tiles + ctx->tune.attn_split_parts - 1) / ctx->tune.attn_split_parts;
    forced = true;
  } else if (jobs > 0 && jobs <= kSlots) {
    const double even_share = static_cast<double>(jobs) * (0.5 * n_kv_tiles) / kSlots;
    if (even_share < 0.9 * n_kv_tiles) part_tiles = static_cast<int>(1.15 * even_share) + 1;
  }
  if (!forced) {
    if (part_tiles < kMinPartTiles) part_tiles = kMinPartTiles;
    int max_parts = kMaxParts;
    if (jobs > 0 && jobs * kMaxParts < kSlots) max_parts = static_cast<int>(std::min<int64_t>(kMaxPartsFew, kSlots / jobs));
    if (part_tiles * max_parts < n_kv_tiles) part_tiles = (n_kv_tiles + max_parts - 1) / max_parts;
  }
  if (part_tiles < 1) part_tiles = 1;
  if (part_tiles > n_kv_tiles) part_tiles = n_kv_tiles > 0 ? n_kv_tiles : 1;
  SplitChoice c;
  c.part_tiles = part_tiles;
  c.parts = (n_kv_tiles + part_tiles - 1) / part_tiles;
  if (c.parts < 1) c.parts = 1;
  // host-side bounds: the grid's z extent, and the partial results must fit what was allocated
  if (c.parts > 65535 || (c.parts > 1 && partial_bytes(ctx, n_rows, c.parts) > scratch_bytes)) {
    c.parts = 1;
    c.part_tiles = n_kv_tiles > 0 ? n_kv_tiles : 1;
  }
  return c;
}

}  // namespace

// Scratch for the partial results, fixed for a layer shape: the largest launch the library cuts by
// itself (as many row blocks as the chip has workgroup slots, 8 parts).
size_t attention_mfma_scratch_bytes(const ifkv_ctx *ctx) {
  const auto &d = ctx->desc;
  const int G = d.n_q_heads / d.n_kv_heads;
  const int64_t rows = static_cast<int64_t>((kSlots + d.n_kv_heads - 1) / d.n_kv_heads) * (128 / G);
  return partial_bytes(ctx, rows, kMaxParts);
}

namespace {

// One launch covers at most 65535 row blocks (the y extent of a grid); more rows than that are
// served by several launches over consecutive row ranges (rows are independent).  Launches of one
// stream run one after the other, so they share the scratch.
constexpr int64_t kMaxRowBlocks = 65535;

hipError_t launch_attention_range(ifkv_ctx *ctx, const uint16_t *q_sel, const int32_t *row_pos, int64_t n_rows,
                                  const uint16_t *k_cache, const uint16_t *v_cache, int64_t n_kv, uint16_t *out,
                                  float *lse_out) {
  const auto &d = ctx->desc;
  const int G = d.n_q_heads / d.n_kv_heads;
  const float scale_log2 = ctx->sm_scale * 1.4426950408889634f;
  const int rpb = 128 / G;
  const unsigned n_rb = static_cast<unsigned>((n_rows + rpb - 1) / rpb);
  const SplitChoice sc = choose_split(ctx, n_rows, n_kv, ctx->scratch_bytes);
  SplitPlan sp;
  sp.part_tiles = sc.part_tiles;
  sp.o_part = nullptr;
  sp.ml_part = nullptr;
  sp.block_tiles = nullptr;
  sp.exact_only = ctx->tune.attn_exact_sweep;
  if (sc.parts > 1) {
    if (ctx->scratch == nullptr || partial_bytes(ctx, n_rows, sc.parts) > ctx->scratch_bytes) return hipErrorInvalidValue;
    const size_t slots = static_cast<size_t>(sc.parts) * static_cast<size_t>(n_rows) * d.n_q_heads;
    char *base = static_cast<char *>(ctx->scratch);
    sp.o_part = reinterpret_cast<float *>(base);
    sp.ml_part = reinterpret_cast<float2 *>(base + align256(slots * D * sizeof(float)));
    sp.block_tiles = reinterpret_cast<int *>(base + align256(slots * D * sizeof(float)) + align256(slots * sizeof(float2)));
  }
  dim3 grid(d.n_kv_heads, n_rb, sc.parts);
  hipLaunchKernelGGL((attn_mfma_kernel<4, 2>), grid, dim3(256), 0, ctx->stream, q_sel, row_pos, static_cast<int>(n_rows),
                     k_cache, v_cache, static_cast<int>(n_kv), out, lse_out, d.n_q_heads, d.n_kv_heads, scale_log2, rpb,
                     cache_layout(ctx), sp);
  if (sc.parts > 1) {
    const int64_t items = n_rows * d.n_q_heads;
    const int64_t per_block = 4 * kCombineItems;  // four wavefronts
    hipLaunchKernelGGL(attn_combine_kernel, dim3(static_cast<unsigned>((items + per_block - 1) / per_block)), dim3(256), 0,
                       ctx->stream, sp, row_pos, static_cast<int>(n_rows), static_cast<int>(n_kv), d.n_q_heads, rpb, out,
                       lse_out);
  }
  return hipGetLastError();
}

}  // namespace

namespace {
int64_t rows_per_launch_of(const ifkv_ctx *ctx) {
  const int G = ctx->desc.n_q_heads / ctx->desc.n_kv_heads;
  int64_t max_rb = kMaxRowBlocks;
  if (ctx->tune.attn_max_row_blocks > 0 && ctx->tune.attn_max_row_blocks < max_rb) max_rb = ctx->tune.attn_max_row_blocks;
  return max_rb * (128 / G);
}
}  // namespace

// What launch_attention_mfma would do for n_rows rows against n_kv keys with a scratch of
// scratch_bytes: the launches, the largest number of kv parts and the smallest part length among
// them, and the most bytes of partial results any of them keeps.  Host arithmetic only.
void attention_mfma_plan(const ifkv_ctx *ctx, int64_t n_rows, int64_t n_kv, size_t scratch_bytes, int64_t out[4]) {
  const int64_t rows_per_launch = rows_per_launch_of(ctx);
  out[0] = out[3] = 0;
  out[1] = 1;
  out[2] = (n_kv + TK - 1) / TK;
  for (int64_t r0 = 0; r0 < n_rows; r0 += rows_per_launch) {
    const int64_t nr = n_rows - r0 < rows_per_launch ? n_rows - r0 : rows_per_launch;
    const SplitChoice sc = choose_split(ctx, nr, n_kv, scratch_bytes);
    ++out[0];
    if (sc.parts > out[1]) out[1] = sc.parts;
    if (sc.part_tiles < out[2]) out[2] = sc.part_tiles;
    if (sc.parts > 1) out[3] = std::max<int64_t>(out[3], static_cast<int64_t>(partial_bytes(ctx, nr, sc.parts)));
  }
}

hipError_t launch_attention_mfma(ifkv_ctx *ctx, const void *q_sel, const int32_t *row_pos, int64_t n_rows,
                                 const void *k_cache, const void *v_cache, int64_t n_kv, void *out,
                                 float *lse_out) {
  const auto &d = ctx->desc;
  const int64_t rows_per_launch = rows_per_launch_of(ctx);
  const int64_t row_elems = static_cast<int64_t>(d.n_q_heads) * D;
  for (int64_t r0 = 0; r0 < n_rows; r0 += rows_per_launch) {
    const int64_t nr = n_rows - r0 < rows_per_launch ? n_rows - r0 : rows_per_launch;
    hipError_t e = launch_attention_range(ctx, static_cast<const uint16_t *>(q_sel) + r0 * row_elems, row_pos + r0, nr,
                                          static_cast<const uint16_t *>(k_cache), static_cast<const uint16_t *>(v_cache),
                                          n_kv, static_cast<uint16_t *>(out) + r0 * row_elems,
                                          lse_out != nullptr ? lse_out + r0 * d.n_q_heads : nullptr);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace ifkv
