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
// Work distribution.  A row block at position p costs p/64 + 1 tiles, so the blocks of one launch
// differ in length by two orders of magnitude while the chip holds only 512 of these workgroups at
// a time (two per CU): handing out whole row blocks leaves an eighth of the machine idle at the
// end of a launch, and cutting the blocks' tiles into equal contiguous shares makes every workgroup
// stream its own stretch of K/V through the fabric (6.8 GB per launch instead of 0.8 GB measured at
// 32K context).  The launch therefore has a fixed number of workgroups per kv head that walk the
// (kv range, row block, tile) line of attention_plan.h in step: at any time they read the same few
// K/V tiles, and all end together.  Pieces that are not a whole row block leave their unnormalised
// O, reference max and sum in a scratch slot and count their tiles on the row block; the workgroup
// that completes the count merges the pieces.  Every workgroup derives the plan by itself from
// row_pos: no extra launch, no host knowledge of the positions, and nobody waits for anybody.
#include <algorithm>

#include "attention_common.h"
#include "attention_plan.h"
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

// ---------------------------------------------------------------------------
// The plan (attention_plan.h) built in LDS by every workgroup for itself: no extra launch, no host
// knowledge of the positions.
// ---------------------------------------------------------------------------
constexpr int kThreads = 256;

struct PlanArgs {
  int n_rb;             // row blocks of this launch (<= kPlanMaxBlocks)
  int wg_per_head;      // workgroups per kv head
  int tail_div;         // the short units at the end of the line are 1/tail_div of a kv range
  int r_min;            // smallest kv range, in tiles (a power of two)
  int slot_cap;         // partial slots per kv head
  float *o_part;        // [n_kv_heads * slot_cap] x [128 * 128]: unnormalised O, see write_partial
  float *ml_part;       // [n_kv_heads * slot_cap] x [128] x 2: (reference max in the log2 domain, sum) per query column
  int *arrived;         // [n_kv_heads][kPlanMaxBlocks + 2]: tiles of a shared row block that are done, then the
                        // units handed out beyond the first W and the workgroups that have left; zero between launches
  unsigned long long *trace;  // tuning aid, normally null: [grid][kTraceWords] time stamps of thread 0 (100 MHz counter)
};
constexpr int kTraceWords = 64;
constexpr size_t kPartFloats = 128 * D;  // O floats per partial slot

struct PlanTables {
  int prefix[kPlanMaxBlocks + 1];
  int r_base[kPlanMaxRanges + 1];
  int r_full[kPlanMaxRanges];
  int r_cnt[kPlanMaxRanges];
  int r_part[kPlanMaxRanges + 1];
  int wave_tmp[kThreads / 64][kPlanRangeChoices + 1];
};

// Exclusive prefix of one value per thread over the workgroup (thread order); *total gets the sum.
// Every thread must call; ends with a barrier, so the scratch row can be reused right away.
__device__ __forceinline__ int block_exclusive_scan(int v, int (*wave_tmp)[kPlanRangeChoices + 1], int *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int u = __shfl_up(incl, o, 64);
    if (lane >= o) incl += u;
  }
  if (lane == 63) wave_tmp[wave][kPlanRangeChoices] = incl;
  __syncthreads();
  int base = incl - v, sum = 0;
#pragma unroll
  for (int w = 0; w < kThreads / 64; ++w) {
    const int x = wave_tmp[w][kPlanRangeChoices];
    if (w < wave) base += x;
    sum += x;
  }
  *total = sum;
  __syncthreads();
  return base;
}

// tiles of row block q (descending length order): that of its last row, positions clamped into the
// cache (rows outside it produce zeros and never extend a block)
__device__ __forceinline__ int block_tiles_of(const int32_t *__restrict__ row_pos, int n_rows, int n_kv, int n_rb,
                                              int rows_per_block, int q) {
  const int rb = n_rb - 1 - q;
  const int last = min((rb + 1) * rows_per_block, n_rows) - 1;
  return min(max(row_pos[last], 0), n_kv - 1) / TK + 1;
}

// number of row blocks with more than x tiles (tile counts do not increase with q)
__device__ __forceinline__ int count_longer(const int *prefix, int n_rb, int x) {
  int a = 0, b = n_rb;  // blocks [0, a) are longer, blocks [b, n_rb) are not
  while (a < b) {
    const int mid = (a + b) >> 1;
    if (prefix[mid + 1] - prefix[mid] > x) a = mid + 1; else b = mid;
  }
  return a;
}

// Every thread of the workgroup must call this.  Returns false (for every thread) if the launch
// does not fit the slots, which the host rules out before launching.
__device__ __forceinline__ bool build_plan(AttnPlan &p, PlanTables &t, const int32_t *__restrict__ row_pos, int n_rows,
                                           int n_kv, int rows_per_block, const PlanArgs &pa) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_rb = pa.n_rb;
  const int lg_min = 31 - __clz(pa.r_min);
  // tiles per row block: prefix sums, and the number of parts for every candidate range length
  const int per = (n_rb + kThreads - 1) / kThreads;
  const int q0 = tid * per;
  int sum = 0;
  int parts[kPlanRangeChoices];
#pragma unroll
  for (int j = 0; j < kPlanRangeChoices; ++j) parts[j] = 0;
  for (int i = 0; i < per; ++i) {
    const int q = q0 + i;
    if (q < n_rb) {
      const int n = block_tiles_of(row_pos, n_rows, n_kv, n_rb, rows_per_block, q);
      sum += n;
#pragma unroll
      for (int j = 0; j < kPlanRangeChoices; ++j) parts[j] += (n + (pa.r_min << j) - 1) >> (lg_min + j);
    }
  }
#pragma unroll
  for (int j = 0; j < kPlanRangeChoices; ++j) {
    const int s = wave_sum_i(parts[j]);
    if (lane == 0) t.wave_tmp[wave][j] = s;
  }
  int total;
  int base = block_exclusive_scan(sum, t.wave_tmp, &total);  // its first barrier also publishes the part counts
  for (int i = 0; i < per; ++i) {  // second walk: the loads hit the cache this time
    const int q = q0 + i;
    if (q < n_rb) {
      t.prefix[q] = base;
      base += block_tiles_of(row_pos, n_rows, n_kv, n_rb, rows_per_block, q);
    }
  }
  if (tid == 0) t.prefix[n_rb] = total;
#pragma unroll
  for (int j = 0; j < kPlanRangeChoices; ++j) {
    int s = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) s += t.wave_tmp[w][j];
    parts[j] = s;
  }
  __syncthreads();
  const int n0 = t.prefix[1];
  const int j = plan_choose_range(parts, n0, total, pa.r_min, pa.wg_per_head, pa.tail_div, pa.slot_cap);
  if (j < 0) return false;
  p.prefix = t.prefix;
  p.r_base = t.r_base;
  p.r_full = t.r_full;
  p.r_cnt = t.r_cnt;
  p.r_part = t.r_part;
  p.n_rb = n_rb;
  p.R = pa.r_min << j;
  p.n_c = (n0 + p.R - 1) / p.R;
  p.total = total;
  plan_set_units(p, pa.wg_per_head, pa.tail_div);
  // per range: row blocks with a part, with a full part; width on the line; then prefix sums over ranges
  const int per_c = (p.n_c + kThreads - 1) / kThreads;  // <= 2
  int width = 0, count = 0;
  for (int i = 0; i < per_c; ++i) {
    const int c = tid * per_c + i;
    if (c < p.n_c) {
      const int cnt = count_longer(t.prefix, n_rb, c * p.R);
      const int full = count_longer(t.prefix, n_rb, (c + 1) * p.R - 1);
      t.r_cnt[c] = cnt;
      t.r_full[c] = full;
      width += full * p.R + (t.prefix[cnt] - t.prefix[full]) - (cnt - full) * c * p.R;
      count += cnt;
    }
  }
  int tot_w, tot_c;
  int wb = block_exclusive_scan(width, t.wave_tmp, &tot_w);
  int cb = block_exclusive_scan(count, t.wave_tmp, &tot_c);
  for (int i = 0; i < per_c; ++i) {
    const int c = tid * per_c + i;
    if (c < p.n_c) {
      const int cnt = t.r_cnt[c], full = t.r_full[c];
      t.r_base[c] = wb;
      t.r_part[c] = cb;
      wb += full * p.R + (t.prefix[cnt] - t.prefix[full]) - (cnt - full) * c * p.R;
      cb += cnt;
    }
  }
  if (tid == 0) {
    t.r_base[p.n_c] = tot_w;
    t.r_part[p.n_c] = tot_c;
  }
  __syncthreads();
  return true;
}

// Partial results travel between workgroups that may sit on different XCDs, whose L2s are not
// coherent with each other.  Cache-wide write-backs or invalidations per piece would cost far more
// than the pieces themselves (and an invalidation throws the K/V tiles out of the L2), so every
// access to a slot is a device-scope relaxed atomic of 8 bytes instead: the store writes through to
// memory, the load does not hit a line another XCD may have changed.
__device__ __forceinline__ void store_coherent(float *p, float a, float b) {
  const uint64_t v = static_cast<uint64_t>(__float_as_uint(a)) | (static_cast<uint64_t>(__float_as_uint(b)) << 32);
  __hip_atomic_store(reinterpret_cast<uint64_t *>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 load_coherent(const float *p) {
  const uint64_t v = __hip_atomic_load(reinterpret_cast<const uint64_t *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float(static_cast<uint32_t>(v)), __uint_as_float(static_cast<uint32_t>(v >> 32)));
}

// Partial result of a piece: accumulator registers 2 x .. 2 x + 1 of d tile dt go to
// [wave][dt * 8 + x][lane], so every store instruction of a wavefront writes 512 consecutive bytes.
__device__ __forceinline__ void write_partial(const WaveState &w, float *o_slot, float *ml_slot, int hf) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float l_tot = w.l_run + __shfl_xor(w.l_run, 32, 64);
  float *dst = o_slot + ((wave * 32) * 64 + lane) * 2;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int x = 0; x < 8; ++x) store_coherent(dst + (dt * 8 + x) * 128, w.O[dt][2 * x], w.O[dt][2 * x + 1]);
  if (hf == 0) store_coherent(ml_slot + 2 * (wave * 32 + (lane & 31)), w.m_run, l_tot);
}

// Merge of the pieces of row block q, in the order of the line (so the result does not depend on
// which workgroup runs it):  O = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s,  M = max_s m_s.
__device__ __forceinline__ void merge_pieces(const AttnPlan &p, int q, const float *o_part, const float *ml_part,
                                             const Column &c, uint16_t *__restrict__ out, float *__restrict__ lse_out,
                                             int n_q_heads, int g, int G) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int hf = lane >> 5;
  const int col = wave * 32 + (lane & 31);
  float m_max = kNoMax;
  plan_for_each_piece(p, q, [&](int slot) { m_max = fmaxf(m_max, load_coherent(ml_part + (static_cast<int64_t>(slot) * 128 + col) * 2).x); });
  f32x16 O[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) O[dt][r] = 0.f;
  float l = 0.f;
  plan_for_each_piece(p, q, [&](int slot) {
    const float2 ml = load_coherent(ml_part + (static_cast<int64_t>(slot) * 128 + col) * 2);
    const float wgt = __builtin_amdgcn_exp2f(ml.x - m_max);  // 0 for a piece that saw no key of this column
    l = fmaf(ml.y, wgt, l);
    const float *src = o_part + static_cast<int64_t>(slot) * kPartFloats + ((wave * 32) * 64 + lane) * 2;
    float2 v[32];  // all loads of a piece are issued before the first is used
#pragma unroll
    for (int x = 0; x < 32; ++x) v[x] = load_coherent(src + x * 128);
#pragma unroll
    for (int x = 0; x < 32; ++x) {
      O[x >> 3][2 * (x & 7)] = fmaf(v[x].x, wgt, O[x >> 3][2 * (x & 7)]);
      O[x >> 3][2 * (x & 7) + 1] = fmaf(v[x].y, wgt, O[x >> 3][2 * (x & 7) + 1]);
    }
  });
  store_output(O, m_max, l, c, out, lse_out, n_q_heads, g, G, hf);
}

// ---------------------------------------------------------------------------
// NWAVES wavefronts, ring of NS LDS stages filled by direct global->LDS loads NS-1 tiles ahead.
// blockIdx.x = w * n_kv_heads + g: consecutive workgroup ids go to consecutive XCDs, so with 8 kv
// heads all workgroups of a head share one XCD's L2.
// ---------------------------------------------------------------------------
template <int NWAVES, int NS>
__global__ __launch_bounds__(NWAVES * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_mfma_kernel(
    const uint16_t *__restrict__ q_sel, const int32_t *__restrict__ row_pos, int n_rows,
    const uint16_t *__restrict__ k_cache, const uint16_t *__restrict__ v_cache, int n_kv,
    uint16_t *__restrict__ out, float *__restrict__ lse_out, int n_q_heads, int n_kv_heads, float scale_log2,
    int rows_per_block, PlanArgs pa) {
  static_assert(NWAVES * 64 == kThreads, "the plan code assumes 256 threads");
  __shared__ __attribute__((aligned(1024))) uint16_t k_lds[NS][TILE_ELEMS];
  __shared__ __attribute__((aligned(1024))) uint16_t v_lds[NS][TILE_ELEMS];
  __shared__ PlanTables tables;
  __shared__ int s_last, s_next;

  const int lane = threadIdx.x & 63;
  const int hf = lane >> 5;
  const int G = n_q_heads / n_kv_heads;
  const int g = blockIdx.x % n_kv_heads;
  const int wg = blockIdx.x / n_kv_heads;

  unsigned long long *trace = (pa.trace != nullptr && threadIdx.x == 0) ? pa.trace + static_cast<size_t>(blockIdx.x) * kTraceWords : nullptr;
  int n_trace = 0;
  auto stamp = [&](unsigned long long tag) {
    if (trace != nullptr && n_trace < kTraceWords) trace[n_trace++] = (wall_clock64() << 8) | tag;
  };
  stamp(1);
  AttnPlan plan;
  if (!build_plan(plan, tables, row_pos, n_rows, n_kv, rows_per_block, pa)) return;  // uniform over the launch, ruled out by the host
  stamp(2);

  const ReadOffsets ro = make_read_offsets(lane);
  const int64_t kv_row_elems = static_cast<int64_t>(n_kv_heads) * D;
  const uint16_t *k_base = k_cache + static_cast<int64_t>(g) * D;
  const uint16_t *v_base = v_cache + static_cast<int64_t>(g) * D;
  const auto dma = make_dma_plan<NWAVES>(kv_row_elems);
  const uint32_t k_lds_addr = __builtin_amdgcn_readfirstlane(lds_address(&k_lds[0][0]));
  const uint32_t v_lds_addr = __builtin_amdgcn_readfirstlane(lds_address(&v_lds[0][0]));
  constexpr uint32_t kStageBytes = TILE_ELEMS * 2;
  float *o_part = pa.o_part + static_cast<int64_t>(g) * pa.slot_cap * kPartFloats;
  float *ml_part = pa.ml_part + static_cast<int64_t>(g) * pa.slot_cap * 256;
  int *arrived = pa.arrived + g * (kPlanMaxBlocks + 2);
  int *next_unit = arrived + kPlanMaxBlocks, *gone = next_unit + 1;

  // A piece counts its tiles on the row block once its partial result has reached memory (the stores
  // write through, see store_coherent, and have completed when the wavefront's memory counter has
  // drained); the workgroup that completes the count merges all pieces of the row block and leaves
  // the counter at zero for the next launch.  Nobody waits for anybody.  The count of a piece is
  // taken after the NEXT piece's kv loop, whose end drains the counter anyway, so the stores'
  // latency is never waited for.
  int pend_q = -1, pend_count = 0;
  auto arrive_pending = [&]() {
    if (pend_q < 0) return;  // uniform over the workgroup
    const int n_tiles = plan_tiles_of(plan, pend_q);
    __syncthreads();  // every wavefront's stores of that piece have completed
    if (threadIdx.x == 0) {
      const int done = __hip_atomic_fetch_add(&arrived[pend_q], pend_count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + pend_count;
      s_last = (done == n_tiles) ? 1 : 0;
      if (done == n_tiles) __hip_atomic_store(&arrived[pend_q], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    stamp(5);
    if (s_last != 0) {
      const int rb = pa.n_rb - 1 - pend_q;
      const Column c = setup_column(row_pos, n_rows, n_kv, rb * rows_per_block, rows_per_block, G, g, n_q_heads,
                                    (threadIdx.x >> 6) * 32 + (lane & 31));
      merge_pieces(plan, pend_q, o_part, ml_part, c, out, lse_out, n_q_heads, g, G);
      stamp(6);
    }
    pend_q = -1;
  };

  // Units: the first W by workgroup index, every further one from the head's counter.  The counter
  // is read when a unit starts and the answer used when it ends, so its latency is never waited for.
  int seg = 0;
  for (int unit = wg; unit < plan.n_units;) {
    int fetched = 0;
    if (threadIdx.x == 0)
      fetched = pa.wg_per_head + __hip_atomic_fetch_add(next_unit, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    plan_for_each_segment(plan, unit, [&](int q, int t0, int t1, int slot) {
    const int n_tiles = plan_tiles_of(plan, q);
    const bool whole = (t0 == 0) && (t1 == n_tiles);
    const int rb = pa.n_rb - 1 - q;
    if (seg > 0) {
      // the previous segment's stores are out and every wavefront is done reading its last tile
      // before the LDS ring is refilled
      __builtin_amdgcn_s_waitcnt(0x0F70);
      __syncthreads();
    }
    ++seg;
    stamp(3);
    const Column c = setup_column(row_pos, n_rows, n_kv, rb * rows_per_block, rows_per_block, G, g, n_q_heads,
                                  (threadIdx.x >> 6) * 32 + (lane & 31));
    bf16x8 qf[8];
    load_q_frags(qf, q_sel, c, hf);

    WaveState w;
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
      issue_tile_dma<NWAVES>(dma, k_lds_addr + t * kStageBytes, v_lds_addr + t * kStageBytes, k_base, v_base,
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
        issue_tile_dma<NWAVES>(dma, k_lds_addr + wr * kStageBytes, v_lds_addr + wr * kStageBytes, k_base, v_base,
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
    __builtin_amdgcn_s_waitcnt(0x0F70);  // drain the look-ahead loads before the LDS is reused or released
    stamp(4);
    if (whole) {
      const float l_tot = w.l_run + __shfl_xor(w.l_run, 32, 64);
      store_output(w.O, w.m_run, l_tot, c, out, lse_out, n_q_heads, g, G, hf);
    } else {
      write_partial(w, o_part + static_cast<int64_t>(slot) * kPartFloats, ml_part + static_cast<int64_t>(slot) * 256, hf);
    }
    arrive_pending();  // the piece before this one: its stores completed while this one was computed
    if (!whole) {
      pend_q = q;
      pend_count = t1 - t0;
    }
    });
    if (threadIdx.x == 0) s_next = fetched;
    __syncthreads();  // (the next write of s_next lies behind the barriers of the next unit's pieces)
    unit = s_next;
  }
  if (pend_q >= 0) {
    __builtin_amdgcn_s_waitcnt(0x0F70);
    arrive_pending();
  }
  // the last workgroup of the head to leave puts the unit counter back to zero for the next launch
  if (threadIdx.x == 0) {
    const int left = __hip_atomic_fetch_add(gone, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1;
    if (left == pa.wg_per_head) {
      __hip_atomic_store(next_unit, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(gone, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  stamp(7);
}

}  // namespace

bool attention_mfma_supported(const ifkv_ctx *ctx) {
  const auto &d = ctx->desc;
  const int G = d.n_q_heads / d.n_kv_heads;
  return d.dtype == IFKV_BF16 && d.head_dim == D && G <= 32;
}

namespace {

size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

// Workgroups per kv head: the chip runs 512 of these workgroups at a time (256 CUs, two each).
int default_wg_per_head(const ifkv_ctx *ctx) {
  const int w = 512 / ctx->desc.n_kv_heads;
  return w > 0 ? w : 1;
}

constexpr int kDefaultRangeTiles = 64;

}  // namespace

constexpr int kDefaultTailDiv = 8;

// Partial slots per kv head: three per kv tile of the longest cache the layer admits (what a launch
// of 30 % of the rows needs with 64-tile ranges), at least 256 and at most 2048, plus those of the
// short units at the end of a launch.  A launch that needs more lengthens its ranges by itself.
int attention_mfma_slot_cap(const ifkv_ctx *ctx) {
  const int64_t tiles = (ctx->desc.max_ctx + TK - 1) / TK;
  const int64_t s = std::min<int64_t>(std::max<int64_t>(3 * tiles, 256), 2048);
  return static_cast<int>(s) + plan_max_tail_units(default_wg_per_head(ctx), kDefaultTailDiv);
}

// Row blocks one launch may hold: the plan's tables, and in the worst case (ranges longer than the
// cache) one part and one full unit per row block plus the short units must fit the slots.
int attention_mfma_max_row_blocks(const ifkv_ctx *ctx) {
  const int by_slots = (attention_mfma_slot_cap(ctx) - plan_max_tail_units(default_wg_per_head(ctx), kDefaultTailDiv)) / 2;
  return std::min(kPlanMaxBlocks, by_slots);
}

size_t attention_mfma_scratch_bytes(const ifkv_ctx *ctx) {
  const size_t slots = static_cast<size_t>(attention_mfma_slot_cap(ctx)) * ctx->desc.n_kv_heads;
  return align256(slots * kPartFloats * sizeof(float)) + align256(slots * 128 * sizeof(float2));
}

size_t attention_mfma_counter_bytes(const ifkv_ctx *ctx) {
  return static_cast<size_t>(ctx->desc.n_kv_heads) * (kPlanMaxBlocks + 2) * sizeof(int);
}

// Host-side bounds of a launch against what was allocated.  Returns false (nothing launched) otherwise.
bool attention_mfma_launch_fits(const ifkv_ctx *ctx, int wg_per_head, int64_t n_rb, int64_t n_kv, int r_min, int tail_div) {
  if (wg_per_head < 1 || wg_per_head > default_wg_per_head(ctx)) return false;
  if (tail_div < 1 || tail_div > kDefaultTailDiv || tail_div > r_min) return false;
  if (n_rb < 1 || n_rb > attention_mfma_max_row_blocks(ctx)) return false;
  if (ctx->scratch == nullptr || attention_mfma_scratch_bytes(ctx) > ctx->scratch_bytes) return false;
  if (ctx->attn_arrived == nullptr) return false;
  // the longest candidate range must cover the cache, so that the fallback (one part per row block) exists
  const int64_t tiles = (n_kv + TK - 1) / TK;
  return r_min >= 1 && (r_min & (r_min - 1)) == 0 && (static_cast<int64_t>(r_min) << (kPlanRangeChoices - 1)) >= tiles;
}

hipError_t launch_attention_mfma(ifkv_ctx *ctx, const void *q_sel, const int32_t *row_pos, int64_t n_rows,
                                 const void *k_cache, const void *v_cache, int64_t n_kv, void *out,
                                 float *lse_out) {
  const auto &d = ctx->desc;
  const int G = d.n_q_heads / d.n_kv_heads;
  const int rpb = 128 / G;
  const float scale_log2 = ctx->sm_scale * 1.4426950408889634f;
  int wg_per_head = default_wg_per_head(ctx);
  if (ctx->tune.attn_wg_per_head > 0 && ctx->tune.attn_wg_per_head < wg_per_head) wg_per_head = ctx->tune.attn_wg_per_head;
  int64_t max_rb = attention_mfma_max_row_blocks(ctx);
  if (ctx->tune.attn_max_row_blocks > 0 && ctx->tune.attn_max_row_blocks < max_rb) max_rb = ctx->tune.attn_max_row_blocks;
  int r_min = ctx->tune.attn_range_tiles > 0 ? ctx->tune.attn_range_tiles : kDefaultRangeTiles;
  const int64_t tiles = (n_kv + TK - 1) / TK;
  while ((static_cast<int64_t>(r_min) << (kPlanRangeChoices - 1)) < tiles) r_min <<= 1;

  const size_t slots = static_cast<size_t>(attention_mfma_slot_cap(ctx)) * d.n_kv_heads;
  char *scratch = static_cast<char *>(ctx->scratch);
  PlanArgs pa;
  pa.wg_per_head = wg_per_head;
  pa.r_min = r_min;
  pa.tail_div = std::min(ctx->tune.attn_tail_div > 0 ? ctx->tune.attn_tail_div : kDefaultTailDiv, r_min);
  pa.slot_cap = attention_mfma_slot_cap(ctx);
  pa.o_part = reinterpret_cast<float *>(scratch);
  pa.ml_part = reinterpret_cast<float *>(scratch + align256(slots * kPartFloats * sizeof(float)));
  pa.arrived = ctx->attn_arrived;
  pa.trace = reinterpret_cast<unsigned long long *>(ctx->tune.attn_trace);

  // More row blocks than one plan holds are served by several launches over consecutive row ranges
  // (rows are independent).  Launches of one stream run one after the other, so they share the slots.
  const int64_t rows_per_launch = max_rb * rpb;
  const int64_t row_elems = static_cast<int64_t>(d.n_q_heads) * D;
  const dim3 grid(static_cast<unsigned>(wg_per_head) * d.n_kv_heads);
  for (int64_t r0 = 0; r0 < n_rows; r0 += rows_per_launch) {
    const int64_t nr = n_rows - r0 < rows_per_launch ? n_rows - r0 : rows_per_launch;
    pa.n_rb = static_cast<int>((nr + rpb - 1) / rpb);
    if (!attention_mfma_launch_fits(ctx, wg_per_head, pa.n_rb, n_kv, r_min, pa.tail_div)) return hipErrorInvalidValue;
    const uint16_t *q_r = static_cast<const uint16_t *>(q_sel) + r0 * row_elems;
    uint16_t *out_r = static_cast<uint16_t *>(out) + r0 * row_elems;
    float *lse_r = lse_out != nullptr ? lse_out + r0 * d.n_q_heads : nullptr;
    hipLaunchKernelGGL((attn_mfma_kernel<4, 2>), grid, dim3(kThreads), 0, ctx->stream, q_r, row_pos + r0,
                       static_cast<int>(nr), static_cast<const uint16_t *>(k_cache),
                       static_cast<const uint16_t *>(v_cache), static_cast<int>(n_kv), out_r, lse_r, d.n_q_heads,
                       d.n_kv_heads, scale_log2, rpb, pa);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace ifkv
