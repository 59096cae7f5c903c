// Stage 4 work plan: which (row block, kv tile) pairs the workgroups of a launch process, in which
// order, and where the partial results of row blocks that several workgroups share are kept.
//
// Row blocks are numbered q = 0.. in descending length (n_q kv tiles; rows ascend, so the last row
// block is the longest).  The kv axis is cut into ranges of R tiles; (range c, row block q) with
// n_q > c R is a "part" of min(R, n_q - c R) tiles.  The parts form one line in the order
// (range, row block, tile): T tiles in total.  The line is cut into units -- R consecutive tiles
// each, and shorter ones over the last stretch -- which the workgroups of a kv head take in the
// order of the line, each fetching its next unit when it starts one (the first W units are dealt
// out by workgroup index).  So at any time the workgroups of a head work on neighbouring units,
// i.e. on the same few K/V tiles, which then come from the L2 instead of the fabric; a workgroup
// that runs faster (the older of the two on a compute unit is given priority by the hardware)
// takes more units; and the short units at the end let all workgroups end together.  A "piece" is
// what lies between two neighbouring boundaries (part or unit boundaries) of the line; a piece that
// is a whole row block is written to the output directly, every other piece leaves a partial
// result in the slot
//     slot = (index of its part along the line) + (index of its unit along the line),
// which grows strictly along the line and is therefore unique.  Pieces, slots and the order in
// which the pieces of a row block are merged do not depend on which workgroup takes which unit, so
// the results are the same bit for bit from run to run.
//
// The functions here only read the plan's tables; they are shared by the kernel (tables in LDS,
// built cooperatively) and by a host routine that the tests use to check coverage and slot
// uniqueness without a GPU.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ifkv {

constexpr int kPlanMaxBlocks = 1024;  // row blocks one launch can plan
constexpr int kPlanMaxRanges = 512;   // kv ranges one launch can plan
constexpr int kPlanRangeChoices = 12; // candidate range lengths R_min << j

struct AttnPlan {
  const int *prefix;   // [n_rb + 1]  tiles of the q longest row blocks
  const int *r_base;   // [n_c + 1]   position on the line where range c begins
  const int *r_full;   // [n_c]       row blocks whose part in range c has R tiles
  const int *r_cnt;    // [n_c]       row blocks that have a part in range c
  const int *r_part;   // [n_c + 1]   parts before range c
  int n_rb, n_c, R;
  int total;           // T
  int main_end;        // the line up to here is cut into units of R tiles (a multiple of R) ...
  int tail_unit;       // ... and the rest into units of this many tiles (the last one may be shorter)
  int n_main;          // main_end / R
  int n_units;         // all units
};

#define IFKV_PLAN_FN __host__ __device__ __forceinline__

IFKV_PLAN_FN int plan_tiles_of(const AttnPlan &p, int q) { return p.prefix[q + 1] - p.prefix[q]; }

IFKV_PLAN_FN int plan_part_len(const AttnPlan &p, int c, int q) {
  const int rest = plan_tiles_of(p, q) - c * p.R;
  return rest < p.R ? rest : p.R;
}

// position on the line of the first tile of part (c, q), q <= r_cnt[c]
IFKV_PLAN_FN int plan_part_start(const AttnPlan &p, int c, int q) {
  const int full = p.r_full[c];
  if (q <= full) return p.r_base[c] + q * p.R;
  return p.r_base[c] + full * p.R + (p.prefix[q] - p.prefix[full]) - (q - full) * c * p.R;
}

// the part that holds position x of the line
IFKV_PLAN_FN void plan_locate(const AttnPlan &p, int x, int &c, int &q) {
  int a = 0, b = p.n_c;  // r_base[a] <= x < r_base[b]
  while (b - a > 1) {
    const int mid = (a + b) >> 1;
    if (p.r_base[mid] <= x) a = mid; else b = mid;
  }
  c = a;
  const int off = x - p.r_base[c];
  const int full = p.r_full[c];
  if (off < full * p.R) {
    q = off / p.R;
    return;
  }
  int lo = full, hi = p.r_cnt[c];  // part_start(lo) <= x < part_start(hi)
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (plan_part_start(p, c, mid) <= x) lo = mid; else hi = mid;
  }
  q = lo;
}

// index, along the line, of the unit that holds position x
IFKV_PLAN_FN int plan_unit_of(const AttnPlan &p, int x) {
  if (x < p.main_end) return x / p.R;
  return p.n_main + (x - p.main_end) / p.tail_unit;
}

IFKV_PLAN_FN void plan_unit_bounds(const AttnPlan &p, int k, int &lo, int &hi) {
  if (k < p.n_main) {
    lo = k * p.R;
    hi = lo + p.R;
  } else {
    lo = p.main_end + (k - p.n_main) * p.tail_unit;
    hi = lo + p.tail_unit < p.total ? lo + p.tail_unit : p.total;
  }
}

// Calls fn(q, t0, t1, slot) for every piece of unit k, in the order of the line: tiles t0 .. t1-1
// of row block q.
template <typename Fn>
IFKV_PLAN_FN void plan_for_each_segment(const AttnPlan &p, int k, Fn &&fn) {
  int lo, hi;
  plan_unit_bounds(p, k, lo, hi);
  int c, q;
  plan_locate(p, lo, c, q);
  while (lo < hi) {
    const int ps = plan_part_start(p, c, q);
    const int pl = plan_part_len(p, c, q);
    const int t0 = c * p.R + (lo - ps);
    const int t1 = c * p.R + (hi - ps < pl ? hi - ps : pl);
    fn(q, t0, t1, p.r_part[c] + q + k);
    lo = ps + (t1 - c * p.R);
    if (++q == p.r_cnt[c]) {
      q = 0;
      ++c;
    }
  }
}

// Calls fn(slot) for every piece of row block q, in the order of the line.
template <typename Fn>
IFKV_PLAN_FN void plan_for_each_piece(const AttnPlan &p, int q, Fn &&fn) {
  const int n = plan_tiles_of(p, q);
  for (int c = 0; c * p.R < n; ++c) {
    const int ps = plan_part_start(p, c, q);
    const int pl = plan_part_len(p, c, q);
    const int c0 = plan_unit_of(p, ps), c1 = plan_unit_of(p, ps + pl - 1);
    for (int ci = c0; ci <= c1; ++ci) fn(p.r_part[c] + q + ci);
  }
}

// Units of a launch: the last stretch of the line, about half a full unit per workgroup, is cut
// into short units of R / tail_div tiles.
IFKV_PLAN_FN int plan_tail_stretch(int R, int W) { return (W * R) / 2; }
// upper bound of the number of units of the last stretch (whatever R is)
IFKV_PLAN_FN int plan_max_tail_units(int W, int tail_div) { return (W / 2 + 1) * tail_div + 2; }

// Range length: the first R_min << j for which the ranges fit the plan's tables and the slots fit
// the capacity.  parts[j] = sum_q ceil(n_q / (R_min << j)); n0 = tiles of the longest row block.
// Slots used are below parts + units.  Returns -1 if no candidate fits.
IFKV_PLAN_FN int plan_choose_range(const int *parts, int n0, int total, int r_min, int W, int tail_div, int slot_cap) {
  for (int j = 0; j < kPlanRangeChoices; ++j) {
    const int64_t R = static_cast<int64_t>(r_min) << j;
    const int64_t n_c = (n0 + R - 1) / R;
    if (n_c <= kPlanMaxRanges && parts[j] + total / R + plan_max_tail_units(W, tail_div) <= slot_cap) return j;
  }
  return -1;
}

// units for a chosen R
IFKV_PLAN_FN void plan_set_units(AttnPlan &p, int W, int tail_div) {
  p.tail_unit = p.R / tail_div > 0 ? p.R / tail_div : 1;
  int m = p.total - plan_tail_stretch(p.R, W);
  if (m < 0) m = 0;
  p.main_end = (m / p.R) * p.R;
  p.n_main = p.main_end / p.R;
  p.n_units = p.n_main + (p.total - p.main_end + p.tail_unit - 1) / p.tail_unit;
}

}  // namespace ifkv
