// Host-side run of the stage-4 work plan (attention_plan.h): the same walk and slot functions the
// kernel uses, over tables filled serially.  Used by the tests to check, without a GPU, that every
// (row block, kv tile) pair is processed exactly once, that no two pieces share a slot and that the
// merge of a row block finds exactly the pieces that were written.
#include <vector>

#include "attention_plan.h"
#include "ifkv_debug.h"

extern "C" int64_t ifkv_attention_plan(const int32_t *block_tiles, int32_t n_rb, int32_t wg_per_head,
                                       int32_t tail_div, int32_t range_tiles, int32_t slot_cap, int32_t *segments,
                                       int64_t max_segments, int32_t *pieces, int64_t max_pieces,
                                       int64_t *n_pieces_out, int32_t *range_out) {
  using namespace ifkv;
  if (block_tiles == nullptr || n_rb < 1 || n_rb > kPlanMaxBlocks || wg_per_head < 1 || tail_div < 1 || tail_div > range_tiles ||
      range_tiles < 1 || (range_tiles & (range_tiles - 1)) != 0 || slot_cap < 1)
    return IFKV_EINVAL;
  for (int q = 0; q < n_rb; ++q)
    if (block_tiles[q] < 1 || (q > 0 && block_tiles[q] > block_tiles[q - 1])) return IFKV_EINVAL;
  std::vector<int> prefix(n_rb + 1, 0);
  int parts[kPlanRangeChoices] = {};
  for (int q = 0; q < n_rb; ++q) {
    prefix[q + 1] = prefix[q] + block_tiles[q];
    for (int j = 0; j < kPlanRangeChoices; ++j) {
      const int64_t R = static_cast<int64_t>(range_tiles) << j;
      parts[j] += static_cast<int>((block_tiles[q] + R - 1) / R);
    }
  }
  const int total = prefix[n_rb];
  const int j = plan_choose_range(parts, block_tiles[0], total, range_tiles, wg_per_head, tail_div, slot_cap);
  if (j < 0) return IFKV_ESHAPE;
  AttnPlan p;
  p.n_rb = n_rb;
  p.R = range_tiles << j;
  p.n_c = (block_tiles[0] + p.R - 1) / p.R;
  p.total = total;
  plan_set_units(p, wg_per_head, tail_div);
  std::vector<int> r_base(p.n_c + 1, 0), r_full(p.n_c, 0), r_cnt(p.n_c, 0), r_part(p.n_c + 1, 0);
  for (int c = 0; c < p.n_c; ++c) {
    int width = 0;
    for (int q = 0; q < n_rb; ++q) {
      const int rest = block_tiles[q] - c * p.R;
      if (rest <= 0) continue;
      ++r_cnt[c];
      if (rest >= p.R) ++r_full[c];
      width += rest < p.R ? rest : p.R;
    }
    r_base[c + 1] = r_base[c] + width;
    r_part[c + 1] = r_part[c] + r_cnt[c];
  }
  p.prefix = prefix.data();
  p.r_base = r_base.data();
  p.r_full = r_full.data();
  p.r_cnt = r_cnt.data();
  p.r_part = r_part.data();
  if (range_out != nullptr) *range_out = p.R;

  int64_t n_seg = 0;
  for (int k = 0; k < p.n_units; ++k)
    plan_for_each_segment(p, k, [&](int q, int t0, int t1, int slot) {
      if (segments != nullptr && n_seg < max_segments) {
        int32_t *s = segments + 6 * n_seg;
        s[0] = k, s[1] = q, s[2] = t0, s[3] = t1, s[4] = slot;
        s[5] = (t0 == 0 && t1 == block_tiles[q]) ? 1 : 0;
      }
      ++n_seg;
    });
  int64_t n_pc = 0;
  for (int q = 0; q < n_rb; ++q)
    plan_for_each_piece(p, q, [&](int slot) {
      if (pieces != nullptr && n_pc < max_pieces) {
        pieces[2 * n_pc] = q;
        pieces[2 * n_pc + 1] = slot;
      }
      ++n_pc;
    });
  if (n_pieces_out != nullptr) *n_pieces_out = n_pc;
  return n_seg;
}
