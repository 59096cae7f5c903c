// Declarations shared by the two scoring translation units.
#pragma once

#include "ifkv_internal.h"

namespace ifkv {

// Largest number of query-row chunks the MFMA scoring pass splits one kv
// head's (prompt row, query head) pairs into.
constexpr int kMaxQChunks = 4;

struct ScoreScratch {
  size_t stats_off;    // float2 [H_q * M]: final (m, 1/Z)
  size_t partial_off;  // float2 [slices][H_q * M]: per-slice (m, Z)
  size_t fused_off;    // chunk table, first rows and rotation table of the fused stage 1 + pass A
  size_t colpart_off;  // float [H_kv * chunks][N]: partial column sums (MFMA pass B)
  size_t total;
};
constexpr int kFusedMaxChunks = 512;
constexpr size_t kFusedTableBytes = kFusedMaxChunks * (32 + 4 + 128 * 4);  // descriptors, first rows, (cos, sin)

// One non-empty chunk of a fused stage 1 + pass A call, in the order of the concatenation.
struct FusedHostChunk {
  const void *k, *v;   // device, packed [len, H_kv, d]; v may be null
  int64_t dst_row;     // first row in the concatenated cache
  double advance;      // rotary phase advance in positions
};
// What the fused sweep replaces: stage 1 (k_out, v_out written) and pass A of stage 2.
struct FusedRepo {
  const FusedHostChunk *chunks;
  int n_chunks;
  void *k_out, *v_out;
};
bool fused_repo_score_supported(const ifkv_ctx *ctx, int m_prompt, int n_chunks);
ScoreScratch score_scratch_layout(const ifkv_ctx *ctx, int64_t n_ctx, int m_prompt);

bool score_mfma_supported(const ifkv_ctx *ctx, int m_prompt);
// pass_b == false: per-block partial (max, sum) of every (head, prompt row); *n_slices_out = number of
// partials per row.  pass_b == true: column sums, reduced into `scores`.  merged_stats (the same value in
// both calls of a pair) says whether the merge kernel runs between them (it must when the prompt keys take
// part) or pass B merges the partials itself; the layout of the partials follows from it.
// `fused` (pass A only): the keys come from the chunk caches, see FusedRepo.
hipError_t launch_score_mfma_passes(ifkv_ctx *ctx, const void *k_global, int64_t n_ctx, const void *q_prompt,
                                    int m_prompt, int *n_slices_out, bool pass_b, int accumulate, float *scores,
                                    const FusedRepo *fused = nullptr, bool merged_stats = false);
// Key ranges (blocks along the context) of the MFMA sweeps: at most one per compute unit.
constexpr int kScoreMaxKeyRanges = 256;

}  // namespace ifkv
