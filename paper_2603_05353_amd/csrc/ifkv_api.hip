// Host side of the C ABI declared in include/ifkv.h: argument validation
// (before any GPU call), host-side bookkeeping (chunk starts, budget), scratch
// management and dispatch to the stage launchers.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "ifkv_calibrate.h"
#include "ifkv_debug.h"
#include "ifkv_internal.h"
#include "score_common.h"

namespace {

thread_local std::string g_create_error;

int fail(ifkv_ctx *ctx, int code, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  if (ctx != nullptr)
    ctx->err = buf;
  else
    g_create_error = buf;
  return code;
}

int hip_fail(ifkv_ctx *ctx, hipError_t e, const char *what) {
  return fail(ctx, IFKV_EHIP, "%s: %s", what, hipGetErrorString(e));
}

// The context's scratch: ONE allocation, on the first stage call that needs scratch, sized for the
// largest request any stage can make under the layer descriptor (the stages run one after the other
// on one stream and share it).  No later call allocates, frees or synchronises.
size_t scratch_bytes_for(const ifkv_ctx *ctx) {
  size_t bytes = ifkv::score_scratch_bytes(ctx, ctx->desc.max_ctx, ctx->desc.max_prompt);
  bytes = std::max(bytes, ifkv::topk_scratch_bytes(ctx, ctx->desc.max_ctx));
  bytes = std::max(bytes, ifkv::attention_scratch_bytes(ctx));
  bytes = std::max(bytes, ifkv::validate_scratch_bytes(ctx));
  return std::max<size_t>(bytes, 256);
}

int ensure_scratch(ifkv_ctx *ctx) {
  if (ctx->scratch != nullptr) return IFKV_OK;
  const size_t bytes = scratch_bytes_for(ctx);
  void *p = nullptr;
  hipError_t e = hipMalloc(&p, bytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(ctx, IFKV_ENOMEM, "scratch allocation of %zu bytes failed: %s", bytes, hipGetErrorString(e));
  }
  // stage 2's arrival counters live apart from the shared scratch (other stages would overwrite them)
  // and must read zero before the first launch; every launch leaves them at zero again
  void *c = nullptr;
  const size_t cbytes = ifkv::kScoreMaxKeyRanges * sizeof(int);
  e = hipMalloc(&c, cbytes);
  if (e == hipSuccess) e = hipMemset(c, 0, cbytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    if (c != nullptr) (void)hipFree(c);
    (void)hipFree(p);
    return fail(ctx, IFKV_ENOMEM, "counter allocation failed: %s", hipGetErrorString(e));
  }
  ctx->score_arrived = static_cast<int *>(c);
  ctx->scratch = p;
  ctx->scratch_bytes = bytes;
  return IFKV_OK;
}

int ensure_inv_freq(ifkv_ctx *ctx) {
  if (ctx->d_inv_freq != nullptr) return IFKV_OK;
  const size_t bytes = sizeof(double) * (ctx->desc.head_dim / 2);
  void *p = nullptr;
  hipError_t e = hipMalloc(&p, bytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(ctx, IFKV_ENOMEM, "frequency table allocation failed: %s", hipGetErrorString(e));
  }
  e = hipMemcpy(p, ctx->inv_freq, bytes, hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    (void)hipFree(p);
    return hip_fail(ctx, e, "hipMemcpy(inv_freq)");
  }
  ctx->d_inv_freq = static_cast<double *>(p);
  return IFKV_OK;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {

const char *ifkv_version(void) { return "0.1"; }

const char *ifkv_last_error(const ifkv_ctx *ctx) {
  return ctx != nullptr ? ctx->err.c_str() : g_create_error.c_str();
}

int ifkv_create(ifkv_ctx **out, const ifkv_layer_desc *desc, void *hip_stream) {
  if (out == nullptr) return fail(nullptr, IFKV_EINVAL, "ifkv_create: out is NULL");
  *out = nullptr;
  if (desc == nullptr) return fail(nullptr, IFKV_EINVAL, "ifkv_create: desc is NULL");
  if (desc->dtype != IFKV_F32 && desc->dtype != IFKV_BF16)
    return fail(nullptr, IFKV_EDTYPE, "ifkv_create: unknown dtype %d", desc->dtype);
  if (desc->pairing != IFKV_ROPE_HALF && desc->pairing != IFKV_ROPE_INTERLEAVED)
    return fail(nullptr, IFKV_EDTYPE, "ifkv_create: unknown rope pairing %d", desc->pairing);
  if (desc->n_q_heads <= 0 || desc->n_kv_heads <= 0 || desc->n_q_heads % desc->n_kv_heads != 0)
    return fail(nullptr, IFKV_EINVAL, "ifkv_create: n_q_heads=%d must be a positive multiple of n_kv_heads=%d",
                desc->n_q_heads, desc->n_kv_heads);
  if (desc->head_dim != 64 && desc->head_dim != 128)
    return fail(nullptr, IFKV_EINVAL, "ifkv_create: head_dim=%d is not supported (64 or 128)", desc->head_dim);
  if (desc->inv_freq == nullptr && !(desc->rope_theta > 0.0))
    return fail(nullptr, IFKV_EINVAL, "ifkv_create: rope_theta must be positive");
  if (!(desc->sm_scale >= 0.f) || !std::isfinite(desc->sm_scale))
    return fail(nullptr, IFKV_EINVAL, "ifkv_create: sm_scale must be finite and >= 0");
  if (desc->max_ctx <= 0 || desc->max_ctx >= (int64_t(1) << 31))
    return fail(nullptr, IFKV_EINVAL, "ifkv_create: max_ctx must be in [1, 2^31)");
  if (desc->max_prompt < 0) return fail(nullptr, IFKV_EINVAL, "ifkv_create: max_prompt must be >= 0");
  int64_t ts = desc->token_stride, hs = desc->head_stride;
  if ((ts == 0) != (hs == 0))
    return fail(nullptr, IFKV_EINVAL, "ifkv_create: token_stride and head_stride must both be 0 (packed) or both be given");
  if (ts == 0) {
    ts = static_cast<int64_t>(desc->n_kv_heads) * desc->head_dim;
    hs = desc->head_dim;
  } else {
    const int64_t vec = desc->dtype == IFKV_BF16 ? 8 : 4;  // elements in 16 bytes
    const int64_t d = desc->head_dim;
    if (ts < d || hs < d || ts % vec != 0 || hs % vec != 0)
      return fail(nullptr, IFKV_EINVAL, "ifkv_create: strides must be multiples of %lld elements and at least head_dim",
                  static_cast<long long>(vec));
    const bool token_major = ts >= (desc->n_kv_heads - 1) * hs + d;
    const bool head_major = hs / ts >= desc->max_ctx - 1 && hs >= (desc->max_ctx - 1) * ts + d;
    if (!token_major && !head_major)
      return fail(nullptr, IFKV_EINVAL, "ifkv_create: token_stride=%lld, head_stride=%lld make rows or heads overlap",
                  static_cast<long long>(ts), static_cast<long long>(hs));
    if (ts > (int64_t(1) << 24) || hs > (int64_t(1) << 40))
      return fail(nullptr, IFKV_EINVAL, "ifkv_create: strides out of range");
  }

  ifkv_ctx *ctx = new (std::nothrow) ifkv_ctx();
  if (ctx == nullptr) return fail(nullptr, IFKV_ENOMEM, "ifkv_create: out of host memory");
  ctx->desc = *desc;
  ctx->desc.inv_freq = nullptr;
  ctx->stream = static_cast<hipStream_t>(hip_stream);
  ctx->token_stride = ts;
  ctx->head_stride = hs;
  ctx->packed = (ts == static_cast<int64_t>(desc->n_kv_heads) * desc->head_dim) && (hs == desc->head_dim);
  ctx->sm_scale = desc->sm_scale > 0.f ? desc->sm_scale : 1.0f / std::sqrt(static_cast<float>(desc->head_dim));
  const int half = desc->head_dim / 2;
  for (int j = 0; j < half; ++j) {
    ctx->inv_freq[j] = desc->inv_freq != nullptr
                           ? desc->inv_freq[j]
                           : std::pow(desc->rope_theta, -2.0 * static_cast<double>(j) / desc->head_dim);
  }
  *out = ctx;
  return IFKV_OK;
}

void ifkv_destroy(ifkv_ctx *ctx) {
  if (ctx == nullptr) return;
  if (ctx->scratch != nullptr) (void)hipFree(ctx->scratch);
  if (ctx->score_arrived != nullptr) (void)hipFree(ctx->score_arrived);
  if (ctx->d_inv_freq != nullptr) (void)hipFree(ctx->d_inv_freq);
  delete ctx;
}

namespace {

struct RepoArgs {
  int32_t n_chunks;
  const void *const *k_chunks;
  const void *const *v_chunks;
  const int32_t *chunk_len;
  const int32_t *chunk_order;
  const int32_t *cached_pos0;
  const int64_t *delta_override;
  void *k_out, *v_out;
  int64_t *chunk_start_out, *n_ctx_out;
};

// Stage 1, host part: argument checks, Eq. (5) (start of every chunk in the concatenation order) and
// the host outputs.  `start` gets the first row of every chunk, *n_ctx_p the number of rows.
int repo_validate(ifkv_ctx *ctx, const RepoArgs &a, std::vector<int64_t> &start, int64_t *n_ctx_p) {
  const int32_t n_chunks = a.n_chunks;
  const void *const *k_chunks = a.k_chunks;
  const void *const *v_chunks = a.v_chunks;
  const int32_t *chunk_len = a.chunk_len, *chunk_order = a.chunk_order;
  void *k_out = a.k_out, *v_out = a.v_out;
  int64_t *chunk_start_out = a.chunk_start_out, *n_ctx_out = a.n_ctx_out;
  if (n_chunks < 0) return fail(ctx, IFKV_EINVAL, "reposition_keys: n_chunks=%d is negative", n_chunks);
  if (n_chunks > 0 && (k_chunks == nullptr || chunk_len == nullptr))
    return fail(ctx, IFKV_EINVAL, "reposition_keys: k_chunks and chunk_len are required");

  // Eq. (5): start of every chunk in the concatenation order
  start.assign(n_chunks > 0 ? n_chunks : 0, 0);
  std::vector<char> seen(n_chunks, 0);
  int64_t n_ctx = 0;
  for (int s = 0; s < n_chunks; ++s) {
    const int c = chunk_order != nullptr ? chunk_order[s] : s;
    if (c < 0 || c >= n_chunks || seen[c])
      return fail(ctx, IFKV_EINVAL, "reposition_keys: chunk_order is not a permutation (slot %d -> %d)", s, c);
    seen[c] = 1;
    if (chunk_len[c] < 0) return fail(ctx, IFKV_EINVAL, "reposition_keys: chunk_len[%d] is negative", c);
    start[c] = n_ctx;
    n_ctx += chunk_len[c];
  }
  if (n_ctx > ctx->desc.max_ctx)
    return fail(ctx, IFKV_ESHAPE, "reposition_keys: %lld context rows exceed max_ctx=%lld",
                static_cast<long long>(n_ctx), static_cast<long long>(ctx->desc.max_ctx));
  for (int c = 0; c < n_chunks; ++c) {
    if (chunk_len[c] > 0) {
      if (k_chunks[c] == nullptr) return fail(ctx, IFKV_EINVAL, "reposition_keys: k_chunks[%d] is NULL", c);
      if (v_chunks != nullptr && v_chunks[c] == nullptr)
        return fail(ctx, IFKV_EINVAL, "reposition_keys: v_chunks[%d] is NULL", c);
      if (!aligned16(k_chunks[c]) || (v_chunks != nullptr && !aligned16(v_chunks[c])))
        return fail(ctx, IFKV_EINVAL, "reposition_keys: chunk %d is not 16-byte aligned", c);
    }
  }
  if (n_ctx > 0) {
    if (k_out == nullptr) return fail(ctx, IFKV_EINVAL, "reposition_keys: k_out is NULL");
    if (v_chunks != nullptr && v_out == nullptr) return fail(ctx, IFKV_EINVAL, "reposition_keys: v_out is NULL");
    if (!aligned16(k_out) || (v_chunks != nullptr && !aligned16(v_out)))
      return fail(ctx, IFKV_EINVAL, "reposition_keys: outputs must be 16-byte aligned");
  }
  if (chunk_start_out != nullptr)
    for (int c = 0; c < n_chunks; ++c) chunk_start_out[c] = start[c];
  if (n_ctx_out != nullptr) *n_ctx_out = n_ctx;
  *n_ctx_p = n_ctx;
  return IFKV_OK;

}

int64_t repo_advance(const RepoArgs &a, const std::vector<int64_t> &start, int c) {
  return a.delta_override != nullptr ? a.delta_override[c]
                                     : start[c] - (a.cached_pos0 != nullptr ? static_cast<int64_t>(a.cached_pos0[c]) : 0);
}

// Stage 1, device part (the stage on its own).
int repo_launch(ifkv_ctx *ctx, const RepoArgs &a, const std::vector<int64_t> &start) {
  const int32_t n_chunks = a.n_chunks;
  const void *const *k_chunks = a.k_chunks;
  const void *const *v_chunks = a.v_chunks;
  const int32_t *chunk_len = a.chunk_len;
  void *k_out = a.k_out, *v_out = a.v_out;
  int rc = ensure_inv_freq(ctx);
  if (rc != IFKV_OK) return rc;

  const int rows_per_tile = ifkv::reposition_rows_per_tile();
  ifkv::RepoBatch batch;
  batch.n = 0;
  batch.total_tiles = 0;
  auto flush = [&]() -> int {
    if (batch.n == 0) return IFKV_OK;
    hipError_t e = ifkv::launch_reposition(ctx, batch, k_out, v_chunks != nullptr ? v_out : nullptr);
    batch.n = 0;
    batch.total_tiles = 0;
    return e == hipSuccess ? IFKV_OK : hip_fail(ctx, e, "reposition kernel launch");
  };
  for (int c = 0; c < n_chunks; ++c) {
    if (chunk_len[c] == 0) continue;
    ifkv::RepoChunk &rc_ = batch.c[batch.n];
    rc_.k = k_chunks[c];
    rc_.v = v_chunks != nullptr ? v_chunks[c] : nullptr;
    rc_.dst_row = start[c];
    const int64_t adv = repo_advance(a, start, c);
    rc_.advance = static_cast<double>(adv);
    rc_.len = chunk_len[c];
    rc_.tile0 = batch.total_tiles;
    batch.total_tiles += (chunk_len[c] + rows_per_tile - 1) / rows_per_tile;
    if (++batch.n == ifkv::kRepoMaxChunks) {
      rc = flush();
      if (rc != IFKV_OK) return rc;
    }
  }
  return flush();
}

int score_validate(ifkv_ctx *ctx, const void *k_global, int64_t n_ctx, const void *q_prompt, int32_t m_prompt,
                   const void *k_prompt, const float *scores) {
  if (n_ctx < 0 || m_prompt < 0) return fail(ctx, IFKV_EINVAL, "score_tokens: negative size");
  if (n_ctx > ctx->desc.max_ctx)
    return fail(ctx, IFKV_ESHAPE, "score_tokens: n_ctx=%lld exceeds max_ctx=%lld", static_cast<long long>(n_ctx),
                static_cast<long long>(ctx->desc.max_ctx));
  if (m_prompt > ctx->desc.max_prompt)
    return fail(ctx, IFKV_ESHAPE, "score_tokens: m_prompt=%d exceeds max_prompt=%d", m_prompt, ctx->desc.max_prompt);
  if (n_ctx == 0) return IFKV_OK;
  if (scores == nullptr) return fail(ctx, IFKV_EINVAL, "score_tokens: scores is NULL");
  if (m_prompt > 0 && (k_global == nullptr || q_prompt == nullptr))
    return fail(ctx, IFKV_EINVAL, "score_tokens: k_global and q_prompt are required");
  if (!aligned16(k_global) || !aligned16(q_prompt) || !aligned16(k_prompt))
    return fail(ctx, IFKV_EINVAL, "score_tokens: inputs must be 16-byte aligned");
  return IFKV_OK;
}

}  // namespace

int ifkv_reposition_keys(ifkv_ctx *ctx, int32_t n_chunks, const void *const *k_chunks,
                         const void *const *v_chunks, const int32_t *chunk_len,
                         const int32_t *chunk_order, const int32_t *cached_pos0,
                         const int64_t *delta_override, void *k_out, void *v_out,
                         int64_t *chunk_start_out, int64_t *n_ctx_out) {
  if (ctx == nullptr) return IFKV_EINVAL;
  const RepoArgs a = {n_chunks, k_chunks, v_chunks, chunk_len, chunk_order, cached_pos0, delta_override,
                      k_out, v_out, chunk_start_out, n_ctx_out};
  std::vector<int64_t> start;
  int64_t n_ctx = 0;
  int rc = repo_validate(ctx, a, start, &n_ctx);
  if (rc != IFKV_OK || n_ctx == 0) return rc;
  return repo_launch(ctx, a, start);
}

int ifkv_reposition_score(ifkv_ctx *ctx, int32_t n_chunks, const void *const *k_chunks,
                          const void *const *v_chunks, const int32_t *chunk_len, const int32_t *chunk_order,
                          const int32_t *cached_pos0, const int64_t *delta_override, void *k_out, void *v_out,
                          int64_t *chunk_start_out, int64_t *n_ctx_out, const void *q_prompt, int32_t m_prompt,
                          const void *k_prompt, int32_t accumulate, float *scores) {
  if (ctx == nullptr) return IFKV_EINVAL;
  const RepoArgs a = {n_chunks, k_chunks, v_chunks, chunk_len, chunk_order, cached_pos0, delta_override,
                      k_out, v_out, chunk_start_out, n_ctx_out};
  std::vector<int64_t> start;
  int64_t n_ctx = 0;
  int rc = repo_validate(ctx, a, start, &n_ctx);
  if (rc != IFKV_OK) return rc;
  rc = score_validate(ctx, k_out, n_ctx, q_prompt, m_prompt, k_prompt, scores);
  if (rc != IFKV_OK || n_ctx == 0) return rc;
  rc = ensure_scratch(ctx);
  if (rc != IFKV_OK) return rc;
  // chunks that hold rows, in the order of the concatenation
  std::vector<ifkv::FusedHostChunk> fc;
  for (int s = 0; s < n_chunks; ++s) {
    const int c = chunk_order != nullptr ? chunk_order[s] : s;
    if (chunk_len[c] == 0) continue;
    fc.push_back({k_chunks[c], v_chunks != nullptr ? v_chunks[c] : nullptr, start[c],
                  static_cast<double>(repo_advance(a, start, c))});
  }
  if (m_prompt > 0 && ifkv::fused_repo_score_supported(ctx, m_prompt, static_cast<int>(fc.size()))) {
    rc = ensure_inv_freq(ctx);
    if (rc != IFKV_OK) return rc;
    const ifkv::FusedRepo fr = {fc.data(), static_cast<int>(fc.size()), k_out, v_chunks != nullptr ? v_out : nullptr};
    hipError_t e = ifkv::launch_score(ctx, k_out, n_ctx, q_prompt, m_prompt, k_prompt, accumulate != 0, scores, &fr);
    return e == hipSuccess ? IFKV_OK : hip_fail(ctx, e, "fused reposition + score launch");
  }
  // otherwise the two stages one after the other
  rc = repo_launch(ctx, a, start);
  if (rc != IFKV_OK) return rc;
  hipError_t e = ifkv::launch_score(ctx, k_out, n_ctx, q_prompt, m_prompt, k_prompt, accumulate != 0, scores);
  return e == hipSuccess ? IFKV_OK : hip_fail(ctx, e, "score kernel launch");
}

int ifkv_score_tokens(ifkv_ctx *ctx, const void *k_global, int64_t n_ctx, const void *q_prompt,
                      int32_t m_prompt, const void *k_prompt, int32_t accumulate, float *scores) {
  if (ctx == nullptr) return IFKV_EINVAL;
  int rc = score_validate(ctx, k_global, n_ctx, q_prompt, m_prompt, k_prompt, scores);
  if (rc != IFKV_OK || n_ctx == 0) return rc;
  rc = ensure_scratch(ctx);
  if (rc != IFKV_OK) return rc;
  hipError_t e = ifkv::launch_score(ctx, k_global, n_ctx, q_prompt, m_prompt, k_prompt, accumulate != 0, scores);
  return e == hipSuccess ? IFKV_OK : hip_fail(ctx, e, "score kernel launch");
}

namespace {

// Argument checks and the budget shared by the two top-k entry points.  Returns IFKV_OK with *k set.
int topk_budget(ifkv_ctx *ctx, int64_t n_ctx, double ratio, int64_t k_override, int64_t *k) {
  if (n_ctx < 0) return fail(ctx, IFKV_EINVAL, "select_topk: n_ctx is negative");
  if (n_ctx > ctx->desc.max_ctx || n_ctx >= (int64_t(1) << 31))
    return fail(ctx, IFKV_ESHAPE, "select_topk: n_ctx=%lld exceeds max_ctx", static_cast<long long>(n_ctx));
  if (k_override >= 0) {
    *k = k_override;
  } else {
    if (!(ratio >= 0.0 && ratio <= 1.0))
      return fail(ctx, IFKV_EINVAL, "select_topk: ratio=%g is outside [0, 1]", ratio);
    *k = static_cast<int64_t>(std::floor(ratio * static_cast<double>(n_ctx)));  // k = floor(rho N)
  }
  if (*k > n_ctx)
    return fail(ctx, IFKV_EINVAL, "select_topk: k=%lld exceeds n_ctx=%lld", static_cast<long long>(*k),
                static_cast<long long>(n_ctx));
  return IFKV_OK;
}

}  // namespace

int ifkv_select_topk(ifkv_ctx *ctx, const float *scores, int64_t n_ctx, double ratio, int64_t k_override,
                     int32_t *idx_out, int64_t *k_out) {
  if (ctx == nullptr) return IFKV_EINVAL;
  int64_t k = 0;
  int rc = topk_budget(ctx, n_ctx, ratio, k_override, &k);
  if (rc != IFKV_OK) return rc;
  if (k_out != nullptr) *k_out = k;
  if (k == 0 || idx_out == nullptr) return IFKV_OK;  // no output buffer: the caller only asks for k
  if (scores == nullptr) return fail(ctx, IFKV_EINVAL, "select_topk: scores is NULL");
  rc = ensure_scratch(ctx);
  if (rc != IFKV_OK) return rc;
  hipError_t e = ifkv::launch_topk(ctx, scores, n_ctx, k, idx_out, ctx->scratch);
  return e == hipSuccess ? IFKV_OK : hip_fail(ctx, e, "top-k kernel launch");
}

int ifkv_select_topk_noalloc(ifkv_ctx *ctx, const float *scores, int64_t n_ctx, double ratio, int64_t k_override,
                             int32_t *idx_out, int64_t *k_out) {
  if (ctx == nullptr) return IFKV_EINVAL;
  int64_t k = 0;
  int rc = topk_budget(ctx, n_ctx, ratio, k_override, &k);
  if (rc != IFKV_OK) return rc;
  if (n_ctx > ifkv::topk_static_max_ctx())
    return fail(ctx, IFKV_ESHAPE, "select_topk_noalloc: n_ctx=%lld exceeds the %lld scores this entry point serves",
                static_cast<long long>(n_ctx), static_cast<long long>(ifkv::topk_static_max_ctx()));
  if (k_out != nullptr) *k_out = k;
  if (k == 0 || idx_out == nullptr) return IFKV_OK;  // no output buffer: the caller only asks for k
  if (scores == nullptr) return fail(ctx, IFKV_EINVAL, "select_topk_noalloc: scores is NULL");
  void *work = nullptr;
  hipError_t e = ifkv::topk_static_scratch(&work);
  if (e != hipSuccess) return hip_fail(ctx, e, "address of the static scratch");
  e = ifkv::launch_topk(ctx, scores, n_ctx, k, idx_out, work);
  return e == hipSuccess ? IFKV_OK : hip_fail(ctx, e, "top-k kernel launch");
}

int ifkv_recompute_attention(ifkv_ctx *ctx, const void *q_sel, const int32_t *row_pos, int64_t n_rows,
                             const void *k_cache, const void *v_cache, int64_t n_kv, void *out,
                             float *lse_out) {
  if (ctx == nullptr) return IFKV_EINVAL;
  if (n_rows < 0 || n_kv < 0) return fail(ctx, IFKV_EINVAL, "recompute_attention: negative size");
  if (n_kv > ctx->desc.max_ctx)
    return fail(ctx, IFKV_ESHAPE, "recompute_attention: n_kv=%lld exceeds max_ctx=%lld",
                static_cast<long long>(n_kv), static_cast<long long>(ctx->desc.max_ctx));
  if (n_rows >= (int64_t(1) << 31)) return fail(ctx, IFKV_ESHAPE, "recompute_attention: too many rows");
  if (n_rows == 0) return IFKV_OK;
  if (n_kv == 0) return fail(ctx, IFKV_EINVAL, "recompute_attention: rows given but the cache is empty");
  if (q_sel == nullptr || row_pos == nullptr || k_cache == nullptr || v_cache == nullptr || out == nullptr)
    return fail(ctx, IFKV_EINVAL, "recompute_attention: NULL pointer");
  if (!aligned16(q_sel) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out))
    return fail(ctx, IFKV_EINVAL, "recompute_attention: tensors must be 16-byte aligned");
  int rc = ensure_scratch(ctx);
  if (rc != IFKV_OK) return rc;
  if (ctx->desc.flags & IFKV_FLAG_VALIDATE) {
    int64_t bad = -1;
    hipError_t ev = ifkv::validate_ascending(ctx, row_pos, n_rows, &bad);
    if (ev != hipSuccess) return hip_fail(ctx, ev, "row_pos check");
    if (bad >= 0)
      return fail(ctx, IFKV_EINVAL, "recompute_attention: row_pos is not strictly ascending at index %lld",
                  static_cast<long long>(bad));
  }
  hipError_t e = ifkv::launch_attention(ctx, q_sel, row_pos, n_rows, k_cache, v_cache, n_kv, out, lse_out);
  return e == hipSuccess ? IFKV_OK : hip_fail(ctx, e, "attention kernel launch");
}

int ifkv_splice_kv(ifkv_ctx *ctx, const void *k_new, const void *v_new, const int32_t *idx, int64_t n_rows,
                   void *k_cache, void *v_cache, int64_t n_kv) {
  if (ctx == nullptr) return IFKV_EINVAL;
  if (n_rows < 0 || n_kv < 0) return fail(ctx, IFKV_EINVAL, "splice_kv: negative size");
  if (n_kv > ctx->desc.max_ctx)
    return fail(ctx, IFKV_ESHAPE, "splice_kv: n_kv=%lld exceeds max_ctx=%lld", static_cast<long long>(n_kv),
                static_cast<long long>(ctx->desc.max_ctx));
  if (n_rows == 0) return IFKV_OK;
  if (k_new == nullptr || idx == nullptr || k_cache == nullptr)
    return fail(ctx, IFKV_EINVAL, "splice_kv: NULL pointer");
  if ((v_new == nullptr) != (v_cache == nullptr))
    return fail(ctx, IFKV_EINVAL, "splice_kv: v_new and v_cache must both be given or both be NULL");
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache))
    return fail(ctx, IFKV_EINVAL, "splice_kv: tensors must be 16-byte aligned");
  if (ctx->desc.flags & IFKV_FLAG_VALIDATE) {
    int rc = ensure_scratch(ctx);
    if (rc != IFKV_OK) return rc;
    int64_t bad = -1;
    hipError_t ev = ifkv::validate_unique(ctx, idx, n_rows, n_kv, &bad);
    if (ev != hipSuccess) return hip_fail(ctx, ev, "idx check");
    if (bad >= 0)
      return fail(ctx, IFKV_EINVAL, "splice_kv: idx names a cache row twice (one of the two entries is index %lld)",
                  static_cast<long long>(bad));
  }
  hipError_t e = ifkv::launch_splice(ctx, k_new, v_new, idx, n_rows, k_cache, v_cache, n_kv);
  return e == hipSuccess ? IFKV_OK : hip_fail(ctx, e, "splice kernel launch");
}

int ifkv_rope_rows(ifkv_ctx *ctx, void *x, const int32_t *pos, int64_t n_rows, int32_t n_heads) {
  if (ctx == nullptr) return IFKV_EINVAL;
  if (n_rows < 0 || n_heads <= 0) return fail(ctx, IFKV_EINVAL, "rope_rows: n_rows must be >= 0 and n_heads > 0");
  if (n_rows >= (int64_t(1) << 31)) return fail(ctx, IFKV_ESHAPE, "rope_rows: too many rows");
  if (n_rows == 0) return IFKV_OK;
  if (x == nullptr || pos == nullptr) return fail(ctx, IFKV_EINVAL, "rope_rows: NULL pointer");
  if (!aligned16(x)) return fail(ctx, IFKV_EINVAL, "rope_rows: x must be 16-byte aligned");
  int rc = ensure_inv_freq(ctx);
  if (rc != IFKV_OK) return rc;
  hipError_t e = ifkv::launch_rope_rows(ctx, x, pos, n_rows, n_heads);
  return e == hipSuccess ? IFKV_OK : hip_fail(ctx, e, "rope_rows kernel launch");
}

int ifkv_chunk_counts(ifkv_ctx *ctx, const int32_t *idx, int64_t k, int32_t n_slots, const int64_t *slot_start,
                      int64_t n_ctx, int32_t *counts_out) {
  if (ctx == nullptr) return IFKV_EINVAL;
  if (k < 0 || n_slots < 0 || n_ctx < 0) return fail(ctx, IFKV_EINVAL, "chunk_counts: negative size");
  if (n_ctx > ctx->desc.max_ctx || k > n_ctx)
    return fail(ctx, IFKV_ESHAPE, "chunk_counts: n_ctx=%lld (k=%lld) exceeds max_ctx=%lld",
                static_cast<long long>(n_ctx), static_cast<long long>(k), static_cast<long long>(ctx->desc.max_ctx));
  if (n_slots == 0) return IFKV_OK;
  if (slot_start == nullptr || counts_out == nullptr || (k > 0 && idx == nullptr))
    return fail(ctx, IFKV_EINVAL, "chunk_counts: NULL pointer");
  for (int32_t s = 0; s < n_slots; ++s) {
    const int64_t lo = slot_start[s], hi = s + 1 < n_slots ? slot_start[s + 1] : n_ctx;
    if (lo < 0 || lo > hi || hi > n_ctx)
      return fail(ctx, IFKV_EINVAL, "chunk_counts: slot_start must ascend within [0, n_ctx] (slot %d)", s);
  }
  // boundaries travel in the kernel arguments, kRepoMaxChunks slots per launch
  for (int32_t s0 = 0; s0 < n_slots; s0 += ifkv::kRepoMaxChunks) {
    ifkv::SlotBounds b;
    b.n = n_slots - s0 < ifkv::kRepoMaxChunks ? n_slots - s0 : ifkv::kRepoMaxChunks;
    for (int32_t t = 0; t <= b.n; ++t)
      b.bound[t] = static_cast<int32_t>(s0 + t < n_slots ? slot_start[s0 + t] : n_ctx);
    hipError_t e = ifkv::launch_chunk_counts(ctx, idx, k, b, counts_out + s0);
    if (e != hipSuccess) return hip_fail(ctx, e, "chunk_counts kernel launch");
  }
  return IFKV_OK;
}

int ifkv_reorder_chunks(ifkv_ctx *ctx, int32_t n_chunks, const int32_t *order_in, const int32_t *slot_counts,
                        const int32_t *chunk_len, int32_t *order_out) {
  if (n_chunks < 0) return fail(ctx, IFKV_EINVAL, "reorder_chunks: negative chunk count");
  if (n_chunks == 0) return IFKV_OK;
  if (slot_counts == nullptr || chunk_len == nullptr || order_out == nullptr)
    return fail(ctx, IFKV_EINVAL, "reorder_chunks: NULL pointer");
  std::vector<int32_t> order(n_chunks);
  std::vector<char> seen(n_chunks, 0);
  for (int32_t s = 0; s < n_chunks; ++s) {
    const int32_t c = order_in != nullptr ? order_in[s] : s;
    if (c < 0 || c >= n_chunks || seen[c]) return fail(ctx, IFKV_EINVAL, "reorder_chunks: order_in is not a permutation");
    seen[c] = 1;
    order[s] = c;
    if (chunk_len[c] < 0 || slot_counts[s] < 0 || slot_counts[s] > chunk_len[c])
      return fail(ctx, IFKV_EINVAL, "reorder_chunks: slot %d has count %d for a chunk of %d rows", s, slot_counts[s],
                  chunk_len[c]);
  }
  // Eq. (9) compared exactly: r_a < r_b  <=>  count_a * len_b < count_b * len_a (empty chunk: r = 0)
  std::vector<int32_t> slot(n_chunks);
  for (int32_t s = 0; s < n_chunks; ++s) slot[s] = s;
  std::stable_sort(slot.begin(), slot.end(), [&](int32_t a, int32_t b) {
    const int64_t la = chunk_len[order[a]], lb = chunk_len[order[b]];
    const int64_t ca = la > 0 ? slot_counts[a] : 0, cb = lb > 0 ? slot_counts[b] : 0;
    return ca * (lb > 0 ? lb : 1) < cb * (la > 0 ? la : 1);
  });
  for (int32_t s = 0; s < n_chunks; ++s) order_out[s] = order[slot[s]];
  return IFKV_OK;
}

int ifkv_set_tuning(ifkv_ctx *ctx, const char *key, int64_t value) {
  if (ctx == nullptr) return IFKV_EINVAL;
  if (key == nullptr) return fail(ctx, IFKV_EINVAL, "set_tuning: key is NULL");
  struct Knob {
    const char *name;
    int *slot;
    int64_t hi;
  } knobs[] = {{"attn_split_parts", &ctx->tune.attn_split_parts, 65535},
               {"attn_part_tiles", &ctx->tune.attn_part_tiles, 1 << 24},
               {"attn_max_row_blocks", &ctx->tune.attn_max_row_blocks, 65535},
               {"attn_exact_sweep", &ctx->tune.attn_exact_sweep, 1},
               {"fused_repo_score", &ctx->tune.fused_repo_score, 1}};
  for (const Knob &k : knobs) {
    if (std::strcmp(key, k.name) != 0) continue;
    if (value < 0 || value > k.hi)
      return fail(ctx, IFKV_EINVAL, "set_tuning: %s=%lld is outside [0, %lld]", key, static_cast<long long>(value),
                  static_cast<long long>(k.hi));
    *k.slot = static_cast<int>(value);
    return IFKV_OK;
  }
  return fail(ctx, IFKV_EINVAL, "set_tuning: unknown key '%s'", key);
}

int ifkv_attention_plan(ifkv_ctx *ctx, int64_t n_rows, int64_t n_kv, int64_t *plan) {
  if (ctx == nullptr) return IFKV_EINVAL;
  if (plan == nullptr) return fail(ctx, IFKV_EINVAL, "attention_plan: plan is NULL");
  if (n_rows < 0 || n_kv < 1 || n_kv > ctx->desc.max_ctx)
    return fail(ctx, IFKV_EINVAL, "attention_plan: n_rows must be >= 0 and n_kv in [1, max_ctx]");
  const size_t scratch = ctx->scratch != nullptr ? ctx->scratch_bytes : scratch_bytes_for(ctx);
  ifkv::attention_plan(ctx, n_rows, n_kv, scratch, plan);
  plan[4] = static_cast<int64_t>(scratch);
  return IFKV_OK;
}

int ifkv_copy_bytes(ifkv_ctx *ctx, void *dst, const void *src, int64_t n_bytes) {
  if (ctx == nullptr) return IFKV_EINVAL;
  if (n_bytes < 0 || (n_bytes & 15) != 0) return fail(ctx, IFKV_EINVAL, "copy_bytes: size must be a multiple of 16");
  if (n_bytes == 0) return IFKV_OK;
  if (dst == nullptr || src == nullptr || !aligned16(dst) || !aligned16(src))
    return fail(ctx, IFKV_EINVAL, "copy_bytes: pointers must be non-NULL and 16-byte aligned");
  hipError_t e = ifkv::launch_copy(ctx, dst, src, n_bytes);
  return e == hipSuccess ? IFKV_OK : hip_fail(ctx, e, "copy kernel launch");
}

int ifkv_mfma_probe(ifkv_ctx *ctx, int pattern, int64_t iterations, float *sink, double *flops_out) {
  if (ctx == nullptr) return IFKV_EINVAL;
  if (pattern != 0 && pattern != 1) return fail(ctx, IFKV_EINVAL, "mfma_probe: pattern must be 0 or 1");
  if (iterations < 1 || iterations > 10000000) return fail(ctx, IFKV_EINVAL, "mfma_probe: iterations out of range");
  if (sink == nullptr) return fail(ctx, IFKV_EINVAL, "mfma_probe: sink is NULL");
  if (flops_out != nullptr) *flops_out = ifkv::mfma_probe_flops((int)iterations);
  hipError_t e = ifkv::launch_mfma_probe(ctx, pattern, (int)iterations, sink);
  return e == hipSuccess ? IFKV_OK : hip_fail(ctx, e, "mfma probe launch");
}

int64_t ifkv_mfma_probe_sink_floats(void) { return (int64_t)ifkv::mfma_probe_sink_floats(); }

}  // extern "C"
