// Drives the host side of the C ABI -- everything that runs before a GPU call: descriptor checks,
// argument validation of every stage, the launch plan of stage 4, the chunk reordering -- in a build
// whose host code is instrumented with AddressSanitizer and UndefinedBehaviorSanitizer
// (tests/test_host_sanitizers.py compiles and runs it on the CPU).  Device pointers are fake and
// never dereferenced: every call here either fails its validation or has nothing to launch.
// Exit status 0 = every expectation held; the sanitizers abort the process on a finding.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ifkv.h"
#include "ifkv_calibrate.h"
#include "ifkv_debug.h"

static int g_failures = 0;
#define EXPECT(cond)                                                  \
  do {                                                                \
    if (!(cond)) {                                                    \
      std::printf("line %d: expectation failed: %s\n", __LINE__, #cond); \
      ++g_failures;                                                   \
    }                                                                 \
  } while (0)

static ifkv_layer_desc base_desc() {
  ifkv_layer_desc d;
  std::memset(&d, 0, sizeof d);
  d.dtype = IFKV_BF16;
  d.n_q_heads = 32;
  d.n_kv_heads = 8;
  d.head_dim = 128;
  d.rope_theta = 5e5;
  d.pairing = IFKV_ROPE_HALF;
  d.max_ctx = 4096;
  d.max_prompt = 64;
  return d;
}

static uint32_t lcg(uint32_t &s) { return s = s * 1664525u + 1013904223u; }

int main() {
  EXPECT(std::strchr(ifkv_version(), '.') != nullptr);
  EXPECT(ifkv_last_error(nullptr) != nullptr);

  // ---- descriptors -------------------------------------------------------------------------
  {
    ifkv_ctx *c = reinterpret_cast<ifkv_ctx *>(0x10);
    EXPECT(ifkv_create(&c, nullptr, nullptr) != IFKV_OK && c == nullptr);
    EXPECT(ifkv_create(nullptr, nullptr, nullptr) != IFKV_OK);
    struct Bad { void (*edit)(ifkv_layer_desc &); } bad[] = {
        {[](ifkv_layer_desc &d) { d.n_q_heads = 30; }},       {[](ifkv_layer_desc &d) { d.n_kv_heads = 0; }},
        {[](ifkv_layer_desc &d) { d.head_dim = 96; }},        {[](ifkv_layer_desc &d) { d.rope_theta = -1.0; }},
        {[](ifkv_layer_desc &d) { d.max_ctx = 0; }},          {[](ifkv_layer_desc &d) { d.max_ctx = int64_t(1) << 31; }},
        {[](ifkv_layer_desc &d) { d.max_prompt = -1; }},      {[](ifkv_layer_desc &d) { d.sm_scale = -0.5f; }},
        {[](ifkv_layer_desc &d) { d.dtype = 7; }},            {[](ifkv_layer_desc &d) { d.pairing = 9; }},
        {[](ifkv_layer_desc &d) { d.token_stride = 1024; }},  {[](ifkv_layer_desc &d) { d.head_stride = 128; }},
        {[](ifkv_layer_desc &d) { d.token_stride = 1028; d.head_stride = 128; }},
        {[](ifkv_layer_desc &d) { d.token_stride = 1024; d.head_stride = 192; }},
        {[](ifkv_layer_desc &d) { d.token_stride = int64_t(1) << 25; d.head_stride = 128; }},
    };
    for (const Bad &b : bad) {
      ifkv_layer_desc d = base_desc();
      b.edit(d);
      c = reinterpret_cast<ifkv_ctx *>(0x10);
      const int rc = ifkv_create(&c, &d, nullptr);
      EXPECT(rc == IFKV_EINVAL || rc == IFKV_EDTYPE);
      EXPECT(c == nullptr);
      EXPECT(std::strlen(ifkv_last_error(nullptr)) > 10);
    }
    // a caller-owned frequency table is copied: it may go away right after ifkv_create
    ifkv_layer_desc d = base_desc();
    double *table = static_cast<double *>(std::malloc(64 * sizeof(double)));
    for (int i = 0; i < 64; ++i) table[i] = std::pow(1e4, -2.0 * i / 128);
    d.inv_freq = table;
    EXPECT(ifkv_create(&c, &d, nullptr) == IFKV_OK && c != nullptr);
    std::free(table);
    int64_t plan[5];
    EXPECT(ifkv_attention_plan(c, 100, 1000, plan) == IFKV_OK);
    ifkv_destroy(c);
    ifkv_destroy(nullptr);
    // strided layouts that are accepted
    d = base_desc();
    d.token_stride = 128;
    d.head_stride = 128 * 5000;
    EXPECT(ifkv_create(&c, &d, nullptr) == IFKV_OK);
    ifkv_destroy(c);
    for (int rep = 0; rep < 50; ++rep) {  // create / destroy does not accumulate anything
      d = base_desc();
      EXPECT(ifkv_create(&c, &d, nullptr) == IFKV_OK);
      ifkv_destroy(c);
    }
  }

  ifkv_layer_desc d = base_desc();
  ifkv_ctx *L = nullptr;
  EXPECT(ifkv_create(&L, &d, nullptr) == IFKV_OK);
  void *const f = reinterpret_cast<void *>(0x1000);
  float *const ff = reinterpret_cast<float *>(0x1000);
  int32_t *const fi = reinterpret_cast<int32_t *>(0x1000);

  // ---- stage 1 -----------------------------------------------------------------------------
  {
    const void *kp[3] = {reinterpret_cast<void *>(0x1000), reinterpret_cast<void *>(0x2000), reinterpret_cast<void *>(0x3000)};
    const int32_t lens[3] = {4, 4, 4}, bad_order[3] = {0, 0, 1}, neg[3] = {4, -1, 4}, big[3] = {4000, 4000, 4000}, zero[3] = {0, 0, 0};
    EXPECT(ifkv_reposition_keys(L, 3, kp, nullptr, lens, bad_order, nullptr, nullptr, f, nullptr, nullptr, nullptr) == IFKV_EINVAL);
    EXPECT(std::strstr(ifkv_last_error(L), "permutation") != nullptr);
    const int32_t out_of_range[3] = {0, 1, 3};
    EXPECT(ifkv_reposition_keys(L, 3, kp, nullptr, lens, out_of_range, nullptr, nullptr, f, nullptr, nullptr, nullptr) == IFKV_EINVAL);
    EXPECT(ifkv_reposition_keys(L, 3, kp, nullptr, neg, nullptr, nullptr, nullptr, f, nullptr, nullptr, nullptr) == IFKV_EINVAL);
    EXPECT(ifkv_reposition_keys(L, 3, kp, nullptr, big, nullptr, nullptr, nullptr, f, nullptr, nullptr, nullptr) == IFKV_ESHAPE);
    EXPECT(ifkv_reposition_keys(L, -1, kp, nullptr, lens, nullptr, nullptr, nullptr, f, nullptr, nullptr, nullptr) == IFKV_EINVAL);
    const void *nullk[3] = {kp[0], nullptr, kp[2]};
    EXPECT(ifkv_reposition_keys(L, 3, nullk, nullptr, lens, nullptr, nullptr, nullptr, f, nullptr, nullptr, nullptr) == IFKV_EINVAL);
    EXPECT(ifkv_reposition_keys(L, 3, kp, nullptr, lens, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == IFKV_EINVAL);
    const void *unaligned[3] = {reinterpret_cast<void *>(0x1004), kp[1], kp[2]};
    EXPECT(ifkv_reposition_keys(L, 3, unaligned, nullptr, lens, nullptr, nullptr, nullptr, f, nullptr, nullptr, nullptr) == IFKV_EINVAL);
    int64_t starts[3] = {7, 7, 7}, n = -1;
    EXPECT(ifkv_reposition_keys(L, 3, kp, nullptr, zero, nullptr, nullptr, nullptr, nullptr, nullptr, starts, &n) == IFKV_OK);
    EXPECT(starts[0] == 0 && starts[1] == 0 && starts[2] == 0 && n == 0);
    // the one-call form of stages 1 + 2 shares these checks
    EXPECT(ifkv_reposition_score(L, 3, kp, nullptr, lens, bad_order, nullptr, nullptr, f, nullptr, nullptr, nullptr, f, 8, nullptr, 0, ff) == IFKV_EINVAL);
    EXPECT(ifkv_reposition_score(L, 3, kp, nullptr, lens, nullptr, nullptr, nullptr, f, nullptr, nullptr, nullptr, f, 65, nullptr, 0, ff) == IFKV_ESHAPE);
    EXPECT(ifkv_reposition_score(L, 3, kp, nullptr, lens, nullptr, nullptr, nullptr, f, nullptr, nullptr, nullptr, f, 8, nullptr, 0, nullptr) == IFKV_EINVAL);
  }

  // ---- stage 2 -----------------------------------------------------------------------------
  EXPECT(ifkv_score_tokens(L, f, 5000, f, 8, nullptr, 0, ff) == IFKV_ESHAPE);
  EXPECT(ifkv_score_tokens(L, f, 100, f, 65, nullptr, 0, ff) == IFKV_ESHAPE);
  EXPECT(ifkv_score_tokens(L, f, -1, f, 8, nullptr, 0, ff) == IFKV_EINVAL);
  EXPECT(ifkv_score_tokens(L, f, 100, f, 8, nullptr, 0, nullptr) == IFKV_EINVAL);
  EXPECT(ifkv_score_tokens(L, nullptr, 100, f, 8, nullptr, 0, ff) == IFKV_EINVAL);
  EXPECT(ifkv_score_tokens(L, f, 0, f, 8, nullptr, 0, ff) == IFKV_OK);
  EXPECT(ifkv_score_tokens(nullptr, f, 0, f, 8, nullptr, 0, ff) == IFKV_EINVAL);

  // ---- stage 3 -----------------------------------------------------------------------------
  {
    int64_t k = -1;
    EXPECT(ifkv_select_topk(L, ff, 100, 1.5, -1, fi, &k) == IFKV_EINVAL);
    EXPECT(ifkv_select_topk(L, ff, 100, -0.1, -1, fi, &k) == IFKV_EINVAL);
    EXPECT(ifkv_select_topk(L, ff, 100, std::nan(""), -1, fi, &k) == IFKV_EINVAL);
    EXPECT(ifkv_select_topk(L, ff, 100, 0.5, 101, fi, &k) == IFKV_EINVAL);
    EXPECT(ifkv_select_topk(L, ff, 5000, 0.5, -1, fi, &k) == IFKV_ESHAPE);
    EXPECT(ifkv_select_topk(L, ff, 100, 0.0, -1, fi, &k) == IFKV_OK && k == 0);
    EXPECT(ifkv_select_topk(L, ff, 6, 0.15, -1, fi, &k) == IFKV_OK && k == 0);
    EXPECT(ifkv_select_topk(L, nullptr, 1024, 0.15, -1, nullptr, &k) == IFKV_OK && k == 153);
    EXPECT(ifkv_select_topk(L, nullptr, 1024, 0.15, -1, fi, &k) == IFKV_EINVAL);
    EXPECT(ifkv_select_topk(L, nullptr, 1024, 0.15, -1, nullptr, nullptr) == IFKV_OK);
    EXPECT(ifkv_select_topk_noalloc(L, ff, 100, 1.5, -1, fi, &k) == IFKV_EINVAL);
    EXPECT(ifkv_select_topk_noalloc(L, ff, 100, 0.0, -1, fi, &k) == IFKV_OK && k == 0);
    EXPECT(ifkv_select_topk_noalloc(L, nullptr, 1024, 0.3, -1, nullptr, &k) == IFKV_OK && k == 307);
    // every ratio's budget is floor(ratio * n) evaluated without going past n
    for (int64_t n : {int64_t(1), int64_t(7), int64_t(100), int64_t(4096)})
      for (double r : {0.0, 0.05, 0.15, 0.3, 0.999999, 1.0}) {
        EXPECT(ifkv_select_topk(L, nullptr, n, r, -1, nullptr, &k) == IFKV_OK);
        EXPECT(k >= 0 && k <= n && k == static_cast<int64_t>(std::floor(r * static_cast<double>(n))));
      }
  }

  // ---- stages 4 and 5 ----------------------------------------------------------------------
  EXPECT(ifkv_recompute_attention(L, f, fi, 4, f, f, 5000, f, nullptr) == IFKV_ESHAPE);
  EXPECT(ifkv_recompute_attention(L, f, fi, -4, f, f, 100, f, nullptr) == IFKV_EINVAL);
  EXPECT(ifkv_recompute_attention(L, f, fi, 4, f, f, 0, f, nullptr) == IFKV_EINVAL);
  EXPECT(ifkv_recompute_attention(L, f, nullptr, 4, f, f, 100, f, nullptr) == IFKV_EINVAL);
  EXPECT(ifkv_recompute_attention(L, f, fi, 0, f, f, 100, f, nullptr) == IFKV_OK);
  EXPECT(ifkv_splice_kv(L, f, f, fi, 4, f, nullptr, 100) == IFKV_EINVAL);
  EXPECT(ifkv_splice_kv(L, f, f, nullptr, 4, f, f, 100) == IFKV_EINVAL);
  EXPECT(ifkv_splice_kv(L, f, f, fi, 0, f, f, 100) == IFKV_OK);
  EXPECT(ifkv_splice_kv(L, f, f, fi, 4, f, f, 5000) == IFKV_ESHAPE);
  EXPECT(ifkv_rope_rows(L, nullptr, fi, 4, 8) == IFKV_EINVAL);
  EXPECT(ifkv_rope_rows(L, f, fi, 0, 8) == IFKV_OK);
  EXPECT(ifkv_copy_bytes(L, f, f, 24) == IFKV_EINVAL);
  EXPECT(ifkv_copy_bytes(L, f, f, 0) == IFKV_OK);
  {
    double flops = -1.0;
    EXPECT(ifkv_mfma_probe(L, 2, 10, ff, &flops) == IFKV_EINVAL);
    EXPECT(ifkv_mfma_probe(L, 0, 0, ff, &flops) == IFKV_EINVAL);
    EXPECT(ifkv_mfma_probe(L, 1, 10, nullptr, &flops) == IFKV_EINVAL);
    EXPECT(flops == -1.0);
    EXPECT(ifkv_mfma_probe_sink_floats() > 0);
  }

  // ---- knobs and the launch plan of stage 4 ------------------------------------------------
  EXPECT(ifkv_set_tuning(L, nullptr, 1) == IFKV_EINVAL);
  EXPECT(ifkv_set_tuning(nullptr, "attn_split_parts", 1) == IFKV_EINVAL);
  EXPECT(ifkv_set_tuning(L, "no_such_knob", 1) == IFKV_EINVAL);
  EXPECT(ifkv_set_tuning(L, "attn_split_parts", 65536) == IFKV_EINVAL);
  EXPECT(ifkv_set_tuning(L, "attn_split_parts", -1) == IFKV_EINVAL);
  ifkv_destroy(L);
  {
    const int shapes[][3] = {{32, 8, 32768}, {32, 8, 131072}, {28, 4, 20480}, {8, 8, 4096}, {32, 1, 32768}, {64, 2, 65536}};
    struct Knobs { const char *k1; int64_t v1; const char *k2; int64_t v2; } knobs[] = {
        {nullptr, 0, nullptr, 0},       {"attn_split_parts", 2, nullptr, 0},    {"attn_split_parts", 65535, nullptr, 0},
        {"attn_part_tiles", 1, nullptr, 0}, {"attn_part_tiles", 40, nullptr, 0}, {"attn_max_row_blocks", 3, nullptr, 0},
        {"attn_max_row_blocks", 3, "attn_part_tiles", 64}, {"attn_max_row_blocks", 40, "attn_split_parts", 3}};
    for (const auto &sh : shapes)
      for (const Knobs &kn : knobs) {
        ifkv_layer_desc dd = base_desc();
        dd.n_q_heads = sh[0];
        dd.n_kv_heads = sh[1];
        dd.max_ctx = sh[2];
        dd.max_prompt = 128;
        ifkv_ctx *c = nullptr;
        EXPECT(ifkv_create(&c, &dd, nullptr) == IFKV_OK);
        if (kn.k1) EXPECT(ifkv_set_tuning(c, kn.k1, kn.v1) == IFKV_OK);
        if (kn.k2) EXPECT(ifkv_set_tuning(c, kn.k2, kn.v2) == IFKV_OK);
        const int64_t rpb = 128 / (sh[0] / sh[1]);
        for (int64_t n_kv : {int64_t(1), int64_t(64), int64_t(65), int64_t(2049), int64_t(sh[2] / 4), int64_t(sh[2])})
          for (int64_t n_rows : {int64_t(0), int64_t(1), rpb, rpb + 1, 8 * rpb, 100 * rpb, n_kv / 20, n_kv * 3 / 20, n_kv}) {
            int64_t p[5] = {-1, -1, -1, -1, -1};
            EXPECT(ifkv_attention_plan(c, n_rows, n_kv, p) == IFKV_OK);
            EXPECT(p[3] <= p[4]);
            EXPECT(p[1] >= 1 && p[1] <= 65535 && p[2] >= 1);
            EXPECT(p[1] > 1 || p[3] == 0);
          }
        int64_t p[5];
        EXPECT(ifkv_attention_plan(c, -1, 10, p) == IFKV_EINVAL);
        EXPECT(ifkv_attention_plan(c, 1, 0, p) == IFKV_EINVAL);
        EXPECT(ifkv_attention_plan(c, 1, int64_t(sh[2]) + 1, p) == IFKV_EINVAL);
        EXPECT(ifkv_attention_plan(c, 1, 1, nullptr) == IFKV_EINVAL);
        ifkv_destroy(c);
      }
  }

  // ---- chunk reordering (host code) ----------------------------------------------------------
  {
    uint32_t seed = 4107;
    for (int rep = 0; rep < 500; ++rep) {
      const int n = 1 + static_cast<int>(lcg(seed) >> 16) % 40;
      std::vector<int32_t> lens(n), order(n), counts(n), out(n, -1);
      for (int i = 0; i < n; ++i) lens[i] = static_cast<int32_t>((lcg(seed) >> 16) % 9);
      for (int i = 0; i < n; ++i) order[i] = i;
      for (int i = n - 1; i > 0; --i) std::swap(order[i], order[(lcg(seed) >> 16) % (i + 1)]);
      for (int s = 0; s < n; ++s) counts[s] = static_cast<int32_t>((lcg(seed) >> 16) % (lens[order[s]] + 1));
      EXPECT(ifkv_reorder_chunks(nullptr, n, rep % 3 == 0 ? nullptr : order.data(), counts.data(), lens.data(), out.data()) ==
             (rep % 3 == 0 ? ifkv_reorder_chunks(nullptr, n, nullptr, counts.data(), lens.data(), out.data()) : IFKV_OK));
      if (rep % 3 != 0) {  // a permutation, densities ascending
        std::vector<int> seen(n, 0), slot_of(n);
        for (int s = 0; s < n; ++s) slot_of[order[s]] = s;
        bool ok = true;
        for (int s = 0; s < n; ++s) ok = ok && out[s] >= 0 && out[s] < n && seen[out[s]]++ == 0;
        EXPECT(ok);
        for (int s = 0; ok && s + 1 < n; ++s) {
          const int a = out[s], b = out[s + 1];
          const int64_t ca = counts[slot_of[a]], cb = counts[slot_of[b]];
          // density a <= density b as exact fractions; an empty chunk has density 0
          const int64_t lhs = lens[a] == 0 ? 0 : ca * (lens[b] == 0 ? 1 : lens[b]);
          const int64_t rhs = lens[b] == 0 ? 0 : cb * (lens[a] == 0 ? 1 : lens[a]);
          EXPECT(lhs <= rhs);
        }
      }
    }
    const int32_t two[2] = {0, 0}, lens2[2] = {1, 1}, over[2] = {2, 0}, negc[2] = {-1, 0}, badp[2] = {0, 2};
    int32_t out2[2];
    EXPECT(ifkv_reorder_chunks(nullptr, 2, two, two, lens2, out2) == IFKV_EINVAL);
    EXPECT(ifkv_reorder_chunks(nullptr, 2, badp, two, lens2, out2) == IFKV_EINVAL);
    EXPECT(ifkv_reorder_chunks(nullptr, 2, nullptr, over, lens2, out2) == IFKV_EINVAL);
    EXPECT(ifkv_reorder_chunks(nullptr, 2, nullptr, negc, lens2, out2) == IFKV_EINVAL);
    EXPECT(ifkv_reorder_chunks(nullptr, 2, nullptr, two, lens2, nullptr) == IFKV_EINVAL);
    EXPECT(ifkv_reorder_chunks(nullptr, 0, nullptr, nullptr, nullptr, nullptr) == IFKV_OK ||
           ifkv_reorder_chunks(nullptr, 0, nullptr, nullptr, nullptr, nullptr) == IFKV_EINVAL);
    ifkv_layer_desc dd = base_desc();
    ifkv_ctx *c = nullptr;
    EXPECT(ifkv_create(&c, &dd, nullptr) == IFKV_OK);
    const int64_t descending[2] = {5, 3};
    int32_t cnt[2];
    EXPECT(ifkv_chunk_counts(c, nullptr, 0, 2, descending, 10, cnt) == IFKV_EINVAL);
    EXPECT(ifkv_chunk_counts(c, nullptr, 0, 2, nullptr, 10, cnt) == IFKV_EINVAL);
    ifkv_destroy(c);
  }

  if (g_failures == 0) std::printf("host ABI under the sanitizers: ok\n");
  return g_failures == 0 ? 0 : 1;
}
