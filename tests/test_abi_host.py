"""CPU-side checks of the C-ABI library: it loads, exports every symbol the
header declares, and rejects invalid arguments before any GPU call."""
import ctypes as C
import os
import re

import pytest

from paper_2603_05353_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    """Every function declared in include/*.h (the method's ABI, the calibration kernels, the tuning aids)."""
    syms = set()
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if not fn.endswith(".h"):
            continue
        with open(os.path.join(inc, fn)) as f:
            text = f.read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        syms |= set(re.findall(r"\b(ifkv_[a-z_]+)\s*\(", text))
    return sorted(syms)


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2603_05353_amd.build import build_library
        build_library()
    return B.load_library()


def test_exports_every_declared_symbol(lib):
    syms = header_symbols()
    assert len(syms) >= 10
    for s in syms:
        assert hasattr(lib, s), s
    assert set(syms) == set(B.EXPORTS)
    assert lib.ifkv_version().decode().count(".") == 1


def _layer(**kw):
    args = dict(dtype="bf16", n_q_heads=32, n_kv_heads=8, head_dim=128, rope_theta=5e5,
                max_ctx=4096, max_prompt=64)
    args.update(kw)
    return B.Layer(**args)


@pytest.mark.parametrize("kw", [
    dict(n_q_heads=30), dict(n_kv_heads=0), dict(head_dim=96), dict(rope_theta=-1.0),
    dict(max_ctx=0), dict(max_ctx=1 << 31), dict(max_prompt=-1), dict(sm_scale=-0.5),
])
def test_create_rejects_bad_descriptors(lib, kw):
    with pytest.raises(B.IfkvError) as e:
        _layer(**kw)
    assert e.value.code in (B.IFKV_EINVAL, B.IFKV_EDTYPE)
    assert len(str(e.value)) > 20


def test_create_ok_without_gpu(lib):
    L = _layer()
    L.close()
    L.close()  # idempotent


def _call(L, name, *args):
    return getattr(L._lib, name)(L._ctx, *args)


def test_reposition_validation(lib):
    L = _layer()
    fake = C.c_void_p(0x1000)  # never dereferenced: validation fails first
    kp = (C.c_void_p * 3)(0x1000, 0x2000, 0x3000)
    lens = (C.c_int32 * 3)(4, 4, 4)
    bad_order = (C.c_int32 * 3)(0, 0, 1)
    rc = _call(L, "ifkv_reposition_keys", 3, kp, None, lens, bad_order, None, None, fake, None, None, None)
    assert rc == B.IFKV_EINVAL and b"permutation" in L._lib.ifkv_last_error(L._ctx)
    neg = (C.c_int32 * 3)(4, -1, 4)
    assert _call(L, "ifkv_reposition_keys", 3, kp, None, neg, None, None, None, fake, None, None, None) == B.IFKV_EINVAL
    big = (C.c_int32 * 3)(4000, 4000, 4000)
    assert _call(L, "ifkv_reposition_keys", 3, kp, None, big, None, None, None, fake, None, None, None) == B.IFKV_ESHAPE
    assert _call(L, "ifkv_reposition_keys", -1, kp, None, lens, None, None, None, fake, None, None, None) == B.IFKV_EINVAL
    nullk = (C.c_void_p * 3)(0x1000, None, 0x3000)
    assert _call(L, "ifkv_reposition_keys", 3, nullk, None, lens, None, None, None, fake, None, None, None) == B.IFKV_EINVAL
    assert _call(L, "ifkv_reposition_keys", 3, kp, None, lens, None, None, None, None, None, None, None) == B.IFKV_EINVAL
    unaligned = (C.c_void_p * 3)(0x1004, 0x2000, 0x3000)
    assert _call(L, "ifkv_reposition_keys", 3, unaligned, None, lens, None, None, None, fake, None, None, None) == B.IFKV_EINVAL
    # host outputs are valid even when nothing has to run: all chunks empty
    zero = (C.c_int32 * 3)(0, 0, 0)
    starts = (C.c_int64 * 3)(7, 7, 7)
    n = C.c_int64(-1)
    assert _call(L, "ifkv_reposition_keys", 3, kp, None, zero, None, None, None, None, None, starts, C.byref(n)) == B.IFKV_OK
    assert list(starts) == [0, 0, 0] and n.value == 0
    L.close()


def test_score_validation(lib):
    L = _layer()
    f = C.c_void_p(0x1000)
    assert _call(L, "ifkv_score_tokens", f, 5000, f, 8, None, 0, f) == B.IFKV_ESHAPE
    assert _call(L, "ifkv_score_tokens", f, 100, f, 65, None, 0, f) == B.IFKV_ESHAPE
    assert _call(L, "ifkv_score_tokens", f, -1, f, 8, None, 0, f) == B.IFKV_EINVAL
    assert _call(L, "ifkv_score_tokens", f, 100, f, 8, None, 0, None) == B.IFKV_EINVAL
    assert _call(L, "ifkv_score_tokens", None, 100, f, 8, None, 0, f) == B.IFKV_EINVAL
    assert _call(L, "ifkv_score_tokens", f, 0, f, 8, None, 0, f) == B.IFKV_OK
    L.close()


def test_topk_validation_and_budget(lib):
    L = _layer()
    f = C.c_void_p(0x1000)
    k = C.c_int64(-1)
    assert _call(L, "ifkv_select_topk", f, 100, 1.5, -1, f, C.byref(k)) == B.IFKV_EINVAL
    assert _call(L, "ifkv_select_topk", f, 100, -0.1, -1, f, C.byref(k)) == B.IFKV_EINVAL
    assert _call(L, "ifkv_select_topk", f, 100, float("nan"), -1, f, C.byref(k)) == B.IFKV_EINVAL
    assert _call(L, "ifkv_select_topk", f, 100, 0.5, 101, f, C.byref(k)) == B.IFKV_EINVAL
    assert _call(L, "ifkv_select_topk", f, 5000, 0.5, -1, f, C.byref(k)) == B.IFKV_ESHAPE
    # k = floor(rho N) is known on the host; k = 0 launches nothing
    assert _call(L, "ifkv_select_topk", f, 100, 0.0, -1, f, C.byref(k)) == B.IFKV_OK and k.value == 0
    assert _call(L, "ifkv_select_topk", f, 6, 0.15, -1, f, C.byref(k)) == B.IFKV_OK and k.value == 0
    # no output buffer: the call only reports k; an output buffer without scores is an error
    assert _call(L, "ifkv_select_topk", None, 1024, 0.15, -1, None, C.byref(k)) == B.IFKV_OK and k.value == 153
    assert _call(L, "ifkv_select_topk", None, 1024, 0.15, -1, f, C.byref(k)) == B.IFKV_EINVAL and k.value == 153
    L.close()


def test_attention_and_splice_validation(lib):
    L = _layer()
    f = C.c_void_p(0x1000)
    assert _call(L, "ifkv_recompute_attention", f, f, 4, f, f, 5000, f, None) == B.IFKV_ESHAPE
    assert _call(L, "ifkv_recompute_attention", f, f, -4, f, f, 100, f, None) == B.IFKV_EINVAL
    assert _call(L, "ifkv_recompute_attention", f, f, 4, f, f, 0, f, None) == B.IFKV_EINVAL
    assert _call(L, "ifkv_recompute_attention", f, None, 4, f, f, 100, f, None) == B.IFKV_EINVAL
    assert _call(L, "ifkv_recompute_attention", f, f, 0, f, f, 100, f, None) == B.IFKV_OK
    assert _call(L, "ifkv_splice_kv", f, f, f, 4, f, None, 100) == B.IFKV_EINVAL
    assert _call(L, "ifkv_splice_kv", f, f, None, 4, f, f, 100) == B.IFKV_EINVAL
    assert _call(L, "ifkv_splice_kv", f, f, f, 0, f, f, 100) == B.IFKV_OK
    assert _call(L, "ifkv_splice_kv", f, f, f, 4, f, f, 5000) == B.IFKV_ESHAPE
    assert _call(L, "ifkv_copy_bytes", f, f, 24) == B.IFKV_EINVAL
    assert _call(L, "ifkv_copy_bytes", f, f, 0) == B.IFKV_OK
    L.close()


def test_product_does_not_import_oracle():
    """The HIP path must not route through the CPU oracle."""
    pkg = os.path.join(ROOT, "paper_2603_05353_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                with open(os.path.join(dirpath, fn)) as f:
                    text = f.read()
                assert "oracle" not in text.lower(), fn
    with open(os.path.join(ROOT, "oracle", "infoflow_oracle.py")) as f:
        assert "paper_2603_05353_amd" not in f.read().replace("from the product", "")


# --------------------------------------------------------------------------
# chunk reordering: the order computation is host-only, so it is checked against the oracle here
# --------------------------------------------------------------------------
def test_reorder_chunks_matches_oracle(lib):
    import numpy as np
    from oracle import infoflow_oracle as O
    g = np.random.Generator(np.random.Philox(key=[41, 7]))
    L = _layer()
    for _ in range(200):
        n = int(g.integers(1, 12))
        lens = g.integers(0, 7, size=n).tolist()
        order = g.permutation(n).tolist()
        counts_by_chunk = [int(g.integers(0, lens[c] + 1)) for c in range(n)]
        slot_counts = [counts_by_chunk[c] for c in order]
        got = L.reorder_chunks(order, slot_counts, lens)
        assert got == O.reorder_chunks(lens, order, counts_by_chunk).tolist()
    # identity order when order_in is NULL; equal densities keep their order
    assert L.reorder_chunks(None, [1, 2, 3], [2, 4, 6]) == [0, 1, 2]
    assert L.reorder_chunks(None, [3, 0, 1], [3, 3, 3]) == [1, 2, 0]
    L.close()


def test_reorder_and_counts_reject_bad_arguments(lib):
    L = _layer()
    for order, counts, lens in [([0, 0], [0, 0], [1, 1]), ([0, 2], [0, 0], [1, 1]), (None, [2, 0], [1, 1]),
                                (None, [-1, 0], [1, 1])]:
        with pytest.raises(B.IfkvError) as e:
            L.reorder_chunks(order, counts, lens)
        assert e.value.code == B.IFKV_EINVAL
    # slot starts must ascend within [0, n_ctx]; checked on the host before any GPU call
    arr = (C.c_int64 * 2)(5, 3)
    out = (C.c_int32 * 2)()
    rc = lib.ifkv_chunk_counts(L._ctx, None, 0, 2, arr, 10, C.cast(out, C.c_void_p))
    assert rc == B.IFKV_EINVAL and b"ascend" in lib.ifkv_last_error(L._ctx)
    rc = lib.ifkv_chunk_counts(L._ctx, None, 0, 2, None, 10, C.cast(out, C.c_void_p))
    assert rc == B.IFKV_EINVAL
    L.close()


def test_mfma_probe_rejects_bad_arguments(lib):
    L = _layer()
    assert lib.ifkv_mfma_probe_sink_floats() > 0
    flops = C.c_double(-1.0)
    fake = C.c_void_p(256)  # never dereferenced: every call below fails validation first
    assert lib.ifkv_mfma_probe(L._ctx, 2, 10, fake, C.byref(flops)) == B.IFKV_EINVAL
    assert lib.ifkv_mfma_probe(L._ctx, 0, 0, fake, C.byref(flops)) == B.IFKV_EINVAL
    assert lib.ifkv_mfma_probe(L._ctx, 0, 10**8, fake, C.byref(flops)) == B.IFKV_EINVAL
    assert lib.ifkv_mfma_probe(L._ctx, 1, 10, None, C.byref(flops)) == B.IFKV_EINVAL
    assert lib.ifkv_mfma_probe(None, 1, 10, fake, C.byref(flops)) == B.IFKV_EINVAL
    assert flops.value == -1.0
    L.close()


def test_set_tuning_validation(lib):
    L = _layer()
    L.set_tuning("attn_split_parts", 3)
    L.set_tuning("attn_part_tiles", 40)
    L.set_tuning("attn_max_row_blocks", 2)
    L.set_tuning("attn_part_tiles", 0)
    L.set_tuning("fused_repo_score", 1)
    L.set_tuning("fused_repo_score", 0)
    L.set_tuning("attn_exact_sweep", 1)
    L.set_tuning("attn_exact_sweep", 0)
    for key, value in [("attn_split_parts", 65536), ("attn_split_parts", -1), ("attn_max_row_blocks", 65536), ("fused_repo_score", 2),
                       ("attn_exact_sweep", 2),
                       ("no_such_knob", 1)]:
        with pytest.raises(B.IfkvError) as e:
            L.set_tuning(key, value)
        assert e.value.code == B.IFKV_EINVAL
    assert lib.ifkv_set_tuning(L._ctx, None, 1) == B.IFKV_EINVAL
    assert lib.ifkv_set_tuning(None, b"attn_split_parts", 1) == B.IFKV_EINVAL
    L.close()


def test_attention_plan_stays_within_the_scratch(lib):
    """Host arithmetic of stage 4's launch plan: whatever the shape and the knobs, the partial results
    of every launch fit the scratch the context allocates once; cuts that would not fit are not made;
    launches with a handful of row blocks are cut finer than the usual 8 parts."""
    shapes = [(32, 8, 32768), (32, 8, 131072), (28, 4, 20480), (8, 8, 4096), (32, 1, 32768), (64, 2, 65536)]
    knobs = [{}, {"attn_split_parts": 2}, {"attn_split_parts": 65535}, {"attn_part_tiles": 1}, {"attn_part_tiles": 40},
             {"attn_max_row_blocks": 3}, {"attn_max_row_blocks": 3, "attn_part_tiles": 64},
             {"attn_max_row_blocks": 40, "attn_split_parts": 3}]
    for hq, hkv, max_ctx in shapes:
        rpb = 128 // (hq // hkv)
        for kn in knobs:
            L = B.Layer("bf16", hq, hkv, 128, 5e5, max_ctx=max_ctx, max_prompt=128, stream=0)
            for key, value in kn.items():
                L.set_tuning(key, value)
            for n_kv in (1, 64, 65, 2049, max_ctx // 4, max_ctx):
                for n_rows in (0, 1, rpb, rpb + 1, 8 * rpb, 100 * rpb, int(0.05 * n_kv), int(0.15 * n_kv), int(0.3 * n_kv), n_kv):
                    p = L.attention_plan(n_rows, n_kv)
                    tag = (hq, hkv, max_ctx, kn, n_kv, n_rows, p)
                    assert p["partial_bytes"] <= p["scratch_bytes"], tag
                    assert 1 <= p["parts"] <= 65535 and p["part_tiles"] >= 1, tag
                    n_rb = -(-n_rows // rpb)
                    max_rb = kn.get("attn_max_row_blocks", 65535)
                    assert p["launches"] == -(-n_rb // max_rb), tag
                    if p["parts"] == 1:
                        assert p["partial_bytes"] == 0, tag
            L.close()
    # the library's own rule
    L = B.Layer("bf16", 32, 8, 128, 5e5, max_ctx=131072, max_prompt=128, stream=0)
    assert L.attention_plan(19661, 131072)["parts"] == 1          # 15 %: more row blocks than slots, never cut
    assert 2 <= L.attention_plan(1638, 32768)["parts"] <= 8       # 5 % of 32K: cut, at most 8 parts
    few = L.attention_plan(8, 131072)                             # one row block per kv head
    assert few["parts"] == 64 and few["part_tiles"] == 32, few
    assert L.attention_plan(128, 131072)["parts"] == 16           # 32 jobs: 16 parts fill the slots
    # a forced cut that cannot fit falls back to no cut
    L.set_tuning("attn_part_tiles", 1)
    big = L.attention_plan(19661, 131072)
    assert big["parts"] == 1 and big["partial_bytes"] == 0, big
    L.close()
    assert lib.ifkv_attention_plan(None, 1, 1, (C.c_int64 * 5)()) == B.IFKV_EINVAL
    L = _layer()
    for bad in [(-1, 10), (1, 0), (1, 10**9)]:
        with pytest.raises(B.IfkvError) as e:
            L.attention_plan(*bad)
        assert e.value.code == B.IFKV_EINVAL
    assert lib.ifkv_attention_plan(L._ctx, 1, 1, None) == B.IFKV_EINVAL
    L.close()


def test_cache_strides_validation(lib):
    """token_stride / head_stride of the layer descriptor: both or neither, 16-byte multiples, at least
    head_dim, and no overlap of the heads of a row or of the rows of a head."""
    ok = [dict(), dict(token_stride=128, head_stride=128 * 5000), dict(token_stride=8 * 128 + 64, head_stride=136),
          dict(token_stride=8 * 128, head_stride=128)]
    for kw in ok:
        B.Layer("bf16", 32, 8, 128, 5e5, max_ctx=4096, max_prompt=16, stream=0, **kw).close()
    bad = [dict(token_stride=1024), dict(head_stride=128), dict(token_stride=1028, head_stride=128),
           dict(token_stride=64, head_stride=128), dict(token_stride=1024, head_stride=192),    # heads of a row overlap
           dict(token_stride=128, head_stride=128 * 4000),                                      # rows of a head overlap (max_ctx 4096)
           dict(token_stride=1 << 25, head_stride=128)]
    for kw in bad:
        with pytest.raises(B.IfkvError) as e:
            B.Layer("bf16", 32, 8, 128, 5e5, max_ctx=4096, max_prompt=16, stream=0, **kw)
        assert e.value.code == B.IFKV_EINVAL, kw


def test_select_topk_reports_k_without_a_buffer(lib):
    L = _layer()
    k = C.c_int64(-1)
    assert lib.ifkv_select_topk(L._ctx, None, 1024, 0.15, -1, None, C.byref(k)) == B.IFKV_OK and k.value == 153
    assert lib.ifkv_select_topk(L._ctx, None, 1000, 0.0, 77, None, C.byref(k)) == B.IFKV_OK and k.value == 77
    assert lib.ifkv_select_topk_noalloc(L._ctx, None, 1024, 0.3, -1, None, C.byref(k)) == B.IFKV_OK and k.value == 307
    assert L.budget_of(1024, 0.15) == 153
    L.close()
