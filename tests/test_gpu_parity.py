"""GPU parity: every stage of the HIP path, called through the C ABI, against
the fp64 CPU oracle on the same seeded inputs.

Tolerances (stated per test):
  stage 1  fp32: 2e-6 * |pair| ; bf16: half a bf16 ulp of the exact value (one
           rounding to storage) + 2e-6 * |pair| for the fp32 rotation
  stage 2  |s - s_ref| <= rtol * (|s_ref| + M/N), rtol 1e-5 (fp32) / 1e-2 (bf16)
  stage 3  bit-exact on identical fp32 input
  stage 4  max-abs 1e-4 (fp32) / 2e-2 (bf16) AND the element-wise rounding bound of
           tests/helpers.attention_error_bound (stays below the signal at any depth)
  stage 5  bit-exact
"""
import numpy as np
import pytest
import torch

from oracle import infoflow_oracle as O
from tests.helpers import (DEV, assert_attention_close, bf16_ulp, make_layer, needle_case, score_tol, to_dev, to_host_bits,
                           to_host_f64)
from workloads import make_recompute_inputs, make_workload, preset, to_f64, to_storage

pytestmark = pytest.mark.gpu

FORCE_GENERIC = 1


def sync():
    torch.cuda.synchronize()


def oracle_inputs(wl):
    sp = wl.spec
    k = [to_f64(c, sp.dtype) for c in wl.k_chunks]
    v = [to_f64(c, sp.dtype) for c in wl.v_chunks]
    return k, v, to_f64(wl.q_prompt, sp.dtype)


def dev_chunks(wl):
    sp = wl.spec
    shape = (0, sp.n_kv_heads, sp.head_dim)
    kd = [to_dev(c.reshape(-1, *shape[1:]), sp.dtype) for c in wl.k_chunks]
    vd = [to_dev(c.reshape(-1, *shape[1:]), sp.dtype) for c in wl.v_chunks]
    return kd, vd


def check_reposition(k_gpu, K_ref, dtype, half):
    """Element-wise bound described in the module docstring."""
    if half == "half":
        d = K_ref.shape[-1]
        pair = np.hypot(K_ref[..., : d // 2], K_ref[..., d // 2:])
        pair = np.concatenate([pair, pair], axis=-1)
    else:
        pr = np.hypot(K_ref[..., 0::2], K_ref[..., 1::2])
        pair = np.repeat(pr, 2, axis=-1)
    err = np.abs(k_gpu - K_ref)
    bound = 2e-6 * pair + 1e-30
    if dtype == "bf16":
        bound = bound + 0.5 * bf16_ulp(K_ref) * 1.001
    worst = (err - bound).max()
    assert worst <= 0, f"reposition error exceeds bound by {worst}"


# ---------------------------------------------------------------------------
# stage 1
# ---------------------------------------------------------------------------
REPO_CASES = [
    ("C1-full", preset("C1")),
    ("C2-ragged", preset("C2", chunk_lens=[70, 0, 33, 129, 16, 1], m_prompt=8)),
    ("C3-permuted", preset("C3", chunk_lens=[96] * 8, m_prompt=8)),
    ("C4-uneven", preset("C4", uneven=(12, 20, 90), m_prompt=8)),
    ("C5-vlm", preset("C5", chunk_lens=[40] * 16 + [24] * 8, m_prompt=8)),
    ("interleaved-bf16", preset("C2", chunk_lens=[50, 31, 64], m_prompt=8, pairing="interleaved")),
    ("interleaved-f32", preset("C1", chunk_lens=[50, 31, 64], m_prompt=8, pairing="interleaved")),
    ("many-chunks", preset("C3", chunk_lens=[5] * 70 + [17] * 3, m_prompt=8)),   # > 64 chunks: two launches
]


@pytest.mark.parametrize("name,spec", REPO_CASES, ids=[c[0] for c in REPO_CASES])
def test_reposition_parity(name, spec):
    wl = make_workload(spec)
    k, v, _ = oracle_inputs(wl)
    K_ref, V_ref, start_ref, N = O.reposition_keys(k, v, wl.chunk_len, wl.chunk_order, spec.rope_theta, spec.pairing)
    L = make_layer(spec, max_ctx=max(N, 1), max_prompt=8)
    kd, vd = dev_chunks(wl)
    k_out, v_out, starts, n_ctx = L.reposition_keys(kd, vd, chunk_order=wl.chunk_order.tolist())
    sync()
    assert n_ctx == N and starts == start_ref.tolist()
    check_reposition(to_host_f64(k_out, spec.dtype), K_ref, spec.dtype, spec.pairing)
    # values: exact gather
    assert np.array_equal(to_host_f64(v_out, spec.dtype), V_ref)
    # the chunk in the first slot is not rotated at all: bit-identical
    c0 = int(wl.chunk_order[0])
    L0 = int(wl.chunk_len[c0])
    assert np.array_equal(to_host_bits(k_out[:L0], spec.dtype).ravel(),
                          to_host_bits(kd[c0], spec.dtype).ravel())
    # keys-only call leaves v untouched and gives the same keys
    k2, v2, _, _ = L.reposition_keys(kd, None, chunk_order=wl.chunk_order.tolist())
    sync()
    assert v2 is None and torch.equal(k2.view(torch.int16 if spec.dtype == "bf16" else torch.int32),
                                      k_out.view(torch.int16 if spec.dtype == "bf16" else torch.int32))
    L.close()


def test_reposition_pos0_and_override():
    spec = preset("C2", chunk_lens=[40, 25, 64], m_prompt=8)
    wl = make_workload(spec)
    k, v, _ = oracle_inputs(wl)
    L = make_layer(spec, max_ctx=wl.n_ctx, max_prompt=8)
    kd, vd = dev_chunks(wl)
    pos0 = [3, 100, 7]
    K_ref, _, _, _ = O.reposition_keys(k, None, wl.chunk_len, None, spec.rope_theta, cached_pos0=pos0)
    k_out, _, _, _ = L.reposition_keys(kd, None, cached_pos0=pos0)
    sync()
    check_reposition(to_host_f64(k_out, "bf16"), K_ref, "bf16", "half")
    over = [0, 0, 129]
    K_ref, _, _, _ = O.reposition_keys(k, None, wl.chunk_len, None, spec.rope_theta, delta_override=over)
    k_out, _, _, _ = L.reposition_keys(kd, None, delta_override=over)
    sync()
    check_reposition(to_host_f64(k_out, "bf16"), K_ref, "bf16", "half")
    L.close()


def test_reposition_large_delta_angles():
    """Phase advances of ~130K positions: angles must be formed in fp64."""
    spec = preset("C1", chunk_lens=[8, 24], m_prompt=8)
    wl = make_workload(spec)
    k, _, _ = oracle_inputs(wl)
    over = [131000, 98765]
    K_ref, _, _, _ = O.reposition_keys(k, None, wl.chunk_len, None, spec.rope_theta, delta_override=over)
    L = make_layer(spec, max_ctx=wl.n_ctx, max_prompt=8)
    kd, _ = dev_chunks(wl)
    k_out, _, _, _ = L.reposition_keys(kd, None, delta_override=over)
    sync()
    check_reposition(to_host_f64(k_out, "f32"), K_ref, "f32", "half")
    L.close()


# ---------------------------------------------------------------------------
# stage 2
# ---------------------------------------------------------------------------
def global_keys(wl):
    """Oracle-side global-frame keys, rounded to the storage dtype so both
    sides score exactly the same stored values."""
    sp = wl.spec
    k, _, q = oracle_inputs(wl)
    K, _, _, N = O.reposition_keys(k, None, wl.chunk_len, wl.chunk_order, sp.rope_theta, sp.pairing)
    K_st = to_storage(K, sp.dtype)
    return K_st, to_f64(K_st, sp.dtype), q


SCORE_CASES = [
    ("C1-full", preset("C1"), 0, 1e-5),
    ("C2-small-alu", preset("C2", chunk_lens=[200, 77, 301], m_prompt=19), FORCE_GENERIC, 1e-2),
    ("C2-small", preset("C2", chunk_lens=[200, 77, 301], m_prompt=19), 0, 1e-2),
    ("C3-small", preset("C3", chunk_lens=[130] * 9, m_prompt=40), 0, 1e-2),
    ("C4-small", preset("C4", uneven=(10, 50, 150), m_prompt=33), 0, 1e-2),
    ("C5-small", preset("C5", chunk_lens=[64] * 16 + [32] * 8, m_prompt=24), 0, 1e-2),
    ("d64-bf16", preset("C2", head_dim=64, n_q_heads=8, n_kv_heads=4, chunk_lens=[100, 50], m_prompt=7), 0, 1e-2),
]


@pytest.mark.parametrize("name,spec,flags,rtol", SCORE_CASES, ids=[c[0] for c in SCORE_CASES])
def test_score_parity(name, spec, flags, rtol):
    wl = make_workload(spec)
    K_st, K64, q64 = global_keys(wl)
    s_ref = O.score_tokens(K64, q64, wl.sm_scale)
    L = make_layer(spec, max_ctx=wl.n_ctx, max_prompt=spec.m_prompt, flags=flags)
    kd = to_dev(K_st, spec.dtype)
    qd = to_dev(wl.q_prompt, spec.dtype)
    s = L.score_tokens(kd, qd)
    sync()
    s = s.cpu().numpy().astype(np.float64)
    assert (np.abs(s - s_ref) <= score_tol(s_ref, spec.m_prompt, rtol)).all(), \
        f"max rel {np.max(np.abs(s - s_ref) / (np.abs(s_ref) + spec.m_prompt / wl.n_ctx))}"
    assert abs(s.sum() - spec.m_prompt) < 1e-3 * spec.m_prompt
    # accumulate adds on top
    s2 = L.score_tokens(kd, qd, scores=torch.from_numpy(s_ref.astype(np.float32)).to(DEV), accumulate=True)
    sync()
    assert (np.abs(s2.cpu().numpy() - 2 * s_ref) <= 2 * score_tol(s_ref, spec.m_prompt, rtol)).all()
    L.close()


# (context lengths, prompt rows, H_q, H_kv): every compiled query-block count of pass A (4, 8, 12, 16),
# several query chunks per kv head, the largest prompt the MFMA path takes (M G = 2048) and the first
# one it hands to the ALU path, and contexts shorter than one key tile
SCORE_SHAPES = [
    ([1], 3, 8, 2), ([63], 32, 8, 2), ([65, 64], 64, 8, 2), ([100, 93], 96, 8, 2), ([70, 121], 128, 8, 2),
    ([150], 130, 8, 2), ([90, 45], 257, 8, 2), ([77], 512, 8, 2), ([77], 513, 8, 2), ([200], 96, 28, 4),
    ([129], 40, 32, 1),
]


@pytest.mark.parametrize("lens,m,hq,hkv", SCORE_SHAPES, ids=[f"N{sum(c[0])}-M{c[1]}-{c[2]}q{c[3]}kv" for c in SCORE_SHAPES])
def test_score_mfma_shapes(lens, m, hq, hkv):
    spec = preset("C2", chunk_lens=lens, m_prompt=m, n_q_heads=hq, n_kv_heads=hkv, seed=20260305 + 50 + m)
    wl = make_workload(spec)
    K_st, K64, q64 = global_keys(wl)
    s_ref = O.score_tokens(K64, q64, wl.sm_scale)
    L = make_layer(spec, max_ctx=wl.n_ctx, max_prompt=m)
    s = L.score_tokens(to_dev(K_st, spec.dtype), to_dev(wl.q_prompt, spec.dtype))
    sync()
    s = s.cpu().numpy().astype(np.float64)
    assert (np.abs(s - s_ref) <= score_tol(s_ref, m, 1e-2)).all(), \
        f"max rel {np.max(np.abs(s - s_ref) / (np.abs(s_ref) + m / wl.n_ctx))}"
    assert abs(s.sum() - m) < 1e-3 * m
    L.close()


@pytest.mark.parametrize("flags", [0, FORCE_GENERIC], ids=["default", "alu"])
def test_score_with_prompt_keys(flags):
    spec = preset("C2", chunk_lens=[90, 41], m_prompt=12)
    wl = make_workload(spec)
    K_st, K64, q64 = global_keys(wl)
    g = np.random.Generator(np.random.Philox(key=[5, 5]))
    kp = to_storage(g.standard_normal((spec.m_prompt, spec.n_kv_heads, spec.head_dim)) * 0.3, "bf16")
    s_ref = O.score_tokens(K64, q64, wl.sm_scale, k_prompt=to_f64(kp, "bf16"))
    L = make_layer(spec, max_ctx=wl.n_ctx, max_prompt=spec.m_prompt, flags=flags)
    s = L.score_tokens(to_dev(K_st, "bf16"), to_dev(wl.q_prompt, "bf16"), k_prompt=to_dev(kp, "bf16"))
    sync()
    s = s.cpu().numpy().astype(np.float64)
    assert (np.abs(s - s_ref) <= score_tol(s_ref, spec.m_prompt, 1e-2)).all()
    assert s.sum() < spec.m_prompt
    L.close()


def test_score_peaky_logits():
    """Logits with a standard deviation of ~4: exercises the running max / rescaling."""
    spec = preset("C2", chunk_lens=[300, 211], m_prompt=16, sigma=2.0)
    wl = make_workload(spec)
    K_st, K64, q64 = global_keys(wl)
    s_ref = O.score_tokens(K64, q64, wl.sm_scale)
    L = make_layer(spec, max_ctx=wl.n_ctx, max_prompt=spec.m_prompt)
    s = L.score_tokens(to_dev(K_st, "bf16"), to_dev(wl.q_prompt, "bf16"))
    sync()
    s = s.cpu().numpy().astype(np.float64)
    assert s_ref.max() > 3 * s_ref.mean()
    assert (np.abs(s - s_ref) <= score_tol(s_ref, spec.m_prompt, 1e-2)).all()
    L.close()


@pytest.mark.parametrize("gain,fused", [(30.0, False), (70.0, False), (200.0, False), (70.0, True)],
                         ids=["logit30", "logit70", "logit200", "logit70-fused-sweep"])
def test_score_prompt_rows_aligned_with_single_keys(gain, fused):
    """Every prompt row points at one key with a logit of `gain` (natural units) while the first keys a
    wavefront sees score near zero: the first sweep of the MFMA path keeps the logit of the first key as
    its reference exponent, so at 70 and 200 its sums leave the range it accepts and the block must repeat
    the sweep with a running maximum; at 30 it must not need to.  `fused`: the same through the sweep
    that reads the chunk caches (ifkv_reposition_score with the fused sweep switched on)."""
    spec = preset("C3", chunk_lens=[300, 211, 150, 600], m_prompt=24)
    wl = make_workload(spec)
    K_st, K64, _ = global_keys(wl)
    N, hq, hkv, d = wl.n_ctx, spec.n_q_heads, spec.n_kv_heads, spec.head_dim
    G = hq // hkv
    g = np.random.Generator(np.random.Philox(key=[77, int(gain)]))
    targets = np.concatenate([[0, 1, 63, 64, 65, N - 1, N - 64, 511, 512], g.integers(0, N, size=64)])
    q = np.empty((spec.m_prompt, hq, d))
    for r in range(spec.m_prompt):
        for h in range(hq):
            kj = K64[targets[(r * hq + h) % len(targets)], h // G]
            q[r, h] = gain * np.sqrt(d) * kj / (kj @ kj)
    q_st = to_storage(q, "bf16")
    s_ref = O.score_tokens(K64, to_f64(q_st, "bf16"), wl.sm_scale)
    assert s_ref[np.unique(targets)].sum() > 0.9 * spec.m_prompt   # the mass sits on the targets
    L = make_layer(spec, max_ctx=N, max_prompt=spec.m_prompt)
    if fused:
        L.set_tuning("fused_repo_score", 1)
        kd, vd = dev_chunks(wl)
        s = L.reposition_score(kd, vd, to_dev(q_st, "bf16"), chunk_order=wl.chunk_order.tolist())[4]
    else:
        s = L.score_tokens(to_dev(K_st, "bf16"), to_dev(q_st, "bf16"))
    sync()
    s = s.cpu().numpy().astype(np.float64)
    assert np.isfinite(s).all()
    assert (np.abs(s - s_ref) <= score_tol(s_ref, spec.m_prompt, 1e-2)).all(), \
        f"max rel {np.max(np.abs(s - s_ref) / (np.abs(s_ref) + spec.m_prompt / N))}"
    assert abs(s.sum() - spec.m_prompt) < 1e-3 * spec.m_prompt
    L.close()


# ---------------------------------------------------------------------------
# stages 1 + 2 in one call (the first scoring sweep reads the chunk caches)
# ---------------------------------------------------------------------------
FUSED_CASES = [
    # name, spec, extras
    ("C2-permuted", preset("C2", chunk_lens=[256, 100, 190, 64, 333], m_prompt=32, permute_order=True), {}),
    ("ragged-with-empty-chunk", preset("C2", chunk_lens=[70, 0, 33, 129, 16, 1, 400], m_prompt=19, permute_order=True), {}),
    ("one-prompt-row", preset("C2", chunk_lens=[300, 211], m_prompt=1), {}),
    ("8-prompt-rows", preset("C3", chunk_lens=[130] * 9, m_prompt=8), {}),
    ("two-query-chunks", preset("C2", chunk_lens=[600, 424], m_prompt=160), {}),                  # 640 query rows per kv head
    ("more-than-64-chunks", preset("C3", chunk_lens=[5] * 70 + [17] * 3 + [240], m_prompt=12), {}),
    ("C5-gqa7", preset("C5", chunk_lens=[200] * 4 + [96] * 3, m_prompt=24), {}),
    ("interleaved", preset("C2", chunk_lens=[150, 31, 264], m_prompt=16, pairing="interleaved", permute_order=True), {}),
    ("cached-from-other-positions", preset("C2", chunk_lens=[90, 141, 130], m_prompt=16), {"cached_pos0": [3, 0, 7]}),
    ("local-geometry", preset("C2", chunk_lens=[90, 141, 130], m_prompt=16), {"delta_override": [0, 0, 0]}),
    ("prompt-keys", preset("C2", chunk_lens=[256, 100, 190], m_prompt=24, permute_order=True), {"with_k_prompt": True}),
    ("keys-only", preset("C2", chunk_lens=[256, 100, 190], m_prompt=24), {"no_v": True}),
    ("head-major-cache", preset("C2", chunk_lens=[256, 100, 190], m_prompt=24, permute_order=True), {"layout": "head-major"}),
    ("fp32-falls-back", preset("C1", chunk_lens=[100, 61, 130], m_prompt=12), {}),
    ("alu-falls-back", preset("C2", chunk_lens=[120, 77], m_prompt=9), {"flags": FORCE_GENERIC}),
]


@pytest.mark.parametrize("fused", [True, False], ids=["fused-sweep", "two-stages"])
@pytest.mark.parametrize("name,spec,extra", FUSED_CASES, ids=[c[0] for c in FUSED_CASES])
def test_reposition_score_in_one_call(name, spec, extra, fused):
    """ifkv_reposition_score against the two calls it stands for (caches and scores bit for bit, also
    when accumulating onto earlier scores) and against the oracle."""
    wl = make_workload(spec)
    k, v, q = oracle_inputs(wl)
    n_ctx = wl.n_ctx
    kw = {}
    if "layout" in extra:
        lay = layouts_for(spec, n_ctx)[extra["layout"]]
        kw = dict(token_stride=lay[0], head_stride=lay[1])
    L = make_layer(spec, max_ctx=n_ctx, max_prompt=spec.m_prompt, flags=extra.get("flags", 0), **kw)
    L.set_tuning("fused_repo_score", 1 if fused else 0)
    kd, vd = dev_chunks(wl)
    if extra.get("no_v"):
        vd = None
    qd = to_dev(wl.q_prompt, spec.dtype)
    order = wl.chunk_order.tolist()
    rk = {key: extra[key] for key in ("cached_pos0", "delta_override") if key in extra}
    kp_st = None
    if extra.get("with_k_prompt"):
        g = np.random.Generator(np.random.Philox(key=[spec.seed, 31]))
        kp_st = to_storage(g.standard_normal((spec.m_prompt, spec.n_kv_heads, spec.head_dim)) * spec.sigma, spec.dtype)
    kpd = None if kp_st is None else to_dev(kp_st, spec.dtype)
    # the two calls
    K1, V1, starts1, N1 = L.reposition_keys(kd, vd, chunk_order=order, **rk)
    s1 = L.score_tokens(K1, qd, k_prompt=kpd)
    # the one call, into caches that hold something else
    K2, V2 = L.empty_cache(n_ctx), (None if vd is None else L.empty_cache(n_ctx))
    K2.fill_(7.0)
    K2, V2, starts2, N2, s2 = L.reposition_score(kd, vd, qd, chunk_order=order, k_out=K2, v_out=V2, k_prompt=kpd, **rk)
    sync()
    assert starts1 == starts2 and N1 == N2 == n_ctx
    assert np.array_equal(to_host_bits(K1, spec.dtype), to_host_bits(K2, spec.dtype))
    if vd is not None:
        assert np.array_equal(to_host_bits(V1, spec.dtype), to_host_bits(V2, spec.dtype))
    assert torch.equal(s1, s2)
    # accumulate: a second layer's scores on top
    s3 = s2.clone()
    L.reposition_score(kd, vd, qd, chunk_order=order, k_out=K2, v_out=V2, k_prompt=kpd, scores=s3, accumulate=True, **rk)
    s4 = s1.clone()
    L.score_tokens(K1, qd, k_prompt=kpd, scores=s4, accumulate=True)
    sync()
    assert torch.equal(s3, s4)
    # the oracle
    K_ref, _, start_ref, _ = O.reposition_keys(k, v, wl.chunk_len, order, spec.rope_theta, spec.pairing,
                                               cached_pos0=rk.get("cached_pos0"), delta_override=rk.get("delta_override"))
    assert starts2 == start_ref.tolist()
    check_reposition(to_host_f64(K2, spec.dtype), K_ref, spec.dtype, spec.pairing)
    s_ref = O.score_tokens(to_host_f64(K2, spec.dtype), q, wl.sm_scale,
                           k_prompt=None if kp_st is None else to_f64(kp_st, spec.dtype))
    rtol = 1e-5 if spec.dtype == "f32" else 1e-2
    assert (np.abs(s2.cpu().numpy() - s_ref) <= score_tol(s_ref, spec.m_prompt, rtol)).all()
    L.close()


# ---------------------------------------------------------------------------
# stage 3
# ---------------------------------------------------------------------------
def topk_case(n, kind, seed):
    g = np.random.Generator(np.random.Philox(key=[seed, n]))
    if kind == "uniform":
        s = g.random(n)
    elif kind == "ties":
        s = g.integers(0, 7, size=n) * 0.125
    elif kind == "equal":
        s = np.full(n, 0.0078125)
    elif kind == "signed":
        s = g.standard_normal(n)
        s[:: 5] = 0.0
        s[1:: 7] = -0.0
    elif kind == "near-uniform":        # what near-uniform attention produces
        s = 0.0078125 * (1 + 1e-6 * g.standard_normal(n))
    else:
        raise ValueError(kind)
    return s.astype(np.float32)


@pytest.mark.parametrize("n", [1, 5, 63, 1000, 8192, 8193, 20000, 32768, 32769, 50000, 140001])
@pytest.mark.parametrize("kind", ["uniform", "ties", "equal", "signed", "near-uniform"])
def test_topk_bit_exact(n, kind):
    s = topk_case(n, kind, 77)
    spec = preset("C1")
    L = make_layer(spec, max_ctx=max(n, 1), max_prompt=8)
    sd = torch.from_numpy(s).to(DEV)
    for k in sorted({0, 1, n // 7, int(0.15 * n), n - 1, n}):
        if k < 0:
            continue
        idx = L.select_topk(sd, k=k)
        sync()
        ref = O.select_topk(s, k)
        assert idx.dtype == torch.int32 and idx.numel() == k
        assert np.array_equal(idx.cpu().numpy().astype(np.int64), ref), (n, kind, k)
    # ratio form
    idx = L.select_topk(sd, ratio=0.15)
    sync()
    assert np.array_equal(idx.cpu().numpy().astype(np.int64), O.select_topk(s, O.budget(n, 0.15)))
    L.close()


def test_topk_unaligned_input():
    s = topk_case(9000, "uniform", 3)
    spec = preset("C1")
    L = make_layer(spec, max_ctx=9000, max_prompt=8)
    buf = torch.zeros(9001, dtype=torch.float32, device=DEV)
    buf[1:] = torch.from_numpy(s).to(DEV)
    idx = L.select_topk(buf[1:], k=1234)
    sync()
    assert np.array_equal(idx.cpu().numpy().astype(np.int64), O.select_topk(s, 1234))
    L.close()


# ---------------------------------------------------------------------------
# stage 4
# ---------------------------------------------------------------------------
def run_attention(spec, q_sel, rows, K_st, V_st, flags=0, tuning=None, max_ctx=None):
    """The library's side of a stage-4 case: (out, lse) as float64 host arrays."""
    L = make_layer(spec, max_ctx=max_ctx or len(K_st), max_prompt=8, flags=flags)
    for key, value in (tuning or {}).items():
        L.set_tuning(key, value)
    out, lse = L.recompute_attention(to_dev(q_sel, spec.dtype), torch.from_numpy(np.asarray(rows).astype(np.int32)).to(DEV),
                                     to_dev(K_st, spec.dtype), to_dev(V_st, spec.dtype), return_lse=True)
    sync()
    L.close()
    return to_host_f64(out, spec.dtype), lse.cpu().numpy().astype(np.float64)


def oracle_attention(q64, rows, K64, V64, scale):
    """(ref, ref_abs, lse_ref): the oracle on V and on |V| (the latter feeds the rounding bound)."""
    ref, lse_ref = O.recompute_attention(q64, rows, K64, V64, scale)
    ref_abs, _ = O.recompute_attention(q64, rows, K64, np.abs(V64), scale)
    return ref, ref_abs, lse_ref


def attention_case(spec, rows, flags=0, q_gain=1.0, tuning=None, n_check=None):
    """Both sides on the spec's workload for the given selected rows, compared element by element
    (the contract's max-abs tolerance and the magnitude-aware bound of tests/helpers.py).  With
    n_check the oracle computes a seeded subsample of the rows (rows are independent)."""
    wl = make_workload(spec)
    K_st, K64, _ = global_keys(wl)
    V_st = np.concatenate([wl.v_chunks[c] for c in wl.chunk_order], axis=0)
    V64 = to_f64(V_st, spec.dtype)
    rows = np.asarray(rows, dtype=np.int64)
    q_sel, _, _ = make_recompute_inputs(wl, rows)
    if q_gain != 1.0:
        q_sel = to_storage(to_f64(q_sel, spec.dtype) * q_gain, spec.dtype)
    out, lse = run_attention(spec, q_sel, rows, K_st, V_st, flags=flags, tuning=tuning, max_ctx=wl.n_ctx)
    pick = np.arange(len(rows))
    if n_check is not None and n_check < len(rows):
        g = np.random.Generator(np.random.Philox(key=[9, 9]))
        pick = np.sort(np.unique(np.concatenate([[0, 1, len(rows) - 1], g.choice(len(rows), n_check, replace=False)])))
    ref, ref_abs, lse_ref = oracle_attention(to_f64(q_sel, spec.dtype)[pick], rows[pick], K64, V64, wl.sm_scale)
    assert_attention_close(out[pick], ref, ref_abs, spec.dtype, lse[pick], lse_ref)
    return out, lse


def sample_rows(n_ctx, k, seed):
    g = np.random.Generator(np.random.Philox(key=[seed, 11]))
    return np.sort(g.choice(n_ctx, size=k, replace=False))


def test_attention_c1_fp32():
    spec = preset("C1")
    rows = sample_rows(1024, 153, 1)
    rows[0] = 0
    attention_case(spec, np.unique(rows))


ATTN_CASES = [
    ("C2-ragged", preset("C2", chunk_lens=[333, 120, 250], m_prompt=8), 105, 0),
    ("C2-ragged-alu", preset("C2", chunk_lens=[333, 120, 250], m_prompt=8), 105, FORCE_GENERIC),
    ("C3-small", preset("C3", chunk_lens=[100] * 11, m_prompt=8), 165, 0),
    ("C4-small", preset("C4", uneven=(9, 60, 180), m_prompt=8), 97, 0),
    ("C5-gqa7", preset("C5", chunk_lens=[64] * 16 + [32] * 8, m_prompt=8), 192, 0),
    ("few-rows", preset("C2", chunk_lens=[500], m_prompt=8), 3, 0),
    ("many-rows-big-blocks", preset("C2", chunk_lens=[640] * 8, m_prompt=8), 4200, 0),
]


@pytest.mark.parametrize("name,spec,k,flags", ATTN_CASES, ids=[c[0] for c in ATTN_CASES])
def test_attention_parity_bf16(name, spec, k, flags):
    n_ctx = int(np.sum(spec.chunk_lens)) if spec.chunk_lens is not None else make_workload(spec).n_ctx
    rows = sample_rows(n_ctx, min(k, n_ctx), 2)
    attention_case(spec, rows, flags=flags, n_check=300 if name.startswith("many-rows") else None)


def test_attention_few_rows_against_a_long_context():
    """A few dozen rows against 20K keys: so few row blocks that the library cuts the kv axis into more
    than its usual 8 parts (8 jobs, 313 tiles: 10 parts of 32 tiles), merged by the combine pass."""
    spec = preset("C3", chunk_lens=[2500] * 8, m_prompt=8)
    rows = np.unique(np.concatenate([sample_rows(20000, 28, 21), [0, 63, 64, 19999]]))
    assert len(rows) <= 32   # one row block per kv head
    attention_case(spec, rows)
    attention_case(spec, rows, q_gain=6.0)


@pytest.mark.parametrize("seed", list(range(24)))
def test_attention_random_shapes_and_knobs(seed):
    """Seeded draws of head counts (group sizes 1 .. 32), chunkings, row sets (a handful of rows up to
    several hundred, with and without the first and the last position), logit sharpness and launch knobs."""
    g = np.random.Generator(np.random.Philox(key=[seed, 31337]))
    h_kv, grp = int(g.choice([1, 2, 4, 8])), int(g.choice([1, 2, 4, 7, 8, 16, 32]))
    while h_kv * grp > 64:
        h_kv //= 2
    lens = [int(x) for x in g.integers(1, 9000 if seed % 4 == 0 else 900, size=int(g.integers(1, 6)))]
    n_ctx = sum(lens)
    k = min(n_ctx, int(g.integers(1, 40))) if seed % 5 == 0 else int(g.integers(1, min(n_ctx, 700) + 1))
    rows = np.sort(g.choice(n_ctx, size=k, replace=False))
    if seed % 3 == 0:
        rows[0] = 0
    if seed % 7 == 0:
        rows[-1] = n_ctx - 1
    tuning = [None, {"attn_part_tiles": int(g.integers(1, 50))}, {"attn_split_parts": int(g.integers(1, 9))},
              {"attn_max_row_blocks": int(g.integers(1, 6))},
              {"attn_max_row_blocks": int(g.integers(1, 6)), "attn_part_tiles": int(g.integers(1, 30))}][seed % 5]
    spec = preset("C2", n_q_heads=h_kv * grp, n_kv_heads=h_kv, chunk_lens=lens, m_prompt=4, seed=20260305 + 900 + seed)
    attention_case(spec, np.unique(rows), tuning=tuning, q_gain=float(g.choice([1.0, 1.0, 6.0])), n_check=64)


# (chunk lengths, selected rows or a count to draw, H_q, H_kv): caches shorter than / equal to / one past a
# key tile, a single row, every row, the largest and the smallest group size the MFMA path takes
ATTN_SHAPES = [
    ([1], [0], 8, 2), ([63], "all", 8, 2), ([64], [0, 63], 8, 2), ([65], [64], 8, 2), ([65], "all", 8, 2),
    ([128, 100], 50, 32, 1), ([300], 200, 8, 8), ([129], [0, 1, 2, 127, 128], 28, 4),
]
# launch shapes: the library's own; kv parts of one tile, so that every row block is cut at every tile
FINE_CUTS = {"attn_part_tiles": 1}


@pytest.mark.parametrize("lens,rows,hq,hkv", ATTN_SHAPES,
                         ids=[f"N{sum(c[0])}-{c[1] if not isinstance(c[1], list) else len(c[1])}rows-{c[2]}q{c[3]}kv" for c in ATTN_SHAPES])
@pytest.mark.parametrize("tuning", [None, FINE_CUTS], ids=["default", "fine-cuts"])
def test_attention_mfma_shapes(lens, rows, hq, hkv, tuning):
    spec = preset("C2", chunk_lens=lens, m_prompt=8, n_q_heads=hq, n_kv_heads=hkv)
    n_ctx = sum(lens)
    if rows == "all":
        rows = np.arange(n_ctx)
    elif isinstance(rows, int):
        rows = sample_rows(n_ctx, rows, 4)
    attention_case(spec, np.asarray(rows, dtype=np.int64), tuning=tuning)


# Whether and where a launch is cut along the kv axis (partial results in scratch, merged by the
# combine pass) and into how many launches a call is split over row ranges is the library's choice;
# every choice must give the same rows.  100 kv tiles, 30 row blocks.
CUT_TUNINGS = [
    ("default", None),
    ("never-cut", {"attn_split_parts": 1}),
    ("2-parts", {"attn_split_parts": 2}),
    ("3-parts", {"attn_split_parts": 3}),
    ("40-tile-parts", {"attn_part_tiles": 40}),     # row blocks of up to 40 tiles stay whole, longer ones get 2 or 3 parts
    ("7-tile-parts", {"attn_part_tiles": 7}),
    ("single-tile-parts", {"attn_part_tiles": 1}),
    ("2-row-blocks-per-launch", {"attn_max_row_blocks": 2}),
    ("3-row-blocks-per-launch-cut-in-4", {"attn_max_row_blocks": 3, "attn_split_parts": 4}),
]


@pytest.mark.parametrize("name,tuning", CUT_TUNINGS, ids=[c[0] for c in CUT_TUNINGS])
def test_attention_cut_along_the_kv_axis(name, tuning):
    """Launches cut along the kv axis (partial results in scratch, merged by the combine pass) and
    calls served by several launches over row ranges, on near-uniform data."""
    spec = preset("C2", chunk_lens=[640] * 10, m_prompt=8)            # 100 kv tiles
    rows = np.unique(np.concatenate([sample_rows(6400, 900, 5), [0, 63, 64, 2111, 2112, 2113, 4223, 4224, 6399]]))
    attention_case(spec, rows, tuning=tuning, n_check=160)


def test_attention_row_ranges_that_are_cut_on_their_own():
    """More jobs than workgroup slots in total (so the call as a whole would not be cut), served in
    two launches over row ranges that each have fewer (so each range is cut along the kv axis by the
    library's own rule): the scratch must serve every range."""
    spec = preset("C2", chunk_lens=[640] * 10, m_prompt=8)            # 100 kv tiles
    rows = sample_rows(6400, 2200, 8)                                  # 69 row blocks x 8 kv heads = 552 jobs
    attention_case(spec, rows, tuning={"attn_max_row_blocks": 60}, n_check=160)


@pytest.mark.parametrize("name,tuning", CUT_TUNINGS, ids=[c[0] for c in CUT_TUNINGS])
def test_attention_needles_at_depth(name, tuning):
    spec = preset("C2", chunk_lens=[6400], m_prompt=8)
    rows, target, q_st, K_st, V_st = needle_case(6400, 32, 8, 700, 3)
    out, lse = run_attention(spec, q_st, rows, K_st, V_st, tuning=tuning)
    g = np.random.Generator(np.random.Philox(key=[10, 9]))
    pick = np.sort(np.unique(np.concatenate([[0, 1, len(rows) - 1], g.choice(len(rows), 150, replace=False)])))
    V64 = to_f64(V_st, "bf16")
    ref, ref_abs, lse_ref = oracle_attention(to_f64(q_st, "bf16")[pick], rows[pick], to_f64(K_st, "bf16"), V64, 128 ** -0.5)
    # the case is what it claims to be: outputs of order one, dominated by the target key's value row
    G = 4
    v_target = V64[target[pick], np.arange(32)[None, :] // G]
    assert np.abs(ref - v_target).max() < 0.2 and np.abs(ref).max(axis=-1).min() > 1.0
    assert_attention_close(out[pick], ref, ref_abs, "bf16", lse[pick], lse_ref)
    # every row of the call, against the value rows themselves (no oracle needed, coarse)
    v_all = V64[target, np.arange(32)[None, :] // G]
    assert np.abs(out - v_all).max() < 0.25


@pytest.mark.parametrize("logit", [70.0, 200.0])
@pytest.mark.parametrize("tuning", [None, {"attn_part_tiles": 7}], ids=["default", "7-tile-parts"])
def test_attention_needles_far_above_the_first_key(logit, tuning):
    """The same needles with logits of 70 and 200: exp(logit - logit of the first key of a sweep) is
    far beyond what the fixed-reference sweep of the MFMA kernel accepts, or overflows fp32 outright, so
    the workgroups must repeat their sweeps with the running maximum and still give finite, right results."""
    spec = preset("C2", chunk_lens=[3000], m_prompt=8)
    rows, target, q_st, K_st, V_st = needle_case(3000, 32, 8, 260, 17, logit=logit)
    out, lse = run_attention(spec, q_st, rows, K_st, V_st, tuning=tuning)
    V64 = to_f64(V_st, "bf16")
    ref, ref_abs, lse_ref = oracle_attention(to_f64(q_st, "bf16"), rows, to_f64(K_st, "bf16"), V64, 128 ** -0.5)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    assert np.abs(ref).max(axis=-1).min() > 1.0
    assert_attention_close(out, ref, ref_abs, "bf16", lse, lse_ref)


@pytest.mark.parametrize("q_gain", [1.0, 2.5, 6.0], ids=["flat", "moderately-peaked", "peaked"])
def test_attention_fixed_reference_sweep_against_the_exact_one(q_gain):
    """The MFMA kernel's two sweeps on the same inputs: the library's own choice (the fixed-reference sweep
    where it is accepted: flat and moderately peaked logits) and the running-maximum sweep forced by the
    knob, each against the oracle, on whole row blocks and on launches cut along the kv axis."""
    spec = preset("C2", chunk_lens=[1500, 700, 1000], m_prompt=8)
    rows = sample_rows(3200, 500, 23)
    rows[0] = 0
    for tuning in (None, {"attn_exact_sweep": 1}, {"attn_part_tiles": 9}, {"attn_part_tiles": 9, "attn_exact_sweep": 1}):
        attention_case(spec, np.unique(rows), tuning=tuning, q_gain=q_gain, n_check=120)


def test_attention_needles_gqa7():
    spec = preset("C5", chunk_lens=[3000], m_prompt=8)
    rows, target, q_st, K_st, V_st = needle_case(3000, 28, 4, 300, 5)
    for tuning in (None, FINE_CUTS):
        out, lse = run_attention(spec, q_st, rows, K_st, V_st, tuning=tuning)
        pick = np.arange(0, len(rows), 3)
        ref, ref_abs, lse_ref = oracle_attention(to_f64(q_st, "bf16")[pick], rows[pick], to_f64(K_st, "bf16"),
                                                 to_f64(V_st, "bf16"), 128 ** -0.5)
        assert np.abs(ref).max(axis=-1).min() > 1.0
        assert_attention_close(out[pick], ref, ref_abs, "bf16", lse[pick], lse_ref)


def test_attention_full_ratio_is_dense_causal():
    spec = preset("C2", chunk_lens=[150, 83], m_prompt=8)
    attention_case(spec, np.arange(233))


@pytest.mark.parametrize("tuning", [None, FINE_CUTS], ids=["default", "fine-cuts"])
def test_attention_peaky_logits(tuning):
    spec = preset("C2", chunk_lens=[700, 301], m_prompt=8, sigma=0.3)
    rows = sample_rows(1001, 150, 4)
    attention_case(spec, rows, q_gain=6.0, tuning=tuning)


@pytest.mark.parametrize("tuning", [None, FINE_CUTS], ids=["default", "fine-cuts"])
def test_attention_out_of_range_rows_give_zeros(tuning):
    spec = preset("C2", chunk_lens=[128], m_prompt=8)
    wl = make_workload(spec)
    K_st, K64, _ = global_keys(wl)
    V_st = wl.v_chunks[0]
    rows = np.array([5, 60, 127], dtype=np.int64)
    q_sel, _, _ = make_recompute_inputs(wl, rows)
    bad = torch.tensor([5, 128, -1], dtype=torch.int32, device=DEV)
    L = make_layer(spec, max_ctx=128, max_prompt=8)
    for key, value in (tuning or {}).items():
        L.set_tuning(key, value)
    out = L.recompute_attention(to_dev(q_sel, "bf16"), bad, to_dev(K_st, "bf16"), to_dev(V_st, "bf16"))
    sync()
    o = to_host_f64(out, "bf16")
    assert np.abs(o[0]).max() > 0 and np.array_equal(o[1:], np.zeros_like(o[1:]))
    L.close()


# ---------------------------------------------------------------------------
# stage 5
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("cfg", ["C1", "C2"])
def test_splice_bit_exact(cfg):
    spec = preset(cfg) if cfg == "C1" else preset("C2", chunk_lens=[300, 211], m_prompt=8)
    wl = make_workload(spec)
    K_st, _, _ = global_keys(wl)
    V_st = np.concatenate([wl.v_chunks[c] for c in wl.chunk_order], axis=0)
    idx = sample_rows(wl.n_ctx, O.budget(wl.n_ctx, 0.15), 6)
    _, k_new, v_new = make_recompute_inputs(wl, idx)
    Kr, Vr = O.splice_kv(K_st, V_st, k_new, v_new, idx)
    L = make_layer(spec, max_ctx=wl.n_ctx, max_prompt=8)
    kd, vd = to_dev(K_st, spec.dtype), to_dev(V_st, spec.dtype)
    idx_d = torch.from_numpy(idx.astype(np.int32)).to(DEV)
    L.splice_kv(to_dev(k_new, spec.dtype), to_dev(v_new, spec.dtype), idx_d, kd, vd)
    sync()
    bits = np.uint16 if spec.dtype == "bf16" else np.uint32
    assert np.array_equal(to_host_bits(kd, spec.dtype), np.ascontiguousarray(Kr).view(bits))
    assert np.array_equal(to_host_bits(vd, spec.dtype), np.ascontiguousarray(Vr).view(bits))
    # keys only; and rows outside the cache are skipped
    kd2 = to_dev(K_st, spec.dtype)
    idx2 = idx_d.clone()
    idx2[0] = wl.n_ctx + 5
    L.splice_kv(to_dev(k_new, spec.dtype), None, idx2, kd2, None)
    sync()
    Kr2, _ = O.splice_kv(K_st, V_st, k_new[1:], v_new[1:], idx[1:])
    assert np.array_equal(to_host_bits(kd2, spec.dtype), np.ascontiguousarray(Kr2).view(bits))
    L.close()


# ---------------------------------------------------------------------------
# composite
# ---------------------------------------------------------------------------
SENTINEL = 0x7F7F      # bf16 bit pattern / low half of the f32 one that fills the padding of strided caches


def strided_cache(L, n_rows):
    """A cache in the layer's layout carved out of a buffer filled with a sentinel, and the buffer."""
    storage = (n_rows - 1) * L.token_stride + (L.n_kv_heads - 1) * L.head_stride + L.head_dim
    base = torch.full((storage,), 0, dtype=L.torch_dtype, device=DEV)
    base.view(torch.int16 if L.dtype == "bf16" else torch.int32).fill_(SENTINEL)
    return torch.as_strided(base, (n_rows, L.n_kv_heads, L.head_dim), (L.token_stride, L.head_stride, 1)), base


def padding_untouched(cache, base):
    """Everything in the buffer that is not an element of the logical cache still holds the sentinel."""
    bits = base.view(torch.int16 if base.dtype == torch.bfloat16 else torch.int32).clone()
    torch.as_strided(bits, cache.shape, cache.stride()).fill_(SENTINEL)
    return bool((bits == SENTINEL).all())


def run_layer_gpu(wl, ratio, flags=0, layout=None):
    sp = wl.spec
    kw = {} if layout is None else dict(token_stride=layout[0], head_stride=layout[1])
    L = make_layer(sp, max_ctx=wl.n_ctx, max_prompt=sp.m_prompt, flags=flags, **kw)
    kd, vd = dev_chunks(wl)
    if layout is None:
        K, V, starts, N = L.reposition_keys(kd, vd, chunk_order=wl.chunk_order.tolist())
    else:
        (K, L._k_base), (V, L._v_base) = strided_cache(L, wl.n_ctx), strided_cache(L, wl.n_ctx)
        K, V, starts, N = L.reposition_keys(kd, vd, chunk_order=wl.chunk_order.tolist(), k_out=K, v_out=V)
    s = L.score_tokens(K, to_dev(wl.q_prompt, sp.dtype))
    idx = L.select_topk(s, ratio=ratio)
    sync()
    return L, K, V, s, idx


@pytest.mark.parametrize("cfg,rtol_sel", [("C1", 1e-5), ("C2", 1e-4)])
def test_composite_layer(cfg, rtol_sel):
    """Whole path, in the order: reposition, score, select, splice, attend."""
    spec = preset(cfg) if cfg == "C1" else preset("C2", chunk_lens=[256] * 6, m_prompt=32)
    composite_case(spec, 0.15, rtol_sel)


@pytest.mark.parametrize("cfg", ["C1", "C2"])
def test_step_replays_from_a_captured_graph(cfg):
    """All five stages enqueue on the stream the layer was created on, allocate nothing once their
    scratch exists and use no memset, so a caller can capture a whole step into a graph.  Every replay
    (with eager work and synchronisations in between) must reproduce the eager step bit for bit."""
    spec = preset(cfg) if cfg == "C1" else preset("C2", chunk_lens=[300, 211, 170, 256], m_prompt=32, permute_order=True)
    wl = make_workload(spec)
    ratio = 0.15
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        L = make_layer(spec, max_ctx=wl.n_ctx, max_prompt=spec.m_prompt)   # binds the current stream
        kd, vd = dev_chunks(wl)
        qd = to_dev(wl.q_prompt, spec.dtype)
        order = wl.chunk_order.tolist()
        K, V, _, N = L.reposition_keys(kd, vd, chunk_order=order)
        scores = L.score_tokens(K, qd)
        idx = L.select_topk(scores, ratio=ratio)
        side.synchronize()
        q_sel, k_new, v_new = make_recompute_inputs(wl, idx.cpu().numpy().astype(np.int64))
        qs, kn, vn = to_dev(q_sel, spec.dtype), to_dev(k_new, spec.dtype), to_dev(v_new, spec.dtype)
        out = torch.empty_like(qs)

        def step():
            L.reposition_keys(kd, vd, chunk_order=order, k_out=K, v_out=V)
            L.score_tokens(K, qd, scores=scores)
            L.select_topk(scores, ratio=ratio, idx_out=idx)
            L.splice_kv(kn, vn, idx, K, V)
            L.recompute_attention(qs, idx, K, V, out=out)

        step()       # eager: also sizes every scratch buffer
        step()
        side.synchronize()
        want = [t.clone() for t in (K, V, scores, idx, out)]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for _ in range(3):
        for t in (K, V, scores, out):
            t.zero_()
        idx.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((K, V, scores, idx, out), want):
            assert torch.equal(got, ref)
    L.close()


def random_shape_spec(seed):
    """A seeded odd-shaped layer: head counts, group sizes, head_dim, chunk lengths (one of them may be
    empty), prompt length and chunk order all drawn, to reach the ragged paths of every kernel."""
    g = np.random.Generator(np.random.Philox(key=[seed, 99]))
    dtype = "f32" if seed % 4 == 0 else "bf16"
    d = 64 if (dtype == "f32" or seed % 3 == 0) else 128
    h_kv = int(g.choice([1, 2, 4, 8]))
    grp = int(g.choice([1, 2, 3, 4, 7, 8]))
    lens = [int(x) for x in g.integers(1, 230, size=int(g.integers(1, 8)))]
    if len(lens) > 2 and seed % 2:
        lens[1] = 0
    base = "C1" if dtype == "f32" else "C2"
    spec = preset(base, n_q_heads=h_kv * grp, n_kv_heads=h_kv, head_dim=d, chunk_lens=lens,
                  m_prompt=int(g.integers(1, 41)), permute_order=True, seed=20260305 + 100 + seed,
                  sigma=1.0 if dtype == "f32" else float(d) ** -0.5)
    return spec, float(g.choice([0.05, 0.15, 0.3, 0.5]))


@pytest.mark.parametrize("seed", list(range(1, 41)))
def test_composite_layer_random_shapes(seed):
    spec, ratio = random_shape_spec(seed)
    composite_case(spec, ratio, 1e-5 if spec.dtype == "f32" else 1e-4)


def composite_case(spec, ratio, rtol_sel, layout=None):
    wl = make_workload(spec)
    k, v, q = oracle_inputs(wl)
    L, K, V, s, idx = run_layer_gpu(wl, ratio, layout=layout)
    # oracle on its own
    Kref, Vref, _, N = O.reposition_keys(k, v, wl.chunk_len, wl.chunk_order, spec.rope_theta, spec.pairing)
    s_ref = O.score_tokens(Kref, q, wl.sm_scale)
    kk = O.budget(N, ratio)
    idx_ref = O.select_topk(s_ref, kk)
    # (i) the GPU selection is exact for the GPU's own fp32 scores
    s_gpu = s.cpu().numpy()
    idx_gpu = idx.cpu().numpy().astype(np.int64)
    assert np.array_equal(idx_gpu, O.select_topk(s_gpu, kk))
    # (ii) against the oracle's set: only tokens within tolerance of the threshold may differ
    thr = np.sort(s_ref)[::-1][kk - 1]
    near = np.abs(s_ref - thr) <= rtol_sel * (thr + spec.m_prompt / N)
    diff = np.setxor1d(idx_gpu, idx_ref)
    assert near[diff].all(), f"{len(diff)} differing tokens, not all near the threshold"
    planted_clear = [j for j in wl.planted if s_ref[j] - thr > rtol_sel * (thr + spec.m_prompt / N)]
    assert set(planted_clear) <= set(idx_gpu.tolist())
    # stages 5 and 4 on the oracle's selection (inputs never come from the GPU path)
    q_sel, k_new, v_new = make_recompute_inputs(wl, idx_ref)
    idx_d = torch.from_numpy(idx_ref.astype(np.int32)).to(DEV)
    L.splice_kv(to_dev(k_new, spec.dtype), to_dev(v_new, spec.dtype), idx_d, K, V)
    out, lse = L.recompute_attention(to_dev(q_sel, spec.dtype), idx_d, K, V, return_lse=True)
    sync()
    # oracle: the same on the GPU-independent side, with stage-1 output rounded to storage
    K_st, V_st = to_storage(Kref, spec.dtype), to_storage(Vref, spec.dtype)
    K2, V2 = O.splice_kv(to_f64(K_st, spec.dtype), to_f64(V_st, spec.dtype),
                         to_f64(k_new, spec.dtype), to_f64(v_new, spec.dtype), idx_ref)
    ref, ref_abs, lse_ref = oracle_attention(to_f64(q_sel, spec.dtype), idx_ref, K2, V2, wl.sm_scale)
    assert_attention_close(to_host_f64(out, spec.dtype), ref, ref_abs, spec.dtype,
                           lse.cpu().numpy().astype(np.float64), lse_ref)
    # stage 1 and stage 5 element by element (the stages above only constrain them through scores and outputs)
    check_reposition(to_host_f64(K, spec.dtype)[np.setdiff1d(np.arange(N), idx_ref)],
                     Kref[np.setdiff1d(np.arange(N), idx_ref)], spec.dtype, spec.pairing)
    bits = np.uint16 if spec.dtype == "bf16" else np.uint32
    assert np.array_equal(to_host_bits(K, spec.dtype)[idx_ref], np.ascontiguousarray(k_new).view(bits))
    assert np.array_equal(to_host_bits(V, spec.dtype)[idx_ref], np.ascontiguousarray(v_new).view(bits))
    if layout is not None:
        assert padding_untouched(K, L._k_base) and padding_untouched(V, L._v_base)
    L.close()


def layouts_for(spec, n_ctx):
    """[H_kv, T_cap, d] (heads outermost, room for 40 more rows), and token-major rows padded by 64
    elements with heads 8 elements apart more than they need."""
    d, h = spec.head_dim, spec.n_kv_heads
    return {"head-major": (d, (n_ctx + 40) * d), "padded-token-major": (h * (d + 8) + 64, d + 8)}


@pytest.mark.parametrize("which", ["head-major", "padded-token-major"])
@pytest.mark.parametrize("cfg", ["C1", "C2", "C2-alu", "C5", "C1-interleaved"])
def test_composite_layer_on_strided_caches(cfg, which):
    """The whole path with the concatenated caches in a layout other than packed [T, H_kv, d]: every
    stage that touches them (1 writes, 2 and 4 read, 5 writes) against the oracle, and nothing written
    outside the logical tensor."""
    spec = {"C1": preset("C1", chunk_lens=[100, 61, 130], m_prompt=12),
            "C1-interleaved": preset("C1", chunk_lens=[100, 61, 130], m_prompt=12, pairing="interleaved"),
            "C2": preset("C2", chunk_lens=[256, 100, 190, 64], m_prompt=32, permute_order=True),
            "C2-alu": preset("C2", chunk_lens=[120, 77], m_prompt=9),
            "C5": preset("C5", chunk_lens=[64] * 6 + [32] * 3, m_prompt=16)}[cfg]
    n_ctx = int(np.sum(spec.chunk_lens))
    layout = layouts_for(spec, n_ctx)[which]
    if cfg == "C2-alu":
        wl = make_workload(spec)
        L, K, V, s, idx = run_layer_gpu(wl, 0.15, flags=FORCE_GENERIC, layout=layout)
        k, v, q = oracle_inputs(wl)
        Kref, Vref, _, N = O.reposition_keys(k, v, wl.chunk_len, wl.chunk_order, spec.rope_theta, spec.pairing)
        check_reposition(to_host_f64(K, spec.dtype), Kref, spec.dtype, spec.pairing)
        s_ref = O.score_tokens(to_host_f64(K, spec.dtype), q, wl.sm_scale)
        assert (np.abs(s.cpu().numpy() - s_ref) <= score_tol(s_ref, spec.m_prompt, 1e-2)).all()
        rows = sample_rows(N, 40, 3)
        q_sel, _, _ = make_recompute_inputs(wl, rows)
        out, lse = L.recompute_attention(to_dev(q_sel, spec.dtype), torch.from_numpy(rows.astype(np.int32)).to(DEV), K, V,
                                         return_lse=True)
        sync()
        ref, ref_abs, lse_ref = oracle_attention(to_f64(q_sel, spec.dtype), rows, to_host_f64(K, spec.dtype),
                                                 to_host_f64(V, spec.dtype), wl.sm_scale)
        assert_attention_close(to_host_f64(out, spec.dtype), ref, ref_abs, spec.dtype, lse.cpu().numpy().astype(np.float64), lse_ref)
        assert padding_untouched(K, L._k_base) and padding_untouched(V, L._v_base)
        L.close()
    else:
        composite_case(spec, 0.15, 1e-5 if spec.dtype == "f32" else 1e-4, layout=layout)


def test_strided_layout_gives_the_same_bits_as_packed():
    """Same inputs, packed and head-major caches: the arithmetic is the same, so scores, selection and
    attention outputs agree bit for bit (100 kv tiles: the attention launch is cut along the kv axis)."""
    spec = preset("C2", chunk_lens=[640] * 10, m_prompt=32)
    wl = make_workload(spec)
    res = []
    for layout in (None, layouts_for(spec, wl.n_ctx)["head-major"]):
        L, K, V, s, idx = run_layer_gpu(wl, 0.1, layout=layout)
        q_sel, _, _ = make_recompute_inputs(wl, idx.cpu().numpy().astype(np.int64))
        out, lse = L.recompute_attention(to_dev(q_sel, spec.dtype), idx, K, V, return_lse=True)
        sync()
        res.append((to_host_bits(K, spec.dtype), s.cpu().numpy(), idx.cpu().numpy(), to_host_bits(out, spec.dtype), lse.cpu().numpy()))
        L.close()
    for a, b in zip(*res):
        assert np.array_equal(a, b)


# ---------------------------------------------------------------------------
# debug mode: device-side checks of what host code cannot see
# ---------------------------------------------------------------------------
def test_validate_flag_reports_bad_row_pos_and_duplicate_idx():
    from paper_2603_05353_amd import IFKV_FLAG_VALIDATE, IfkvError
    spec = preset("C2", chunk_lens=[300, 211], m_prompt=8)
    wl = make_workload(spec)
    K_st, K64, _ = global_keys(wl)
    V_st = np.concatenate([wl.v_chunks[c] for c in wl.chunk_order], axis=0)
    rows = sample_rows(511, 70, 2)
    q_sel, k_new, v_new = make_recompute_inputs(wl, rows)
    L = make_layer(spec, max_ctx=511, max_prompt=8, flags=IFKV_FLAG_VALIDATE)
    Ln = make_layer(spec, max_ctx=511, max_prompt=8)
    Kd, Vd, qd = to_dev(K_st, "bf16"), to_dev(V_st, "bf16"), to_dev(q_sel, "bf16")
    good = torch.from_numpy(rows.astype(np.int32)).to(DEV)
    # good input: same result as without the flag
    out_v = L.recompute_attention(qd, good, Kd, Vd)
    out_n = Ln.recompute_attention(qd, good, Kd, Vd)
    sync()
    assert torch.equal(out_v, out_n)
    for pos, what in [(17, "equal"), (40, "descending"), (69, "descending")]:
        bad = good.clone()
        bad[pos] = bad[pos - 1] if what == "equal" else bad[pos - 1] - 3
        with pytest.raises(IfkvError) as e:
            L.recompute_attention(qd, bad, Kd, Vd)
        assert e.value.code == -1 and f"index {pos}" in str(e.value)
    # splice: duplicates are refused and nothing is written; unique indices (in any order) pass
    K2 = Kd.clone()
    dup = good.clone()
    dup[33] = dup[5]
    with pytest.raises(IfkvError) as e:
        L.splice_kv(to_dev(k_new, "bf16"), to_dev(v_new, "bf16"), dup, K2, Vd.clone())
    assert e.value.code == -1 and ("index 33" in str(e.value) or "index 5" in str(e.value))
    sync()
    assert torch.equal(K2, Kd)
    perm = torch.randperm(70, generator=torch.Generator().manual_seed(3))
    L.splice_kv(to_dev(k_new[perm.numpy()], "bf16"), to_dev(v_new[perm.numpy()], "bf16"), good[perm.to(DEV)], K2, Vd.clone())
    sync()
    Kr, _ = O.splice_kv(K_st, V_st, k_new, v_new, rows)
    assert np.array_equal(to_host_bits(K2, "bf16"), np.ascontiguousarray(Kr).view(np.uint16))
    L.close(), Ln.close()


# ---------------------------------------------------------------------------
# caller-supplied frequency table
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("cfg,pairing", [("C1", "half"), ("C2", "half"), ("C2", "interleaved")])
def test_custom_frequency_table_on_the_gpu(cfg, pairing):
    """inv_freq of the layer descriptor replaces the geometric table of Eq. (4) pair by pair, in the
    re-rotation of cached keys and in the rotary embedding of fresh rows."""
    spec = preset(cfg, chunk_lens=[90, 41, 130], m_prompt=8, pairing=pairing, permute_order=True)
    half = spec.head_dim // 2
    freqs = np.array([0.37 / (1 + j) + (0.011 if j % 3 == 0 else 0.0) + 0.002 * ((7 * j) % 5) for j in range(half)])
    wl = make_workload(spec)
    k, v, _ = oracle_inputs(wl)
    L = make_layer(spec, max_ctx=wl.n_ctx, max_prompt=8, inv_freq=freqs.tolist())
    kd, vd = dev_chunks(wl)
    pos0 = [3, 0, 7]
    K, V, starts, N = L.reposition_keys(kd, vd, chunk_order=wl.chunk_order.tolist(), cached_pos0=pos0)
    sync()
    K_ref, V_ref, start_ref, _ = O.reposition_keys(k, v, wl.chunk_len, wl.chunk_order, spec.rope_theta, pairing,
                                                   cached_pos0=pos0, freqs=freqs)
    assert starts == start_ref.tolist()
    check_reposition(to_host_f64(K, spec.dtype), K_ref, spec.dtype, pairing)
    # the default table gives something else entirely: the custom one was really used
    K_def, _, _, _ = O.reposition_keys(k, v, wl.chunk_len, wl.chunk_order, spec.rope_theta, pairing, cached_pos0=pos0)
    assert np.abs(to_host_f64(K, spec.dtype) - K_def).max() > 0.05 * np.abs(K_def).max()
    g = np.random.Generator(np.random.Philox(key=[5, 5]))
    x_st = to_storage(g.standard_normal((40, 3, spec.head_dim)) * 0.3, spec.dtype)
    pos = np.sort(g.choice(140000, size=40, replace=False)).astype(np.int32)
    xd = to_dev(x_st, spec.dtype)
    L.rope_rows(xd, torch.from_numpy(pos).to(DEV))
    sync()
    check_reposition(to_host_f64(xd, spec.dtype), O.rope_rows(to_f64(x_st, spec.dtype), pos, spec.rope_theta, pairing, freqs=freqs),
                     spec.dtype, pairing)
    L.close()


# ---------------------------------------------------------------------------
# rotary embedding of recomputed rows
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("cfg,pairing,heads", [("C1", "half", 8), ("C2", "half", 32), ("C2", "half", 8),
                                               ("C2", "interleaved", 32), ("C5", "half", 4), ("C1", "interleaved", 3)])
def test_rope_rows_parity(cfg, pairing, heads):
    spec = preset(cfg, pairing=pairing)
    g = np.random.Generator(np.random.Philox(key=[77, heads]))
    R, d = 333, spec.head_dim
    x64 = g.standard_normal((R, heads, d)) * 0.3
    pos = np.sort(g.choice(140000, size=R, replace=False)).astype(np.int32)
    pos[0], pos[1] = 0, 1
    x_st = to_storage(x64, spec.dtype)
    L = make_layer(spec, max_ctx=1024, max_prompt=8)
    xd = to_dev(x_st, spec.dtype)
    L.rope_rows(xd, torch.from_numpy(pos).to(DEV))
    sync()
    ref = O.rope_rows(to_f64(x_st, spec.dtype), pos, spec.rope_theta, pairing)
    got = to_host_f64(xd, spec.dtype)
    check_reposition(got, ref, spec.dtype, pairing)
    assert np.array_equal(to_host_bits(xd, spec.dtype)[0], np.ascontiguousarray(x_st[0]).view(np.uint16 if spec.dtype == "bf16" else np.uint32))   # position 0: cos = 1, sin = 0, bit-exact
    L.close()


# ---------------------------------------------------------------------------
# prompt rows through the attention stage: the glue a layer's recompute pass needs
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("cfg", ["C1", "C2"])
def test_prompt_rows_and_selected_rows_in_one_attention_call(cfg):
    """Prompt tokens are always computed fresh ("KV Recomputation"): their keys get rotary positions
    N..N+M-1 (ifkv_rope_rows), are appended to the spliced cache, and their queries run through the
    attention stage together with the selected context rows (row_pos beyond N, n_kv = N + M).  Both
    sides take the stored prompt keys after the rotation, so the attention check is not loosened by it."""
    spec = preset(cfg, chunk_lens=[210, 97, 160, 133], m_prompt=24)
    wl = make_workload(spec)
    N, M = wl.n_ctx, spec.m_prompt
    K_st, K64, q_prompt64 = global_keys(wl)
    V_st = np.concatenate([wl.v_chunks[c] for c in wl.chunk_order], axis=0)
    g = np.random.Generator(np.random.Philox(key=[spec.seed, 31]))
    kp_raw = to_storage(g.standard_normal((M, spec.n_kv_heads, spec.head_dim)) * spec.sigma, spec.dtype)
    vp_st = to_storage(g.standard_normal((M, spec.n_kv_heads, spec.head_dim)) * spec.sigma, spec.dtype)
    sel = sample_rows(N, 90, 3)
    q_sel, _, _ = make_recompute_inputs(wl, sel)
    rows = np.concatenate([sel, np.arange(N, N + M)]).astype(np.int64)
    q_all = np.concatenate([q_sel, to_storage(q_prompt64, spec.dtype)], axis=0)

    L = make_layer(spec, max_ctx=N + M, max_prompt=M)
    Kd = to_dev(np.concatenate([K_st, kp_raw], axis=0), spec.dtype)
    Vd = to_dev(np.concatenate([V_st, vp_st], axis=0), spec.dtype)
    pos_p = torch.arange(N, N + M, dtype=torch.int32, device=DEV)
    L.rope_rows(Kd[N:], pos_p)                      # in place on the appended rows
    out, lse = L.recompute_attention(to_dev(q_all, spec.dtype), torch.from_numpy(rows.astype(np.int32)).to(DEV),
                                     Kd, Vd, return_lse=True)
    sync()
    kp_ref = O.rope_rows(to_f64(kp_raw, spec.dtype), np.arange(N, N + M), spec.rope_theta, spec.pairing)
    check_reposition(to_host_f64(Kd[N:], spec.dtype), kp_ref, spec.dtype, spec.pairing)
    K_all64 = np.concatenate([K64, to_host_f64(Kd[N:], spec.dtype)], axis=0)
    V_all64 = np.concatenate([to_f64(V_st, spec.dtype), to_f64(vp_st, spec.dtype)], axis=0)
    ref, ref_abs, lse_ref = oracle_attention(to_f64(q_all, spec.dtype), rows, K_all64, V_all64, wl.sm_scale)
    assert_attention_close(to_host_f64(out, spec.dtype), ref, ref_abs, spec.dtype,
                           lse.cpu().numpy().astype(np.float64), lse_ref)
    L.close()


# ---------------------------------------------------------------------------
# the other RoPE geometries of the appendix ("RoPE Geometry"), expressed through delta_override
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("geometry", ["HL-TP", "HL-HP", "TL-TP"])
def test_scores_under_other_rope_geometries(geometry):
    """Head-local context (every chunk keeps positions 0..len-1), tail-local context (every chunk ends
    right before the prompt: advance N - len_i) and the two prompt placements (tail = global position N,
    head = right after the longest chunk).  Reading: "immediately before/after" is taken per chunk.
    The library only sees phase advances and already-rotated prompt queries; the scores and the selected
    set must match the oracle run with the same advances."""
    from workloads import rope_at
    spec = preset("C2", chunk_lens=[180, 75, 260, 141], m_prompt=16, permute_order=True)
    wl = make_workload(spec)
    k, _, q = oracle_inputs(wl)
    N, lens, order = wl.n_ctx, [int(x) for x in wl.chunk_len], wl.chunk_order.tolist()
    adv = [N - L_i for L_i in lens] if geometry == "TL-TP" else [0] * len(lens)
    if geometry == "HL-HP":   # prompt moved from N.. to max(len).. : queries rotate by the difference
        q = rope_at(q, float(max(lens) - N), spec.rope_theta, spec.pairing)
    q_st = to_storage(q, spec.dtype)
    q = to_f64(q_st, spec.dtype)
    L = make_layer(spec, max_ctx=N, max_prompt=spec.m_prompt)
    kd, _ = dev_chunks(wl)
    K, _, _, _ = L.reposition_keys(kd, None, chunk_order=order, delta_override=adv)
    s = L.score_tokens(K, to_dev(q_st, spec.dtype))
    idx = L.select_topk(s, ratio=0.15)
    sync()
    K_ref, _, _, _ = O.reposition_keys(k, None, lens, order, spec.rope_theta, spec.pairing, delta_override=adv)
    check_reposition(to_host_f64(K, spec.dtype), K_ref, spec.dtype, spec.pairing)
    # score the stored keys the GPU produced, so both sides see identical inputs
    s_ref = O.score_tokens(to_host_f64(K, spec.dtype), q, wl.sm_scale)
    s_h = s.cpu().numpy()
    assert (np.abs(s_h - s_ref) <= score_tol(s_ref, spec.m_prompt, 1e-2)).all()
    assert np.array_equal(idx.cpu().numpy().astype(np.int64), O.select_topk(s_h, O.budget(N, 0.15)))
    L.close()


# ---------------------------------------------------------------------------
# chunk reordering
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("n_slots,n_ctx,k", [(1, 100, 30), (4, 1024, 153), (64, 32768, 4915), (100, 5000, 700),
                                              (7, 50, 0), (5, 40, 40)])
def test_chunk_counts_bit_exact(n_slots, n_ctx, k):
    g = np.random.Generator(np.random.Philox(key=[n_slots, n_ctx]))
    cuts = np.sort(g.choice(n_ctx + 1, size=n_slots - 1, replace=True)) if n_slots > 1 else np.array([], dtype=np.int64)
    starts = np.concatenate([[0], cuts]).astype(np.int64)           # empty slots allowed
    lens = np.diff(np.concatenate([starts, [n_ctx]])).astype(np.int64)
    idx = np.sort(g.choice(n_ctx, size=k, replace=False)).astype(np.int32)
    spec = preset("C2", chunk_lens=[int(n_ctx)], m_prompt=8)
    L = make_layer(spec, max_ctx=n_ctx, max_prompt=8)
    got = L.chunk_counts(torch.from_numpy(idx).to(DEV), starts.tolist(), n_ctx)
    sync()
    want = O.chunk_selection_counts(idx.astype(np.int64), lens.tolist(), None)   # slots in identity order
    assert np.array_equal(got.cpu().numpy().astype(np.int64), want)
    L.close()


def test_reorder_two_pass_flow():
    """First-stage selection under the local geometry, Eq. (9), new order, second pass under the
    GLOBAL geometry of the new order -- GPU against oracle at every hand-over."""
    spec = preset("C2", chunk_lens=[200, 96, 310, 128, 64, 226], m_prompt=24, permute_order=True)
    wl = make_workload(spec)
    k, v, q = oracle_inputs(wl)
    ratio = 0.15
    n = len(wl.chunk_len)
    order = wl.chunk_order.tolist()
    L = make_layer(spec, max_ctx=wl.n_ctx, max_prompt=spec.m_prompt)
    kd, vd = dev_chunks(wl)
    qd = to_dev(wl.q_prompt, spec.dtype)
    # pass 1 on the GPU: phase advance 0 for every chunk
    K1, _, starts, N = L.reposition_keys(kd, None, chunk_order=order, delta_override=[0] * n)
    s1 = L.score_tokens(K1, qd)
    idx1 = L.select_topk(s1, ratio=ratio)
    slot_start = [starts[c] for c in order]
    counts = L.chunk_counts(idx1, slot_start, N)
    sync()
    # the keys of pass 1 are the cached keys, bit for bit
    assert np.array_equal(to_host_bits(K1, spec.dtype), np.concatenate([wl.k_chunks[c] for c in order], axis=0))
    # counts: exact for the GPU's own selection
    idx1_h = idx1.cpu().numpy().astype(np.int64)
    counts_h = counts.cpu().numpy().astype(np.int64)
    want_counts = O.chunk_selection_counts(idx1_h, wl.chunk_len, order)       # per chunk id
    assert np.array_equal(counts_h, want_counts[order])
    new_order = L.reorder_chunks(order, counts_h.tolist(), wl.chunk_len.tolist())
    assert new_order == O.reorder_chunks(wl.chunk_len, order, want_counts).tolist()
    # the oracle's own first pass: selections may differ only near the threshold, so per-chunk counts
    # differ by at most the number of such tokens
    ref_order, ref_counts, ref_idx = O.reorder_pass(k, wl.chunk_len, order, spec.rope_theta, spec.pairing, q,
                                                    wl.sm_scale, ratio)
    assert np.abs(ref_counts - want_counts).sum() <= 2 * len(np.setxor1d(ref_idx, idx1_h)) <= 8
    if np.array_equal(ref_counts, want_counts):
        assert new_order == ref_order.tolist()
    # pass 2: the normal path on the new order
    K2, V2, starts2, N2 = L.reposition_keys(kd, vd, chunk_order=new_order)
    s2 = L.score_tokens(K2, qd)
    idx2 = L.select_topk(s2, ratio=ratio)
    sync()
    Kref, _, start_ref, _ = O.reposition_keys(k, v, wl.chunk_len, new_order, spec.rope_theta, spec.pairing)
    assert starts2 == start_ref.tolist() and N2 == N
    s_ref = O.score_tokens(Kref, q, wl.sm_scale)
    s2_h = s2.cpu().numpy().astype(np.float64)
    assert (np.abs(s2_h - s_ref) <= score_tol(s_ref, spec.m_prompt, 1e-2)).all()
    assert np.array_equal(idx2.cpu().numpy().astype(np.int64), O.select_topk(s2.cpu().numpy(), O.budget(N, ratio)))
    L.close()
