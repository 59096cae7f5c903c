"""CPU checks of the stage-4 comparison itself (tests/helpers.assert_attention_close): it must
accept what the kernel's arithmetic can legitimately produce and reject wrong second products at
any depth.  The mistakes are planted in copies of the ORACLE's output, never in a kernel."""
import numpy as np
import pytest

from oracle import infoflow_oracle as O
from tests.helpers import assert_attention_close
from workloads import f64_to_bf16_bits, bf16_bits_to_f64


def rng(seed):
    return np.random.Generator(np.random.Philox(key=[seed, 4]))


def bf16_round(x):
    return bf16_bits_to_f64(f64_to_bf16_bits(x))


@pytest.fixture(scope="module")
def deep_case():
    """Near-uniform attention over up to 3000 keys with sigma_V = 128^-1/2: what the benchmark
    workloads look like, outputs of ~3e-3 at depth."""
    g = rng(1)
    N, Hq, Hkv, d = 3000, 4, 2, 128
    sig = d ** -0.5
    K = bf16_round(g.standard_normal((N, Hkv, d)) * sig)
    V = bf16_round(g.standard_normal((N, Hkv, d)) * sig)
    rows = np.array([0, 5, 40, 127, 128, 700, 1500, 2999])
    Q = bf16_round(g.standard_normal((len(rows), Hq, d)) * sig)
    ref, lse = O.recompute_attention(Q, rows, K, V, d ** -0.5)
    ref_abs, _ = O.recompute_attention(Q, rows, K, np.abs(V), d ** -0.5)
    return dict(rows=rows, Q=Q, K=K, V=V, ref=ref, ref_abs=ref_abs, lse=lse, scale=d ** -0.5)


def kernel_like(c):
    """The bf16 kernel's rounding points re-enacted in numpy: fp32 probabilities against a running
    reference, the normaliser from the unrounded values, bf16-rounded probabilities in the second
    product, one rounding of the result to bf16."""
    Q, K, V, rows = c["Q"], c["K"], c["V"], c["rows"]
    G = Q.shape[1] // K.shape[1]
    out = np.zeros_like(c["ref"])
    for r, p in enumerate(rows):
        for h in range(Q.shape[1]):
            lg = (c["scale"] * (K[: p + 1, h // G] @ Q[r, h])).astype(np.float32)
            e = np.exp(lg - lg.max()).astype(np.float32)
            out[r, h] = bf16_round((bf16_round(e)[None, :] @ V[: p + 1, h // G])[0] / np.float32(e.sum(dtype=np.float32)))
    return out


def test_bound_accepts_the_kernels_own_rounding(deep_case):
    c = deep_case
    assert_attention_close(kernel_like(c), c["ref"], c["ref_abs"], "bf16", c["lse"] + 3e-4, c["lse"])


def old_check(out, ref):
    return np.abs(out - ref).max() <= 2e-2


def test_swapped_columns_are_rejected(deep_case):
    c = deep_case
    bad = c["ref"].copy()
    bad[..., [3, 77]] = bad[..., [77, 3]]
    assert old_check(bad[4:], c["ref"][4:])            # the fixed absolute tolerance alone does not notice at depth
    with pytest.raises(AssertionError):
        assert_attention_close(bad, c["ref"], c["ref_abs"], "bf16")
    with pytest.raises(AssertionError):                # not even on the deep rows alone
        assert_attention_close(bad[5:], c["ref"][5:], c["ref_abs"][5:], "bf16")


def test_zero_output_at_depth_is_rejected(deep_case):
    c = deep_case
    bad = c["ref"].copy()
    bad[c["rows"] >= 128] = 0.0
    assert old_check(bad[5:], c["ref"][5:])            # positions 700 and beyond: zeros pass the absolute tolerance
    with pytest.raises(AssertionError):
        assert_attention_close(bad, c["ref"], c["ref_abs"], "bf16")
    # every deep row fails on its own
    for r in np.nonzero(c["rows"] >= 128)[0]:
        with pytest.raises(AssertionError):
            assert_attention_close(bad[r:r + 1], c["ref"][r:r + 1], c["ref_abs"][r:r + 1], "bf16")


def test_dropped_tile_and_wrong_normaliser_are_rejected(deep_case):
    c = deep_case
    r = 6                                               # position 1500
    p = int(c["rows"][r])
    G = c["Q"].shape[1] // c["K"].shape[1]
    # keys 64..127 left out of the second product (the normaliser still counts them)
    bad = c["ref"].copy()
    for h in range(c["Q"].shape[1]):
        lg = c["scale"] * (c["K"][: p + 1, h // G] @ c["Q"][r, h])
        w = np.exp(lg - lg.max())
        w /= w.sum()
        w[64:128] = 0
        bad[r, h] = w @ c["V"][: p + 1, h // G]
    assert old_check(bad, c["ref"])
    with pytest.raises(AssertionError):
        assert_attention_close(bad, c["ref"], c["ref_abs"], "bf16")
    # a normaliser off by 3 %
    with pytest.raises(AssertionError):
        assert_attention_close(c["ref"] * 1.03, c["ref"], c["ref_abs"], "bf16")
    # log-sum-exp off by 5e-3 is caught by the tight LSE bound
    with pytest.raises(AssertionError):
        assert_attention_close(c["ref"], c["ref"], c["ref_abs"], "bf16", c["lse"] + 5e-3, c["lse"])


def test_fp32_bound(deep_case):
    c = deep_case
    ok = c["ref"].astype(np.float32).astype(np.float64)
    assert_attention_close(ok, c["ref"], c["ref_abs"], "f32", c["lse"], c["lse"])
    with pytest.raises(AssertionError):
        assert_attention_close(c["ref"] * (1 + 1e-3), c["ref"], c["ref_abs"], "f32")
