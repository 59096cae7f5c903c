"""Test-side plumbing: numpy storage arrays <-> torch device tensors, and the
tolerance forms used by the parity tests."""
import numpy as np
import torch

from workloads import to_f64, to_storage

DEV = "cuda:0"


def to_dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).view(torch.bfloat16).to(DEV)
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(DEV)


def to_host_f64(t: torch.Tensor, dtype: str) -> np.ndarray:
    """Device tensor in storage dtype -> exact float64 numpy array."""
    if dtype == "bf16":
        return to_f64(t.cpu().contiguous().view(torch.int16).numpy().view(np.uint16), "bf16")
    return t.cpu().numpy().astype(np.float64)


def to_host_bits(t: torch.Tensor, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return t.cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
    return t.cpu().numpy().view(np.uint32)


def bf16_ulp(x: np.ndarray) -> np.ndarray:
    """Spacing of bfloat16 (8 significand bits) at |x| (x != 0)."""
    ax = np.maximum(np.abs(x), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 7)


def make_layer(spec, max_ctx, max_prompt, flags=0, **kw):
    from paper_2603_05353_amd import Layer
    return Layer(spec.dtype, spec.n_q_heads, spec.n_kv_heads, spec.head_dim, spec.rope_theta,
                 max_ctx=max_ctx, max_prompt=max_prompt, pairing=spec.pairing, flags=flags, **kw)


def score_tol(s_ref: np.ndarray, m_prompt: int, rtol: float) -> np.ndarray:
    """|s - s_ref| <= rtol * (|s_ref| + M/N): relative to the larger of the
    score and the mean score, so near-zero scores do not demand absolute zero."""
    return rtol * (np.abs(s_ref) + m_prompt / len(s_ref))


# ---------------------------------------------------------------------------
# stage 4: what "equal to the oracle" means for the attention output
# ---------------------------------------------------------------------------
ATTN_ABS_TOL = {"f32": 1e-4, "bf16": 2e-2}      # the contract's max-abs bounds
LSE_TOL = {"f32": 1e-4, "bf16": 1e-3}           # logits, exponentials and row sums are fp32 in both kernels


def attention_error_bound(ref: np.ndarray, ref_abs: np.ndarray, dtype: str) -> np.ndarray:
    """Element-wise bound on |out - ref| that follows from the kernel's arithmetic, where
    ref = sum_j w_j v_j is the exact output and ref_abs = sum_j w_j |v_j| (the oracle run on |V|).

    bf16 kernel: logits, exponentials and the normaliser are fp32 (relative error ~1e-6); each
    probability is rounded to bf16 before the second product (relative error <= 2^-8 each, so the
    numerator moves by at most 2^-8 * sum_j w_j |v_j|); the result is rounded once to bf16
    (<= 2^-8 of its magnitude).  fp32 kernel: accumulation error only.
    Unlike a fixed absolute tolerance this stays below the signal at any depth: near-uniform
    attention over p keys gives |ref| ~ sigma_V / sqrt(p) while the bound is ~ 2^-8 * 0.8 sigma_V."""
    if dtype == "bf16":
        eps = 2.0 ** -8
        return eps * (1 + eps) * ref_abs + eps * np.abs(ref) + 4e-6 * ref_abs + 1e-30
    return 2e-5 * ref_abs + 1e-30


def assert_attention_close(out, ref, ref_abs, dtype, lse=None, lse_ref=None):
    """The contract's absolute tolerance AND the magnitude-aware bound, element by element."""
    assert out.shape == ref.shape
    if ref.size == 0:  # an empty selection (k = 0): nothing to compare
        return
    err = np.abs(out - ref)
    assert err.max() <= ATTN_ABS_TOL[dtype], f"max-abs error {err.max()}"
    excess = err - attention_error_bound(ref, ref_abs, dtype)
    if excess.max() > 0:
        w = np.unravel_index(np.argmax(excess), excess.shape)
        raise AssertionError(f"attention output differs from the oracle beyond the rounding bound at {w}: "
                             f"|{out[w]} - {ref[w]}| = {err[w]}, bound {err[w] - excess[w]}; "
                             f"{int((excess > 0).sum())} of {excess.size} elements")
    if lse is not None:
        e = np.abs(lse - lse_ref).max()
        assert e <= LSE_TOL[dtype], f"log-sum-exp differs by {e}"


def needle_case(n_kv, hq, hkv, n_rows, seed, logit=24.0):
    """Inputs whose outputs are O(1) at any depth: V ~ N(0, 1), and every query column is aligned
    with ONE key of its prefix so strongly that the output is that key's value row to within a few
    per cent.  The target keys cover, per row: position 0, the row's own position, the first and
    last key of its last tile, the last key of the tile before, keys 63 and 64, and seeded random
    positions -- so a wrong or dropped product in any tile class (first, middle in either LDS
    stage, last masked, any piece of a cut row block) moves some output by O(1)."""
    g = np.random.Generator(np.random.Philox(key=[seed, 41]))
    d = 128
    K64 = g.standard_normal((n_kv, hkv, d)) * d ** -0.5
    V64 = g.standard_normal((n_kv, hkv, d))
    rows = np.sort(g.choice(n_kv, size=n_rows, replace=False))
    rows[0], rows[-1] = 0, n_kv - 1
    rows = np.unique(rows)
    G = hq // hkv
    Q64 = np.zeros((len(rows), hq, d))
    target = np.zeros((len(rows), hq), dtype=np.int64)
    for r, p in enumerate(rows):
        p = int(p)
        fixed = [0, p, 64 * (p // 64), max(64 * (p // 64) - 1, 0), min(63, p), min(64, p), p // 2]
        for h in range(hq):
            j = fixed[h] if h < len(fixed) else int(g.integers(0, p + 1))
            target[r, h] = j
            kj = K64[j, h // G]
            Q64[r, h] = (logit * d ** 0.5) * kj / (kj @ kj)     # the target's logit is `logit` whatever its norm
    K_st, V_st, q_st = (to_storage(x, "bf16") for x in (K64, V64, Q64))
    return rows, target, q_st, K_st, V_st
