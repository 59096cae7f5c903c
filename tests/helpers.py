"""Test-side plumbing: numpy storage arrays <-> torch device tensors, and the
tolerance forms used by the parity tests."""
import numpy as np
import torch

from workloads import to_f64

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
