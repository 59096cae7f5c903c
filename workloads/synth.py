"""Seeded synthetic workloads shaped like the paper's multi-chunk KV-reuse setting.

What is modelled (and only that): a set of context chunks that were prefilled
independently, so each chunk's keys carry rotary positions 0..len-1 (Method,
"Input Chunking and Prefilling"); a chunk order; a prompt whose queries carry
rotary positions N..N+M-1 (the GLOBAL geometry of the "RoPE Geometry"
paragraph); and, for the recompute stages, freshly "projected" rows for a given
selected set.  Real model weights and datasets are not available, so values are
Gaussian with a few *planted* tokens whose global-frame keys are aligned with
the prompt, which gives the scoring stage something to find.

Everything is drawn in fp64 from numpy's counter-based Philox generator, rounded
once (round-to-nearest-even) to the storage dtype, and handed out as numpy
arrays: float32 arrays for "f32", uint16 bit patterns for "bf16".  The same
bits go to the CPU oracle and to the GPU library.

The only arithmetic here is what a model would have done *before* the path
starts: the rotary embedding of Eq. (3)-(4) applied at an absolute position.
None of the five stages' arithmetic lives in this module.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

BASE_SEED = 20260305


# --------------------------------------------------------------------------
# storage-dtype helpers
# --------------------------------------------------------------------------
def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round to bfloat16 (nearest-even) and return the 16-bit patterns."""
    f32 = np.ascontiguousarray(x, dtype=np.float32)
    bits = f32.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))
    return ((bits + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(u: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns exactly to float64."""
    u = np.ascontiguousarray(u, dtype=np.uint16)
    return (u.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return f64_to_bf16_bits(x)
    raise ValueError(f"unknown dtype {dtype!r}")


def to_f64(x: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a stored array to float64."""
    if dtype == "f32":
        return np.asarray(x, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        return bf16_bits_to_f64(x)
    raise ValueError(f"unknown dtype {dtype!r}")


# --------------------------------------------------------------------------
# model-side rotary embedding (input construction only)
# --------------------------------------------------------------------------
def inv_freq(head_dim: int, theta: float) -> np.ndarray:
    """theta_i = base^(-2i/d), i = 0..d/2-1 (Eq. 4, with the base a parameter)."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    return np.power(np.float64(theta), -2.0 * i / np.float64(head_dim))


def rope_at(x: np.ndarray, pos, theta: float, pairing: str = "half") -> np.ndarray:
    """Apply the rotation of Eq. (3) at absolute position(s) `pos`.

    x: [T, H, d] float64; pos: scalar or [T].  Pairing "half" couples
    (x_i, x_{i+d/2}); "interleaved" couples (x_{2i}, x_{2i+1}).
    """
    x = np.asarray(x, dtype=np.float64)
    T, H, d = x.shape
    p = np.broadcast_to(np.asarray(pos, dtype=np.float64), (T,))
    ang = p[:, None] * inv_freq(d, theta)[None, :]          # [T, d/2]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    out = np.empty_like(x)
    if pairing == "half":
        a, b = x[..., : d // 2], x[..., d // 2:]
        out[..., : d // 2] = a * c - b * s
        out[..., d // 2:] = a * s + b * c
    elif pairing == "interleaved":
        a, b = x[..., 0::2], x[..., 1::2]
        out[..., 0::2] = a * c - b * s
        out[..., 1::2] = a * s + b * c
    else:
        raise ValueError(pairing)
    return out


# --------------------------------------------------------------------------
# specification
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class WorkloadSpec:
    name: str
    dtype: str                      # "f32" | "bf16"
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    rope_theta: float
    m_prompt: int
    ratios: Sequence[float]
    # chunks: either explicit lengths, or (n_chunks, lo, hi) drawn uniformly
    chunk_lens: Optional[Sequence[int]] = None
    uneven: Optional[Sequence[int]] = None      # (n_chunks, lo, hi) inclusive
    permute_order: bool = False
    sigma: float = 1.0              # per-component std of Q, K, V
    planted_count: Optional[int] = None
    planted_frac: float = 0.0
    plant_gain: float = 3.0         # planted key += gain * sigma * unit direction
    key_norm_lognormal: float = 0.0  # per-token key scale exp(N(0, s^2))
    lowrank_chunks: Sequence[int] = ()   # chunk ids whose keys are low-rank
    lowrank_rank: int = 32
    pairing: str = "half"
    seed: int = BASE_SEED

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


def _c5_lens() -> List[int]:
    return [1024] * 16 + [512] * 8


PRESETS: Dict[str, WorkloadSpec] = {
    # Tiny single layer, fp32.
    "C1": WorkloadSpec("C1", "f32", 8, 8, 64, 1e4, 32, (0.15,),
                       chunk_lens=[256] * 4, sigma=1.0, planted_count=16,
                       seed=BASE_SEED + 1),
    # Llama-3-8B-shaped layer, 8K context.
    "C2": WorkloadSpec("C2", "bf16", 32, 8, 128, 5e5, 64, (0.15,),
                       chunk_lens=[512] * 16, sigma=128 ** -0.5,
                       planted_frac=0.05, seed=BASE_SEED + 2),
    # Same layer, 32K context, permuted chunk order.
    "C3": WorkloadSpec("C3", "bf16", 32, 8, 128, 5e5, 128, (0.05, 0.15, 0.30),
                       chunk_lens=[512] * 64, permute_order=True,
                       sigma=128 ** -0.5, planted_frac=0.05, seed=BASE_SEED + 3),
    # Long context, uneven chunks, heavy-tailed key norms.
    "C4": WorkloadSpec("C4", "bf16", 32, 8, 128, 5e5, 128, (0.10,),
                       uneven=(128, 512, 1536), sigma=128 ** -0.5,
                       planted_frac=0.02, key_norm_lognormal=0.5,
                       seed=BASE_SEED + 4),
    # VLM-shaped layer: 16 image chunks (low-rank keys) + 8 text chunks,
    # placed in a seeded random slot order.
    "C5": WorkloadSpec("C5", "bf16", 28, 4, 128, 1e6, 96, (0.15,),
                       chunk_lens=_c5_lens(), permute_order=True,
                       sigma=128 ** -0.5, planted_frac=0.05,
                       lowrank_chunks=tuple(range(16)), lowrank_rank=32,
                       seed=BASE_SEED + 5),
}


def preset(name: str, **overrides) -> WorkloadSpec:
    """A BASELINE configuration, optionally with fields replaced (e.g. a
    shorter `chunk_lens` for tests that must finish in seconds)."""
    return dataclasses.replace(PRESETS[name], **overrides)


# --------------------------------------------------------------------------
# workload
# --------------------------------------------------------------------------
@dataclass
class Workload:
    spec: WorkloadSpec
    chunk_len: np.ndarray          # int32 [n_chunks], by chunk id
    chunk_order: np.ndarray        # int32 [n_chunks], slot -> chunk id
    chunk_start: np.ndarray        # int64 [n_chunks], by chunk id (start row in the concatenation)
    n_ctx: int
    k_chunks: List[np.ndarray]     # storage arrays [len_i, H_kv, d], chunk-local rotary positions
    v_chunks: List[np.ndarray]
    q_prompt: np.ndarray           # storage [M, H_q, d], rotary positions N..N+M-1
    planted: np.ndarray            # int64 sorted global indices of planted tokens
    k_global32: np.ndarray = field(repr=False, default=None)  # float32 [N,H_kv,d] global-frame keys before rounding
    v_global32: np.ndarray = field(repr=False, default=None)

    @property
    def sm_scale(self) -> float:
        return float(self.spec.head_dim) ** -0.5


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def make_workload(spec: WorkloadSpec) -> Workload:
    H_q, H_kv, d = spec.n_q_heads, spec.n_kv_heads, spec.head_dim
    G = spec.group
    assert H_q % H_kv == 0 and d % 2 == 0

    # ---- chunk geometry ---------------------------------------------------
    if spec.chunk_lens is not None:
        lens = np.asarray(spec.chunk_lens, dtype=np.int32)
    else:
        n, lo, hi = spec.uneven
        lens = _rng(spec.seed, 0).integers(lo, hi + 1, size=n).astype(np.int32)
    n_chunks = len(lens)
    if spec.permute_order:
        order = _rng(spec.seed, 1).permutation(n_chunks).astype(np.int32)
    else:
        order = np.arange(n_chunks, dtype=np.int32)
    slot_start = np.zeros(n_chunks, dtype=np.int64)
    slot_start[1:] = np.cumsum(lens[order].astype(np.int64))[:-1]
    chunk_start = np.zeros(n_chunks, dtype=np.int64)
    chunk_start[order] = slot_start
    N = int(lens.sum())
    M = spec.m_prompt

    # ---- prompt queries at rotary positions N..N+M-1 ------------------------
    q_raw = _rng(spec.seed, 2).standard_normal((M, H_q, d)) * spec.sigma
    q_rot = rope_at(q_raw, N + np.arange(M), spec.rope_theta, spec.pairing)
    q_prompt = to_storage(q_rot, spec.dtype)
    q_st = to_f64(q_prompt, spec.dtype)

    # shared direction per kv group: normalised mean of that group's stored queries
    u = q_st.reshape(M, H_kv, G, d).mean(axis=(0, 2))            # [H_kv, d]
    u /= np.linalg.norm(u, axis=-1, keepdims=True)

    # ---- planted token positions -----------------------------------------------
    n_plant = spec.planted_count if spec.planted_count is not None else int(round(spec.planted_frac * N))
    n_plant = min(n_plant, N)
    planted = np.sort(_rng(spec.seed, 3).choice(N, size=n_plant, replace=False)).astype(np.int64)
    is_planted = np.zeros(N, dtype=bool)
    is_planted[planted] = True

    # ---- per-chunk keys/values, built in the global frame then rotated back -----
    k_chunks: List[np.ndarray] = [None] * n_chunks
    v_chunks: List[np.ndarray] = [None] * n_chunks
    k_global32 = np.empty((N, H_kv, d), dtype=np.float32)
    v_global32 = np.empty((N, H_kv, d), dtype=np.float32)
    lowrank = set(int(c) for c in spec.lowrank_chunks)
    basis = None
    if lowrank:
        basis = _rng(spec.seed, 4).standard_normal((H_kv, spec.lowrank_rank, d)) \
            * (spec.sigma / np.sqrt(spec.lowrank_rank))
    for cid in range(n_chunks):
        L = int(lens[cid])
        r0 = int(chunk_start[cid])
        g = _rng(spec.seed, 100 + cid)
        if cid in lowrank:
            z = g.standard_normal((L, H_kv, spec.lowrank_rank))
            kg = np.einsum("thr,hrd->thd", z, basis)
            kg += 0.05 * spec.sigma * g.standard_normal((L, H_kv, d))
        else:
            kg = g.standard_normal((L, H_kv, d)) * spec.sigma
        if spec.key_norm_lognormal > 0:
            kg *= np.exp(spec.key_norm_lognormal * g.standard_normal((L, 1, 1)))
        vg = g.standard_normal((L, H_kv, d)) * spec.sigma
        mask = is_planted[r0:r0 + L]
        if mask.any():
            kg[mask] += spec.plant_gain * spec.sigma * u[None, :, :]
        k_global32[r0:r0 + L] = kg
        v_global32[r0:r0 + L] = vg
        # what the offline per-chunk prefill would have cached: the same key
        # at rotary position p instead of r0 + p, i.e. rotated back by r0.
        k_loc = rope_at(kg, -float(r0), spec.rope_theta, spec.pairing) if L else kg
        k_chunks[cid] = to_storage(k_loc, spec.dtype)
        v_chunks[cid] = to_storage(vg, spec.dtype)

    return Workload(spec=spec, chunk_len=lens, chunk_order=order, chunk_start=chunk_start,
                    n_ctx=N, k_chunks=k_chunks, v_chunks=v_chunks, q_prompt=q_prompt,
                    planted=planted, k_global32=k_global32, v_global32=v_global32)


def make_recompute_inputs(wl: Workload, idx: np.ndarray, stream: int = 7):
    """Rows a model would hand to the recompute stages for the selected set
    `idx` (ascending global positions): queries at their global rotary
    position, and freshly projected K/V rows modelled as the global-frame cached
    row plus a small seeded perturbation, so that a splice is observable.

    Returns (q_sel [R,H_q,d], k_new [R,H_kv,d], v_new [R,H_kv,d]) in storage dtype.
    """
    spec = wl.spec
    idx = np.asarray(idx, dtype=np.int64)
    R = len(idx)
    g = _rng(spec.seed, stream)
    q_raw = g.standard_normal((R, spec.n_q_heads, spec.head_dim)) * spec.sigma
    q_sel = rope_at(q_raw, idx, spec.rope_theta, spec.pairing) if R else q_raw
    k_new = wl.k_global32[idx].astype(np.float64) \
        + 0.1 * spec.sigma * g.standard_normal((R, spec.n_kv_heads, spec.head_dim))
    v_new = wl.v_global32[idx].astype(np.float64) \
        + 0.1 * spec.sigma * g.standard_normal((R, spec.n_kv_heads, spec.head_dim))
    return (to_storage(q_sel, spec.dtype), to_storage(k_new, spec.dtype),
            to_storage(v_new, spec.dtype))
