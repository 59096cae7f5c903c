"""CPU oracle for InfoFlow KV's per-layer selective-recompute path (fp64, numpy).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
five stages compute.  Only the tests, the smoke check and the benchmark's
`cpu_baseline` leg may import it; the product (the HIP library and its Python
binding) never does, and it imports nothing from the product.  It shares no
code, tables or helpers with the GPU path.

Every function takes float64 arrays (stored bf16/fp32 values widened exactly by
the caller) and returns float64 / integer arrays with no intermediate rounding.

Parity pins (tests/test_oracle_pins.py): each function below is pinned against
closed forms, brute force on tiny inputs and textbook routines; the paper
prints no worked numeric example of the method, so beyond those pins the
expected values are fixed by the definitions alone.

Readings taken where the paper is silent are stated at each function.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np


# ---------------------------------------------------------------------------
# Stage 1 -- global position reconstruction and key re-rotation
# ---------------------------------------------------------------------------
def rope_frequencies(head_dim: int, theta: float) -> np.ndarray:
    """Angular frequencies of Eq. (4): theta_i = base**(-2 i / d), i < d/2.
    The base is a parameter because the evaluated model families use bases
    other than the 10000 printed in the equation."""
    return np.array([theta ** (-2.0 * i / head_dim) for i in range(head_dim // 2)],
                    dtype=np.float64)


def chunk_starts(chunk_len: Sequence[int], chunk_order: Optional[Sequence[int]]) -> Tuple[np.ndarray, int]:
    """Delta_i of Eq. (5): the start of chunk i in the concatenated context.

    `chunk_order[s]` is the chunk placed in slot s (None = natural order).
    Returns (start per chunk id, N).  The first slot starts at 0.
    """
    n = len(chunk_len)
    order = list(range(n)) if chunk_order is None else [int(c) for c in chunk_order]
    if sorted(order) != list(range(n)):
        raise ValueError("chunk_order is not a permutation")
    start = np.zeros(n, dtype=np.int64)
    run = 0
    for c in order:
        start[c] = run
        run += int(chunk_len[c])
    return start, run


def rotate_pairs(x: np.ndarray, angle: np.ndarray, pairing: str) -> np.ndarray:
    """Rotate each 2-D pair of the last axis by +angle (matrix of Eq. 3:
    a' = a cos - b sin, b' = a sin + b cos).  x: [..., d]; angle broadcastable
    to [..., d/2].  Reading: "half" pairs (x_i, x_{i+d/2}) (the convention of
    the Llama/Qwen checkpoints the paper evaluates); "interleaved" pairs
    (x_{2i}, x_{2i+1})."""
    d = x.shape[-1]
    c, s = np.cos(angle), np.sin(angle)
    y = np.empty_like(x, dtype=np.float64)
    if pairing == "half":
        a, b = x[..., : d // 2], x[..., d // 2:]
        y[..., : d // 2] = a * c - b * s
        y[..., d // 2:] = a * s + b * c
    elif pairing == "interleaved":
        a, b = x[..., 0::2], x[..., 1::2]
        y[..., 0::2] = a * c - b * s
        y[..., 1::2] = a * s + b * c
    else:
        raise ValueError(pairing)
    return y


def reposition_keys(k_chunks: List[np.ndarray], v_chunks: Optional[List[np.ndarray]],
                    chunk_len: Sequence[int], chunk_order: Optional[Sequence[int]],
                    theta: float, pairing: str = "half",
                    cached_pos0: Optional[Sequence[int]] = None,
                    delta_override: Optional[Sequence[int]] = None,
                    freqs: Optional[np.ndarray] = None):
    """Eq. (5) + Eq. (3): a key cached at chunk-local position p of chunk i sits
    at global position g = Delta_i + p, so its rotary phase must advance by
    Delta_i * theta_j in every pair j (rotations compose additively).  Values
    carry no rotary phase and are only concatenated.

    cached_pos0[i]: rotary position the chunk's first row was cached at
    (default 0); the phase advance is then Delta_i - pos0_i.
    delta_override[i]: use this phase advance instead (other RoPE geometries);
    rows are still placed by the concatenation order.

    Returns (K_glob [N,H,d], V_cat [N,H,d] or None, start per chunk, N).
    """
    start, N = chunk_starts(chunk_len, chunk_order)
    H, d = None, None
    for kc in k_chunks:
        if kc.shape[0] > 0 or kc.ndim == 3:
            H, d = kc.shape[1], kc.shape[2]
            break
    th = rope_frequencies(d, theta) if freqs is None else np.asarray(freqs, dtype=np.float64)
    K = np.zeros((N, H, d), dtype=np.float64)
    V = np.zeros((N, H, d), dtype=np.float64) if v_chunks is not None else None
    for i, kc in enumerate(k_chunks):
        L = int(chunk_len[i])
        if L == 0:
            continue
        if delta_override is not None:
            adv = int(delta_override[i])
        else:
            adv = int(start[i]) - (int(cached_pos0[i]) if cached_pos0 is not None else 0)
        phi = np.float64(adv) * th                      # [d/2]
        K[start[i]: start[i] + L] = rotate_pairs(np.asarray(kc[:L], dtype=np.float64), phi, pairing)
        if V is not None:
            V[start[i]: start[i] + L] = v_chunks[i][:L]
    return K, V, start, N


# ---------------------------------------------------------------------------
# Stage 2 -- prompt-conditioned attention-norm score
# ---------------------------------------------------------------------------
def score_tokens(k_glob: np.ndarray, q_prompt: np.ndarray, sm_scale: float,
                 k_prompt: Optional[np.ndarray] = None) -> np.ndarray:
    """Eq. (7): s_j = sum_i A_ij, A the prompt-to-context attention matrix.

    Readings: logits are sm_scale * q.k; query head h reads kv head h // G
    (contiguous groups); A is the softmax over the N context columns
    (context-only domain) unless `k_prompt` [M,H_kv,d] is given, in which case
    each prompt row's softmax also runs over the prompt positions it can see
    causally (rows 0..i), and those columns are dropped afterwards; the
    per-head scores are averaged over all query heads, so that in the
    context-only domain sum_j s_j = M.

    k_glob [N,H_kv,d], q_prompt [M,H_q,d] -> s [N] float64.
    """
    N, H_kv, d = k_glob.shape
    M, H_q, _ = q_prompt.shape
    G = H_q // H_kv
    s = np.zeros(N, dtype=np.float64)
    for h in range(H_q):
        g = h // G
        logits = sm_scale * (q_prompt[:, h, :] @ k_glob[:, g, :].T)          # [M, N]
        if k_prompt is not None:
            lp = sm_scale * (q_prompt[:, h, :] @ k_prompt[:, g, :].T)        # [M, M]
            lp = np.where(np.tril(np.ones((M, M), dtype=bool)), lp, -np.inf)
            full = np.concatenate([logits, lp], axis=1)
        else:
            full = logits
        full = full - full.max(axis=1, keepdims=True)
        e = np.exp(full)
        A = e / e.sum(axis=1, keepdims=True)
        s += A[:, :N].sum(axis=0)
    return s / H_q


# ---------------------------------------------------------------------------
# Stage 3 -- global top-k
# ---------------------------------------------------------------------------
def budget(n_ctx: int, ratio: float) -> int:
    """k = floor(rho * N) ("Chunk Reordering", first paragraph); N counts
    context tokens only."""
    return int(math.floor(float(ratio) * int(n_ctx)))


def select_topk(scores: np.ndarray, k: int) -> np.ndarray:
    """Eq. (8): the k context tokens with the largest scores, one global set
    with no per-chunk quota.  Readings: equal scores are resolved in favour of
    the smaller index; the set is returned in ascending index order."""
    s = np.asarray(scores)
    if not 0 <= k <= len(s):
        raise ValueError("k out of range")
    by_score = np.argsort(-s.astype(np.float64), kind="stable")   # stable: ties keep index order
    return np.sort(by_score[:k]).astype(np.int64)


# ---------------------------------------------------------------------------
# Stage 4 -- causal attention of the selected rows over the full prefix
# ---------------------------------------------------------------------------
def recompute_attention(q_sel: np.ndarray, row_pos: np.ndarray, k_cache: np.ndarray,
                        v_cache: np.ndarray, sm_scale: float):
    """"KV Recomputation" paragraph: each selected token runs an ordinary
    forward pass at its global position over the concatenated sequence, i.e.
    row r (global position p_r) attends causally to cache rows 0..p_r
    inclusive.  Query head h reads kv head h // G.

    q_sel [R,H_q,d], row_pos [R], caches [n_kv,H_kv,d] ->
    (out [R,H_q,d], lse [R,H_q]) with lse the natural-log sum-exp of the
    scaled logits.
    """
    R, H_q, d = q_sel.shape
    H_kv = k_cache.shape[1]
    G = H_q // H_kv
    out = np.zeros((R, H_q, d), dtype=np.float64)
    lse = np.zeros((R, H_q), dtype=np.float64)
    for r in range(R):
        p = int(row_pos[r])
        for g in range(H_kv):
            Kp = k_cache[: p + 1, g, :]                              # [p+1, d]
            Vp = v_cache[: p + 1, g, :]
            q = q_sel[r, g * G:(g + 1) * G, :]                       # [G, d]
            logit = sm_scale * (q @ Kp.T)                            # [G, p+1]
            m = logit.max(axis=1, keepdims=True)
            e = np.exp(logit - m)
            z = e.sum(axis=1, keepdims=True)
            out[r, g * G:(g + 1) * G, :] = (e / z) @ Vp
            lse[r, g * G:(g + 1) * G] = (m + np.log(z))[:, 0]
    return out, lse


# ---------------------------------------------------------------------------
# Stage 5 -- splice recomputed rows into the cache
# ---------------------------------------------------------------------------
def splice_kv(k_cache: np.ndarray, v_cache: np.ndarray, k_new: np.ndarray,
              v_new: np.ndarray, idx: np.ndarray):
    """"KV Recomputation" paragraph, last sentence: recomputed K/V rows replace
    the cached rows of the selected tokens; every other row is reused as is.
    Returns new arrays (inputs are not modified)."""
    K = np.array(k_cache, copy=True)
    V = np.array(v_cache, copy=True)
    idx = np.asarray(idx, dtype=np.int64)
    K[idx] = k_new
    V[idx] = v_new
    return K, V


# ---------------------------------------------------------------------------
# Composite
# ---------------------------------------------------------------------------
# ---------------------------------------------------------------------------
# Rotary embedding of freshly projected rows at their global positions
# ---------------------------------------------------------------------------
def rope_rows(x: np.ndarray, pos: np.ndarray, theta: float, pairing: str = "half",
              freqs: Optional[np.ndarray] = None) -> np.ndarray:
    """"KV Recomputation": the forward pass of a selected token runs at the
    token's position in the concatenated sequence, so its freshly projected
    query and key rows get the rotary embedding of Eq. (3)-(4) at that position:
    row r, pair j is turned by pos[r] * theta_j.  x [R, H, d]; pos [R] (integers)."""
    d = x.shape[-1]
    th = rope_frequencies(d, theta) if freqs is None else np.asarray(freqs, dtype=np.float64)
    out = np.empty_like(np.asarray(x, dtype=np.float64))
    for r in range(x.shape[0]):
        out[r] = rotate_pairs(np.asarray(x[r], dtype=np.float64), np.float64(int(pos[r])) * th, pairing)
    return out


# ---------------------------------------------------------------------------
# Chunk reordering (optional step before the path, "Chunk Reordering")
# ---------------------------------------------------------------------------
def chunk_selection_counts(idx: np.ndarray, chunk_len: Sequence[int],
                           chunk_order: Optional[Sequence[int]]) -> np.ndarray:
    """Numerator of Eq. (9): |S ∩ C_i| for every chunk i, where idx holds the
    selected global row indices and chunk i occupies rows
    [Delta_i, Delta_i + len_i) of the concatenation.  Returned per chunk id."""
    start, _ = chunk_starts(chunk_len, chunk_order)
    counts = np.zeros(len(chunk_len), dtype=np.int64)
    for i in range(len(chunk_len)):
        lo, hi = int(start[i]), int(start[i]) + int(chunk_len[i])
        counts[i] = sum(1 for j in np.asarray(idx).tolist() if lo <= j < hi)
    return counts


def reorder_chunks(chunk_len: Sequence[int], chunk_order: Optional[Sequence[int]],
                   counts: Sequence[int]) -> np.ndarray:
    """"Chunk Reordering": chunks with a larger density r_i = |S ∩ C_i| / |C_i|
    (Eq. 9) are placed closer to the prompt, i.e. later in the concatenation;
    chunks with equal r_i keep their current relative order.  Reading where the
    paper is silent: an empty chunk has r_i = 0; densities are compared exactly
    (as fractions), so equality means equality.

    Returns the new slot -> chunk order."""
    from fractions import Fraction
    n = len(chunk_len)
    order = list(range(n)) if chunk_order is None else [int(c) for c in chunk_order]
    dens = [Fraction(int(counts[c]), int(chunk_len[c])) if int(chunk_len[c]) > 0 else Fraction(0) for c in range(n)]
    # insertion sort on the current order, ascending density: stable by construction
    out: List[int] = []
    for c in order:
        pos = len(out)
        while pos > 0 and dens[out[pos - 1]] > dens[c]:
            pos -= 1
        out.insert(pos, c)
    return np.asarray(out, dtype=np.int64)


def reorder_pass(k_chunks, chunk_len, chunk_order, theta, pairing, q_prompt, sm_scale, ratio):
    """First-stage selection of "Chunk Reordering" with the local-context
    geometry the paper uses for it (appendix "RoPE Geometry", last paragraph):
    every chunk keeps its chunk-local rotary positions (phase advance 0), the
    prompt stays at its global position; one global top-k over the scores;
    Eq. (9) per chunk; new order.  Returns (new_order, counts, idx)."""
    n = len(chunk_len)
    K, _, _, N = reposition_keys(k_chunks, None, chunk_len, chunk_order, theta, pairing,
                                 delta_override=[0] * n)
    s = score_tokens(K, q_prompt, sm_scale)
    idx = select_topk(s, budget(N, ratio))
    counts = chunk_selection_counts(idx, chunk_len, chunk_order)
    return reorder_chunks(chunk_len, chunk_order, counts), counts, idx


def recompute_layer(k_chunks, v_chunks, chunk_len, chunk_order, theta, pairing,
                    q_prompt, sm_scale, ratio, make_rows):
    """One layer of the path in the paper's order: assemble and re-rotate,
    score, select, then recompute.  Reading: a standard forward pass of the
    selected tokens sees their freshly projected K/V, so the recomputed rows
    are spliced in first and the attention runs over the spliced cache.

    make_rows(idx) -> (q_sel, k_new, v_new) in float64 supplies what the
    model's projections would (they are outside this path).
    """
    K, V, start, N = reposition_keys(k_chunks, v_chunks, chunk_len, chunk_order, theta, pairing)
    s = score_tokens(K, q_prompt, sm_scale)
    idx = select_topk(s, budget(N, ratio))
    q_sel, k_new, v_new = make_rows(idx)
    K2, V2 = splice_kv(K, V, k_new, v_new, idx)
    out, lse = recompute_attention(q_sel, idx, K2, V2, sm_scale)
    return dict(k=K2, v=V2, scores=s, idx=idx, out=out, lse=lse, start=start, n_ctx=N)
