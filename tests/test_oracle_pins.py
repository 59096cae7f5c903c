"""Pins for the CPU oracle: closed forms, brute force on tiny inputs, textbook
routines and invariants.  Nothing here re-uses the oracle's own formulae: the
independent side of every comparison is written out in this file (complex
multiplication for rotations, explicit Python loops for softmax sums, scipy for
textbook routines)."""
import cmath
import math
import os

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import infoflow_oracle as O
from workloads import make_recompute_inputs, make_workload, preset, to_f64

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.Generator(np.random.Philox(key=[seed, 99]))


# --------------------------------------------------------------------------
# independent helpers
# --------------------------------------------------------------------------
def rope_scratch_complex(x, pos, theta, pairing):
    """RoPE from scratch at absolute positions via complex multiplication:
    (a + ib) * exp(i * pos * theta_j).  x [T,H,d]."""
    T, H, d = x.shape
    y = np.zeros_like(x)
    for t in range(T):
        for h in range(H):
            for j in range(d // 2):
                ia, ib = (j, j + d // 2) if pairing == "half" else (2 * j, 2 * j + 1)
                w = cmath.exp(1j * pos[t] * theta ** (-2.0 * j / d))
                z = complex(x[t, h, ia], x[t, h, ib]) * w
                y[t, h, ia], y[t, h, ib] = z.real, z.imag
    return y


def brute_scores(K, Q, scale, G):
    N, M, Hq = K.shape[0], Q.shape[0], Q.shape[1]
    s = [0.0] * N
    for h in range(Hq):
        for i in range(M):
            lg = [scale * sum(Q[i, h, c] * K[j, h // G, c] for c in range(K.shape[2])) for j in range(N)]
            mx = max(lg)
            ex = [math.exp(v - mx) for v in lg]
            z = sum(ex)
            for j in range(N):
                s[j] += ex[j] / z / Hq
    return np.array(s)


def brute_causal_attention(Q, K, V, scale, G):
    """Dense causal self-attention, row t sees rows 0..t.  Python loops."""
    T, Hq, d = Q.shape
    out = np.zeros((T, Hq, d))
    for t in range(T):
        for h in range(Hq):
            lg = np.array([scale * float(np.dot(Q[t, h], K[j, h // G])) for j in range(t + 1)])
            w = softmax(lg)
            acc = np.zeros(d)
            for j in range(t + 1):
                acc += w[j] * V[j, h // G]
            out[t, h] = acc
    return out


# --------------------------------------------------------------------------
# stage 1
# --------------------------------------------------------------------------
@pytest.mark.parametrize("pairing", ["half", "interleaved"])
def test_reposition_equals_rope_from_scratch(pairing):
    """Re-rotating a locally-rotated key by Delta equals rotating the raw key
    at the global position (rotations compose: R(a)R(b) = R(a+b))."""
    g = rng(1)
    theta, H, d = 10000.0, 2, 8
    lens = [3, 0, 5, 2]
    order = [2, 0, 3, 1]
    raw = [g.standard_normal((L, H, d)) for L in lens]
    cached = [rope_scratch_complex(raw[i], list(range(lens[i])), theta, pairing) for i in range(4)]
    vals = [g.standard_normal((L, H, d)) for L in lens]
    K, V, start, N = O.reposition_keys(cached, vals, lens, order, theta, pairing)
    assert N == 10
    # brute-force starts: walk the slots
    exp_start = {2: 0, 0: 5, 3: 8, 1: 10}
    for c in range(4):
        assert start[c] == exp_start[c]
        want = rope_scratch_complex(raw[c], [exp_start[c] + p for p in range(lens[c])], theta, pairing)
        np.testing.assert_allclose(K[exp_start[c]:exp_start[c] + lens[c]], want, rtol=0, atol=1e-13)
        assert np.array_equal(V[exp_start[c]:exp_start[c] + lens[c]], vals[c])


def test_reposition_slot0_identity_and_norms():
    g = rng(2)
    lens = [4, 6]
    k = [g.standard_normal((L, 3, 16)) for L in lens]
    K, _, start, N = O.reposition_keys(k, None, lens, None, 5e5)
    assert np.array_equal(K[:4], k[0])              # Delta = 0: cos 1, sin 0 exactly
    assert not np.allclose(K[4:], k[1])
    # per-pair norms preserved
    def pair_norm(x):
        return np.hypot(x[..., :8], x[..., 8:])
    np.testing.assert_allclose(pair_norm(K[4:]), pair_norm(k[1]), rtol=1e-14)


def test_reposition_hand_value_and_direction():
    """d = 2 has a single pair of frequency 1: a key (1, 0) cached in a chunk
    that starts at position L turns into (cos L, sin L) -- counter-clockwise."""
    L = 3
    k = [np.zeros((L, 1, 2)), np.array([[[1.0, 0.0]], [[0.0, 1.0]]])]
    K, _, _, _ = O.reposition_keys(k, None, [L, 2], None, 10000.0)
    np.testing.assert_allclose(K[L, 0], [math.cos(L), math.sin(L)], atol=1e-15)
    np.testing.assert_allclose(K[L + 1, 0], [-math.sin(L), math.cos(L)], atol=1e-15)


def test_reposition_frequency_index():
    """Pair j rotates at base**(-2j/d): pair 0 fastest (frequency 1), the last
    pair slowest; checked pair by pair against math.pow."""
    d, base, L = 8, 100.0, 7
    k = [np.zeros((L, 1, d)), np.zeros((1, 1, d))]
    k[1][0, 0, : d // 2] = 1.0       # a = 1, b = 0 in every pair
    K, _, _, _ = O.reposition_keys(k, None, [L, 1], None, base)
    for j in range(d // 2):
        ang = L * math.pow(base, -2.0 * j / d)
        assert abs(K[L, 0, j] - math.cos(ang)) < 1e-14
        assert abs(K[L, 0, j + d // 2] - math.sin(ang)) < 1e-14
    assert abs(O.rope_frequencies(d, base)[0] - 1.0) == 0.0


def test_reposition_relative_position_invariance():
    """q.k depends only on the position difference: shifting the chunk start
    and the query position by the same amount leaves the logit unchanged."""
    g = rng(3)
    theta, d = 10000.0, 16
    kraw = g.standard_normal((1, 1, d))
    qraw = g.standard_normal((1, 1, d))
    logits = []
    for shift in (0, 11, 400):
        pad = [np.zeros((shift, 1, d)), rope_scratch_complex(kraw, [0], theta, "half")]
        K, _, _, N = O.reposition_keys(pad, None, [shift, 1], None, theta)
        q = rope_scratch_complex(qraw, [N + 5], theta, "half")
        logits.append(float(np.dot(q[0, 0], K[shift, 0])))
    assert abs(logits[0] - logits[1]) < 1e-12 and abs(logits[0] - logits[2]) < 1e-12


def test_reposition_pos0_and_override():
    g = rng(4)
    theta, d = 10000.0, 8
    raw = g.standard_normal((3, 1, d))
    # chunk cached at positions 7..9, lands at 4..6 -> advance by -3
    cached = rope_scratch_complex(raw, [7, 8, 9], theta, "half")
    K, _, _, _ = O.reposition_keys([np.zeros((4, 1, d)), cached], None, [4, 3], None, theta,
                                   cached_pos0=[0, 7])
    np.testing.assert_allclose(K[4:], rope_scratch_complex(raw, [4, 5, 6], theta, "half"), atol=1e-13)
    # override: advance 0 keeps the local frame but rows still move
    K0, _, _, _ = O.reposition_keys([np.zeros((4, 1, d)), cached], None, [4, 3], None, theta,
                                    delta_override=[0, 0])
    assert np.array_equal(K0[4:], cached)


def test_chunk_starts_rejects_non_permutation():
    with pytest.raises(ValueError):
        O.chunk_starts([2, 2, 2], [0, 0, 1])


def test_generator_caches_reposition_to_global_frame():
    """The synthetic chunk caches were derived from global-frame keys; the
    oracle must bring the stored local keys back to them (up to the storage
    rounding of the cache)."""
    wl = make_workload(preset("C3", chunk_lens=[40, 24, 56, 8], m_prompt=8))
    sp = wl.spec
    k = [to_f64(c, sp.dtype) for c in wl.k_chunks]
    K, _, start, N = O.reposition_keys(k, None, wl.chunk_len, wl.chunk_order, sp.rope_theta)
    assert np.array_equal(start, wl.chunk_start) and N == wl.n_ctx
    err = np.abs(K - wl.k_global32.astype(np.float64)).max()
    assert err < 2 ** -8 * np.abs(wl.k_global32).max() * 1.5


# --------------------------------------------------------------------------
# stage 2
# --------------------------------------------------------------------------
def test_score_brute_force_gqa():
    g = rng(10)
    N, M, Hq, Hkv, d = 7, 3, 4, 2, 6
    K = g.standard_normal((N, Hkv, d))
    Q = g.standard_normal((M, Hq, d))
    s = O.score_tokens(K, Q, 0.37)
    np.testing.assert_allclose(s, brute_scores(K, Q, 0.37, Hq // Hkv), rtol=1e-12)


def test_score_invariants():
    g = rng(11)
    N, M, Hq, Hkv, d = 50, 5, 6, 3, 8
    K = g.standard_normal((N, Hkv, d)) * 2
    Q = g.standard_normal((M, Hq, d)) * 2
    s = O.score_tokens(K, Q, d ** -0.5)
    assert abs(s.sum() - M) < 1e-12
    assert (s >= 0).all() and (s <= M).all()
    # permutation equivariance over context tokens
    perm = g.permutation(N)
    np.testing.assert_allclose(O.score_tokens(K[perm], Q, d ** -0.5), s[perm], rtol=1e-12)
    # identical keys -> uniform attention
    Ku = np.repeat(K[:1], N, axis=0)
    np.testing.assert_allclose(O.score_tokens(Ku, Q, d ** -0.5), np.full(N, M / N), rtol=1e-13)


def test_score_single_row_is_textbook_softmax():
    g = rng(12)
    K = g.standard_normal((9, 1, 4))
    Q = g.standard_normal((1, 1, 4))
    want = softmax(0.5 * (K[:, 0, :] @ Q[0, 0]))
    np.testing.assert_allclose(O.score_tokens(K, Q, 0.5), want, rtol=1e-13)


def test_score_with_prompt_keys_brute_force():
    """Real-forward domain: row i also sees prompt positions 0..i."""
    g = rng(13)
    N, M, d = 5, 3, 4
    K = g.standard_normal((N, 1, d))
    Q = g.standard_normal((M, 1, d))
    Kp = g.standard_normal((M, 1, d))
    want = np.zeros(N)
    for i in range(M):
        lg = [0.5 * float(Q[i, 0] @ K[j, 0]) for j in range(N)] + \
             [0.5 * float(Q[i, 0] @ Kp[t, 0]) for t in range(i + 1)]
        w = softmax(np.array(lg))
        want += w[:N]
    np.testing.assert_allclose(O.score_tokens(K, Q, 0.5, k_prompt=Kp), want, rtol=1e-12)
    assert O.score_tokens(K, Q, 0.5, k_prompt=Kp).sum() < M


def test_planted_tokens_need_global_positions():
    """Planted tokens were built in the GLOBAL frame: scoring re-rotated keys
    finds them, scoring the chunk-local keys as cached does not (the paper's
    finding that rankings under a mismatched geometry are misleading)."""
    wl = make_workload(preset("C1"))
    sp = wl.spec
    k = [to_f64(c, sp.dtype) for c in wl.k_chunks]
    q = to_f64(wl.q_prompt, sp.dtype)
    K, _, _, N = O.reposition_keys(k, None, wl.chunk_len, wl.chunk_order, sp.rope_theta)
    kk = O.budget(N, 0.15)
    assert kk == 153
    S = set(O.select_topk(O.score_tokens(K, q, wl.sm_scale), kk).tolist())
    assert set(wl.planted.tolist()) <= S
    K_local = np.concatenate(k, axis=0)
    s_loc = O.score_tokens(K_local, q, wl.sm_scale)
    S_loc = set(O.select_topk(s_loc, len(wl.planted)).tolist())
    s_glob = O.score_tokens(K, q, wl.sm_scale)
    S_top = set(O.select_topk(s_glob, len(wl.planted)).tolist())
    later = set(int(j) for j in wl.planted if j >= 256)          # chunks with Delta != 0
    assert len(later & S_top) >= 0.9 * len(later)
    assert len(later & S_loc) <= 0.5 * len(later)


# --------------------------------------------------------------------------
# stage 3
# --------------------------------------------------------------------------
def test_budget_golden():
    with open(os.path.join(GOLDEN, "budget.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 5
    for n, rho, k in rows:
        assert O.budget(int(n), float(rho)) == int(k)


def test_topk_brute_force_and_ties():
    g = rng(20)
    for trial in range(20):
        n = int(g.integers(1, 40))
        s = g.integers(0, 5, size=n).astype(np.float32) * 0.25     # many exact ties
        k = int(g.integers(0, n + 1))
        # brute force: repeatedly take the largest remaining, lowest index first
        remaining = list(range(n))
        chosen = []
        for _ in range(k):
            best = remaining[0]
            for j in remaining:
                if s[j] > s[best]:
                    best = j
            chosen.append(best)
            remaining.remove(best)
        got = O.select_topk(s, k)
        assert got.tolist() == sorted(chosen)
        if 0 < k < n:
            rest = np.setdiff1d(np.arange(n), got)
            assert s[got].min() >= s[rest].max()


def test_topk_edges():
    s = np.array([0.5, 0.1, 0.9], dtype=np.float32)
    assert O.select_topk(s, 0).tolist() == []
    assert O.select_topk(s, 3).tolist() == [0, 1, 2]
    assert O.select_topk(s, 1).tolist() == [2]
    with pytest.raises(ValueError):
        O.select_topk(s, 4)


# --------------------------------------------------------------------------
# stage 4
# --------------------------------------------------------------------------
def test_attention_full_ratio_is_dense_causal():
    g = rng(30)
    T, Hq, Hkv, d = 9, 4, 2, 6
    Q = g.standard_normal((T, Hq, d))
    K = g.standard_normal((T, Hkv, d))
    V = g.standard_normal((T, Hkv, d))
    out, lse = O.recompute_attention(Q, np.arange(T), K, V, 0.41)
    np.testing.assert_allclose(out, brute_causal_attention(Q, K, V, 0.41, 2), rtol=1e-12, atol=1e-14)
    # LSE against scipy
    for t in range(T):
        for h in range(Hq):
            lg = 0.41 * (K[: t + 1, h // 2] @ Q[t, h])
            assert abs(lse[t, h] - logsumexp(lg)) < 1e-12


def test_attention_row_independence_and_special_cases():
    g = rng(31)
    T, Hq, Hkv, d = 12, 2, 2, 4
    Q = g.standard_normal((T, Hq, d))
    K = g.standard_normal((T, Hkv, d))
    V = g.standard_normal((T, Hkv, d))
    dense, _ = O.recompute_attention(Q, np.arange(T), K, V, 0.5)
    rows = np.array([0, 3, 4, 11])
    sub, _ = O.recompute_attention(Q[rows], rows, K, V, 0.5)
    np.testing.assert_allclose(sub, dense[rows], rtol=1e-14)
    # first position attends to itself only
    np.testing.assert_allclose(sub[0], V[0], rtol=1e-15)
    # constant V -> output equals that row whatever the weights
    Vc = np.repeat(V[:1], T, axis=0)
    outc, _ = O.recompute_attention(Q, np.arange(T), K, Vc, 0.5)
    np.testing.assert_allclose(outc, np.broadcast_to(V[0], outc.shape), rtol=1e-13)


def test_attention_gqa_equals_replicated_mha():
    g = rng(32)
    T, Hq, Hkv, d = 6, 6, 2, 4
    Q = g.standard_normal((T, Hq, d))
    K = g.standard_normal((T, Hkv, d))
    V = g.standard_normal((T, Hkv, d))
    a, la = O.recompute_attention(Q, np.arange(T), K, V, 0.5)
    b, lb = O.recompute_attention(Q, np.arange(T), np.repeat(K, 3, axis=1), np.repeat(V, 3, axis=1), 0.5)
    np.testing.assert_allclose(a, b, rtol=1e-14)
    np.testing.assert_allclose(la, lb, rtol=1e-14)


# --------------------------------------------------------------------------
# stage 5 and composite
# --------------------------------------------------------------------------
def test_splice_exact():
    g = rng(40)
    K = g.standard_normal((10, 2, 4))
    V = g.standard_normal((10, 2, 4))
    idx = np.array([1, 4, 9])
    kn = g.standard_normal((3, 2, 4))
    vn = g.standard_normal((3, 2, 4))
    K2, V2 = O.splice_kv(K, V, kn, vn, idx)
    assert np.array_equal(K2[idx], kn) and np.array_equal(V2[idx], vn)
    rest = np.setdiff1d(np.arange(10), idx)
    assert np.array_equal(K2[rest], K[rest]) and np.array_equal(V2[rest], V[rest])
    K3, V3 = O.splice_kv(K2, V2, kn, vn, idx)                     # idempotent
    assert np.array_equal(K3, K2) and np.array_equal(V3, V2)
    assert not np.shares_memory(K2, K)


def test_composite_full_ratio_equals_dense_causal_over_repositioned_cache():
    wl = make_workload(preset("C1", chunk_lens=[5, 3, 4], m_prompt=4, planted_count=2,
                              n_q_heads=4, n_kv_heads=2, head_dim=8))
    sp = wl.spec
    k = [to_f64(c, sp.dtype) for c in wl.k_chunks]
    v = [to_f64(c, sp.dtype) for c in wl.v_chunks]
    q = to_f64(wl.q_prompt, sp.dtype)
    Kg, Vg, _, N = O.reposition_keys(k, v, wl.chunk_len, wl.chunk_order, sp.rope_theta)
    g = rng(50)
    Qall = g.standard_normal((N, sp.n_q_heads, sp.head_dim))

    def rows(idx):
        return Qall[idx], Kg[idx], Vg[idx]

    res = O.recompute_layer(k, v, wl.chunk_len, wl.chunk_order, sp.rope_theta, sp.pairing,
                            q, wl.sm_scale, 1.0, rows)
    assert res["idx"].tolist() == list(range(N))
    want = brute_causal_attention(Qall, Kg, Vg, wl.sm_scale, sp.group)
    np.testing.assert_allclose(res["out"], want, rtol=1e-12, atol=1e-14)


def test_composite_splice_precedes_attention():
    """A selected row must see its own freshly projected K/V (a standard
    forward pass): with V_new = 0 at a single selected row at position 0 the
    output of that row is zero."""
    wl = make_workload(preset("C1", chunk_lens=[6, 6], m_prompt=4, planted_count=1,
                              n_q_heads=2, n_kv_heads=2, head_dim=8))
    sp = wl.spec
    k = [to_f64(c, sp.dtype) for c in wl.k_chunks]
    v = [to_f64(c, sp.dtype) for c in wl.v_chunks]
    q = to_f64(wl.q_prompt, sp.dtype)

    def rows(idx):
        R = len(idx)
        return (np.ones((R, 2, 8)), np.ones((R, 2, 8)), np.zeros((R, 2, 8)))

    res = O.recompute_layer(k, v, wl.chunk_len, wl.chunk_order, sp.rope_theta, sp.pairing,
                            q, wl.sm_scale, 1.0, rows)
    assert np.array_equal(res["out"], np.zeros_like(res["out"]))


def test_recompute_inputs_shapes_and_rope():
    wl = make_workload(preset("C2", chunk_lens=[16, 16], m_prompt=4))
    idx = np.array([0, 5, 31])
    q, kn, vn = make_recompute_inputs(wl, idx)
    assert q.shape == (3, 32, 128) and kn.shape == (3, 8, 128) and vn.dtype == np.uint16


# --------------------------------------------------------------------------
# chunk reordering (Eq. 9)
# --------------------------------------------------------------------------
def test_chunk_counts_bruteforce_and_hand_case():
    # hand case: chunks of 3, 2, 4 rows in order [2, 0, 1] -> chunk 2 rows 0..3, chunk 0 rows 4..6, chunk 1 rows 7..8
    lens, order = [3, 2, 4], [2, 0, 1]
    idx = np.array([0, 3, 4, 8])
    assert O.chunk_selection_counts(idx, lens, order).tolist() == [1, 1, 2]
    g = rng(31)
    for _ in range(20):
        n = int(g.integers(1, 7))
        lens = g.integers(0, 9, size=n).tolist()
        order = g.permutation(n).tolist()
        N = sum(lens)
        k = int(g.integers(0, N + 1))
        idx = np.sort(g.choice(N, size=k, replace=False)) if N else np.array([], dtype=np.int64)
        # independent side: label every row with its chunk, then count labels
        owner = []
        for c in order:
            owner += [c] * lens[c]
        want = [sum(1 for j in idx.tolist() if owner[j] == c) for c in range(n)]
        assert O.chunk_selection_counts(idx, lens, order).tolist() == want
        assert sum(want) == k


def test_reorder_is_stable_ascending_density():
    # densities 2/4, 1/2 (equal), 0/3, 3/3: ascending; the two equal ones keep their current relative order
    lens, counts = [4, 2, 3, 3], [2, 1, 0, 3]
    assert O.reorder_chunks(lens, [0, 1, 2, 3], counts).tolist() == [2, 0, 1, 3]
    assert O.reorder_chunks(lens, [1, 0, 3, 2], counts).tolist() == [2, 1, 0, 3]
    # densest chunk ends next to the prompt (last slot); all-equal densities change nothing
    assert O.reorder_chunks([5, 5, 5], [2, 0, 1], [1, 1, 1]).tolist() == [2, 0, 1]
    # empty chunk counts as density 0
    assert O.reorder_chunks([0, 4, 4], None, [0, 1, 2]).tolist() == [0, 1, 2]
    assert O.reorder_chunks([4, 0, 4], None, [2, 0, 1]).tolist() == [1, 2, 0]
    # against Python's stable sort on exact fractions
    from fractions import Fraction
    g = rng(32)
    for _ in range(50):
        n = int(g.integers(1, 9))
        lens = g.integers(1, 6, size=n).tolist()
        counts = [int(g.integers(0, L + 1)) for L in lens]
        order = g.permutation(n).tolist()
        want = sorted(order, key=lambda c: Fraction(counts[c], lens[c]))
        assert O.reorder_chunks(lens, order, counts).tolist() == want


def test_reorder_pass_is_local_geometry_then_density_sort():
    """The first pass scores the chunks' keys exactly as cached (chunk-local rotary positions: the
    concatenation of the chunk caches, no rotation) against the prompt at its global position,
    takes one global top-k, and sorts the chunks by Eq. (9).  Every step is redone here with
    independent pieces: numpy concatenation, the brute-force scores, a sort on (-score, index),
    row labels and Python's stable sort on exact fractions."""
    from fractions import Fraction
    spec = preset("C1", chunk_lens=[9, 14, 5, 11], m_prompt=3, permute_order=True, n_q_heads=2, n_kv_heads=1,
                  head_dim=8, planted_count=4)
    wl = make_workload(spec)
    kc = [to_f64(c, spec.dtype) for c in wl.k_chunks]
    q = to_f64(wl.q_prompt, spec.dtype)
    ratio = 0.3
    new_order, counts, idx = O.reorder_pass(kc, wl.chunk_len, wl.chunk_order, spec.rope_theta, spec.pairing, q,
                                            wl.sm_scale, ratio)
    order = [int(c) for c in wl.chunk_order]
    K_local = np.concatenate([kc[c] for c in order], axis=0)
    s = brute_scores(K_local, q, wl.sm_scale, 2)
    k = int(math.floor(ratio * K_local.shape[0]))
    want_idx = sorted(sorted(range(len(s)), key=lambda j: (-s[j], j))[:k])
    assert idx.tolist() == want_idx
    owner = []
    for c in order:
        owner += [c] * int(wl.chunk_len[c])
    want_counts = [sum(1 for j in want_idx if owner[j] == c) for c in range(4)]
    assert counts.tolist() == want_counts
    want_order = sorted(order, key=lambda c: Fraction(want_counts[c], int(wl.chunk_len[c])))
    assert new_order.tolist() == want_order


# --------------------------------------------------------------------------
# rotary embedding of recomputed rows
# --------------------------------------------------------------------------
def test_rope_rows_against_complex_multiplication_and_composition():
    g = rng(51)
    for pairing in ("half", "interleaved"):
        x = g.standard_normal((7, 3, 8))
        pos = np.array([0, 1, 5, 17, 1000, 40000, 131071])
        got = O.rope_rows(x, pos, 10000.0, pairing)
        assert np.allclose(got, rope_scratch_complex(x, pos, 10000.0, pairing), rtol=0, atol=1e-9)
        assert np.array_equal(got[0], x[0])                       # position 0: identity
        # rotations add: rotating rows placed at p by a further q equals placing them at p + q
        again = O.rope_rows(got, np.full(7, 23), 10000.0, pairing)
        assert np.allclose(again, O.rope_rows(x, pos + 23, 10000.0, pairing), rtol=0, atol=1e-9)
        # per-pair norms are preserved
        n0 = np.hypot(x[..., :4], x[..., 4:]) if pairing == "half" else np.hypot(x[..., 0::2], x[..., 1::2])
        n1 = np.hypot(got[..., :4], got[..., 4:]) if pairing == "half" else np.hypot(got[..., 0::2], got[..., 1::2])
        assert np.allclose(n0, n1, rtol=1e-12)


# --------------------------------------------------------------------------
# caller-supplied frequency table (Eq. 4 replaced by an explicit table, e.g. a
# frequency-rescaled one for long-context checkpoints)
# --------------------------------------------------------------------------
def _custom_freqs(half):
    """A table that is neither geometric nor monotone, so that a transposed,
    reversed, truncated or ignored table cannot reproduce it."""
    return np.array([0.37 / (1 + j) + (0.011 if j % 3 == 0 else 0.0) + 0.002 * ((7 * j) % 5) for j in range(half)])


@pytest.mark.parametrize("pairing", ["half", "interleaved"])
def test_custom_frequency_table_is_used_pair_by_pair(pairing):
    g = rng(61)
    d, H = 16, 2
    freqs = _custom_freqs(d // 2)
    lens = [3, 4, 2]
    order = [2, 0, 1]
    pos0 = [0, 5, 1]
    chunks = [g.standard_normal((L, H, d)) for L in lens]
    K, _, start, N = O.reposition_keys(chunks, None, lens, order, theta=123.0, pairing=pairing,
                                       cached_pos0=pos0, freqs=freqs)
    assert start.tolist() == [2, 5, 0] and N == 9      # slots: chunk 2 (2 rows), chunk 0 (3), chunk 1 (4)
    for c, L in enumerate(lens):
        adv = int(start[c]) - pos0[c]
        for p in range(L):
            for h in range(H):
                for j in range(d // 2):
                    ia, ib = (j, j + d // 2) if pairing == "half" else (2 * j, 2 * j + 1)
                    z = complex(chunks[c][p, h, ia], chunks[c][p, h, ib]) * cmath.exp(1j * adv * freqs[j])
                    assert abs(K[start[c] + p, h, ia] - z.real) < 1e-12
                    assert abs(K[start[c] + p, h, ib] - z.imag) < 1e-12
    # the table replaces the base entirely: a different base gives the same result,
    # and leaving the table out (same base) gives a different one
    K2, _, _, _ = O.reposition_keys(chunks, None, lens, order, theta=5e5, pairing=pairing, cached_pos0=pos0, freqs=freqs)
    assert np.array_equal(K, K2)
    K3, _, _, _ = O.reposition_keys(chunks, None, lens, order, theta=123.0, pairing=pairing, cached_pos0=pos0)
    assert np.abs(K - K3).max() > 0.1
    # rows at given positions: the same table, pair by pair
    x = g.standard_normal((5, H, d))
    pos = np.array([0, 1, 9, 1000, 131071])
    y = O.rope_rows(x, pos, 123.0, pairing, freqs=freqs)
    for r in range(5):
        for h in range(H):
            for j in range(d // 2):
                ia, ib = (j, j + d // 2) if pairing == "half" else (2 * j, 2 * j + 1)
                z = complex(x[r, h, ia], x[r, h, ib]) * cmath.exp(1j * int(pos[r]) * freqs[j])
                assert abs(y[r, h, ia] - z.real) < 1e-9 and abs(y[r, h, ib] - z.imag) < 1e-9
    # geometric table passed explicitly == the default built from the base
    geo = np.array([123.0 ** (-2.0 * j / d) for j in range(d // 2)])
    assert np.array_equal(O.rope_rows(x, pos, 123.0, pairing, freqs=geo), O.rope_rows(x, pos, 123.0, pairing))
