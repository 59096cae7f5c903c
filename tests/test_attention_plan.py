"""CPU checks of the stage-4 work plan (csrc/attention_plan.h) through its host entry point: the walk
every workgroup makes over the (row block, kv tile) line, the slots its partial results go to and the
list of pieces the merge of a row block reads.  The checks are written against what the plan must
achieve (exact cover, unique slots, merge sees what was written, even shares), not against its
formulas."""
import ctypes as C

import numpy as np
import pytest

import paper_2603_05353_amd.binding as B


@pytest.fixture(scope="module")
def lib():
    return B.load_library()


def run_plan(lib, tiles, W, tail_div, R, cap):
    tiles = np.ascontiguousarray(tiles, dtype=np.int32)
    total = int(tiles.sum())
    max_seg = 2 * total + 16
    seg = np.zeros((max_seg, 6), dtype=np.int32)
    pcs = np.zeros((max_seg, 2), dtype=np.int32)
    n_pc = C.c_int64(-1)
    r_out = C.c_int32(-1)
    i32p = C.POINTER(C.c_int32)
    n = lib.ifkv_attention_plan(tiles.ctypes.data_as(i32p), len(tiles), W, tail_div, R, cap,
                                seg.ctypes.data_as(i32p), max_seg, pcs.ctypes.data_as(i32p), max_seg,
                                C.byref(n_pc), C.byref(r_out))
    if n < 0:
        return n, None, None, None
    assert n <= max_seg and n_pc.value <= max_seg
    return n, seg[:n], pcs[:n_pc.value], r_out.value


def check_plan(tiles, W, tail_div, seg, pcs, cap, R):
    tiles = np.asarray(tiles)
    covered = [np.zeros(n, dtype=np.int32) for n in tiles]
    slots = {}
    unit_tiles = {}
    last_unit = -1
    for k, q, t0, t1, slot, whole in seg.tolist():
        assert k >= last_unit, "segments come in the order of the units"
        last_unit = k
        assert 0 <= q < len(tiles) and 0 <= t0 < t1 <= tiles[q]
        covered[q][t0:t1] += 1
        unit_tiles[k] = unit_tiles.get(k, 0) + t1 - t0
        assert whole == int(t0 == 0 and t1 == tiles[q])
        assert (t0 // R) == ((t1 - 1) // R), "a piece stays inside one kv range"
        if not whole:
            assert 0 <= slot < cap
            assert slot not in slots, "two pieces share a slot"
            slots[slot] = q
    for q, cov in enumerate(covered):
        assert (cov == 1).all(), f"row block {q}: tiles covered {np.unique(cov)} times"
    # the merge of a row block reads exactly the slots its pieces were written to, in ascending order
    # (= the order of the line: a fixed order, whoever merges)
    by_q = {}
    for q, slot in pcs.tolist():
        by_q.setdefault(q, []).append(slot)
    written = {}
    for slot, q in slots.items():
        written.setdefault(q, []).append(slot)
    for q in range(len(tiles)):
        got = by_q.get(q, [])
        assert got == sorted(got)
        want = sorted(written.get(q, []))
        if want:
            assert got == want
        else:
            assert len(got) == 1          # a whole row block: one piece, never merged
    # units: numbered 0 .. n-1 without gaps; full ones of R tiles first, then short ones of
    # R / tail_div tiles over the last stretch (about half a full unit per workgroup)
    total = int(tiles.sum())
    n_units = max(unit_tiles) + 1
    assert sorted(unit_tiles) == list(range(n_units))
    sizes = np.array([unit_tiles[k] for k in range(n_units)])
    short = max(1, R // tail_div)
    n_full = int((sizes == R).sum()) if short != R else None
    if short != R:
        assert (sizes[:n_full] == R).all() and (sizes[n_full:-1] == short).all() and 0 < sizes[-1] <= short
        tail = total - n_full * R
        assert tail == total or W * R // 2 <= tail < W * R // 2 + R
    else:
        assert (sizes[:-1] == R).all() and 0 < sizes[-1] <= R


def c3_like(n_rb, max_tiles, seed):
    g = np.random.Generator(np.random.Philox(key=[seed, 5]))
    return np.sort(g.integers(1, max_tiles + 1, size=n_rb))[::-1]


# (name, tiles per row block, workgroups per head, tail_div, shortest range)
CASES = [
    ("one-block", [7], 4, 1, 2),
    ("one-tile", [1], 64, 8, 64),
    ("equal-blocks", [16] * 10, 8, 1, 4),
    ("c3-like", c3_like(154, 512, 1), 64, 8, 64),
    ("c3-5pct", c3_like(52, 512, 2), 64, 8, 64),
    ("c2-like", c3_like(38, 128, 3), 64, 8, 64),
    ("c5-like", c3_like(171, 320, 4), 128, 8, 64),
    ("c4-like", c3_like(410, 2048, 5), 64, 8, 64),
    ("tiny-ranges", c3_like(40, 50, 6), 7, 1, 1),
    ("ragged-small", c3_like(300, 9, 7), 5, 2, 4),
    ("many-short", [1] * 1024, 64, 8, 64),
    ("one-workgroup", c3_like(20, 100, 8), 1, 8, 16),
    ("staircase", list(range(64, 0, -1)), 16, 4, 8),
]


@pytest.mark.parametrize("name,tiles,W,tail_div,R", CASES, ids=[c[0] for c in CASES])
def test_plan_covers_every_tile_once(lib, name, tiles, W, tail_div, R):
    cap = 8192
    n, seg, pcs, r_out = run_plan(lib, tiles, W, tail_div, R, cap)
    assert n > 0
    check_plan(tiles, W, tail_div, seg, pcs, cap, r_out)


def test_plan_lengthens_its_ranges_to_fit_the_slots(lib):
    tiles = c3_like(154, 512, 1)
    seen = []
    for cap in (4096, 1600, 900, 700):
        n, seg, pcs, r_out = run_plan(lib, tiles, 64, 8, 64, cap)
        assert n > 0
        check_plan(tiles, 64, 8, seg, pcs, cap, r_out)
        seen.append(r_out)
    assert seen[0] == 64 and seen == sorted(seen) and seen[-1] > 64
    # worst case the host sizes for: one part and one full unit per row block plus the short units
    worst = 2 * 154 + (64 // 2 + 1) * 8 + 2
    n, seg, pcs, r_out = run_plan(lib, tiles, 64, 8, 64, worst)
    assert n > 0
    check_plan(tiles, 64, 8, seg, pcs, worst, r_out)
    assert run_plan(lib, tiles, 64, 8, 64, 100)[0] == B.IFKV_ESHAPE


def test_plan_keeps_workgroups_on_neighbouring_tiles(lib):
    """What the range-major line is for: any 64 consecutive units (what the workgroups of a head hold
    at one time) touch a small set of kv tiles, so they are served by one L2."""
    tiles = c3_like(154, 512, 1)
    n, seg, pcs, R = run_plan(lib, tiles, 64, 8, 64, 4096)
    by_unit = {}
    for k, q, t0, t1, slot, whole in seg.tolist():
        by_unit.setdefault(k, set()).update(range(t0, t1))
    n_units = max(by_unit) + 1
    for k0 in range(0, n_units - 64, 16):
        touched = set()
        for k in range(k0, k0 + 64):
            touched |= by_unit[k]
        assert len(touched) <= 2 * R      # at most two ranges in flight


def test_plan_rejects_bad_arguments(lib):
    i32p = C.POINTER(C.c_int32)
    t = np.array([3, 5], dtype=np.int32)    # increasing: not "longest first"
    assert lib.ifkv_attention_plan(t.ctypes.data_as(i32p), 2, 4, 1, 2, 64, None, 0, None, 0, None, None) == B.IFKV_EINVAL
    t = np.array([5, 3], dtype=np.int32)
    assert lib.ifkv_attention_plan(t.ctypes.data_as(i32p), 2, 4, 1, 3, 64, None, 0, None, 0, None, None) == B.IFKV_EINVAL
    assert lib.ifkv_attention_plan(t.ctypes.data_as(i32p), 2, 4, 4, 2, 64, None, 0, None, 0, None, None) == B.IFKV_EINVAL
    assert lib.ifkv_attention_plan(t.ctypes.data_as(i32p), 0, 4, 1, 2, 64, None, 0, None, 0, None, None) == B.IFKV_EINVAL
    assert lib.ifkv_attention_plan(None, 2, 4, 1, 2, 64, None, 0, None, 0, None, None) == B.IFKV_EINVAL
    # counting only
    assert lib.ifkv_attention_plan(t.ctypes.data_as(i32p), 2, 4, 1, 2, 64, None, 0, None, 0, None, None) > 0
