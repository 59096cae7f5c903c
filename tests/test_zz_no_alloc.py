"""The entry point that allocates nothing (ifkv_select_topk_noalloc) against ifkv_select_topk, through
the C ABI: two calls in a row, the second with a smaller input, both large enough to use the static
device scratch (more than 32768 scores), plus one that needs no scratch at all; bit-exact, and
equal to the oracle's selection on the same fp32 scores."""
import numpy as np
import pytest
import torch

from oracle import infoflow_oracle as O
from tests.helpers import DEV, make_layer
from workloads import preset

pytestmark = pytest.mark.gpu


def scores(n, seed):
    g = np.random.Generator(np.random.Philox(key=[seed, 77]))
    s = g.random(n).astype(np.float32)
    s[g.choice(n, n // 50, replace=False)] = s[0]          # ties
    return s


def test_select_topk_noalloc_matches_select_topk():
    spec = preset("C4")
    L = make_layer(spec, max_ctx=200000, max_prompt=8)
    # the new entry point first, on a context that has never allocated its scratch
    for n, ratio in [(140001, 0.1), (50000, 0.3), (1000, 0.15), (140001, 0.02)]:
        s_h = scores(n, n)
        s_d = torch.from_numpy(s_h).to(DEV)
        idx = torch.full((n,), -7, dtype=torch.int32, device=DEV)
        got = L.select_topk_noalloc(s_d, idx, ratio=ratio)
        torch.cuda.synchronize()
        want = L.select_topk(s_d, ratio=ratio)
        torch.cuda.synchronize()
        k = O.budget(n, ratio)
        assert got.shape[0] == want.shape[0] == k
        assert torch.equal(got, want)
        assert np.array_equal(got.cpu().numpy().astype(np.int64), O.select_topk(s_h, k))
        assert (idx[k:] == -7).all()
    # beyond the static array: refused with a clear error, nothing launched
    from paper_2603_05353_amd import IfkvError
    Lb = make_layer(spec, max_ctx=(1 << 22) + 4096, max_prompt=8)
    big = torch.zeros((1 << 22) + 1, dtype=torch.float32, device=DEV)
    with pytest.raises(IfkvError) as e:
        Lb.select_topk_noalloc(big, torch.empty(16, dtype=torch.int32, device=DEV), k=16)
    assert "exceeds" in str(e.value)
    Lb.close()
    L.close()
