"""The library's length-based load balancing (paper section 3.1.1) against the oracle: a host-only call,
so it runs without a GPU.  Integer work: every output must match exactly."""
import numpy as np
import pytest
import torch

import paper_2512_07710_amd as moe
from oracle.length_balance import balance_lengths


def _lens(seed, n, kind):
    rng = np.random.default_rng(seed)
    if kind == "lognormal":          # long-tailed generation lengths, clipped to a 32k context
        v = np.clip(rng.lognormal(6.5, 1.0, n), 16, 32768).astype(np.int64)
    elif kind == "ties":             # few distinct values: the tie rules decide almost everything
        v = rng.integers(0, 4, n).astype(np.int64) * 100
    else:                            # wide range incl. zeros and values above 2^31
        v = rng.integers(0, 2**40, n).astype(np.int64)
        v[rng.random(n) < 0.1] = 0
    return v


@pytest.mark.parametrize("kind", ["lognormal", "ties", "wide"])
@pytest.mark.parametrize("n,G", [(0, 3), (1, 1), (5, 8), (64, 8), (1000, 7), (4096, 64), (20000, 256)])
@pytest.mark.parametrize("equal", [False, True])
def test_matches_oracle(kind, n, G, equal):
    v = _lens(n * 31 + G, n, kind)
    got = moe.moe_balance_lengths(torch.from_numpy(v), G, equal)
    want = balance_lengths(v.tolist(), G, equal)
    assert got[0].tolist() == want[0]
    assert got[1].tolist() == want[1]
    assert got[2].tolist() == want[2]
    assert got[3].tolist() == want[3]


def test_rejects_bad_arguments():
    lib = moe.load_library()
    v = torch.tensor([3, -1, 2], dtype=torch.int64)
    with pytest.raises(moe.MoEError):
        moe.moe_balance_lengths(v, 2)
    with pytest.raises(moe.MoEError):
        moe.moe_balance_lengths(torch.tensor([1, 2], dtype=torch.int64), 0)
    with pytest.raises(moe.MoEError):
        moe.moe_balance_lengths(torch.tensor([1, 2], dtype=torch.int32), 2)
    ok = torch.tensor([1, 2], dtype=torch.int64)
    buf = torch.empty(4, dtype=torch.int64)
    assert lib.moe_balance_lengths(ok.data_ptr(), 2, 2, 0, None, buf.data_ptr(), buf.data_ptr(), buf.data_ptr()) == -1
    assert lib.moe_balance_lengths(ok.data_ptr(), -1, 2, 0, buf.data_ptr(), buf.data_ptr(), buf.data_ptr(),
                                   buf.data_ptr()) == -1
    assert lib.moe_balance_lengths(None, 0, 2, 1, None, None, None, buf.data_ptr()) == -1
