"""The entry point that allocates nothing: moe_route_replay_noalloc against moe_route_replay, through the C ABI.

Two calls in a row on the same stream, the second with a smaller batch (the static scratch array still holds the
first call's histograms), then a single-block batch, a batch with bad ids, and the empty batch.  Every output must
equal the context-based call's bit for bit, and the oracle's permutation.
"""
import numpy as np
import pytest
import torch

from oracle import moe_layer as om

pytestmark = pytest.mark.gpu


def _log(T, E, k, seed, zipf=False):
    rng = np.random.default_rng(seed)
    if zipf:
        p = (np.arange(E) + 1.0) ** -1.2
        p /= p.sum()
        ids = np.stack([rng.choice(E, size=k, replace=False, p=p) for _ in range(T)])
    else:
        ids = np.stack([rng.permutation(E)[:k] for _ in range(T)])
    w = rng.dirichlet(np.ones(k), T)
    return ids.astype(np.int32), w.astype(np.float32)


def _outputs(T, k, E, fill):
    dev = "cuda"
    N = max(T * k, 1)
    return dict(topk_idx=torch.full((max(T, 1), k), fill, dtype=torch.int32, device=dev),
                topk_w=torch.full((max(T, 1), k), float(fill), dtype=torch.float32, device=dev),
                offsets=torch.full((E + 1,), fill, dtype=torch.int32, device=dev),
                perm=torch.full((N,), fill, dtype=torch.int32, device=dev),
                inv_perm=torch.full((N,), fill, dtype=torch.int32, device=dev))


def _compare(gpu_lib, T, E, k, ids, w, expect_flags=(0, 0)):
    ids_d, w_d = torch.from_numpy(ids).cuda(), torch.from_numpy(w).cuda()
    ref = _outputs(T, k, E, -7)
    ctx = gpu_lib.moe_create(T, 128, E, k, 128)
    try:
        gpu_lib.moe_route_replay(ctx, None, ids_d, w_d, ref["topk_idx"], ref["topk_w"], ref["offsets"], ref["perm"],
                                 ref["inv_perm"])
        torch.cuda.synchronize()
        ref_status = gpu_lib.moe_check_ids(ctx)
    finally:
        gpu_lib.moe_destroy(ctx)
    got = _outputs(T, k, E, -9)
    flags = torch.full((2,), 5, dtype=torch.int32, device="cuda")
    gpu_lib.moe_route_replay_noalloc(None, T, E, k, ids_d, w_d, got["topk_idx"], got["topk_w"], got["offsets"],
                                     got["perm"], got["inv_perm"], flags)
    torch.cuda.synchronize()
    n_valid = int(ref["offsets"][E].item())
    for name in ("topk_idx", "offsets"):
        assert torch.equal(got[name], ref[name]), name
    assert torch.equal(got["topk_w"].view(torch.int32), ref["topk_w"].view(torch.int32))
    assert torch.equal(got["inv_perm"], ref["inv_perm"])
    assert torch.equal(got["perm"][:n_valid], ref["perm"][:n_valid])
    assert tuple(flags.tolist()) == expect_flags
    assert ref_status == (0 if expect_flags == (0, 0) else -3)
    if expect_flags == (0, 0):
        offsets, perm, inv_perm = om.permute(ids, E)
        assert np.array_equal(got["offsets"].cpu().numpy(), offsets)
        assert np.array_equal(got["perm"].cpu().numpy(), perm)
        assert np.array_equal(got["inv_perm"].cpu().numpy(), inv_perm)


def test_noalloc_replay_matches_the_context_call_twice_in_a_row(gpu_lib):
    # 32768 assignments in 16 chunks over 128 experts, Zipf-skewed as in the imbalanced replay workload
    ids, w = _log(4096, 128, 8, seed=3, zipf=True)
    _compare(gpu_lib, 4096, 128, 8, ids, w)
    # a smaller batch right behind it: 5 chunks, other E and k; the scratch array still holds the first call's counts
    ids, w = _log(1500, 40, 6, seed=4)
    _compare(gpu_lib, 1500, 40, 6, ids, w)
    # one chunk: the single-block kernel
    ids, w = _log(300, 200, 5, seed=5)
    _compare(gpu_lib, 300, 200, 5, ids, w)
    # the largest batch the array holds: 2^20 assignments
    ids, w = _log(65536, 256, 16, seed=6)
    _compare(gpu_lib, 65536, 256, 16, ids, w)


def test_noalloc_replay_flags_and_limits(gpu_lib):
    ids, w = _log(3000, 16, 4, seed=7)
    bad = ids.copy()
    bad[17, 2] = 16                       # outside [0,E)
    _compare(gpu_lib, 3000, 16, 4, bad, w, expect_flags=(1, 0))
    dup = ids.copy()
    dup[2999, 3] = dup[2999, 0]           # repeated inside a token
    _compare(gpu_lib, 3000, 16, 4, dup, w, expect_flags=(0, 1))
    _compare(gpu_lib, 3000, 16, 4, ids, w)        # and the flags are clear again on the next call
    # without a flag pointer the call still works
    got = _outputs(3000, 4, 16, -1)
    gpu_lib.moe_route_replay_noalloc(None, 3000, 16, 4, torch.from_numpy(ids).cuda(), torch.from_numpy(w).cuda(),
                                     got["topk_idx"], got["topk_w"], got["offsets"], got["perm"], got["inv_perm"], None)
    torch.cuda.synchronize()
    assert np.array_equal(got["perm"].cpu().numpy(), om.permute(ids, 16)[1])
    # beyond the scratch array: refused, nothing written
    e = torch.empty(1, dtype=torch.int32, device="cuda")
    f = torch.empty(1, dtype=torch.float32, device="cuda")
    with pytest.raises(gpu_lib.MoEError):
        gpu_lib.moe_route_replay_noalloc(None, 65537, 256, 16, e, f, e, f, got["offsets"], e, e, None)
    # the empty batch writes offsets only
    off = torch.full((17,), 3, dtype=torch.int32, device="cuda")
    gpu_lib.moe_route_replay_noalloc(None, 0, 16, 4, None, None, None, None, off, None, None, None)
    torch.cuda.synchronize()
    assert torch.all(off == 0)
