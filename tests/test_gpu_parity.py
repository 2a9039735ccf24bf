"""GPU parity: every stage of the HIP path against the CPU oracle, through the C ABI.

Bars: ids / permutation / offsets / e4m3 codes / scales bit-exact; routed ids
bit-exact wherever the oracle's k-th vs (k+1)-th score gap exceeds 1e-4 (closer
calls are counted and reported); gate weights |dw| <= 1e-6 + 1e-5*w; layer output
relative L2 (whole tensor) <= 2e-3 on identical quantised inputs.
"""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import fp_formats as ff
from oracle import moe_layer as om
from workloads import CONFIGS, MoEConfig, make_inputs

pytestmark = pytest.mark.gpu

REL_L2_BAR = 2e-3
GAP_BAR = 1e-4


def _bits(x):
    return x.cpu().view(torch.int16).numpy().view(np.uint16)


def _host(inp):
    out = {}
    for k, v in inp.items():
        if isinstance(v, torch.Tensor):
            out[k] = _bits(v) if v.dtype == torch.bfloat16 else v.cpu().numpy()
        else:
            out[k] = v
    return out


def _dev(inp, dev="cuda:0"):
    return {k: (v.to(dev) if isinstance(v, torch.Tensor) else v) for k, v in inp.items()}


def _rel_l2(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b.astype(np.float64)) / max(np.linalg.norm(b.astype(np.float64)), 1e-300))


def _compare_routing(h, layer, bias=None):
    """Routed-mode ids/weights vs the oracle; returns the oracle result and the set of tokens to exclude."""
    cfg = h["cfg"]
    idx_o, w_o, logits = om.route(h["x"], h["W_r"], cfg.k, bias)
    idx_g = layer.topk_idx.cpu().numpy()
    w_g = layer.topk_w.cpu().numpy()
    score = logits if bias is None else logits + bias.astype(np.float64)[None, :]
    srt = -np.sort(-score, axis=1)
    gap_k = srt[:, cfg.k - 1] - srt[:, cfg.k] if cfg.k < cfg.E else np.full(cfg.T, np.inf)
    inner_gap = (srt[:, :cfg.k - 1] - srt[:, 1:cfg.k]).min(axis=1) if cfg.k > 1 else np.full(cfg.T, np.inf)
    same_seq = np.all(idx_o == idx_g, axis=1)
    same_set = np.array([set(a) == set(b) for a, b in zip(idx_o.tolist(), idx_g.tolist())])
    # clear-cut tokens must match exactly
    clear = (gap_k > GAP_BAR) & (inner_gap > GAP_BAR)
    assert np.all(same_seq[clear]), f"{(~same_seq[clear]).sum()} clear-cut tokens routed differently"
    assert np.all(same_set[gap_k > GAP_BAR]), "expert set differs where the k/k+1 gap is large"
    near_set = int((~same_set).sum())
    near_order = int((same_set & ~same_seq).sum())
    print(f"[routing] near-tie set mismatches: {near_set}, order-only mismatches: {near_order} of {cfg.T} tokens")
    ok = same_seq
    assert np.all(np.abs(w_g[ok] - w_o[ok]) <= 1e-6 + 1e-5 * w_o[ok])
    assert np.allclose(w_g.sum(1), 1.0, atol=1e-5)
    return idx_o, w_o, ~same_seq


def _check_permutation(idx, E, layer):
    offsets, perm, inv_perm = om.permute(idx, E)
    assert np.array_equal(layer.offsets.cpu().numpy(), offsets)
    assert np.array_equal(layer.perm.cpu().numpy(), perm)
    assert np.array_equal(layer.inv_perm.cpu().numpy(), inv_perm)
    return offsets, perm, inv_perm


def _run_and_check_layer(gpu_lib, cfg: MoEConfig, mode: str, seed=None, log=None):
    """Full layer at `cfg` (must be small enough for the whole oracle).  log = (ids, weights) replaces the
    replay log that would otherwise be the oracle's own routing."""
    inp = make_inputs(cfg, seed=seed)
    h, dv = _host(inp), _dev(inp)
    layer = gpu_lib.MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F)
    bias_h = h.get("sel_bias")
    try:
        if mode == "routed":
            layer.route(dv["x"], dv["W_r"], dv.get("sel_bias"))
            torch.cuda.synchronize()
            _compare_routing(h, layer, bias_h)
        else:
            if log is not None:
                log_idx, log_w = log
            elif cfg.log == "zipf":
                log_idx, log_w = h["logged_idx"], h["logged_w"]
            else:
                log_idx, log_w, _ = om.route(h["x"], h["W_r"], cfg.k, bias_h)
            layer.route_replay(dv["x"], torch.from_numpy(log_idx).cuda(), torch.from_numpy(log_w).cuda())
            torch.cuda.synchronize()
            assert np.array_equal(layer.topk_idx.cpu().numpy(), log_idx)
            assert np.array_equal(layer.topk_w.cpu().numpy(), log_w)
        assert gpu_lib.moe_check_ids(layer.ctx) == 0
        # from here on the oracle follows the GPU's routing decision, so near-tie tokens stay comparable
        idx = layer.topk_idx.cpu().numpy()
        w = layer.topk_w.cpu().numpy()
        offsets, perm, inv_perm = _check_permutation(idx, cfg.E, layer)

        layer.quantize(dv["x"])
        xq_o, xs_o = om.gather_quantize(h["x"], perm, cfg.k)
        assert np.array_equal(layer.xq.cpu().numpy()[:cfg.N], xq_o)
        assert np.array_equal(layer.xs.cpu().numpy().T[:cfg.N], xs_o)      # device layout is [d/128, N]

        layer.expert_ffn(dv)
        y_o, hq_o, hs_o = om.expert_ffn(xq_o, xs_o, offsets, h["W1q"], h["W3q"], h["W2q"], h["s1"], h["s3"], h["s2"])
        hq_g, hs_g = layer.hidden()
        hq_g, hs_g = hq_g.cpu().numpy()[:cfg.N], np.ascontiguousarray(hs_g.cpu().numpy().T[:cfg.N])
        code_mismatch = float((hq_g != hq_o).mean())
        scale_rel = float(np.abs(hs_g - hs_o).max() / np.abs(hs_o).max())
        print(f"[{cfg.name}/{mode}] hq code mismatch fraction {code_mismatch:.2e}, hs max rel diff {scale_rel:.2e}")
        # The FP8 matrix cores align the products of a dot product to the largest one and drop
        # low-order bits, so g and u carry an absolute error of ~1e-5 of their terms' magnitude.
        # Elements of h formed by cancellation can therefore land a few codes away; what is
        # gated is how rare that is and how little of the tensor's energy it moves.
        dec_g = ff.e4m3_decode(hq_g) * np.repeat(hs_g.astype(np.float64), 128, axis=1)
        dec_o = ff.e4m3_decode(hq_o) * np.repeat(hs_o.astype(np.float64), 128, axis=1)
        h_rel = _rel_l2(dec_g, dec_o)
        step = np.maximum(np.abs(ff.e4m3_decode(hq_o)) / 8.0, 2.0 ** -9) * np.repeat(hs_o.astype(np.float64), 128, axis=1)
        far = float((np.abs(dec_g - dec_o) > 1.001 * step + 1e-4 * np.abs(dec_o)).mean())
        y_perm_g = layer.y_perm.cpu().numpy()[:cfg.N]
        y_iso = np.zeros_like(y_o)
        for e in range(cfg.E):
            a, b = offsets[e], offsets[e + 1]
            if b > a:
                y_iso[a:b] = om.block_scaled_matmul(hq_g[a:b], hs_g[a:b], h["W2q"][e], h["s2"][e])
        iso_rel = _rel_l2(y_perm_g, y_iso)
        yp_rel = _rel_l2(y_perm_g, y_o)
        print(f"[{cfg.name}/{mode}] dequantised h rel-L2 {h_rel:.3e}, codes beyond one step {far:.2e}, "
              f"y_perm rel-L2 {yp_rel:.3e}, GEMM2 alone (oracle on the GPU's hq/hs) {iso_rel:.3e}")
        assert code_mismatch < 5e-3
        assert far < 2e-4
        assert np.allclose(hs_g, hs_o, rtol=2e-4)
        assert yp_rel <= REL_L2_BAR
        # stage-isolated: the oracle's second GEMM on the GPU's own hq/hs must agree tightly
        assert iso_rel <= 1e-4

        y_f32 = torch.full((cfg.T, cfg.d), float("nan"), dtype=torch.float32, device="cuda")
        layer.combine(y_f32)
        y_g = layer.y.float().cpu().numpy()
        y64, y_bits = om.combine(y_o, inv_perm, w)
        y_ref = ff.bf16_bits_to_f64(y_bits)
        rel = _rel_l2(y_g, y_ref)
        per_tok = np.linalg.norm(y_g - y_ref, axis=1) / np.maximum(np.linalg.norm(y_ref, axis=1), 1e-300)
        # the sums before the output rounding: the bf16 output is exactly their rounding, and against the oracle's
        # unrounded output they show the layer's error without the whole-step differences of two rounded values
        y32 = y_f32.cpu().numpy()
        assert np.array_equal(ff.f64_to_bf16_bits(y32.astype(np.float64)), _bits(layer.y))
        pre = _rel_l2(y32, y64)
        print(f"[{cfg.name}/{mode}] layer rel-L2 {rel:.3e} (bar {REL_L2_BAR}), per-token max {per_tok.max():.3e}; "
              f"before the output rounding {pre:.3e}")
        assert rel <= REL_L2_BAR
        assert pre <= REL_L2_BAR
        # combine alone, on the GPU's own y_perm, is exact up to fp32 summation
        _, bits_iso = om.combine(y_perm_g.astype(np.float64), inv_perm, w)
        iso = ff.bf16_bits_to_f64(bits_iso)
        flips = float((y_g != iso).mean())                # fp32-vs-fp64 sums landing on another bf16 value
        assert flips < 1e-3 and _rel_l2(y_g, iso) <= 1e-6 + 0.01 * np.sqrt(flips)
        return layer.y.clone(), layer.perm.clone()
    finally:
        layer.close()


def test_config0_routed(gpu_lib):
    _run_and_check_layer(gpu_lib, CONFIGS[0], "routed")


def _replay_of_own_routing_is_bitwise_identical(gpu_lib, cfg):
    """Replay fed with the GPU's own routed ids and weights must reproduce every output bit, on both FFN paths."""
    inp = _dev(make_inputs(cfg))
    layer = gpu_lib.MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F)
    try:
        for fused in (False, True):
            acts = ("xq_tok", "xs_tok") if fused else ("xq", "xs")
            layer.forward_routed(inp["x"], inp["W_r"], inp.get("sel_bias"), inp, fused=fused)
            torch.cuda.synchronize()
            keep = {n: getattr(layer, n).clone() for n in ("topk_idx", "topk_w", "offsets", "perm", "inv_perm", "y_perm", "y") + acts}
            for n in ("offsets", "perm", "inv_perm", "y_perm", "y") + acts:
                getattr(layer, n).zero_()
            layer.forward_replay(inp["x"], keep["topk_idx"], keep["topk_w"], inp, fused=fused)
            torch.cuda.synchronize()
            for n, v in keep.items():
                assert torch.equal(getattr(layer, n).view(torch.uint8), v.view(torch.uint8)), (n, fused)
    finally:
        layer.close()


def test_config0_replay_equals_routed_bitwise(gpu_lib):
    _run_and_check_layer(gpu_lib, CONFIGS[0], "replay")
    _replay_of_own_routing_is_bitwise_identical(gpu_lib, CONFIGS[0])


@pytest.mark.parametrize("seed", [11, 12])
def test_small_ragged_shapes(gpu_lib, seed):
    """Several tiles and a ragged tail per expert; an expert-starved layout (k small, E large)."""
    cfg = MoEConfig("ragged", T=333, d=384, E=5, k=3, F=640, modes=("routed",), seed=seed)
    _run_and_check_layer(gpu_lib, cfg, "routed")
    cfg = MoEConfig("sparse", T=37, d=256, E=200, k=2, F=128, modes=("routed",), seed=seed)
    _run_and_check_layer(gpu_lib, cfg, "routed")


def test_single_k_block_in_both_gemms(gpu_lib):
    """d = F = 128: each GEMM's K loop has exactly one block (prologue and drain only), output tiles half empty."""
    _run_and_check_layer(gpu_lib, MoEConfig("tiny", T=400, d=128, E=4, k=2, F=128, modes=("routed",), seed=21), "routed")
    _run_and_check_layer(gpu_lib, MoEConfig("tiny3", T=300, d=384, E=3, k=1, F=384, modes=("routed",), seed=22), "routed")


def test_k_equals_e_and_single_expert(gpu_lib):
    _run_and_check_layer(gpu_lib, MoEConfig("dense", T=130, d=256, E=4, k=4, F=256, modes=("routed",), seed=5), "routed")
    _run_and_check_layer(gpu_lib, MoEConfig("one", T=200, d=128, E=1, k=1, F=384, modes=("routed",), seed=6), "routed")


def test_config1_routed_and_replay(gpu_lib):
    _run_and_check_layer(gpu_lib, CONFIGS[1], "routed")
    _run_and_check_layer(gpu_lib, CONFIGS[1], "replay")
    _replay_of_own_routing_is_bitwise_identical(gpu_lib, CONFIGS[1])


def test_exact_tie_lowest_index(gpu_lib):
    cfg = MoEConfig("tie", T=64, d=128, E=8, k=3, F=128, modes=("routed",), seed=3)
    inp = make_inputs(cfg, with_experts=False)
    W = inp["W_r"].clone()
    W[6] = W[2]
    W[7] = W[2]
    layer = gpu_lib.MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F)
    try:
        layer.route(inp["x"].cuda(), W.cuda(), None)
        torch.cuda.synchronize()
        idx_o, w_o, _ = om.route(_bits(inp["x"]), W.numpy(), cfg.k)
        assert np.array_equal(layer.topk_idx.cpu().numpy(), idx_o)
    finally:
        layer.close()


def test_quantize_plain_and_edge_values(gpu_lib):
    """Plain (no fan-out) quantisation incl. zero groups, powers of two, tiny and huge magnitudes."""
    g = torch.Generator().manual_seed(0)
    x = torch.randn((257, 512), generator=g) * torch.exp2(torch.randint(-12, 12, (257, 1), generator=g).float())
    x[3, 128:256] = 0
    x[4, :] = 0
    x[5, :128] = torch.exp2(torch.randint(-3, 4, (128,), generator=g).float())
    x[6, 7] = 3.0e38
    x[7, :] = -x[8, :]
    xb = x.to(torch.bfloat16)
    layer = gpu_lib.MoELayer(1, 128, 1, 1, 128)
    try:
        q = torch.empty((257, 512), dtype=torch.uint8, device="cuda")
        s = torch.empty((4, 257), dtype=torch.float32, device="cuda")          # group-major scale planes
        gpu_lib.moe_quantize_fp8(layer.ctx, xb.cuda(), 257, 512, 128, None, 1, q, s)
        torch.cuda.synchronize()
        q_o, s_o = om.quantize_rows(ff.bf16_bits_to_f64(_bits(xb)))
        assert np.array_equal(s.cpu().numpy().T, s_o)
        assert np.array_equal(q.cpu().numpy(), q_o)
        # rows_in = 0 is legal and touches nothing
        gpu_lib.moe_quantize_fp8(layer.ctx, xb.cuda(), 0, 512, 128, None, 1, q, s)
        with pytest.raises(gpu_lib.MoEError):
            gpu_lib.moe_quantize_fp8(layer.ctx, xb.cuda(), 257, 512, 64, None, 1, q, s)
    finally:
        layer.close()


def test_replay_rejects_nothing_but_flags_bad_ids(gpu_lib):
    """Ids outside [0,E) and ids repeated inside a token never fault: the call goes through, a device flag is
    raised that moe_check_ids reports once, and the permutation is the stable sort of what was given."""
    cfg = MoEConfig("bad", T=16, d=128, E=4, k=2, F=128, modes=("replay",))
    layer = gpu_lib.MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F)
    try:
        rng = np.random.default_rng(16)
        good = np.stack([rng.permutation(4)[:2] for _ in range(16)]).astype(np.int32)     # distinct inside a token
        w = torch.full((16, 2), 0.5)
        idx = torch.from_numpy(good.copy())
        idx[5, 1] = 9
        idx[6, 0] = -2
        layer.route_replay(None, idx.cuda(), w.cuda())
        assert gpu_lib.moe_check_ids(layer.ctx) == -3
        assert gpu_lib.moe_check_ids(layer.ctx) == 0                   # reported once, then cleared
        layer.route_replay(None, torch.from_numpy(good).cuda(), w.cuda())
        assert gpu_lib.moe_check_ids(layer.ctx) == 0
        _check_permutation(good, 4, layer)
        # a token that names the same expert twice: flagged, and still sorted like any other assignment
        dup = good.copy()
        dup[11, 1] = dup[11, 0]
        layer.route_replay(None, torch.from_numpy(dup).cuda(), w.cuda())
        assert gpu_lib.moe_check_ids(layer.ctx) == -3
        _check_permutation(dup, 4, layer)
        assert gpu_lib.moe_check_ids(layer.ctx) == 0
    finally:
        layer.close()


@pytest.mark.parametrize("T,E,k", [(5000, 64, 6), (300, 200, 16)])
def test_replay_duplicate_check_at_several_chunks(gpu_lib, T, E, k):
    """The duplicate check in the three-kernel permutation (more than 2048 assignments) and in the single-block
    one: a clean log passes, one repeated id anywhere in it is found."""
    rng = np.random.default_rng(T)
    good = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    w = torch.full((T, k), 1.0 / k)
    layer = gpu_lib.MoELayer(T, 128, E, k, 128)
    try:
        layer.route_replay(None, torch.from_numpy(good).cuda(), w.cuda())
        assert gpu_lib.moe_check_ids(layer.ctx) == 0
        for t, a, b in ((0, 0, k - 1), (T - 1, k - 2, k - 1), (T // 2, 1, 3)):
            dup = good.copy()
            dup[t, b] = dup[t, a]
            layer.route_replay(None, torch.from_numpy(dup).cuda(), w.cuda())
            assert gpu_lib.moe_check_ids(layer.ctx) == -3, (t, a, b)
            _check_permutation(dup, E, layer)
    finally:
        layer.close()


def test_zeroed_expert_contributes_exactly_zero(gpu_lib):
    """Unit weight scales and small-integer codes, one expert's down projection all zero.  That expert's rows
    of y_perm must be exactly 0.  g and u are exact integers on both sides here, so many h/s land on e4m3
    ties and the few ulps between the fp32 and the fp64 silu decide them: the hidden codes are compared by
    mismatch rate (each mismatch one code step), and the down projection is compared on the GPU's own
    codes.  (Exactness of the fp32 accumulation itself is pinned through moe_linear_fp8 in
    test_linear_small_integer_codes_are_exact.)"""
    cfg = MoEConfig("ints", T=96, d=256, E=3, k=2, F=128, modes=("replay",), seed=9)
    rng = np.random.default_rng(9)
    pool = ff.e4m3_encode(np.array([0, 1, 2, -1, -2, 0.5, -0.5, 0], dtype=np.float64))
    W1q = pool[rng.integers(0, 8, (3, 128, 256))]
    W3q = pool[rng.integers(0, 8, (3, 128, 256))]
    W2q = pool[rng.integers(0, 8, (3, 256, 128))]
    W2q[1] = 0
    ones = lambda *s: np.ones(s, np.float32)
    s1, s3, s2 = ones(3, 1, 2), ones(3, 1, 2), ones(3, 2, 1)
    idx = np.stack([rng.permutation(3)[:2] for _ in range(96)]).astype(np.int32)
    w = np.full((96, 2), 0.5, np.float32)
    offsets, perm, inv_perm = om.permute(idx, 3)
    xq = pool[rng.integers(0, 8, (192, 256))]
    xs = ones(192, 2)
    layer = gpu_lib.MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F)
    try:
        t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
        layer.route_replay(None, t(idx), t(w))
        layer.xq.copy_(t(xq))
        layer.xs.copy_(t(xs.T))
        layer.expert_ffn(dict(W1q=t(W1q), W3q=t(W3q), W2q=t(W2q), s1=t(s1), s3=t(s3), s2=t(s2)))
        torch.cuda.synchronize()
        y_o, hq_o, hs_o = om.expert_ffn(xq, xs, offsets, W1q, W3q, W2q, s1, s3, s2)
        y_g = layer.y_perm.cpu().numpy()
        a, b = offsets[1], offsets[2]
        assert b > a and np.all(y_g[a:b] == 0.0)
        hq_g, hs_g = layer.hidden()
        hq_g, hs_g = hq_g.cpu().numpy(), np.ascontiguousarray(hs_g.cpu().numpy().T)
        assert np.allclose(hs_g, hs_o, rtol=2e-4)
        diff = hq_g != hq_o
        # a mismatch is one code step (adjacent magnitudes, same sign); +0/-0 are codes 0x00/0x80
        step = np.abs((hq_g & 0x7F).astype(np.int32) - (hq_o & 0x7F).astype(np.int32))
        print(f"[ints] hidden code mismatches {diff.mean():.2e}, largest step {step.max()}")
        assert diff.mean() < 2e-2 and step.max() <= 1
        for e in range(3):
            a, b = int(offsets[e]), int(offsets[e + 1])
            iso = om.block_scaled_matmul(hq_g[a:b], hs_g[a:b], W2q[e], s2[e])
            assert _rel_l2(y_g[a:b], iso) <= 1e-4
    finally:
        layer.close()


def test_run_twice_bit_identical(gpu_lib):
    cfg = CONFIGS[0]
    inp = _dev(make_inputs(cfg))
    layer = gpu_lib.MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F)
    try:
        outs = []
        for _ in range(2):
            layer.forward_routed(inp["x"], inp["W_r"], None, inp)
            torch.cuda.synchronize()
            outs.append((layer.y.clone(), layer.perm.clone(), layer.topk_idx.clone(), layer.y_perm.clone()))
        for a, b in zip(*outs):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
    finally:
        layer.close()
