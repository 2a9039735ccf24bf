"""Pins of the MoE-layer oracle against brute force, closed forms, invariants and
special cases that reduce to library routines (CPU only).

The paper prints no worked example of the layer (its numbers are whole-pipeline),
so every pin here is definitional: see each test's docstring.
"""
import itertools
import math

import numpy as np
import pytest
import torch
from scipy.special import softmax as scipy_softmax

from oracle import fp_formats as ff
from oracle import moe_layer as om
from workloads import CONFIGS, make_inputs


def _np(t):
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


@pytest.fixture(scope="module")
def cfg0():
    inp = make_inputs(CONFIGS[0])
    return {k: (_np(v) if isinstance(v, torch.Tensor) else v) for k, v in inp.items()}


# ----------------------------------------------------------------------------- top-k
def _brute_topk(row, k):
    """Selection by repeated arg-max scan, earliest index wins an exact tie."""
    taken, out = set(), []
    for _ in range(k):
        best = None
        for e, s in enumerate(row):
            if e in taken:
                continue
            if best is None or s > row[best]:
                best = e
        taken.add(best)
        out.append(best)
    return out


def test_topk_exhaustive_orderings_with_ties():
    """Every ordering of a 6-value multiset with repeated values, all k."""
    vals = [0.5, 0.5, -1.0, 2.0, 2.0, 0.0]
    for p in set(itertools.permutations(vals)):
        row = np.array([p], dtype=np.float64)
        for k in range(1, 7):
            assert om.topk_select(row, k)[0].tolist() == _brute_topk(list(p), k)


def test_topk_random_vs_brute_force():
    rng = np.random.default_rng(0)
    score = np.round(rng.standard_normal((200, 17)), 1)      # rounding plants many ties
    for k in (1, 3, 8, 17):
        got = om.topk_select(score, k)
        for t in range(score.shape[0]):
            assert got[t].tolist() == _brute_topk(score[t].tolist(), k)


def test_selection_bias_changes_ids_not_weights():
    """Bias enters the selection score only; weights come from the unbiased logits."""
    rng = np.random.default_rng(1)
    x = torch.randn(16, 128).to(torch.bfloat16)
    xb = _np(x)
    W = rng.standard_normal((8, 128)).astype(np.float32)
    bias = np.zeros(8, np.float32)
    bias[5] = 100.0
    idx, w, logits = om.route(xb, W, 2, bias)
    assert np.all(idx[:, 0] == 5)
    sel = np.take_along_axis(logits, idx.astype(np.int64), 1)
    assert np.allclose(w, scipy_softmax(sel, axis=1), rtol=1e-6)


# ----------------------------------------------------------------------------- gate weights
def test_gate_weights_closed_forms(cfg0):
    logits = om.router_logits(cfg0["x"], cfg0["W_r"])
    # logits equal an independently computed fp64 product
    ref = torch.from_numpy(cfg0["x"].view(np.int16)).view(torch.bfloat16).double() @ torch.from_numpy(cfg0["W_r"]).double().T
    assert np.allclose(logits, ref.numpy(), rtol=0, atol=1e-12)
    E = logits.shape[1]
    for k in (1, 2, 5, E):
        idx = om.topk_select(logits, k)
        w = om.gate_weights(logits, idx).astype(np.float64)
        assert np.allclose(w.sum(1), 1.0, atol=1e-6)
        # softmax over all experts, then renormalise over the selected ones
        p = scipy_softmax(logits, axis=1)
        psel = np.take_along_axis(p, idx.astype(np.int64), 1)
        assert np.allclose(w, psel / psel.sum(1, keepdims=True), rtol=1e-6, atol=1e-9)
        assert np.all(np.diff(w, axis=1) <= 1e-7)             # descending score => descending weight
    assert np.array_equal(om.gate_weights(logits, om.topk_select(logits, 1)), np.ones((logits.shape[0], 1), np.float32))
    idxE = om.topk_select(logits, E)
    wE = om.gate_weights(logits, idxE)
    assert np.allclose(wE, np.take_along_axis(scipy_softmax(logits, axis=1), idxE.astype(np.int64), 1), rtol=1e-6)


def test_each_token_gets_k_distinct_experts(cfg0):
    idx, _, _ = om.route(cfg0["x"], cfg0["W_r"], 2)
    assert idx.shape == (64, 2) and idx.min() >= 0 and idx.max() < 8
    assert np.all(idx[:, 0] != idx[:, 1])


def test_exact_tie_lowest_index_wins():
    """Two identical router rows give identical logits; the lower index must come first."""
    x = _np(torch.randn(32, 128).to(torch.bfloat16))
    W = np.random.default_rng(2).standard_normal((8, 128)).astype(np.float32)
    W[6] = W[2]
    idx, w, _ = om.route(x, W, 8)
    pos2 = np.argmax(idx == 2, axis=1)
    pos6 = np.argmax(idx == 6, axis=1)
    assert np.all(pos6 == pos2 + 1)


# ----------------------------------------------------------------------------- permutation
def _check_perm_invariants(idx, E, offsets, perm, inv_perm):
    N = idx.size
    flat = idx.reshape(-1)
    assert offsets[0] == 0 and offsets[E] == N and np.all(np.diff(offsets) >= 0)
    assert np.array_equal(np.sort(perm), np.arange(N))
    assert np.array_equal(perm[inv_perm], np.arange(N))
    assert np.array_equal(inv_perm[perm], np.arange(N))
    for e in range(E):
        seg = perm[offsets[e]:offsets[e + 1]]
        assert np.all(flat[seg] == e)
        assert np.all(np.diff(seg) > 0)                       # stability
    assert np.array_equal(np.diff(offsets), np.bincount(flat, minlength=E))


def test_permute_invariants_and_stable_sort():
    rng = np.random.default_rng(5)
    for (T, k, E) in ((64, 2, 8), (100, 6, 64), (7, 3, 5), (1, 1, 1), (33, 4, 300)):
        idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
        offsets, perm, inv_perm = om.permute(idx, E)
        _check_perm_invariants(idx, E, offsets, perm, inv_perm)
        assert np.array_equal(perm, np.argsort(idx.reshape(-1), kind="stable"))


def test_permute_empty_experts_and_skew():
    idx = np.array([[0, 3], [0, 3], [3, 0]], dtype=np.int32)
    offsets, perm, inv_perm = om.permute(idx, 6)
    assert offsets.tolist() == [0, 3, 3, 3, 6, 6, 6]
    assert perm.tolist() == [0, 2, 5, 1, 3, 4]
    assert inv_perm.tolist() == [0, 3, 1, 4, 5, 2]


# ----------------------------------------------------------------------------- quantisation
def test_quantize_rows_invariants():
    rng = np.random.default_rng(11)
    v = rng.standard_normal((37, 384)).astype(np.float32)
    v[3, 128:256] = 0.0                                      # an all-zero group
    v[5, :128] = np.exp2(rng.integers(-3, 4, 128)).astype(np.float32)   # powers of two
    v[5, 0] = 8.0
    codes, s = om.quantize_rows(v.astype(np.float64))
    dec = ff.e4m3_decode(codes).reshape(37, 3, 128)
    vg = v.reshape(37, 3, 128).astype(np.float64)
    amax = np.abs(vg).max(2)
    assert s.dtype == np.float32 and codes.dtype == np.uint8
    assert s[3, 1] == 1.0 and np.all(codes[3, 128:256] == 0)
    nz = amax > 0
    assert np.all(np.abs(dec).max(2)[nz] == 448.0)           # the group maximum always lands on 448
    # reconstruction error is at most half an e4m3 step at that magnitude (+ fp32 rounding of x/s)
    r = np.abs(vg / s[:, :, None].astype(np.float64))
    step = np.where(r < 2.0 ** -6, 2.0 ** -9, np.exp2(np.floor(np.log2(np.maximum(r, 1e-300))) - 3))
    err = np.abs(vg - dec * s[:, :, None].astype(np.float64))
    assert np.all(err <= s[:, :, None] * (0.5 * step) * (1 + 1e-6))
    # powers of two scaled by a power-of-two-free factor 8/448: x/s = x*56 exactly representable?
    # 56*2^j = 1.75*2^(j+5): three mantissa bits -> exact
    assert np.allclose(dec[5, 0] * s[5, 0], vg[5, 0], rtol=1e-7)


def test_quantize_rows_matches_float32_arithmetic_and_torch_cast():
    """Same recipe in numpy float32 arithmetic with torch's float8 cast as the encoder."""
    rng = np.random.default_rng(12)
    v = (rng.standard_normal((64, 256)) * np.exp2(rng.integers(-6, 6, (64, 1)))).astype(np.float32)
    codes, s = om.quantize_rows(v.astype(np.float64))
    vg = v.reshape(64, 2, 128)
    amax = np.abs(vg).max(2)
    s32 = amax / np.float32(448.0)
    r32 = vg / s32[:, :, None]
    ref = torch.from_numpy(r32).to(torch.float8_e4m3fn).view(torch.uint8).numpy().reshape(64, 256)
    assert np.array_equal(s, s32)
    assert np.array_equal(codes, ref)


def test_gather_quantize_follows_perm(cfg0):
    idx, _, _ = om.route(cfg0["x"], cfg0["W_r"], 2)
    offsets, perm, inv_perm = om.permute(idx, 8)
    xq, xs = om.gather_quantize(cfg0["x"], perm, 2)
    plain_q, plain_s = om.quantize_rows(ff.bf16_bits_to_f64(cfg0["x"]))
    for p in range(perm.size):
        assert np.array_equal(xq[p], plain_q[perm[p] // 2])
        assert np.array_equal(xs[p], plain_s[perm[p] // 2])


# ----------------------------------------------------------------------------- expert FFN
def _dequant_weight(wq, ws):
    """codes [R,C] + block scales [R/128,C/128] -> fp64 matrix, via torch's float8 decode."""
    w = torch.from_numpy(wq).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    return w * np.kron(ws.astype(np.float64), np.ones((128, 128)))


def _dequant_rows(q, s):
    v = torch.from_numpy(q).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    return v * np.repeat(s.astype(np.float64), 128, axis=1)


def test_block_scaled_matmul_equals_dequantised_matmul(cfg0):
    rng = np.random.default_rng(13)
    aq = rng.integers(0, 256, (19, 256)).astype(np.uint8)
    aq[(aq & 0x7F) == 0x7F] = 0x10
    a_s = rng.uniform(0.01, 2.0, (19, 2)).astype(np.float32)
    wq = rng.integers(0, 256, (384, 256)).astype(np.uint8)
    wq[(wq & 0x7F) == 0x7F] = 0x90
    w_s = rng.uniform(0.001, 0.1, (3, 2)).astype(np.float32)
    got = om.block_scaled_matmul(aq, a_s, wq, w_s)
    ref = _dequant_rows(aq, a_s) @ _dequant_weight(wq, w_s).T
    assert got.shape == (19, 384)
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-9)
    # not symmetric in its operands: a transposed-weight mistake would show
    assert not np.allclose(got[:, :256], om.block_scaled_matmul(aq, a_s, wq[:256].T.copy(), w_s[:2].T.copy()))


def test_integer_inputs_give_exact_integers():
    """Unit scales and small-integer codes: every partial sum is an integer, no rounding anywhere."""
    rng = np.random.default_rng(14)
    ints = np.array([0, 1, 2, 3, 4, -1, -2, -3, -4], dtype=np.float64)
    a = rng.choice(ints, (9, 256))
    w = rng.choice(ints, (128, 256))
    aq, wq = ff.e4m3_encode(a), ff.e4m3_encode(w)
    assert np.array_equal(ff.e4m3_decode(aq), a)
    out = om.block_scaled_matmul(aq, np.ones((9, 2), np.float32), wq, np.ones((1, 2), np.float32))
    assert np.array_equal(out, a @ w.T)


def test_single_expert_reduces_to_dense_swiglu(cfg0):
    """E=1, k=1: the layer is one dense SwiGLU FFN on dequantised matrices."""
    c = cfg0
    x = c["x"]
    T = x.shape[0]
    idx = np.zeros((T, 1), np.int32)
    w = np.ones((T, 1), np.float32)
    out = om.moe_layer(x, 1, idx, w, c["W1q"][:1], c["W3q"][:1], c["W2q"][:1], c["s1"][:1], c["s3"][:1], c["s2"][:1])
    assert np.array_equal(out["perm"], np.arange(T))
    xd = _dequant_rows(out["xq"], out["xs"])
    g = xd @ _dequant_weight(c["W1q"][0], c["s1"][0]).T
    u = xd @ _dequant_weight(c["W3q"][0], c["s3"][0]).T
    h = (g * (1.0 / (1.0 + np.exp(-g)))) * u
    # same h quantisation recipe, float32 arithmetic + torch cast
    h32 = h.astype(np.float32).reshape(T, -1, 128)
    hs = np.abs(h32).max(2) / np.float32(448.0)
    hq = torch.from_numpy(h32 / hs[:, :, None]).to(torch.float8_e4m3fn).view(torch.uint8).numpy().reshape(T, -1)
    agree = (hq == out["hq"]).mean()
    assert agree > 0.999                                     # fp64 summation order may flip a boundary case
    y = _dequant_rows(out["hq"], out["hs"]) @ _dequant_weight(c["W2q"][0], c["s2"][0]).T
    assert np.allclose(out["y"], y, rtol=1e-10, atol=1e-12)
    assert np.allclose(out["hs"], hs, rtol=1e-6)


def _dense_layer_bruteforce(c, idx, w):
    """Token-by-token, expert-by-expert evaluation with no permutation machinery."""
    x = ff.bf16_bits_to_f64(c["x"])
    T, d = x.shape
    y = np.zeros((T, d))
    W1 = [_dequant_weight(c["W1q"][e], c["s1"][e]) for e in range(c["W1q"].shape[0])]
    W3 = [_dequant_weight(c["W3q"][e], c["s3"][e]) for e in range(c["W1q"].shape[0])]
    W2 = [_dequant_weight(c["W2q"][e], c["s2"][e]) for e in range(c["W1q"].shape[0])]

    def q128(vec):
        out = np.empty_like(vec)
        for g0 in range(0, vec.size, 128):
            blk = vec[g0:g0 + 128].astype(np.float32)
            amax = np.abs(blk).max()
            s = np.float32(1.0) if amax == 0 else amax / np.float32(448.0)
            code = torch.from_numpy(blk / s).to(torch.float8_e4m3fn)
            out[g0:g0 + 128] = code.to(torch.float64).numpy() * np.float64(s)
        return out

    for t in range(T):
        xt = q128(x[t])
        for j in range(idx.shape[1]):
            e = int(idx[t, j])
            g = W1[e] @ xt
            u = W3[e] @ xt
            h = np.array([gi / (1.0 + math.exp(-gi)) * ui for gi, ui in zip(g, u)])
            y[t] += float(w[t, j]) * (W2[e] @ q128(h))
    return y


def test_whole_layer_config0_vs_dense_bruteforce(cfg0):
    c = cfg0
    out = om.moe_layer_routed(c["x"], c["W_r"], 2, None, c["W1q"], c["W3q"], c["W2q"], c["s1"], c["s3"], c["s2"])
    ref = _dense_layer_bruteforce(c, out["topk_idx"], out["topk_w"])
    rel = np.linalg.norm(out["y"] - ref) / np.linalg.norm(ref)
    # identical up to h-quantisation boundary flips caused by summation order
    assert rel < 2e-3, rel
    per_tok = np.linalg.norm(out["y"] - ref, axis=1) / np.linalg.norm(ref, axis=1)
    assert np.median(per_tok) < 1e-12
    # the rounded output is the rounding of the unrounded one
    assert np.array_equal(out["y_bits"], ff.f64_to_bf16_bits(out["y"]))


def test_replay_with_routed_log_reproduces_routed_output(cfg0):
    c = cfg0
    a = om.moe_layer_routed(c["x"], c["W_r"], 2, None, c["W1q"], c["W3q"], c["W2q"], c["s1"], c["s3"], c["s2"])
    b = om.moe_layer_replay(c["x"], 8, a["topk_idx"], a["topk_w"], c["W1q"], c["W3q"], c["W2q"], c["s1"], c["s3"], c["s2"])
    for key in ("offsets", "perm", "inv_perm", "xq", "xs", "hq", "hs", "y", "y_bits"):
        assert np.array_equal(a[key], b[key]), key


def test_replay_follows_the_log_not_the_router(cfg0):
    c = cfg0
    a = om.moe_layer_routed(c["x"], c["W_r"], 2, None, c["W1q"], c["W3q"], c["W2q"], c["s1"], c["s3"], c["s2"])
    log_idx = a["topk_idx"].copy()
    log_w = np.full_like(a["topk_w"], 0.5)
    log_idx[7] = [(a["topk_idx"][7, 0] + 1) % 8, (a["topk_idx"][7, 0] + 2) % 8]
    log_idx[7] = sorted(set(range(8)) - set(a["topk_idx"][7].tolist()))[:2]
    b = om.moe_layer_replay(c["x"], 8, log_idx, log_w, c["W1q"], c["W3q"], c["W2q"], c["s1"], c["s3"], c["s2"])
    assert np.array_equal(b["topk_idx"], log_idx) and np.array_equal(b["topk_w"], log_w)
    ref = _dense_layer_bruteforce(c, log_idx, log_w)
    assert np.linalg.norm(b["y"] - ref) / np.linalg.norm(ref) < 2e-3
    assert np.linalg.norm(b["y"][7] - a["y"][7]) > 0.1 * np.linalg.norm(a["y"][7])


def test_zeroed_expert_contributes_zero_and_weights_scale_linearly(cfg0):
    c = cfg0
    idx, w, _ = om.route(c["x"], c["W_r"], 2)
    W2z = c["W2q"].copy()
    W2z[3] = 0
    out = om.moe_layer(c["x"], 8, idx, w, c["W1q"], c["W3q"], W2z, c["s1"], c["s3"], c["s2"])
    a, b = out["offsets"][3], out["offsets"][4]
    assert b > a and np.all(out["y_perm"][a:b] == 0.0)
    base = om.moe_layer(c["x"], 8, idx, w, c["W1q"], c["W3q"], c["W2q"], c["s1"], c["s3"], c["s2"])
    dbl = om.moe_layer(c["x"], 8, idx, (2 * w).astype(np.float32), c["W1q"], c["W3q"], c["W2q"], c["s1"], c["s3"], c["s2"])
    assert np.array_equal(dbl["y"], 2 * base["y"])
    # permuting tokens permutes the output rows
    p = np.random.default_rng(0).permutation(c["x"].shape[0])
    pm = om.moe_layer(c["x"][p], 8, idx[p], w[p], c["W1q"], c["W3q"], c["W2q"], c["s1"], c["s3"], c["s2"])
    assert np.allclose(pm["y"], base["y"][p], rtol=1e-12, atol=1e-14)


def test_combine_is_weighted_gather():
    rng = np.random.default_rng(21)
    T, k, d = 9, 3, 16
    y_perm = rng.standard_normal((T * k, d))
    inv = rng.permutation(T * k).astype(np.int32)
    w = rng.uniform(0, 1, (T, k)).astype(np.float32)
    y, bits = om.combine(y_perm, inv, w)
    for t in range(T):
        ref = sum(float(w[t, j]) * y_perm[inv[t * k + j]] for j in range(k))
        assert np.allclose(y[t], ref, rtol=1e-14)
    assert np.array_equal(bits, ff.f64_to_bf16_bits(y))


# --------------------------------------------------------------------------- ids-only replay
def test_replay_ids_closed_forms():
    """Weights recomputed over the logged ids: brute force, permutation equivariance, k = E, own ids."""
    from scipy.special import softmax
    rng = np.random.default_rng(5)
    T, d, E, k = 12, 128, 8, 3
    x = ff.f64_to_bf16_bits(rng.standard_normal((T, d)))
    W_r = rng.standard_normal((E, d)).astype(np.float32) / np.sqrt(d)
    ids = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    idx, w, logits = om.route_replay_ids(x, W_r, ids)
    assert np.array_equal(idx, ids)
    xf = ff.bf16_bits_to_f64(x)
    for t in range(T):                                   # token by token, expert by expert
        lg = np.array([sum(float(xf[t, c]) * float(W_r[e, c]) for c in range(d)) for e in ids[t]])
        p = np.exp(lg - lg.max())
        assert np.allclose(w[t], p / p.sum(), rtol=1e-6, atol=1e-7)
    assert np.allclose(w.sum(axis=1), 1.0, atol=1e-6)
    # reordering the logged slots reorders the weights and nothing else
    order = np.array([2, 0, 1])
    _, w2, _ = om.route_replay_ids(x, W_r, ids[:, order])
    assert np.array_equal(w2, w[:, order])
    # k = E: the plain softmax over all experts, in the logged order
    all_ids = np.tile(np.arange(E, dtype=np.int32)[::-1], (T, 1))
    _, w_all, lg_all = om.route_replay_ids(x, W_r, all_ids)
    assert np.allclose(w_all, softmax(lg_all, axis=1)[:, ::-1], rtol=1e-6, atol=1e-7)
    # logging the router's own choice reproduces the routed weights bit for bit
    r_idx, r_w, _ = om.route(x, W_r, k)
    _, w3, _ = om.route_replay_ids(x, W_r, r_idx)
    assert np.array_equal(w3, r_w)
    # the log decides the ids even where the router would choose otherwise
    assert not np.array_equal(ids, r_idx)


# --------------------------------------------------------------------------- block-wise weight quantisation
def test_quantize_blocks_invariants_and_torch_recipe():
    rng = np.random.default_rng(11)
    w = rng.standard_normal((256, 384)) / 30.0
    w[:128, 128:256] = 0.0                                # an all-zero block
    w[128:, :128] = np.exp2(rng.integers(-6, 3, (128, 128)))   # powers of two: exact
    w[130, 300] = 7.5                                      # an outlier that owns its block's scale
    wb = ff.bf16_bits_to_f64(ff.f64_to_bf16_bits(w))       # the trainer's weights are bf16
    q, s = om.quantize_blocks(wb)
    assert q.shape == (256, 384) and s.shape == (2, 3) and s.dtype == np.float32
    dec = ff.e4m3_decode(q)
    for bi in range(2):
        for bj in range(3):
            blk = wb[bi * 128:(bi + 1) * 128, bj * 128:(bj + 1) * 128]
            d_blk = dec[bi * 128:(bi + 1) * 128, bj * 128:(bj + 1) * 128]
            if np.abs(blk).max() == 0:
                assert s[bi, bj] == 1.0 and not q[bi * 128:(bi + 1) * 128, bj * 128:(bj + 1) * 128].any()
                continue
            assert np.abs(d_blk).max() == 448.0            # the block maximum lands on the largest code
            assert s[bi, bj] == np.float32(np.abs(blk).max() / 448.0)
            half_step = np.maximum(np.abs(d_blk) / 16.0, 2.0 ** -10)       # half an e4m3 step at that magnitude
            assert np.all(np.abs(blk / np.float64(s[bi, bj]) - d_blk) <= half_step * (1 + 1e-6))
    assert s[1, 2] == np.float32(7.5 / 448.0)
    # powers of two divided by a power-of-two-times-7/4 scale: check against plain float32 arithmetic + torch's cast
    wt = torch.from_numpy(wb.astype(np.float32))
    st = torch.from_numpy(s)
    rt = (wt.view(2, 128, 3, 128) / st[:, None, :, None]).reshape(256, 384)
    q_t = rt.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(q, q_t)
    # a matrix whose 128-row blocks consist of identical rows: block scales = row-group scales
    row = rng.standard_normal((1, 256))
    wr = ff.bf16_bits_to_f64(ff.f64_to_bf16_bits(np.repeat(row, 128, axis=0)))
    qb, sb = om.quantize_blocks(wr)
    qr, sr = om.quantize_rows(wr)
    assert np.array_equal(qb, qr) and np.array_equal(np.repeat(sb, 128, axis=0), sr)
