"""Plain CPU oracle of one MoE-layer forward pass (routed or Router Replay).

TEST INFRASTRUCTURE ONLY.  Only tests/, the smoke check and the benchmark's
cpu_baseline leg may import this; the HIP path shares no code with it.

What is computed (paper sections 2.4.4 "Router Replay" and 3.1.2 "FP8
quantisation for rollout"; the paper gives no formulas for the layer, so the
standard definitions below are the reading taken):

  routed   logits = x W_r^T; top-k experts by (logit + selection bias),
           ties to the lower index, slots in descending score order; gate
           weights = softmax over the k selected unbiased logits.
  replay   the logged expert ids and gate weights are used verbatim
           (router decisions recorded at rollout are reused by the trainer);
           ids-only form: the ids are reused, the weights are the softmax of
           this engine's own logits over the logged ids.
  weights  block-wise quantisation of a weight matrix: one scale per 128x128
           block, same scale and rounding rule as for activations.
  permute  stable counting sort of the T*k (token, slot) assignments by expert.
  quantise each row, per 128 contiguous elements: s = amax/448 (1 if amax=0),
           code = e4m3(x/s); s and x/s are rounded to fp32 before use.
  experts  g = xq W1^T, u = xq W3^T with per-128-block rescaling by
           (activation scale x weight block scale); h = silu(g)*u; h is
           quantised like x; y_perm = hq W2^T, same rescaling.
  combine  y[t] = sum_j w[t,j] * y_perm[row of (t,j)], rounded to bf16 once.

All arithmetic is float64 except the rounding points named above.
"""
from __future__ import annotations

import numpy as np

from .fp_formats import E4M3_MAX, e4m3_decode, e4m3_encode, bf16_bits_to_f64, f64_to_bf16_bits

G = 128  # quantisation group / block edge


# --------------------------------------------------------------------------- routing
def router_logits(x_bits: np.ndarray, W_r: np.ndarray) -> np.ndarray:
    """logit[t,e] = sum_c x[t,c] * W_r[e,c] in float64; x given as bf16 bit patterns."""
    return bf16_bits_to_f64(x_bits) @ np.asarray(W_r, dtype=np.float64).T


def topk_select(score: np.ndarray, k: int) -> np.ndarray:
    """ids of the k largest scores per row, descending, equal scores -> lower index first."""
    order = np.argsort(-score, axis=1, kind="stable")
    return order[:, :k].astype(np.int32)


def gate_weights(logits: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """softmax over the selected logits of each row (fp64), stored as fp32."""
    sel = np.take_along_axis(logits, idx.astype(np.int64), axis=1)
    m = sel.max(axis=1, keepdims=True)
    p = np.exp(sel - m)
    return (p / p.sum(axis=1, keepdims=True)).astype(np.float32)


def route(x_bits, W_r, k, sel_bias=None):
    """Routed mode: (topk_idx [T,k] i32, topk_w [T,k] f32, logits [T,E] f64)."""
    logits = router_logits(x_bits, W_r)
    score = logits if sel_bias is None else logits + np.asarray(sel_bias, dtype=np.float64)[None, :]
    idx = topk_select(score, k)
    return idx, gate_weights(logits, idx), logits


def route_replay(logged_idx, logged_w):
    """Replay mode: the log is the routing decision (section 2.4.4)."""
    return np.array(logged_idx, dtype=np.int32, copy=True), np.array(logged_w, dtype=np.float32, copy=True)


def route_replay_ids(x_bits, W_r, logged_idx):
    """Ids-only Router Replay (section 2.4.4 read literally: the router DECISIONS are reused).

    The logged expert ids are taken verbatim; the gate weights are recomputed from this engine's own
    logits, w[t,j] = softmax over logit[t, logged_idx[t,:]].  Returns (idx i32, w f32, logits f64).
    """
    logits = router_logits(x_bits, W_r)
    idx = np.array(logged_idx, dtype=np.int32, copy=True)
    return idx, gate_weights(logits, idx), logits


def permute(topk_idx: np.ndarray, E: int):
    """Stable counting sort of flat assignments i = t*k+j by expert id.

    Returns offsets [E+1], perm [N] (sorted position -> flat assignment) and
    inv_perm [N] (flat assignment -> sorted position), all int32.
    """
    flat = np.asarray(topk_idx, dtype=np.int64).reshape(-1)
    N = flat.size
    counts = np.zeros(E, dtype=np.int64)
    for e in flat:
        counts[e] += 1
    offsets = np.zeros(E + 1, dtype=np.int64)
    for e in range(E):
        offsets[e + 1] = offsets[e] + counts[e]
    cursor = offsets[:-1].copy()
    perm = np.empty(N, dtype=np.int32)
    inv_perm = np.empty(N, dtype=np.int32)
    for i in range(N):
        p = cursor[flat[i]]
        cursor[flat[i]] += 1
        perm[p] = i
        inv_perm[i] = p
    return offsets.astype(np.int32), perm, inv_perm


# --------------------------------------------------------------------------- quantisation
def quantize_rows(v: np.ndarray):
    """Per-row, per-128-group e4m3 quantisation of fp32-representable values.

    v [R,C] float64 holding values exactly representable in fp32.  Returns
    codes u8 [R,C] and scales f32 [R,C/128].  s = fp32(amax/448) (1 if the
    group is all zero), r = fp32(v/s), code = e4m3(r).
    """
    R, C = v.shape
    assert C % G == 0
    vg = v.reshape(R, C // G, G)
    amax = np.abs(vg).max(axis=2)
    s = (amax / E4M3_MAX).astype(np.float32)
    s = np.where(amax == 0, np.float32(1.0), s)
    r = (vg / s.astype(np.float64)[:, :, None]).astype(np.float32)
    codes = e4m3_encode(r.astype(np.float64)).reshape(R, C)
    return codes, s


def quantize_blocks(w: np.ndarray):
    """Block-wise weight quantisation (section 3.1.2: weights are quantised block-wise when the trainer
    pushes them to the rollout engine).

    w [R,C] float64 holding fp32-representable values, R and C multiples of 128.  One fp32 scale per
    128x128 block: s = fp32(amax/448) (1 if the block is all zero), code = e4m3(fp32(w/s)).
    Returns codes u8 [R,C] and scales f32 [R/128, C/128].
    """
    R, C = w.shape
    assert R % G == 0 and C % G == 0
    codes = np.zeros((R, C), dtype=np.uint8)
    scales = np.ones((R // G, C // G), dtype=np.float32)
    for bi in range(R // G):
        for bj in range(C // G):
            blk = w[bi * G:(bi + 1) * G, bj * G:(bj + 1) * G]
            amax = np.abs(blk).max()
            s = np.float32(1.0) if amax == 0 else np.float32(amax / E4M3_MAX)
            r = (blk / np.float64(s)).astype(np.float32)
            codes[bi * G:(bi + 1) * G, bj * G:(bj + 1) * G] = e4m3_encode(r.astype(np.float64))
            scales[bi, bj] = s
    return codes, scales


def gather_quantize(x_bits: np.ndarray, perm: np.ndarray, k: int):
    """Expert-ordered quantised activations: sorted row p comes from token perm[p]//k."""
    tok = np.asarray(perm, dtype=np.int64) // k
    return quantize_rows(bf16_bits_to_f64(x_bits)[tok])


# --------------------------------------------------------------------------- experts
def block_scaled_matmul(aq, a_s, wq, w_s) -> np.ndarray:
    """out[p,n] = sum_kb a_s[p,kb] * w_s[n//128,kb] * sum_{c in kb} dec(aq[p,c]) * dec(wq[n,c]).

    aq [M,K] u8, a_s [M,K/128] f32, wq [Nn,K] u8, w_s [Nn/128,K/128] f32.
    """
    A = e4m3_decode(aq)
    W = e4m3_decode(wq)
    M, K = A.shape
    Nn = W.shape[0]
    out = np.zeros((M, Nn), dtype=np.float64)
    a_s = np.asarray(a_s, dtype=np.float64)
    w_s = np.asarray(w_s, dtype=np.float64)
    for kb in range(K // G):
        part = A[:, kb * G:(kb + 1) * G] @ W[:, kb * G:(kb + 1) * G].T
        scale = a_s[:, kb][:, None] * np.repeat(w_s[:, kb], G)[None, :]
        out += scale * part
    return out


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def expert_ffn_rows(xq, xs, W1q, s1, W3q, s3, W2q, s2):
    """One expert's SwiGLU FFN on its rows.  Returns (y [M,d] f64, hq u8 [M,F], hs f32 [M,F/128])."""
    g = block_scaled_matmul(xq, xs, W1q, s1)
    u = block_scaled_matmul(xq, xs, W3q, s3)
    h = silu(g) * u
    hq, hs = quantize_rows(h.astype(np.float32).astype(np.float64))
    y = block_scaled_matmul(hq, hs, W2q, s2)
    return y, hq, hs


def expert_ffn(xq_perm, xs_perm, offsets, W1q, W3q, W2q, s1, s3, s2, experts=None):
    """Grouped FFN over expert-sorted rows.  Returns (y_perm f64 [N,d], hq, hs).

    `experts` restricts the work to some experts (other rows are left zero).
    """
    N = xq_perm.shape[0]
    d = W2q.shape[1]
    F = W1q.shape[1]
    y = np.zeros((N, d), dtype=np.float64)
    hq = np.zeros((N, F), dtype=np.uint8)
    hs = np.ones((N, F // G), dtype=np.float32)
    for e in (range(W1q.shape[0]) if experts is None else experts):
        a, b = int(offsets[e]), int(offsets[e + 1])
        if a == b:
            continue
        y[a:b], hq[a:b], hs[a:b] = expert_ffn_rows(xq_perm[a:b], xs_perm[a:b], W1q[e], s1[e],
                                                   W3q[e], s3[e], W2q[e], s2[e])
    return y, hq, hs


# --------------------------------------------------------------------------- combine
def combine(y_perm: np.ndarray, inv_perm: np.ndarray, topk_w: np.ndarray):
    """y[t] = sum_j w[t,j] * y_perm[inv_perm[t*k+j]] in fp64; also its bf16 rounding."""
    T, k = topk_w.shape
    rows = np.asarray(inv_perm, dtype=np.int64).reshape(T, k)
    w = np.asarray(topk_w, dtype=np.float64)
    y = np.zeros((T, y_perm.shape[1]), dtype=np.float64)
    for j in range(k):
        y += w[:, j][:, None] * y_perm[rows[:, j]]
    return y, f64_to_bf16_bits(y)


# --------------------------------------------------------------------------- whole layer
def moe_layer(x_bits, E, topk_idx, topk_w, W1q, W3q, W2q, s1, s3, s2):
    """Everything after routing.  Returns a dict with every intermediate."""
    T, k = topk_idx.shape
    offsets, perm, inv_perm = permute(topk_idx, E)
    xq, xs = gather_quantize(x_bits, perm, k)
    y_perm, hq, hs = expert_ffn(xq, xs, offsets, W1q, W3q, W2q, s1, s3, s2)
    y, y_bits = combine(y_perm, inv_perm, topk_w)
    return dict(offsets=offsets, perm=perm, inv_perm=inv_perm, xq=xq, xs=xs, hq=hq, hs=hs,
                y_perm=y_perm, y=y, y_bits=y_bits)


def moe_layer_routed(x_bits, W_r, k, sel_bias, W1q, W3q, W2q, s1, s3, s2):
    idx, w, logits = route(x_bits, W_r, k, sel_bias)
    out = moe_layer(x_bits, W_r.shape[0], idx, w, W1q, W3q, W2q, s1, s3, s2)
    out.update(topk_idx=idx, topk_w=w, logits=logits)
    return out


def moe_layer_replay(x_bits, E, logged_idx, logged_w, W1q, W3q, W2q, s1, s3, s2):
    idx, w = route_replay(logged_idx, logged_w)
    out = moe_layer(x_bits, E, idx, w, W1q, W3q, W2q, s1, s3, s2)
    out.update(topk_idx=idx, topk_w=w)
    return out
