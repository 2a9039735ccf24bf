"""The five synthetic MoE-layer workloads and their seeded generators.

Only inputs are made here: activations x (bf16), router weights W_r (fp32),
an optional selection bias, expert weights already stored as e4m3 codes with
one fp32 scale per 128x128 block, and routing logs for replay mode.  Expert
weights are inputs of the layer in their quantised form (the rollout engine
receives block-quantised weights from the trainer; FP8 rollout, section
3.1.2), so the generator may produce the codes any way it likes; it uses
torch's own float8_e4m3fn cast.  Nothing here is imported by the oracle's or
the HIP path's arithmetic.

Draw order for one config (each stream has its own generator, seeded from
(seed, stream tag), so any part can be regenerated alone):
  "x"      activations            N(0,1) fp32 -> bf16 (round to nearest even)
  "wr"     router weights         N(0,1/d) fp32
  "e<i>"   expert i: W1, W3, W2   N(0,1/d) fp32 -> codes + block scales
  "log"    replay log (config 3)  Zipf ids, Dirichlet weights, mismatch mask
  "out"    outlier mask (config 4)
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Iterable, Optional

import torch

QBLOCK = 128          # quantisation block edge (weights 128x128, activations 1x128)
E4M3_MAX = 448.0      # largest finite e4m3 magnitude


@dataclasses.dataclass(frozen=True)
class MoEConfig:
    name: str
    T: int            # tokens
    d: int            # hidden size
    E: int            # experts
    k: int            # experts per token
    F: int            # expert FFN width
    modes: tuple      # subset of ("routed", "replay")
    bias: str = "none"        # "none" | "balanced"
    log: str = "routed"       # where the replay log comes from: "routed" | "zipf"
    outliers: float = 0.0     # probability of a +-20 sigma activation
    seed: int = 0

    @property
    def N(self) -> int:
        return self.T * self.k

    def gemm_flop(self) -> int:
        return 6 * self.N * self.d * self.F

    def weight_bytes(self) -> int:
        return 3 * self.E * self.d * self.F


CONFIGS = (
    MoEConfig("cfg0_tiny", T=64, d=128, E=8, k=2, F=256, modes=("routed",), seed=0),
    MoEConfig("cfg1_decode", T=256, d=4096, E=64, k=6, F=1408, modes=("routed", "replay"), seed=1),
    MoEConfig("cfg2_rollout_balanced", T=4096, d=5120, E=128, k=8, F=1536, modes=("routed",),
              bias="balanced", seed=2),
    MoEConfig("cfg3_replay_zipf", T=4096, d=5120, E=128, k=8, F=1536, modes=("replay",),
              log="zipf", seed=3),
    MoEConfig("cfg4_longctx", T=32768, d=7168, E=256, k=8, F=2048, modes=("routed", "replay"),
              outliers=1e-3, seed=4),
)


def _gen(seed: int, tag: str, device) -> torch.Generator:
    """A generator whose seed depends on (seed, tag) only."""
    h = 1469598103934665603
    for ch in f"{seed}:{tag}".encode():
        h = ((h ^ ch) * 1099511628211) & 0xFFFFFFFFFFFFFFFF
    g = torch.Generator(device=device)
    g.manual_seed(h & 0x7FFFFFFFFFFFFFFF)
    return g


def quantize_block128(w: torch.Tensor):
    """fp32 [R,C] -> (uint8 e4m3 codes [R,C], fp32 scales [R/128, C/128]).

    scale = max|w| over the 128x128 block / 448 (1.0 for an all-zero block).
    """
    R, C = w.shape
    assert R % QBLOCK == 0 and C % QBLOCK == 0
    wb = w.view(R // QBLOCK, QBLOCK, C // QBLOCK, QBLOCK)
    amax = wb.abs().amax(dim=(1, 3))
    s = amax / E4M3_MAX
    s = torch.where(amax == 0, torch.ones_like(s), s)
    q = (wb / s[:, None, :, None]).to(torch.float8_e4m3fn).view(torch.uint8)
    return q.reshape(R, C), s.to(torch.float32)


def make_expert_weights(cfg: MoEConfig, experts: Optional[Iterable[int]] = None,
                        device="cpu", seed: Optional[int] = None) -> Dict[str, torch.Tensor]:
    """Expert weights as codes + scales for `experts` (default: all).

    Returns W1q,W3q [n,F,d] u8, W2q [n,d,F] u8, s1,s3 [n,F/128,d/128] f32,
    s2 [n,d/128,F/128] f32, with n = len(experts) in the order given.
    """
    seed = cfg.seed if seed is None else seed
    ids = list(range(cfg.E)) if experts is None else list(experts)
    n, d, F = len(ids), cfg.d, cfg.F
    out = {
        "W1q": torch.empty((n, F, d), dtype=torch.uint8, device=device),
        "W3q": torch.empty((n, F, d), dtype=torch.uint8, device=device),
        "W2q": torch.empty((n, d, F), dtype=torch.uint8, device=device),
        "s1": torch.empty((n, F // QBLOCK, d // QBLOCK), dtype=torch.float32, device=device),
        "s3": torch.empty((n, F // QBLOCK, d // QBLOCK), dtype=torch.float32, device=device),
        "s2": torch.empty((n, d // QBLOCK, F // QBLOCK), dtype=torch.float32, device=device),
    }
    std = 1.0 / math.sqrt(d)
    for j, e in enumerate(ids):
        g = _gen(seed, f"e{e}", device)
        for wname, sname, shape in (("W1q", "s1", (F, d)), ("W3q", "s3", (F, d)), ("W2q", "s2", (d, F))):
            w = torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std
            q, s = quantize_block128(w)
            out[wname][j] = q
            out[sname][j] = s
    return out


def _zipf_ids(T: int, E: int, k: int, s: float, g: torch.Generator, device) -> torch.Tensor:
    """k distinct ids per token, drawn without replacement with p_e ~ (e+1)^-s (Gumbel top-k)."""
    logp = -s * torch.log(torch.arange(1, E + 1, device=device, dtype=torch.float64))
    u = torch.rand((T, E), generator=g, device=device, dtype=torch.float64).clamp_(1e-300, 1.0)
    gumbel = -torch.log((-torch.log(u)).clamp_(min=1e-300))
    return torch.topk(logp[None, :] + gumbel, k, dim=1).indices.to(torch.int32)


def make_replay_log(cfg: MoEConfig, device="cpu", seed: Optional[int] = None):
    """Config-3 style log: Zipf(1.2) ids, Dirichlet(1) weights, and the planted sets.

    Returns (planted_idx [T,k] i32, logged_idx [T,k] i32, logged_w [T,k] f32,
    differs [T] bool).  `planted_idx` are the experts the router is steered
    towards by the activations; `logged_idx` equals it except on the ~3 % of
    tokens flagged in `differs`, which carry a fresh independent draw.
    """
    seed = cfg.seed if seed is None else seed
    g = _gen(seed, "log", device)
    planted = _zipf_ids(cfg.T, cfg.E, cfg.k, 1.2, g, device)
    fresh = _zipf_ids(cfg.T, cfg.E, cfg.k, 1.2, g, device)
    differs = torch.rand((cfg.T,), generator=g, device=device) < 0.03
    logged = torch.where(differs[:, None], fresh, planted)
    ex = -torch.log(torch.rand((cfg.T, cfg.k), generator=g, device=device, dtype=torch.float64).clamp_(1e-300, 1.0))
    w = (ex / ex.sum(dim=1, keepdim=True)).to(torch.float32)
    return planted, logged.contiguous(), w.contiguous(), differs


def _balanced_bias(x: torch.Tensor, W_r: torch.Tensor, k: int, iters: int = 300):
    """Selection bias that evens out the per-expert top-k load (config 2).

    Fixed-point iteration b_e += 0.05*(mean-load_e)/mean on the top-k counts of
    logit+b; the bias with the smallest max|load-mean|/mean seen is returned
    together with that imbalance.
    """
    logits = x.to(torch.float64) @ W_r.to(torch.float64).T
    T, E = logits.shape
    mean = T * k / E
    b = torch.zeros(E, dtype=torch.float64, device=x.device)
    best, best_b = float("inf"), b.clone()
    for _ in range(iters):
        sel = torch.topk(logits + b, k, dim=1).indices
        load = torch.bincount(sel.flatten(), minlength=E).to(torch.float64)
        imb = float(((load - mean).abs().max() / mean).item())
        if imb < best:
            best, best_b = imb, b.clone()
        if imb <= 0.02:
            break
        b = b + 0.05 * (mean - load) / mean
    return best_b.to(torch.float32), best


def make_inputs(cfg: MoEConfig, device="cpu", seed: Optional[int] = None,
                with_experts: bool = True) -> Dict[str, object]:
    """All inputs of one config on `device`.

    Keys: x (bf16 [T,d]), W_r (f32 [E,d]), sel_bias (f32 [E] or None), the
    expert-weight tensors of make_expert_weights (if with_experts), and for a
    Zipf-log config planted_idx / logged_idx / logged_w / differs.
    """
    seed = cfg.seed if seed is None else seed
    T, d, E, k = cfg.T, cfg.d, cfg.E, cfg.k
    out: Dict[str, object] = {"cfg": cfg, "seed": seed}
    W_r = torch.randn((E, d), generator=_gen(seed, "wr", device), device=device, dtype=torch.float32) / math.sqrt(d)
    x = torch.randn((T, d), generator=_gen(seed, "x", device), device=device, dtype=torch.float32)
    if cfg.outliers > 0:
        go = _gen(seed, "out", device)
        mask = torch.rand((T, d), generator=go, device=device) < cfg.outliers
        sign = torch.where(torch.rand((T, d), generator=go, device=device) < 0.5, -1.0, 1.0)
        x = torch.where(mask, 20.0 * sign, x)
    if cfg.log == "zipf":
        planted, logged, lw, differs = make_replay_log(cfg, device, seed)
        dirs = W_r / (W_r * W_r).sum(dim=1, keepdim=True)          # W_r[e]/|W_r[e]|^2
        onehot = torch.zeros((T, E), device=device, dtype=torch.float32)
        onehot.scatter_(1, planted.long(), 1.0)
        x = x + 8.0 * (onehot @ dirs)
        out.update(planted_idx=planted, logged_idx=logged, logged_w=lw, differs=differs)
    out["x"] = x.to(torch.bfloat16).contiguous()
    out["W_r"] = W_r.contiguous()
    out["sel_bias"] = None
    if cfg.bias == "balanced":
        b, imb = _balanced_bias(out["x"], W_r, k)
        out["sel_bias"] = b.contiguous()
        out["bias_imbalance"] = imb
    if with_experts:
        out.update(make_expert_weights(cfg, None, device, seed))
    return out
