#!/usr/bin/env python3
"""Benchmark of the MoE-layer forward pass on one MI355X.

One step = one pass of the whole hot path (route or replay, permutation, FP8
quantise + expert-order fan-out, gate/up GEMM + SwiGLU + re-quantise, down GEMM,
combine) over one batch of synthetic input that is already resident in HBM.
Prints ONE JSON line.  `value` is the FP8 GEMM work of the layer (6*N*d*F FLOP)
divided by the whole step's time, in TFLOP/s, for routed mode; replay-mode and
per-stage figures ride along in the same line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP8_PEAK_TFLOPS = 5000.0   # MI355X dense FP8 MFMA peak
HBM_PEAK_GBS = 8000.0      # MI355X HBM3E
CALIB_BYTES = 1 << 30      # size of the plain device copy that calibrates the HBM byte counters


def _measured_traffic(config_index):
    """HBM bytes per launch of the gate/up GEMM, as recorded in the committed counter summary
    (profiles/ffn_gemm_cfg<i>_hbm_traffic.txt, line 'gemm1_hbm_bytes_per_launch: <number>'); None if absent."""
    path = os.path.join(ROOT, "profiles", f"ffn_gemm_cfg{config_index}_hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("gemm1_hbm_bytes_per_launch:"):
                    return float(line.split(":", 1)[1].strip())
    except OSError:
        pass
    return None


def _cpu_baseline(cfg, inp_small):
    """Time the oracle, as it stands, on a bounded slice of the workload (host cores)."""
    import numpy as np
    from oracle import moe_layer as om
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    t0 = time.perf_counter()
    om.moe_layer_routed(*inp_small)
    dt = time.perf_counter() - t0
    Ts, Es = inp_small[0].shape[0], inp_small[1].shape[0]
    ks = inp_small[2]
    flop = 6.0 * Ts * ks * cfg.d * cfg.F
    return {"value": flop / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "tokens_per_s": Ts / dt, "seconds": dt,
            "sample": f"whole layer (oracle route, permute, quantise, FFN, combine) on tokens 0..{Ts - 1} "
                      f"routed over experts 0..{Es - 1} with k={ks} (={Ts * ks // Es} rows per expert), full d={cfg.d}, F={cfg.F}"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="index into the five workloads (default: the largest)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2512_07710_amd as moe
    from workloads import CONFIGS, make_inputs

    if not os.path.exists(moe.LIB_PATH):
        from paper_2512_07710_amd.build import build
        build()
    moe.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    cfg = CONFIGS[args.config]
    inp = make_inputs(cfg, device=dev)
    torch.cuda.synchronize()
    layer = moe.MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, device=dev)
    x, W_r, bias = inp["x"], inp["W_r"], inp.get("sel_bias")
    # a plain copy of known size: under `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` its counters give the
    # factor that turns the same counters of the GEMM kernels into bytes
    calib = torch.empty(CALIB_BYTES, dtype=torch.uint8, device=dev)
    calib_dst = torch.empty_like(calib)
    calib_dst.copy_(calib)
    del calib, calib_dst
    K, W = args.steps, args.warmup

    def step_routed():
        layer.forward_routed(x, W_r, bias, inp)

    # the replay log: config 3 brings its own; otherwise the routed decision of this very input
    step_routed()
    torch.cuda.synchronize()
    if cfg.log == "zipf":
        log_idx, log_w = inp["logged_idx"], inp["logged_w"]
    else:
        log_idx, log_w = layer.topk_idx.clone(), layer.topk_w.clone()

    def step_replay():
        layer.forward_replay(x, log_idx, log_w, inp)

    def timed(fn):
        for _ in range(W):
            fn()
        torch.cuda.synchronize()
        moe.moe_profile_enable(layer.ctx, True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            fn()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        g1, g2, calls = moe.moe_profile_read(layer.ctx)
        moe.moe_profile_enable(layer.ctx, False)
        return dt / K * 1e3, g1, g2, calls

    head_mode = "routed" if "routed" in cfg.modes else "replay"
    ms_routed = g1 = g2 = None
    if "routed" in cfg.modes:
        ms_routed, g1, g2, _ = timed(step_routed)
    ms_replay, g1r, g2r, _ = timed(step_replay)
    if head_mode == "replay":
        g1, g2 = g1r, g2r
    ms_head = ms_routed if head_mode == "routed" else ms_replay

    # per-stage times (diagnostic pass, outside the headline timing)
    def stage_ms(fn, reps=10):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        fn()
        torch.cuda.synchronize()
        ev[0].record()
        for _ in range(reps):
            fn()
        ev[1].record()
        torch.cuda.synchronize()
        return ev[0].elapsed_time(ev[1]) / reps

    stages = {
        "route": stage_ms(lambda: layer.route(x, W_r, bias)) if "routed" in cfg.modes else None,
        "route_replay": stage_ms(lambda: layer.route_replay(x, log_idx, log_w)),
    }
    (step_routed if head_mode == "routed" else step_replay)()
    stages["quantize"] = stage_ms(lambda: layer.quantize_tokens(x))          # once per token (the timed path)
    stages["expert_ffn"] = stage_ms(lambda: layer.expert_ffn_gather(inp))     # gathers inside the gate/up GEMM
    stages["combine"] = stage_ms(layer.combine)
    # the unfused alternative: expert-ordered copy of the activations, then the plain grouped FFN
    stages["quantize_fanout_unfused"] = stage_ms(lambda: layer.quantize(x))
    stages["expert_ffn_unfused"] = stage_ms(lambda: layer.expert_ffn(inp))

    N, d, F, T, k = cfg.N, cfg.d, cfg.F, cfg.T, cfg.k
    flop = 6.0 * N * d * F
    gemm1_flop = 4.0 * N * d * F
    q_bytes = 2.0 * T * d + T * d + 4.0 * T * d / 128          # token-order quantisation: read bf16, write codes + scales
    qf_bytes = 2.0 * T * d + N * d + 4.0 * N * d / 128         # with the k-fold fan-out of the unfused path
    c_bytes = 4.0 * N * d + 8.0 * N + 2.0 * T * d
    roof = {"bound": "mfma", "kernel": "ffn_gemm<gate/up, gather> (token gather + GEMM1 + SwiGLU + h re-quantisation)",
            "achieved": gemm1_flop / (g1 * 1e-3) / 1e12, "peak": FP8_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": gemm1_flop / (g1 * 1e-3) / 1e12 / FP8_PEAK_TFLOPS, "traffic": _measured_traffic(args.config),
            "algorithmic_bytes": 2.0 * cfg.E * d * F + T * d + N * F,       # weights, token-order codes, hq
            "avg_launch_ms": g1, "flop_per_launch": gemm1_flop}
    out = {
        "metric": "MoE-layer fwd FP8 TFLOP/s (% MFMA peak) + tokens/s, routed vs replay",
        "value": flop / (ms_head * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_head, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "fp8", "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {cfg.name}: T={T} d={d} E={cfg.E} k={k} F={F}, mode={head_mode}",
                   "T": T, "d": d, "E": cfg.E, "k": k, "F": F, "mode": head_mode},
        "pct_mfma_peak_whole_step": 100.0 * flop / (ms_head * 1e-3) / 1e12 / FP8_PEAK_TFLOPS,
        "tokens_per_s": T / (ms_head * 1e-3),
        "routed": None if ms_routed is None else {"ms_per_step": ms_routed, "tokens_per_s": T / (ms_routed * 1e-3),
                                                  "tflops": flop / (ms_routed * 1e-3) / 1e12},
        "replay": {"ms_per_step": ms_replay, "tokens_per_s": T / (ms_replay * 1e-3),
                   "tflops": flop / (ms_replay * 1e-3) / 1e12},
        "stages_ms": stages,
        "kernels": {"gemm1_ms": g1, "gemm2_ms": g2,
                    "gemm1_tflops": gemm1_flop / (g1 * 1e-3) / 1e12,
                    "gemm2_tflops": 2.0 * N * d * F / (g2 * 1e-3) / 1e12,
                    "quantize_fanout_GBs": qf_bytes / (stages["quantize_fanout_unfused"] * 1e-3) / 1e9,
                    "quantize_fanout_frac_hbm": qf_bytes / (stages["quantize_fanout_unfused"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    "quantize_GBs": q_bytes / (stages["quantize"] * 1e-3) / 1e9,
                    "quantize_frac_hbm": q_bytes / (stages["quantize"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    "combine_GBs": c_bytes / (stages["combine"] * 1e-3) / 1e9,
                    "combine_frac_hbm": c_bytes / (stages["combine"] * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "roofline": roof,
    }
    # the entry points beyond the five core calls, timed outside the headline region (same resident inputs)
    ext = {}
    if "routed" in cfg.modes:
        ext["route_replay_ids_ms"] = stage_ms(lambda: layer.route_replay_ids(x, W_r, log_idx))
    rows_w = min(cfg.E * F, 16 * 4096)                        # a slab of bf16 gate weights of 16*4096 rows
    w_bf16 = torch.randn((rows_w, d), device=dev, dtype=torch.float32).mul_(d ** -0.5).to(torch.bfloat16)
    wq = torch.empty((rows_w, d), dtype=torch.uint8, device=dev)
    wsc = torch.empty((rows_w // 128, d // 128), dtype=torch.float32, device=dev)
    t_wq = stage_ms(lambda: moe.moe_quantize_weights_fp8(layer.ctx, w_bf16, rows_w, d, wq, wsc))
    ext["weight_quant_ms"] = t_wq
    ext["weight_quant_GBs"] = 3.0 * rows_w * d / (t_wq * 1e-3) / 1e9
    ext["weight_quant_frac_hbm"] = ext["weight_quant_GBs"] / HBM_PEAK_GBS
    rows_l = min(8192, N)                                     # dense linear: [rows_l, d] x [rows_w, d]^T
    if rows_l * rows_w <= N * d:                              # y_perm doubles as the output buffer
        xs_l = layer.xs[:, :rows_l].contiguous()
        t_lin = stage_ms(lambda: moe.moe_linear_fp8(layer.ctx, layer.xq, xs_l, rows_l, d, wq, wsc, rows_w,
                                                    layer.y_perm), reps=5)
        ext["dense_linear_ms"] = t_lin
        ext["dense_linear_tflops"] = 2.0 * rows_l * d * rows_w / (t_lin * 1e-3) / 1e12
        ext["dense_linear_shape"] = [rows_l, d, rows_w]
    # the same layer with the expert outputs kept as 16-bit block-scaled rows between the down GEMM and the combine
    # (half the bytes of that round trip; the headline above keeps fp32 rows)
    i16 = {}
    if "routed" in cfg.modes:
        i16["routed_ms_per_step"] = timed(lambda: layer.forward_routed(x, W_r, bias, inp, fused="i16"))[0]
    ms_i16, _, g2_i16, _ = timed(lambda: layer.forward_replay(x, log_idx, log_w, inp, fused="i16"))
    i16["replay_ms_per_step"] = ms_i16
    i16["gemm2_ms"] = g2_i16
    i16["combine_ms"] = stage_ms(layer.combine_i16)
    ci_bytes = 2.0 * N * d + 4.0 * N * d / 128 + 8.0 * N + 2.0 * T * d
    i16["combine_GBs"] = ci_bytes / (i16["combine_ms"] * 1e-3) / 1e9
    i16["combine_frac_hbm"] = i16["combine_GBs"] / HBM_PEAK_GBS
    head_i16 = i16.get("routed_ms_per_step", ms_i16) if head_mode == "routed" else ms_i16
    i16["tflops"] = flop / (head_i16 * 1e-3) / 1e12
    i16["tokens_per_s"] = T / (head_i16 * 1e-3)
    ext["i16_expert_outputs"] = i16
    out["extensions"] = ext
    del w_bf16, wq, wsc
    if not args.no_cpu_baseline:
        Ts, Es = min(1024, T), min(8, cfg.E)
        ks = min(k, Es)
        xb = x[:Ts].cpu().view(torch.int16).numpy().view(np.uint16)
        small = (xb, W_r[:Es].cpu().numpy(), ks, None,
                 inp["W1q"][:Es].cpu().numpy(), inp["W3q"][:Es].cpu().numpy(), inp["W2q"][:Es].cpu().numpy(),
                 inp["s1"][:Es].cpu().numpy(), inp["s3"][:Es].cpu().numpy(), inp["s2"][:Es].cpu().numpy())
        out["cpu_baseline"] = _cpu_baseline(cfg, small)
    layer.close()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
