#!/usr/bin/env python3
"""Benchmark of the MoE-layer forward pass on one MI355X.

One step = one pass of the whole hot path (route or replay, permutation, FP8 quantisation of the tokens,
gather-fused gate/up GEMM + SwiGLU + re-quantisation, down GEMM, combine) over one batch of synthetic input
that is already resident in HBM.  Prints ONE JSON line.  `value` is the FP8 GEMM work of the layer
(6*N*d*F FLOP) divided by the whole step's time, in TFLOP/s, at configs[4] in routed mode; replay-mode,
per-stage and per-kernel figures, the other configurations, the machine's measured ceilings and the CPU
oracle's rate ride along in the same line.
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
MFMA_BOUND_ROWS = 315      # mean rows per expert above which the grouped GEMM is matrix-bound: 2*rows FLOP per
                           # weight byte against the ridge of 5000 TFLOP/s / 8 TB/s = 625 FLOP/B


def _recorded_traffic(config_index):
    """HBM bytes per launch of the gate/up GEMM as RECORDED in the committed counter summary
    (profiles/ffn_gemm_cfg<i>_hbm_traffic.txt, line 'gemm1_hbm_bytes_per_launch: <number>'); None if absent.
    Counters cannot be read inside a timed run: this is a stored figure, not a live one."""
    path = os.path.join(ROOT, "profiles", f"ffn_gemm_cfg{config_index}_hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("gemm1_hbm_bytes_per_launch:"):
                    return float(line.split(":", 1)[1].strip()), os.path.relpath(path, ROOT)
    except OSError:
        pass
    return None, None


def _cpu_baseline(cfg, inp_small):
    """Time the oracle, as it stands, on a bounded slice of the workload (host cores)."""
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


def _stage_ms(torch, fn, reps=10):
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    fn()
    torch.cuda.synchronize()
    ev[0].record()
    for _ in range(reps):
        fn()
    ev[1].record()
    torch.cuda.synchronize()
    return ev[0].elapsed_time(ev[1]) / reps


def _ceilings(torch, moe, ctx, dev):
    """What this machine delivers to the simplest possible kernels, measured in this run."""
    nbytes = 1 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty_like(src)
    t_copy = _stage_ms(torch, lambda: moe.moe_probe_copy(ctx, src, dst, nbytes), reps=10)
    del src, dst
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    blocks, steps = 256 * 4, 2048
    flop = blocks * 8 * steps * 16 * 2.0 * 32 * 32 * 64
    t_bare = _stage_ms(torch, lambda: moe.moe_probe_fp8_mfma(ctx, blocks, steps, False, sink), reps=3)
    t_scaled = _stage_ms(torch, lambda: moe.moe_probe_fp8_mfma(ctx, blocks, steps, True, sink), reps=3)
    return {"copy_GBs": 2.0 * nbytes / (t_copy * 1e-3) / 1e9,
            "fp8_mfma_loop_tflops": flop / (t_bare * 1e-3) / 1e12,
            "fp8_mfma_loop_with_block_scaling_tflops": flop / (t_scaled * 1e-3) / 1e12,
            "note": "measured in this run: 1 GiB streaming copy (read + write bytes); register-only loop of "
                    "v_mfma_f32_32x32x64_f8f6f4 on random operand bits, bare and with the 16 fp32 multiply-adds per "
                    "product that per-128-block scaling needs (no LDS, no memory).  Reported beside the published "
                    "peaks, which stay the denominators of every `frac`."}


def _measure(torch, moe, cfg, config_index, dev, K, W, detail):
    """Times one configuration; returns (result dict, layer, inputs) - layer and inputs only if detail."""
    from workloads import make_inputs
    inp = make_inputs(cfg, device=dev)
    torch.cuda.synchronize()
    layer = moe.MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.F, device=dev)
    x, W_r, bias = inp["x"], inp["W_r"], inp.get("sel_bias")

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
        moe.moe_profile_enable(layer.ctx, True)       # HIP events around the two GEMM kernels, on the library's stream
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

    N, d, F, T, k, E = cfg.N, cfg.d, cfg.F, cfg.T, cfg.k, cfg.E
    counts = (layer.offsets[1:] - layer.offsets[:-1]).cpu()
    e_active = int((counts > 0).sum())
    flop = 6.0 * N * d * F
    gemm1_flop = 4.0 * N * d * F
    gemm1_bytes = 2.0 * e_active * d * F + T * d + N * F       # weights of the experts in use, token-order codes, hq
    gemm2_bytes = 1.0 * e_active * d * F + N * F + 4.0 * N * d
    mfma_bound = N / E >= MFMA_BOUND_ROWS
    if mfma_bound:
        roof = {"bound": "mfma", "achieved": gemm1_flop / (g1 * 1e-3) / 1e12, "peak": FP8_PEAK_TFLOPS, "unit": "TFLOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": gemm1_bytes / (g1 * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["kernel"] = "ffn_gemm<gate/up, gather> (token gather + GEMM1 + SwiGLU + h re-quantisation)"
    roof["rule"] = (f"mean rows per expert {N / E:.0f} {'>=' if mfma_bound else '<'} {MFMA_BOUND_ROWS}: "
                    f"{'matrix-bound' if mfma_bound else 'weight streaming, HBM-bound'}")
    res = {
        "workload": f"configs[{config_index}] {cfg.name}: T={T} d={d} E={E} k={k} F={F}",
        "mode": head_mode, "ms_per_step": ms_head, "tokens_per_s": T / (ms_head * 1e-3),
        "tflops": flop / (ms_head * 1e-3) / 1e12,
        "routed_ms": ms_routed, "replay_ms": ms_replay,
        "gemm1_ms": g1, "gemm2_ms": g2,
        "gemm1_tflops": gemm1_flop / (g1 * 1e-3) / 1e12, "gemm2_tflops": 2.0 * N * d * F / (g2 * 1e-3) / 1e12,
        "gemm1_GBs": gemm1_bytes / (g1 * 1e-3) / 1e9, "gemm2_GBs": gemm2_bytes / (g2 * 1e-3) / 1e9,
        "roofline": roof,
    }
    if not detail:
        layer.close()
        return res, None, None
    res["_private"] = dict(step_routed=step_routed, step_replay=step_replay, log_idx=log_idx, log_w=log_w,
                           gemm1_flop=gemm1_flop, gemm1_bytes=gemm1_bytes, flop=flop)
    return res, layer, inp


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="index into the five workloads (default: the largest)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the compact figures of configs 1-3")
    ap.add_argument("--no-extensions", action="store_true",
                    help="skip the entry points beyond the core calls and the ceiling probes (clean kernel traces)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2512_07710_amd as moe
    from workloads import CONFIGS

    if not os.path.exists(moe.LIB_PATH):
        from paper_2512_07710_amd.build import build
        build()
    moe.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    K, W = args.steps, args.warmup

    # the other configurations first (small, a few seconds together), each with the roofline that bounds it
    others = {}
    if not args.no_other_configs:
        for ci in (1, 2, 3):
            if ci == args.config:
                continue
            r, _, _ = _measure(torch, moe, CONFIGS[ci], ci, dev, max(K, 20), max(W, 3), detail=False)
            others[f"cfg{ci}"] = r
            torch.cuda.empty_cache()

    cfg = CONFIGS[args.config]
    # a plain copy of known size: under `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` its counters give the
    # factor that turns the same counters of the GEMM kernels into bytes
    calib = torch.empty(CALIB_BYTES, dtype=torch.uint8, device=dev)
    calib_dst = torch.empty_like(calib)
    calib_dst.copy_(calib)
    del calib, calib_dst
    res, layer, inp = _measure(torch, moe, cfg, args.config, dev, K, W, detail=True)
    priv = res.pop("_private")
    x, W_r, bias = inp["x"], inp["W_r"], inp.get("sel_bias")
    log_idx, log_w = priv["log_idx"], priv["log_w"]
    head_mode, ms_head = res["mode"], res["ms_per_step"]
    N, d, F, T, k = cfg.N, cfg.d, cfg.F, cfg.T, cfg.k

    # per-stage times (diagnostic pass, outside the headline timing)
    stages = {
        "route": _stage_ms(torch, lambda: layer.route(x, W_r, bias)) if "routed" in cfg.modes else None,
        "route_replay": _stage_ms(torch, lambda: layer.route_replay(x, log_idx, log_w)),
    }
    (priv["step_routed"] if head_mode == "routed" else priv["step_replay"])()
    stages["quantize"] = _stage_ms(torch, lambda: layer.quantize_tokens(x))          # once per token (the timed path)
    stages["expert_ffn"] = _stage_ms(torch, lambda: layer.expert_ffn_gather(inp))     # gathers inside the gate/up GEMM
    stages["combine"] = _stage_ms(torch, layer.combine)
    # the unfused alternative: expert-ordered copy of the activations, then the plain grouped FFN
    stages["quantize_fanout_unfused"] = _stage_ms(torch, lambda: layer.quantize(x))
    stages["expert_ffn_unfused"] = _stage_ms(torch, lambda: layer.expert_ffn(inp))

    q_bytes = 2.0 * T * d + T * d + 4.0 * T * d / 128          # token-order quantisation: read bf16, write codes + scales
    qf_bytes = 2.0 * T * d + N * d + 4.0 * N * d / 128         # with the k-fold fan-out of the unfused path
    c_bytes = 4.0 * N * d + 8.0 * N + 2.0 * T * d
    r_bytes = 2.0 * T * d + 8.0 * N
    roof = dict(res["roofline"])
    traffic, src = _recorded_traffic(args.config)
    roof.update({"traffic": traffic,
                 "traffic_source": None if src is None else f"recorded in {src} (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE "
                                                            "runs of this command), not measured in this run",
                 "algorithmic_bytes": priv["gemm1_bytes"], "avg_launch_ms": res["gemm1_ms"],
                 "flop_per_launch": priv["gemm1_flop"]})
    kernels = {"gemm1_ms": res["gemm1_ms"], "gemm2_ms": res["gemm2_ms"],
               "gemm1_tflops": res["gemm1_tflops"], "gemm2_tflops": res["gemm2_tflops"],
               "gemm1_frac_mfma": res["gemm1_tflops"] / FP8_PEAK_TFLOPS, "gemm2_frac_mfma": res["gemm2_tflops"] / FP8_PEAK_TFLOPS,
               "gemm1_frac_hbm": res["gemm1_GBs"] / HBM_PEAK_GBS, "gemm2_frac_hbm": res["gemm2_GBs"] / HBM_PEAK_GBS,
               "quantize_fanout_GBs": qf_bytes / (stages["quantize_fanout_unfused"] * 1e-3) / 1e9,
               "quantize_fanout_frac_hbm": qf_bytes / (stages["quantize_fanout_unfused"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
               "quantize_GBs": q_bytes / (stages["quantize"] * 1e-3) / 1e9,
               "quantize_frac_hbm": q_bytes / (stages["quantize"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
               "combine_GBs": c_bytes / (stages["combine"] * 1e-3) / 1e9,
               "combine_frac_hbm": c_bytes / (stages["combine"] * 1e-3) / 1e9 / HBM_PEAK_GBS}
    if stages["route"]:
        kernels["route_GBs"] = r_bytes / (stages["route"] * 1e-3) / 1e9
        kernels["route_frac_hbm"] = kernels["route_GBs"] / HBM_PEAK_GBS
    out = {
        "metric": "MoE-layer fwd FP8 TFLOP/s (% MFMA peak) + tokens/s, routed vs replay",
        "value": res["tflops"], "unit": "TFLOP/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_head, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "fp8", "data": "synthetic",
        "config": {"workload": f"{res['workload']}, mode={head_mode}",
                   "T": T, "d": d, "E": cfg.E, "k": k, "F": F, "mode": head_mode},
        "pct_mfma_peak_whole_step": 100.0 * res["tflops"] / FP8_PEAK_TFLOPS,
        "tokens_per_s": res["tokens_per_s"],
        "routed": None if res["routed_ms"] is None else {"ms_per_step": res["routed_ms"], "tokens_per_s": T / (res["routed_ms"] * 1e-3),
                                                         "tflops": priv["flop"] / (res["routed_ms"] * 1e-3) / 1e12},
        "replay": {"ms_per_step": res["replay_ms"], "tokens_per_s": T / (res["replay_ms"] * 1e-3),
                   "tflops": priv["flop"] / (res["replay_ms"] * 1e-3) / 1e12},
        "stages_ms": stages,
        "kernels": kernels,
        "roofline": roof,
        "ceilings": None if args.no_extensions else _ceilings(torch, moe, layer.ctx, dev),
        "configs": others,
    }
    # the entry points beyond the five core calls, timed outside the headline region (same resident inputs)
    ext = {}
    if args.no_extensions:
        rows_l = rows_w = 0
    elif "routed" in cfg.modes:
        ext["route_replay_ids_ms"] = _stage_ms(torch, lambda: layer.route_replay_ids(x, W_r, log_idx))
    if not args.no_extensions:
        rows_w = min(cfg.E * F, 16 * 4096)                    # a slab of bf16 gate weights of 16*4096 rows
        w_bf16 = torch.randn((rows_w, d), device=dev, dtype=torch.float32).mul_(d ** -0.5).to(torch.bfloat16)
        wq = torch.empty((rows_w, d), dtype=torch.uint8, device=dev)
        wsc = torch.empty((rows_w // 128, d // 128), dtype=torch.float32, device=dev)
        t_wq = _stage_ms(torch, lambda: moe.moe_quantize_weights_fp8(layer.ctx, w_bf16, rows_w, d, wq, wsc))
        ext["weight_quant_ms"] = t_wq
        ext["weight_quant_GBs"] = 3.0 * rows_w * d / (t_wq * 1e-3) / 1e9
        ext["weight_quant_frac_hbm"] = ext["weight_quant_GBs"] / HBM_PEAK_GBS
        rows_l = min(8192, N)                                 # dense linear: [rows_l, d] x [rows_w, d]^T
    if rows_l and rows_l * rows_w <= N * d:                   # y_perm doubles as the output buffer
        xs_l = layer.xs[:, :rows_l].contiguous()
        t_lin = _stage_ms(torch, lambda: moe.moe_linear_fp8(layer.ctx, layer.xq, xs_l, rows_l, d, wq, wsc, rows_w,
                                                            layer.y_perm), reps=5)
        ext["dense_linear_ms"] = t_lin
        ext["dense_linear_tflops"] = 2.0 * rows_l * d * rows_w / (t_lin * 1e-3) / 1e12
        ext["dense_linear_shape"] = [rows_l, d, rows_w]
    out["extensions"] = ext
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
