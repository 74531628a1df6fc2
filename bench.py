#!/usr/bin/env python3
"""Benchmark of the decode-time MoE block on one MI355X.

Workload (default): one Mixtral-8x7B-shaped MoE layer in bf16 (H 4096, F 14336,
8 experts, adaptive top-2 with threshold 0.2), all experts resident in HBM,
256 AR(1)-correlated batch-1 decode tokens cycled.  A step is one token through
the whole block: gate + adaptive test, residency lookup, expert GEMVs, combine.
Inputs are synthetic and already in HBM when the timed region starts.

Prints one JSON line: decode tokens/s for the layer, the roofline figures of
the dominant kernel (gate/up GEMV) from HIP-event timing, and the CPU checker
timed on a bounded sample of the same tokens as a baseline.
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

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2048)
    ap.add_argument("--warmup", type=int, default=256)
    ap.add_argument("--tokens", type=int, default=256, help="distinct decode tokens cycled through")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget for the CPU-checker baseline (0 = skip)")
    ap.add_argument("--workload", default="mixtral_layer_bf16", choices=["mixtral_layer_bf16", "tiny_f32"])
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2408_10284_amd import binding as B
    from paper_2408_10284_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    if not os.path.exists(B.LIB_PATH):
        from paper_2408_10284_amd import build
        build.build(verbose=False)

    if args.workload == "tiny_f32":
        shape, tau, act = synth.TINY, 0.3, "f32"
        X = synth.iid_tokens(args.tokens, shape.H, seed=1, dtype="f32")
    else:
        shape, tau, act = synth.MIXTRAL_LAYER, 0.2, "bf16"
        X = synth.ar1_tokens(args.tokens, shape.H, 0.8, seed=1, dtype="bf16")
    esz = 4 if act == "f32" else 2
    dt = B.F32 if act == "f32" else B.BF16

    t_setup = time.time()
    ctx, cfg = B.adapmoe_create(shape.H, shape.F, shape.N, shape.L, dt, max_B=1)
    nbytes = B.adapmoe_expert_bytes(cfg)
    keep = []

    def dev(a):
        if act == "f32":
            return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
        return torch.from_numpy(synth.bf16_bits(a).view(np.int16)).cuda()

    def bits(a):
        return a if act == "f32" else synth.bf16_bits(a)

    wg = synth.router_weights(shape, 0)
    wg_d = dev(wg)
    B.adapmoe_set_router(ctx, 0, wg_d)
    B.adapmoe_set_tau(ctx, [tau])
    experts = []
    for e in range(shape.N):
        w1, w3, w2 = synth.expert_weights(shape, 0, e)
        experts.append((w1, w3, w2))
        img = np.empty(nbytes, dtype=np.uint8)
        B.adapmoe_pack_expert(cfg, bits(w1), bits(w3), bits(w2), img)
        t = torch.from_numpy(img).cuda()
        keep.append(t)
        B.adapmoe_bind_expert_dev(ctx, 0, e, t)
    xd = dev(X).reshape(args.tokens, shape.H)
    y = torch.empty((1, shape.H), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    rows = [xd[i:i + 1] for i in range(args.tokens)]
    ptrs = [r.data_ptr() for r in rows]
    t_setup = time.time() - t_setup

    # the gate's decisions for these tokens (needed to count the bytes the kernels read)
    ids = torch.empty((args.tokens, 2), dtype=torch.int32, device="cuda")
    w = torch.empty((args.tokens, 2), dtype=torch.float32, device="cuda")
    k = torch.empty(args.tokens, dtype=torch.int32, device="cuda")
    for i in range(args.tokens):
        B.moe_gate(ctx, 0, ptrs[i], 1, ids[i:i + 1], w[i:i + 1], k[i:i + 1])
    torch.cuda.synchronize()
    k_host = k.cpu().numpy()

    def run(n, start=0):
        for s in range(n):
            B.moe_layer_step(ctx, 0, ptrs[(start + s) % args.tokens], 1, y, stream)

    run(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps, args.warmup)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    B.adapmoe_check(ctx)
    elapsed = t1 - t0
    tok_s = args.steps / elapsed
    us_per_layer = elapsed / args.steps * 1e6

    # second pass with HIP events around each kernel launch, on the launch stream
    B.adapmoe_profile(ctx, True)
    run(args.steps, args.warmup)
    torch.cuda.synchronize()
    n_gu, ms_gu = B.adapmoe_profile_read(ctx, 0)
    n_dn, ms_dn = B.adapmoe_profile_read(ctx, 1)
    n_gt, ms_gt = B.adapmoe_profile_read(ctx, 2)
    B.adapmoe_profile(ctx, False)
    ks = np.array([k_host[(args.warmup + s) % args.tokens] for s in range(args.steps)], dtype=np.float64)
    bytes_gu = float(ks.sum()) * 2 * shape.H * shape.F * esz      # W1 and W3 of every activated expert
    bytes_dn = float(ks.sum()) * shape.H * shape.F * esz          # W2 of every activated expert
    gu_gbs = bytes_gu / (ms_gu * 1e-3) / 1e9
    dn_gbs = bytes_dn / (ms_dn * 1e-3) / 1e9
    ffn_gbs = (bytes_gu + bytes_dn) / ((ms_gu + ms_dn) * 1e-3) / 1e9

    cpu = None
    if args.cpu_seconds > 0:
        cpu = cpu_baseline(args, shape, X, wg, experts, tau)

    out = {
        "metric": "decode tokens/s + us per MoE layer; expert-GEMV HBM GB/s as % of peak",
        "value": round(tok_s, 2),
        "unit": "tokens/s (one MoE layer, batch 1)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(elapsed / args.steps * 1e3, 6),
        "us_per_layer": round(us_per_layer, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": act, "data": "synthetic",
        "config": {"workload": f"{args.workload}: H={shape.H} F={shape.F} N={shape.N} L=1, tau={tau}, "
                               f"{args.tokens} AR(1) decode tokens cycled, experts resident in HBM",
                   "mean_k": round(float(ks.mean()), 4), "single_expert_ratio": round(float((ks == 1).mean()), 4),
                   "setup_s": round(t_setup, 1)},
        "roofline": {"bound": "hbm", "kernel": "ffn_gateup_kernel", "achieved": round(gu_gbs, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(gu_gbs / HBM_PEAK_GBS, 4), "traffic": None,
                     "avg_us": round(ms_gu / max(n_gu, 1) * 1e3, 2), "launches": n_gu,
                     "bytes_per_launch": round(bytes_gu / max(n_gu, 1))},
        "kernels": {"ffn_down_kernel": {"achieved_GBs": round(dn_gbs, 1), "frac": round(dn_gbs / HBM_PEAK_GBS, 4),
                                        "avg_us": round(ms_dn / max(n_dn, 1) * 1e3, 2)},
                    "gate_kernel": {"avg_us": round(ms_gt / max(n_gt, 1) * 1e3, 2)},
                    "ffn_both": {"achieved_GBs": round(ffn_gbs, 1), "frac": round(ffn_gbs / HBM_PEAK_GBS, 4)},
                    "whole_step_GBs": round((bytes_gu + bytes_dn) / elapsed / 1e9, 1)},
        "cpu_baseline": cpu,
    }
    torch.cuda.synchronize()
    B.adapmoe_destroy(ctx)
    print(json.dumps(out))


def cpu_baseline(args, shape, X, wg, experts, tau):
    """The CPU checker, as it stands, on the first tokens of the same stream."""
    import numpy as np
    from oracle import expert as OE
    from oracle import gate as OG
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = 1
    n = 0
    t0 = time.perf_counter()
    c0 = time.process_time()
    while n < args.tokens:
        g = OG.adaptive_gate(X[n], wg, np.float32(tau))
        OE.moe_block(X[n], experts, g["ids"], g["w"], g["k"])
        n += 1
        if time.perf_counter() - t0 > args.cpu_seconds:
            break
    dt = time.perf_counter() - t0
    cpu_t = time.process_time() - c0
    return {"value": round(n / dt, 4), "unit": "tokens/s (one MoE layer, batch 1)", "cores": int(threads), "kind": "oracle",
            "sample": f"first {n} of the {args.tokens} tokens, float64 NumPy checker, {dt:.1f} s wall, "
                      f"cpu/wall {cpu_t / dt:.1f}, host has {os.cpu_count()} logical CPUs"}


if __name__ == "__main__":
    main()
