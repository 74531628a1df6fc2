#!/usr/bin/env python3
"""Benchmark of the decode-time MoE block on one MI355X.

Default workload `mixtral_layer_bf16`: one Mixtral-8x7B-shaped MoE layer in bf16
(H 4096, F 14336, 8 experts, adaptive top-2 with threshold 0.2), all experts
resident in HBM, 256 AR(1)-correlated batch-1 decode tokens cycled.  A step is
one token through the whole block: gate + adaptive test, residency lookup,
expert GEMVs, combine.  Inputs are synthetic and already in HBM when the timed
region starts.

Prints one JSON line: decode tokens/s for the layer, the roofline figures of the
dominant kernel from HIP-event timing on the launch stream (with a load-only
kernel of the same access pattern timed beside it), and the CPU checker timed on
a bounded sample of the same tokens as a baseline.  With no flags the record also
carries, under "stacks", short runs of the 32-layer resident stack, the 32-layer
batched stack and the int4 layer.

Other workloads (same JSON shape, selected with --workload):
  mixtral_layer_int4     same layer with group-64 int4 experts (dequantisation fused)
  mixtral_layer_int2     same layer with group-64 2-bit experts
  mixtral22_layer_bf16 / _int4 / _int2   one layer with Mixtral-8x22B expert shapes (H 6144, F 16384)
  mixtral_stack_resident 32 layers, all experts resident in HBM (90 GB bf16), batch-1 decode through the whole stack
  mixtral_stack_offload  L-layer stack, experts in host memory (pinned, or pageable with --staging), bounded HBM
                         cache sized by the planner, LRU + next-layer prefetch (host-link bound);
                         --dtype int4|int2, --model 8x22b, --layers, --cache, --lookahead, --tiles
  mixtral_batched        16 decode streams per step, experts resident, MFMA grouped GEMM
  tiny_f32               the small fp32 layer
--opt NAME=VALUE sets a library option (adapmoe_set_option) for the benchmarked context.
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
METRIC = "decode tokens/s + \u00b5s per MoE layer; expert-GEMV HBM GB/s as % of peak"   # the metric string of the benchmark spec


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--tokens", type=int, default=256, help="distinct decode tokens cycled through")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget for the CPU-checker baseline (0 = skip)")
    ap.add_argument("--workload", default="mixtral_layer_bf16",
                    choices=["mixtral_layer_bf16", "mixtral_layer_int4", "mixtral_layer_int2", "tiny_f32", "mixtral_stack_offload",
                             "mixtral_batched", "mixtral_stack_resident", "mixtral22_layer_bf16", "mixtral22_layer_int4",
                             "mixtral22_layer_int2"])
    ap.add_argument("--stacks", type=int, default=None,
                    help="1: add short runs of the multi-layer and int4 workloads to the record (default for the default workload), 0: do not")
    ap.add_argument("--layers", type=int, default=None, help="layers of the stack workloads (default: offload 14, batched 32)")
    ap.add_argument("--cache", type=int, default=None, help="total cache slots of the offload workload (default 2 per layer)")
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "int4", "int2"], help="expert storage of the offload workload")
    ap.add_argument("--tiles", type=int, default=0, help="offload workload: tile-wise loading with this many gate/up tiles (0 = whole images)")
    ap.add_argument("--staging", type=int, default=0,
                    help="offload workload: expert images in pageable host memory, loads staged through this many pinned buffers "
                         "(for stacks larger than the box lets a process pin, e.g. --layers 32 in bf16)")
    ap.add_argument("--staging-threads", type=int, default=8, help="offload workload: host threads that fill a staging buffer together")
    ap.add_argument("--lookahead", type=int, default=1, help="offload workload: layers predicted and prefetched ahead (1..3)")
    ap.add_argument("--model", default="8x7b", choices=["8x7b", "8x22b"],
                    help="offload workload: expert shapes and depth of Mixtral-8x7B (H 4096, F 14336, 32 layers) or of "
                         "Mixtral-8x22B (H 6144, F 16384, 56 layers; quantised experts only, staged from pageable memory)")
    ap.add_argument("--graph", action="store_true", help="mixtral_stack_resident: replay one captured HIP graph per token")
    ap.add_argument("--opt", action="append", default=[], metavar="NAME=VALUE",
                    help="library option for the benchmarked context, e.g. GATEUP_BLOCKS=768 (names of adapmoe_set_option)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference kernel for the HBM byte counters)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2408_10284_amd import binding as B
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    if not os.path.exists(B.LIB_PATH):
        from paper_2408_10284_amd import build
        build.build(verbose=False)
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    if args.workload == "mixtral_stack_offload":
        out = bench_stack_offload(args)
    elif args.workload == "mixtral_batched":
        out = bench_batched(args)
    elif args.workload == "mixtral_stack_resident":
        out = bench_stack_resident(args)
    else:
        out = bench_layer(args)
        want_stacks = args.stacks if args.stacks is not None else int(args.workload == "mixtral_layer_bf16" and args.steps is None)
        if want_stacks:
            out["stacks"] = bench_stacks(args)
    print(json.dumps(out))


def apply_options(ctx, args):
    from paper_2408_10284_amd import binding as B
    for item in args.opt:
        name, value = item.split("=")
        B.adapmoe_set_option(ctx, getattr(B, "OPT_" + name.upper()), int(value))


class _LazyList:
    """list-like whose items are produced on first use (expert matrices read back from device images)."""

    def __init__(self, n, make):
        self.n, self.make, self.cache = n, make, {}

    def __len__(self):
        return self.n

    def __getitem__(self, i):
        if i not in self.cache:
            self.cache[i] = self.make(i)
        return self.cache[i]


def cpu_baseline_stack(shape, routers, images_dev, taus, h0, gamma, budget_s, n_layers, what):
    """The CPU checker's multi-layer loop (oracle/stack.py), as it stands, on the first tokens of the same stream
    through the first `n_layers` layers (reading the experts back from the device images costs more time than
    evaluating them, so the sample is bounded by layers as well as by tokens).  The rate is scaled to the full depth."""
    import numpy as np
    import torch
    from oracle import expert as OE
    from oracle import stack as OS
    from paper_2408_10284_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = 1
    L = min(n_layers, shape.L)
    cache = {}

    def mats(l, e):
        if (l, e) not in cache:
            img = images_dev[l][e]
            if shape.dtype == "bf16":
                cache[(l, e)] = synth.unpack_image_bf16(img.view(torch.int16).cpu().numpy().view(np.uint16), shape.H, shape.F)
            else:
                dec = synth.decode_int4_image if shape.dtype == "int4g64" else synth.decode_int2_image
                cache[(l, e)] = tuple(OE.decode_int4(q, s, z) for (q, s, z) in dec(img.cpu().numpy(), shape.H, shape.F))
        return cache[(l, e)]

    routers_f32 = [routers[l].float().cpu().numpy() for l in range(L)]
    n = 0
    t0 = time.perf_counter()
    while n < h0.shape[0] and time.perf_counter() - t0 < budget_s:
        OS.run_stack(h0[n:n + 1].astype(np.float64), routers_f32, [np.float32(t) for t in taus[:L]],
                     lambda l, e, x: OE.expert_ffn(x, *mats(l, e)), gamma, store=synth.bf16_round)
        n += 1
    dt = time.perf_counter() - t0
    return {"value": round(n * L / dt / shape.L, 4), "unit": f"tokens/s ({shape.L}-layer stack)", "cores": int(threads), "kind": "oracle",
            "sample": f"{what}: first {n} token(s) through the first {L} of {shape.L} layers with the float64 NumPy checker "
                      f"(oracle/stack.py), {dt:.1f} s wall incl. reading the experts back from HBM; rate scaled to {shape.L} layers; "
                      f"host has {os.cpu_count()} logical CPUs"}


def read_decisions(ctx, logbuf, n_records, max_B, Bt):
    """(ids [n,Bt,2], k [n,Bt]) from a decision-log buffer."""
    rec = logbuf[:n_records].cpu().numpy().reshape(n_records, 6 * max_B)
    return rec[:, :2 * Bt].reshape(n_records, Bt, 2), rec[:, 2 * Bt:3 * Bt]


def bench_stacks(args):
    """Short runs of the other workloads of the path, for the default record: the 32-layer stack with all experts
    resident at batch 1 and with 16 streams (the same 90 GB of images), and the int4 layer."""
    import copy
    out = {}
    shared = {}
    a = copy.copy(args)
    a.steps, a.warmup, a.layers, a.graph = 64, 8, None, False
    a.cpu_seconds = min(args.cpu_seconds, 12.0)
    try:
        out["mixtral_stack_resident"] = bench_stack_resident(a, shared)
        a.steps, a.warmup = 24, 4
        out["mixtral_batched"] = bench_batched(a, shared)
    finally:
        shared.clear()
        import torch
        torch.cuda.empty_cache()
    a = copy.copy(args)
    a.workload, a.steps, a.warmup, a.gpu_images = "mixtral_layer_int4", 1024, 128, True
    a.cpu_seconds = min(args.cpu_seconds, 10.0)
    out["mixtral_layer_int4"] = bench_layer(a)
    for rec in out.values():      # the sub-records repeat only what differs from the headline record
        for key in ("metric", "n_gpus", "higher_is_better", "scaling", "vs_baseline", "data"):
            rec.pop(key, None)
    return out


# --------------------------------------------------------------------------- one layer, batch 1 ----

def bench_layer(args):
    import numpy as np
    import torch

    from paper_2408_10284_amd import binding as B
    from paper_2408_10284_amd import synth

    steps = args.steps if args.steps is not None else 2048
    warmup = args.warmup if args.warmup is not None else 256
    wl = args.workload
    big = wl.startswith("mixtral22")                 # Mixtral-8x22B expert shape (Sec. 6.1): H 6144, F 16384
    Hh, Ff = (6144, 16384) if big else (4096, 14336)
    gpu_images = big or getattr(args, "gpu_images", False)    # images drawn and packed on the GPU (seconds instead of minutes)
    if wl == "tiny_f32":
        shape, tau, act, dt = synth.TINY, 0.3, "f32", B.F32
        X = synth.iid_tokens(args.tokens, shape.H, seed=1, dtype="f32")
    elif wl.endswith("int4") or wl.endswith("int2"):
        four = wl.endswith("int4")
        shape = synth.MoEShape(Hh, Ff, 8, 1, "int4g64" if four else "int2g64")
        tau, act, dt = 0.2, "bf16", (B.INT4G64 if four else B.INT2G64)
        X = synth.ar1_tokens(args.tokens, shape.H, 0.8, seed=1, dtype="bf16")
    else:
        shape, tau, act, dt = synth.MoEShape(Hh, Ff, 8, 1, "bf16"), 0.2, "bf16", B.BF16
        X = synth.ar1_tokens(args.tokens, shape.H, 0.8, seed=1, dtype="bf16")

    t_setup = time.time()
    ctx, cfg = B.adapmoe_create(shape.H, shape.F, shape.N, shape.L, dt, max_B=1)
    apply_options(ctx, args)
    nbytes = B.adapmoe_expert_bytes(cfg)
    keep = []

    def dev(a):
        if act == "f32":
            return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
        return torch.from_numpy(synth.bf16_bits(a).view(np.int16)).cuda()

    if gpu_images:
        wg_t = synth.router_bf16_torch(shape, 0, 0)
        wg = wg_t.float().cpu().numpy()
        wg_d = wg_t
    else:
        wg = synth.router_weights(shape, 0)
        wg_d = dev(wg)
    B.adapmoe_set_router(ctx, 0, wg_d)
    B.adapmoe_set_tau(ctx, [tau])
    experts = []        # what the CPU baseline evaluates: float32 matrices (codes, scales, zeros for int4), or None = decode the image
    for e in range(shape.N):
        if gpu_images:
            gen = {B.INT4G64: synth.expert_image_int4_torch, B.INT2G64: synth.expert_image_int2_torch}.get(dt, synth.expert_image_bf16_torch)
            t = gen(shape, 0, e, 0)
            assert t.numel() * t.element_size() == nbytes
            keep.append(t)
            experts.append(None)
            B.adapmoe_bind_expert_dev(ctx, 0, e, t)
            continue
        w1, w3, w2 = synth.expert_weights(shape, 0, e)
        img = np.empty(nbytes, dtype=np.uint8)
        if dt in (B.INT4G64, B.INT2G64):
            quant, pack = ((synth.quantize_int4_g64, B.adapmoe_pack_expert_int4) if dt == B.INT4G64
                           else (synth.quantize_int2_g64, B.adapmoe_pack_expert_int2))
            qs = [quant(m) for m in (w1, w3, w2)]
            pack(cfg, *[a for (q, s, z) in qs for a in (q, s.view(np.uint16), z.view(np.uint16))], img)
            experts.append(qs)
        elif dt == B.BF16:
            B.adapmoe_pack_expert(cfg, synth.bf16_bits(w1), synth.bf16_bits(w3), synth.bf16_bits(w2), img)
            experts.append((w1, w3, w2))
        else:
            B.adapmoe_pack_expert(cfg, w1, w3, w2, img)
            experts.append((w1, w3, w2))
        t = torch.from_numpy(img).cuda()
        keep.append(t)
        B.adapmoe_bind_expert_dev(ctx, 0, e, t)
    if gpu_images:
        torch.cuda.synchronize()

        def image_mats(e):      # canonical matrices of expert e for the CPU baseline, read back from the image
            if dt == B.BF16:
                return synth.unpack_image_bf16(keep[e].view(torch.int16).cpu().numpy().view(np.uint16), shape.H, shape.F)
            dec = synth.decode_int4_image if dt == B.INT4G64 else synth.decode_int2_image
            return dec(keep[e].cpu().numpy(), shape.H, shape.F)
        experts = _LazyList(shape.N, image_mats)
    xd = dev(X).reshape(args.tokens, shape.H)
    y = torch.empty((1, shape.H), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    ptrs = [xd[i:i + 1].data_ptr() for i in range(args.tokens)]
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

    run(warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(steps, warmup)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    B.adapmoe_check(ctx)
    elapsed = t1 - t0

    # second pass with a pair of HIP events tied to each kernel dispatch, on the launch stream (the kernel's execution time)
    B.adapmoe_profile(ctx, True)
    run(steps, warmup)
    torch.cuda.synchronize()
    n_gu, ms_gu = B.adapmoe_profile_read(ctx, 0)
    n_dn, ms_dn = B.adapmoe_profile_read(ctx, 1)
    n_gt, ms_gt = B.adapmoe_profile_read(ctx, 2)
    n_fu, ms_fu = B.adapmoe_profile_read(ctx, 6)
    B.adapmoe_profile(ctx, False)
    fused = n_gu == 0 and n_fu > 0          # ADAPMOE_FUSED: both GEMVs in one launch, timed as one kernel
    if fused:
        n_gu, ms_gu, n_dn, ms_dn = n_fu, ms_fu * 2.0 / 3.0, n_fu, ms_fu / 3.0
    ks = np.array([k_host[(warmup + s) % args.tokens] for s in range(steps)], dtype=np.float64)
    per_matrix = nbytes / 3.0                                     # bytes of one of the three matrices of an expert
    bytes_gu = float(ks.sum()) * 2 * per_matrix                   # W1 and W3 of every activated expert
    bytes_dn = float(ks.sum()) * per_matrix                       # W2 of every activated expert
    gu_gbs = bytes_gu / (ms_gu * 1e-3) / 1e9
    dn_gbs = bytes_dn / (ms_dn * 1e-3) / 1e9
    ffn_gbs = (bytes_gu + bytes_dn) / ((ms_gu + ms_dn) * 1e-3) / 1e9

    quantised = dt in (B.INT4G64, B.INT2G64)
    # what this machine's memory system does on a plain device-to-device copy (1 GiB read + 1 GiB written per copy)
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(5):
        dst.copy_(src)
    ev1.record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * float(1 << 30) / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del src, dst

    # what the memory system delivers for the gate/up kernel's access pattern with no arithmetic at all: a load-only
    # kernel of the library, same number of workgroups, same bytes as a launch with one and with two activated experts
    probe = None
    if not quantised and not fused and shape.H * (4 if act == "f32" else 2) in (1024, 2048, 4096, 8192, 16384):
        row_bytes = shape.H * (4 if act == "f32" else 2)
        wgs = B.adapmoe_get_option(ctx, B.OPT_GATEUP_BLOCKS)
        pbuf = torch.empty(2 * 2 * shape.F * row_bytes, dtype=torch.uint8, device="cuda").fill_(1)
        us = {kx: B.adapmoe_stream_probe(pbuf, kx * 2 * shape.F, row_bytes, 2, row_bytes, wgs, 20) for kx in (1, 2)}
        del pbuf
        n1, n2 = float((ks == 1).sum()), float((ks == 2).sum())
        avg = (n1 * us[1] + n2 * us[2]) / max(n1 + n2, 1.0)
        probe = {"pattern": "a wavefront reads whole row pairs one after the other, two 16 KiB buffers in flight, "
                            f"{wgs} workgroups of 256 threads, loads only",
                 "us_one_expert": round(us[1], 2), "us_two_experts": round(us[2], 2),
                 "GBs_two_experts": round(2 * 2 * per_matrix / (us[2] * 1e-6) / 1e9, 1),
                 "us_for_this_run's_k": round(avg, 2), "kernel_over_probe": round(ms_gu / max(n_gu, 1) * 1e3 / avg, 4)}

    cpu = cpu_baseline_layer(args, shape, X, wg, experts, tau, quantised) if args.cpu_seconds > 0 else None
    gu_name = "ffn_fused_kernel" if fused else ("ffn_gateup_quant_kernel" if quantised else "ffn_gateup_kernel")
    # HBM bytes per launch from the committed counter runs of this workload.  Those runs launch every one of the
    # 256 tokens once, so their per-launch average belongs to the mean k of the token set; it is scaled to the
    # mean k of the launches timed here (one launch reads k experts).
    per_launch_ref = {"mixtral_layer_bf16": measured_traffic(gu_name),
                      "mixtral_layer_int4": measured_traffic("ffn_gateup_quant_kernel<4", "pmc_traffic_int4.json")}.get(args.workload)
    traffic = round(per_launch_ref / float(k_host.mean()) * float(ks.mean())) if per_launch_ref and args.tokens == 256 else None
    out = {
        "metric": METRIC, "value": round(steps / elapsed, 2), "unit": "tokens/s (one MoE layer, batch 1)",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(elapsed / steps * 1e3, 6), "us_per_layer": round(elapsed / steps * 1e6, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {B.INT4G64: "int4", B.INT2G64: "int2"}.get(dt, act), "data": "synthetic",
        "config": {"workload": f"{args.workload}: H={shape.H} F={shape.F} N={shape.N} L=1, tau={tau}, "
                               f"{args.tokens} AR(1) decode tokens cycled, experts resident in HBM",
                   "mean_k": round(float(ks.mean()), 4), "single_expert_ratio": round(float((ks == 1).mean()), 4),
                   "expert_bytes": nbytes, "setup_s": round(t_setup, 1)},
        "roofline": {"bound": "hbm", "kernel": gu_name, "achieved": round(gu_gbs, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(gu_gbs / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "traffic_note": "HBM bytes per launch (read + written) from profiles/pmc_traffic*.json, scaled from the mean k of "
                                     "the counter runs to the mean k of the launches timed here",
                     "avg_us": round(ms_gu / max(n_gu, 1) * 1e3, 2), "launches": n_gu,
                     "bytes_per_launch": round(bytes_gu / max(n_gu, 1)),
                     "measured_device_copy_GBs": round(copy_gbs, 1), "frac_of_device_copy": round(gu_gbs / copy_gbs, 4),
                     "stream_probe": probe},
        "kernels": {"down": {"achieved_GBs": round(dn_gbs, 1), "frac": round(dn_gbs / HBM_PEAK_GBS, 4),
                             "avg_us": round(ms_dn / max(n_dn, 1) * 1e3, 2)},
                    "gate": {"avg_us": round(ms_gt / max(n_gt, 1) * 1e3, 2)},
                    "ffn_both": {"achieved_GBs": round(ffn_gbs, 1), "frac": round(ffn_gbs / HBM_PEAK_GBS, 4)},
                    "whole_step_GBs": round((bytes_gu + bytes_dn) / elapsed / 1e9, 1),
                    "whole_step_frac": round((bytes_gu + bytes_dn) / elapsed / 1e9 / HBM_PEAK_GBS, 4)},
        "cpu_baseline": cpu,
    }
    torch.cuda.synchronize()
    B.adapmoe_destroy(ctx)
    return out


def measured_traffic(kernel, summary="pmc_traffic.json"):
    """HBM bytes per launch (read + write) of `kernel` from the committed rocprofv3 --pmc summary
    of this workload (FETCH_SIZE and WRITE_SIZE scaled by a plain copy), or None."""
    path = os.path.join(ROOT, "profiles", summary)
    try:
        with open(path) as f:
            data = json.load(f)
        for name, v in data["kernels"].items():
            if kernel in name:
                return round(v["fetch_bytes_per_launch"] + v["write_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        pass
    return None


def cpu_baseline_layer(args, shape, X, wg, experts, tau, int4):
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
        if int4:
            # the checker decodes the activated experts from the same codes, scales and zeros
            ex = {e: tuple(OE.decode_int4(q, s, z) for (q, s, z) in experts[e]) for e in g["ids"][: g["k"]]}
            OE.combine(g["ids"], g["w"], g["k"], lambda e: OE.expert_ffn(X[n], *ex[e]))
        else:
            OE.moe_block(X[n], experts, g["ids"], g["w"], g["k"])
        n += 1
        if time.perf_counter() - t0 > args.cpu_seconds:
            break
    dt = time.perf_counter() - t0
    cpu_t = time.process_time() - c0
    return {"value": round(n / dt, 4), "unit": "tokens/s (one MoE layer, batch 1)", "cores": int(threads), "kind": "oracle",
            "sample": f"first {n} of the {args.tokens} tokens, float64 NumPy checker, {dt:.1f} s wall, "
                      f"cpu/wall {cpu_t / dt:.1f}, host has {os.cpu_count()} logical CPUs"}


# --------------------------------------------------------------------------- stack helpers ----

def build_stack(shape, seed, keep_on_device, pin_host, pageable=False):
    """Routers and expert images of an L-layer stack drawn on the GPU.  Returns
    (routers_dev[L], images_dev[L][N] or None, images_host[L][N] or None)."""
    import torch

    from paper_2408_10284_amd import synth
    routers, dev, host = [], [], []
    for l in range(shape.L):
        routers.append(synth.router_bf16_torch(shape, l, seed))
        drow, hrow = [], []
        for e in range(shape.N):
            if shape.dtype == "int2g64":
                img = synth.expert_image_int2_torch(shape, l, e, seed)
            elif shape.dtype == "int4g64":
                img = synth.expert_image_int4_torch(shape, l, e, seed)
            else:
                img = synth.expert_image_bf16_torch(shape, l, e, seed)
            if pin_host:
                h = torch.empty(img.numel(), dtype=img.dtype, pin_memory=not pageable)
                h.copy_(img)
                hrow.append(h)
            if keep_on_device:
                drow.append(img)
        dev.append(drow)
        host.append(hrow)
    torch.cuda.synchronize()
    return routers, (dev if keep_on_device else None), (host if pin_host else None)


def profile_gate_statistics(shape, routers, images_dev, taus, h0, gamma):
    """Offline profiling (Sec. 4.4.1): single-expert probability a_l and prefetch
    accuracy beta_l of every layer, from the library's own gate decisions on a
    warm-up stream with all experts resident.  Values rounded to 1/1024."""
    import numpy as np
    import torch

    from paper_2408_10284_amd import binding as B
    L, N, H = shape.L, shape.N, shape.H
    dt = {"int4g64": B.INT4G64, "int2g64": B.INT2G64}.get(shape.dtype, B.BF16)
    ctx, cfg = B.adapmoe_create(H, shape.F, N, L, dt, max_B=1)
    try:
        for l in range(L):
            B.adapmoe_set_router(ctx, l, routers[l])
            for e in range(N):
                B.adapmoe_bind_expert_dev(ctx, l, e, images_dev[l][e])
        B.adapmoe_set_tau(ctx, taus)
        n = h0.shape[0]
        ids = torch.empty((n, L, 2), dtype=torch.int32, device="cuda")
        w = torch.empty((n, L, 2), dtype=torch.float32, device="cuda")
        k = torch.empty((n, L), dtype=torch.int32, device="cuda")
        pids = torch.empty((n, L, 2), dtype=torch.int32, device="cuda")
        pk = torch.empty((n, L), dtype=torch.int32, device="cuda")
        x = torch.empty((1, H), dtype=torch.bfloat16, device="cuda")
        y = torch.empty((1, H), dtype=torch.float32, device="cuda")
        cos = []
        for t in range(n):
            h = h0[t:t + 1].clone()
            xprev = None
            for l in range(L):
                B.moe_residual_rmsnorm(ctx, h, y if l > 0 else None, gamma, x, 1)
                if t < 4:
                    xf = x.float()
                    if xprev is not None:
                        cos.append(float(torch.nn.functional.cosine_similarity(xf, xprev).item()))
                    xprev = xf.clone()
                B.moe_gate(ctx, l, x, 1, ids[t, l:l + 1], w[t, l:l + 1], k[t, l:l + 1], pids[t, l:l + 1], pk[t, l:l + 1])
                B.moe_expert_ffn(ctx, l, x, 1, ids[t, l:l + 1], w[t, l:l + 1], k[t, l:l + 1], y)
        B.adapmoe_check(ctx)
        ids, k, pids, pk = ids.cpu().numpy(), k.cpu().numpy(), pids.cpu().numpy(), pk.cpu().numpy()
    finally:
        B.adapmoe_destroy(ctx)
    a = np.zeros(L)
    beta = np.zeros(L)
    for l in range(L):
        a[l] = np.mean(k[:, l] == 1)
        if l == 0:
            beta[l] = 0.0       # nothing predicts layer 0
            continue
        hit = tot = 0
        for t in range(n):
            act = set(ids[t, l, :k[t, l]].tolist())
            pred = set(pids[t, l - 1, :pk[t, l - 1]].tolist())
            hit += len(act & pred)
            tot += len(act)
        beta[l] = hit / tot
    return np.round(a * 1024) / 1024, np.round(beta * 1024) / 1024, float(np.mean(cos)) if cos else None


# --------------------------------------------------------------------------- offloaded stack ----

def bench_stack_offload(args):
    import numpy as np
    import torch

    from paper_2408_10284_amd import binding as B
    from paper_2408_10284_amd import synth

    # The test machines pin at most ~46 GB of host memory (hipHostMalloc fails beyond), so the
    # bf16 default is 14 layers = 112 experts = 39.5 GB with the cache-to-experts ratio of the 32-layer
    # workload (2 slots per layer, 25 %); --layers 32 needs a box that can pin 90 GB.  The int4
    # workload (25.4 GB) runs all 32 layers with 128 slots.
    int4 = args.dtype in ("int4", "int2")      # quantised images: all 32 layers fit the pinning limit
    big = args.model == "8x22b"
    if big and not int4:
        print("bench.py: --model 8x22b takes --dtype int4 or int2 (its bf16 experts, 270 GB, do not fit the box's host memory)", file=sys.stderr)
        sys.exit(2)
    L = args.layers or (56 if big else (32 if int4 else 14))
    Hm, Fm = (6144, 16384) if big else (4096, 14336)
    shape = synth.MoEShape(Hm, Fm, 8, L, {"int4": "int4g64", "int2": "int2g64"}.get(args.dtype, "bf16"))
    if big and not args.staging and L > 24:
        args.staging = 4                       # 448 experts of 170 MB are more than a process may pin here
    C = args.cache if args.cache is not None else (4 * L if int4 else 2 * L)
    steps = args.steps if args.steps is not None else 48
    warmup = args.warmup if args.warmup is not None else 16
    gamma = 0.3
    taus = synth.tau_profile(L)
    t_setup = time.time()
    routers, images_dev, images_host = build_stack(shape, 0, keep_on_device=True, pin_host=True, pageable=args.staging > 0)
    H0 = torch.from_numpy(synth.ar1_tokens(64 + warmup + steps, shape.H, 0.8, seed=1, dtype="f32")).cuda()
    a, beta, cos = profile_gate_statistics(shape, routers, images_dev, taus, H0[:64], gamma)
    slots, plan_cost = B.cache_plan(L, shape.N, C, a, beta)
    del images_dev
    torch.cuda.empty_cache()

    ctx, cfg = B.adapmoe_create(shape.H, shape.F, shape.N, L, {"int4": B.INT4G64, "int2": B.INT2G64}.get(args.dtype, B.BF16),
                                max_B=1, trace_capacity=1 << 20)
    apply_options(ctx, args)
    nbytes = B.adapmoe_expert_bytes(cfg)
    for l in range(L):
        B.adapmoe_set_router(ctx, l, routers[l])
        for e in range(shape.N):
            B.adapmoe_register_expert(ctx, l, e, images_host[l][e], nbytes)
    B.adapmoe_set_tau(ctx, taus)
    B.cache_alloc(ctx, slots)
    if args.tiles:
        B.adapmoe_set_tiles(ctx, args.tiles)
    if args.staging:
        B.adapmoe_set_staging(ctx, args.staging, args.staging_threads)
    B.adapmoe_set_lookahead(ctx, args.lookahead)
    t_setup = time.time() - t_setup

    x = torch.empty((1, shape.H), dtype=torch.bfloat16, device="cuda")
    y = torch.empty((1, shape.H), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def run(first, n):
        for t in range(first, first + n):
            h = H0[64 + t:64 + t + 1].clone()
            B.moe_stack_token(ctx, t, h, x, y, 1, gamma, stream)

    run(0, warmup)
    torch.cuda.synchronize()
    B.adapmoe_trace_read(ctx, 1 << 20)          # drop the warm-up events
    c0 = B.adapmoe_counters(ctx)
    B.adapmoe_profile(ctx, True)                # kernel durations of the timed steps (their sum = time the compute stream worked)
    t0 = time.perf_counter()
    run(warmup, steps)
    B.adapmoe_check(ctx, stream)
    t1 = time.perf_counter()
    c1 = B.adapmoe_counters(ctx)
    compute_busy = sum(B.adapmoe_profile_read(ctx, c)[1] for c in (0, 1, 2)) * 1e-3
    B.adapmoe_profile(ctx, False)
    elapsed = t1 - t0
    d = {k: c1[k] - c0[k] for k in c1}
    demand = d["hits"] + d["misses"] + d["bypasses"]
    h2d_gbs = d["h2d_bytes"] / elapsed / 1e9
    # on-demand loads per token and layer, measured (cache events) against the planner's model f_{l,t_l} (Eq.15)
    per_layer = np.zeros(L)
    for (_t, l, kind, _e, _v, _s) in B.adapmoe_trace_read(ctx, 1 << 20):
        if kind in ("MISS", "BYPASS"):
            per_layer[l] += 1
    per_layer /= steps
    model = np.array([B.cache_cost(shape.N, slots[l], float(a[l]), float(beta[l])) for l in range(L)])

    # pinned-copy reference: the same expert images copied back to back on one stream
    buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    r0 = time.perf_counter()
    ref_imgs = [images_host[i % L][i % shape.N] for i in range(8)]
    if args.staging:      # the link's rate is a property of pinned memory: copy one image into a pinned buffer and send that
        pinned = torch.empty(images_host[0][0].numel(), dtype=images_host[0][0].dtype, pin_memory=True)
        pinned.copy_(images_host[0][0])
        ref_imgs = [pinned] * 8
        buf.view(pinned.dtype).copy_(pinned, non_blocking=True)
        torch.cuda.synchronize()
        r0 = time.perf_counter()
    for i in range(8):
        buf.view(images_host[0][0].dtype).copy_(ref_imgs[i], non_blocking=True)
    torch.cuda.synchronize()
    link_gbs = 8 * nbytes / (time.perf_counter() - r0) / 1e9
    copy_busy = d["h2d_bytes"] / (link_gbs * 1e9)            # time the side stream needs for the copies at the link's rate
    # time during which both streams worked: at least copy + compute - elapsed, at most the shorter of the two
    overlap_lo = max(0.0, min(copy_busy, compute_busy, copy_busy + compute_busy - elapsed))
    overlap_hi = min(copy_busy, compute_busy)
    served = d["hits_after_prefetch"] + d["misses"] + d["bypasses"]
    # CPU baseline: the checker's stack on the same tokens (expert images read back from pinned memory), compute only
    class _HostImages:
        def __getitem__(self, l):
            return [images_host[l][e] for e in range(shape.N)]
    cpu = (cpu_baseline_stack(shape, routers, _HostImages(), taus, H0[64 + warmup:].cpu().numpy(), gamma, min(args.cpu_seconds, 12.0),
                              2 if int4 else 8, "the timed stream, no transfers on the CPU side") if args.cpu_seconds > 0 else None)

    out = {
        "metric": METRIC, "value": round(steps / elapsed, 3), "unit": f"tokens/s ({L}-layer stack, batch 1, offloaded experts)",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(elapsed / steps * 1e3, 3),
        "us_per_layer": round(elapsed / steps / L * 1e6, 1),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"mixtral_stack_offload ({args.model}, {args.dtype}): H={shape.H} F={shape.F} N=8 L={L}, {L * 8} experts ({L * 8 * nbytes / 1e9:.1f} GB) in "
                               + (f"pageable host memory staged through {args.staging} pinned buffers" if args.staging else "pinned host memory")
                               + f", cache of {C} slots sized by the planner, LRU + prefetch {args.lookahead} layer(s) ahead, "
                               f"{'tile-wise loading (' + str(args.tiles) + ' tiles)' if args.tiles else 'whole-image loading'}, gamma={gamma}",
                   "slots_per_layer": slots, "planner_cost": round(plan_cost, 4),
                   "a_l_mean": round(float(a.mean()), 4), "beta_l_mean": round(float(beta[1:].mean()), 4) if L > 1 else None,
                   "cos_successive_inputs": cos, "setup_s": round(t_setup, 1)},
        "roofline": {"bound": "host-link", "achieved": round(h2d_gbs, 2), "peak": round(link_gbs, 2), "unit": "GB/s",
                     "frac": round(h2d_gbs / link_gbs, 4), "traffic": None,
                     "note": "peak = measured back-to-back pinned host-to-HBM copies of the same images on this box"},
        "cache": {"demanded": demand, "hit_rate": round(d["hits"] / max(demand, 1), 4),
                  "hits_after_prefetch": d["hits_after_prefetch"], "on_demand_loads": d["misses"] + d["bypasses"],
                  "prefetch_loads": d["prefetch_loads"], "prefetch_touches": d["prefetch_touches"],
                  "single_expert_ratio": round(d["single_expert"] / max(d["tokens_gated"], 1), 4),
                  "h2d_GB": round(d["h2d_bytes"] / 1e9, 2),
                  "loads_per_token": round((d["misses"] + d["bypasses"] + d["prefetch_loads"]) / steps, 2),
                  "prefetch_landed_outside_budget": d["prefetch_landed"],
                  "experts_evaluated_tile_wise": d["tiled_ffn"]},
        "on_demand_loads_per_token": {"planner_model": round(float(model.sum()), 3), "measured": round(float(per_layer.sum()), 3),
                                      "per_layer_planner": [round(float(v), 3) for v in model],
                                      "per_layer_measured": [round(float(v), 3) for v in per_layer],
                                      "note": "model = sum of f_{l,t_l} (Eq.15) with the profiled a_l, beta_l; it takes the cached set "
                                              "for a random one, LRU with routing locality does better"},
        "overlap": {"copy_busy_s": round(copy_busy, 4), "compute_busy_s": round(compute_busy, 4), "elapsed_s": round(elapsed, 4),
                    "both_streams_busy_s": [round(overlap_lo, 4), round(overlap_hi, 4)],
                    "frac_of_copy_time_hidden_behind_compute": [round(overlap_lo / max(copy_busy, 1e-9), 4), round(overlap_hi / max(copy_busy, 1e-9), 4)],
                    "frac_of_loaded_demands_transferred_ahead_of_time": round(d["hits_after_prefetch"] / max(served, 1), 4),
                    "note": "copy_busy = bytes / measured link rate; compute_busy = sum of kernel durations; the time both streams "
                            "worked lies between copy + compute - elapsed and the shorter of the two (pairs are lower, upper bound). "
                            "The link is the bottleneck here: compute is a few percent of the time, so what prefetch hides is the "
                            "wait of a demand, counted as the share of experts that had to come over the link and were already "
                            "there when demanded"},
        "cpu_baseline": cpu,
    }
    torch.cuda.synchronize()
    B.adapmoe_destroy(ctx)
    return out


# --------------------------------------------------------------------------- batched, resident ----

def shared_stack(shape, shared):
    """Routers and device images of the 32-layer bf16 stack, built once for the workloads that share them."""
    key = (shape.H, shape.F, shape.N, shape.L, shape.dtype)
    if shared is None:
        return build_stack(shape, 0, keep_on_device=True, pin_host=False)[:2]
    if key not in shared:
        shared[key] = build_stack(shape, 0, keep_on_device=True, pin_host=False)[:2]
    return shared[key]


def bench_batched(args, shared=None):
    import numpy as np
    import torch

    from paper_2408_10284_amd import binding as B
    from paper_2408_10284_amd import synth

    L = args.layers or 32
    Bt = 16
    shape = synth.MoEShape(4096, 14336, 8, L, "bf16")
    steps = args.steps if args.steps is not None else 64
    warmup = args.warmup if args.warmup is not None else 8
    gamma = 0.3
    taus = synth.tau_profile(L)
    t_setup = time.time()
    routers, images_dev = shared_stack(shape, shared)
    ctx, cfg = B.adapmoe_create(shape.H, shape.F, shape.N, L, B.BF16, max_B=Bt)
    apply_options(ctx, args)
    nbytes = B.adapmoe_expert_bytes(cfg)
    for l in range(L):
        B.adapmoe_set_router(ctx, l, routers[l])
        for e in range(shape.N):
            B.adapmoe_bind_expert_dev(ctx, l, e, images_dev[l][e])
    B.adapmoe_set_tau(ctx, taus)
    n_tok = warmup + steps
    Xs = synth.ar1_streams(n_tok, Bt, shape.H, 0.8, seed=1, dtype="f32")
    H0 = torch.from_numpy(Xs).cuda()
    t_setup = time.time() - t_setup
    x = torch.empty((Bt, shape.H), dtype=torch.bfloat16, device="cuda")
    y = torch.empty((Bt, shape.H), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def run(first, n):
        for t in range(first, first + n):
            h = H0[t].clone()
            B.moe_stack_token(ctx, t, h, x, y, Bt, gamma, stream)

    run(0, warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(warmup, steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    B.adapmoe_check(ctx)

    # instrumented pass: kernel durations from events tied to the dispatches, and the gate decisions of every
    # layer step (decision log), which give the experts each launch really streamed and the pairs it really computed
    n_prof = min(steps, 16)
    logbuf = torch.zeros((n_prof * L, 6 * Bt), dtype=torch.int32, device="cuda")
    B.adapmoe_set_decision_log(ctx, logbuf, n_prof * L)
    B.adapmoe_profile(ctx, True)
    run(warmup, n_prof)
    torch.cuda.synchronize()
    prof = {c: B.adapmoe_profile_read(ctx, c) for c in (2, 3, 4, 5)}
    B.adapmoe_profile(ctx, False)
    B.adapmoe_set_decision_log(ctx, None, 0)
    ids, kk = read_decisions(ctx, logbuf, n_prof * L, Bt, Bt)
    touched = pairs = 0
    for r in range(n_prof * L):
        act = set()
        for b in range(Bt):
            act.update(int(e) for e in ids[r, b, :kk[r, b]])
        touched += len(act)
        pairs += int(kk[r].sum())
    touched /= n_prof * L          # experts streamed per layer step
    pairs /= n_prof * L            # (token, expert) pairs per layer step
    n_l = prof[4][0]
    per_matrix = nbytes / 3.0
    gu_us = prof[4][1] / max(n_l, 1) * 1e3
    dn_us = prof[5][1] / max(prof[5][0], 1) * 1e3
    gu_gbs = touched * 2 * per_matrix / (gu_us * 1e-6) / 1e9
    own_flops = pairs * 2 * 3 * shape.H * shape.F          # multiply-adds of the method itself, both GEMMs
    issued_flops = touched * 16 * 2 * 3 * shape.H * shape.F  # what the 16-column matrix instructions execute
    cpu = (cpu_baseline_stack(shape, routers, images_dev, taus, Xs[warmup:, 0, :], gamma, args.cpu_seconds, 3, "stream 0 of the 16")
           if args.cpu_seconds > 0 else None)
    # the grouped GEMM's access pattern with loads only: 512 bytes of each of 32 rows per step, one workgroup per compute unit
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    pbuf = torch.empty(8 * 2 * shape.F * shape.H * 2, dtype=torch.uint8, device="cuda").fill_(1)
    probe_us = B.adapmoe_stream_probe(pbuf, 8 * 2 * shape.F, shape.H * 2, 32, 512, cus, 10)
    del pbuf
    probe = {"pattern": f"a wavefront reads 512 bytes of each of 32 rows per step, two 16 KiB buffers in flight, {cus} workgroups of "
                        "256 threads, loads only, W1 and W3 of 8 experts",
             "us": round(probe_us, 1), "GBs": round(8 * 2 * per_matrix / (probe_us * 1e-6) / 1e9, 1),
             "kernel_GBs_over_probe_GBs": round(gu_gbs / (8 * 2 * per_matrix / (probe_us * 1e-6) / 1e9), 4)}
    out = {
        "metric": METRIC, "value": round(Bt * steps / elapsed, 2), "unit": f"tokens/s ({L}-layer stack, {Bt} decode streams per step)",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(elapsed / steps * 1e3, 3),
        "us_per_layer": round(elapsed / steps / L * 1e6, 1),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"mixtral_batched: H=4096 F=14336 N=8 L={L}, {Bt} AR(1) streams, experts resident in HBM "
                               f"({L * 8 * nbytes / 1e9:.1f} GB), MFMA grouped GEMM over tokens bucketed by expert, gamma={gamma}",
                   "experts_streamed_per_layer_step": round(touched, 3), "token_expert_pairs_per_layer_step": round(pairs, 2),
                   "setup_s": round(t_setup, 1)},
        "roofline": {"bound": "hbm", "kernel": "grouped_gateup_stream_kernel", "achieved": round(gu_gbs, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gu_gbs / HBM_PEAK_GBS, 4),
                     "traffic": measured_traffic("grouped_gateup_stream_kernel", "pmc_traffic_batched.json"),
                     "avg_us": round(gu_us, 1), "launches": n_l,
                     "bytes_per_launch": round(touched * 2 * per_matrix),
                     "note": "bytes = W1 and W3 of the experts the launches really streamed (from the decision log)",
                     "stream_probe": probe},
        "kernels": {"grouped_down_mfma_kernel": {"avg_us": round(dn_us, 1), "achieved_GBs": round(touched * per_matrix / (dn_us * 1e-6) / 1e9, 1)},
                    "bucket_gather_kernel": {"avg_us": round(prof[3][1] / max(prof[3][0], 1) * 1e3, 2)},
                    "gate_kernel": {"avg_us": round(prof[2][1] / max(prof[2][0], 1) * 1e3, 2)},
                    "mfma": {"own_flops_per_layer_step": round(own_flops), "issued_flops_per_layer_step": round(issued_flops),
                             "util_own_of_2.5PFLOPs": round(own_flops / ((gu_us + dn_us) * 1e-6) / 2.5e15, 5),
                             "util_issued_of_2.5PFLOPs": round(issued_flops / ((gu_us + dn_us) * 1e-6) / 2.5e15, 5),
                             "note": "own = the (token, expert) pairs the gate activated; issued = 16 token columns per "
                                     "streamed expert, the shape of the matrix instruction (most columns are padding)"}},
        "cpu_baseline": cpu,
    }
    torch.cuda.synchronize()
    B.adapmoe_destroy(ctx)
    return out


# --------------------------------------------------------------------------- batch 1, resident stack ----

def bench_stack_resident(args, shared=None):
    import numpy as np
    import torch

    from paper_2408_10284_amd import binding as B
    from paper_2408_10284_amd import synth

    L = args.layers or 32
    shape = synth.MoEShape(4096, 14336, 8, L, "bf16")
    steps = args.steps if args.steps is not None else 128
    warmup = args.warmup if args.warmup is not None else 16
    gamma = 0.3
    taus = synth.tau_profile(L)
    t_setup = time.time()
    routers, images_dev = shared_stack(shape, shared)
    ctx, cfg = B.adapmoe_create(shape.H, shape.F, shape.N, L, B.BF16, max_B=1)
    apply_options(ctx, args)
    nbytes = B.adapmoe_expert_bytes(cfg)
    for l in range(L):
        B.adapmoe_set_router(ctx, l, routers[l])
        for e in range(shape.N):
            B.adapmoe_bind_expert_dev(ctx, l, e, images_dev[l][e])
    B.adapmoe_set_tau(ctx, taus)
    H0_host = synth.ar1_tokens(warmup + steps, shape.H, 0.8, seed=1, dtype="f32")
    H0 = torch.from_numpy(H0_host).cuda()
    t_setup = time.time() - t_setup
    x = torch.empty((1, shape.H), dtype=torch.bfloat16, device="cuda")
    y = torch.empty((1, shape.H), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    hbuf = torch.empty((1, shape.H), dtype=torch.float32, device="cuda")
    graph = None
    if args.graph:
        # the whole token step (4 launches per layer) as one graph; the residual stream lives in hbuf
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            hbuf.copy_(H0[0:1])
            B.moe_stack_token(ctx, 0, hbuf, x, y, 1, gamma, side)
            side.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                B.moe_stack_token(ctx, 0, hbuf, x, y, 1, gamma, torch.cuda.current_stream())
        stream.wait_stream(side)

    def run(first, n):
        for t in range(first, first + n):
            if graph is not None:
                hbuf.copy_(H0[t:t + 1])
                graph.replay()
            else:
                h = H0[t:t + 1].clone()
                B.moe_stack_token(ctx, t, h, x, y, 1, gamma, stream)

    run(0, warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(warmup, steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    B.adapmoe_check(ctx)
    graph_steps, graph = graph is not None, None      # the instrumented pass below runs eagerly

    # instrumented pass: kernel durations (events tied to the dispatches) and the k of every layer step (decision log)
    n_prof = min(steps, 32)
    logbuf = torch.zeros((n_prof * L, 6), dtype=torch.int32, device="cuda")
    B.adapmoe_set_decision_log(ctx, logbuf, n_prof * L)
    B.adapmoe_profile(ctx, True)
    run(warmup, n_prof)
    torch.cuda.synchronize()
    n_gu, ms_gu = B.adapmoe_profile_read(ctx, 0)
    n_dn, ms_dn = B.adapmoe_profile_read(ctx, 1)
    n_gt, ms_gt = B.adapmoe_profile_read(ctx, 2)
    B.adapmoe_profile(ctx, False)
    B.adapmoe_set_decision_log(ctx, None, 0)
    _, kk = read_decisions(ctx, logbuf, n_prof * L, 1, 1)
    mean_k = float(kk.mean())
    per_matrix = nbytes / 3.0
    gu_gbs = mean_k * 2 * per_matrix / (ms_gu / max(n_gu, 1) * 1e-3) / 1e9
    dn_gbs = mean_k * per_matrix / (ms_dn / max(n_dn, 1) * 1e-3) / 1e9
    cpu = (cpu_baseline_stack(shape, routers, images_dev, taus, H0_host[warmup:], gamma, args.cpu_seconds, 8, "the timed stream")
           if args.cpu_seconds > 0 else None)
    out = {
        "metric": METRIC, "value": round(steps / elapsed, 2), "unit": f"tokens/s ({L}-layer stack, batch 1, experts resident)",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(elapsed / steps * 1e3, 3),
        "us_per_layer": round(elapsed / steps / L * 1e6, 1),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"mixtral_stack_resident: H=4096 F=14336 N=8 L={L}, one AR(1) stream, experts resident in HBM "
                               f"({L * 8 * nbytes / 1e9:.1f} GB), residual + RMS norm between blocks, gamma={gamma}"
                               + (", one HIP graph replay per token" if graph_steps else ""),
                   "mean_k": round(mean_k, 4), "single_expert_ratio": round(float((kk == 1).mean()), 4), "setup_s": round(t_setup, 1)},
        "roofline": {"bound": "hbm", "kernel": "ffn_gateup_kernel", "achieved": round(gu_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gu_gbs / HBM_PEAK_GBS, 4), "traffic": None,
                     "avg_us": round(ms_gu / max(n_gu, 1) * 1e3, 2), "launches": n_gu,
                     "bytes_per_launch": round(mean_k * 2 * per_matrix)},
        "kernels": {"down": {"achieved_GBs": round(dn_gbs, 1), "frac": round(dn_gbs / HBM_PEAK_GBS, 4), "avg_us": round(ms_dn / max(n_dn, 1) * 1e3, 2)},
                    "norm_gate": {"avg_us": round(ms_gt / max(n_gt, 1) * 1e3, 2)},
                    "whole_step_GBs": round(mean_k * nbytes * L / (elapsed / steps) / 1e9, 1),
                    "whole_step_frac": round(mean_k * nbytes * L / (elapsed / steps) / 1e9 / HBM_PEAK_GBS, 4)},
        "cpu_baseline": cpu,
    }
    torch.cuda.synchronize()
    B.adapmoe_destroy(ctx)
    return out


if __name__ == "__main__":
    main()
