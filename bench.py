#!/usr/bin/env python3
"""Benchmark of the sliced, group-dequantised linear hot path on one MI355X.

Workload (default): the Llama-2-7B-shaped decoder linears at batch M=1
(q/k/v/o 4096x4096, gate/up 11008x4096, down 4096x11008; 32 blocks = 224
linears), 8-bit parent with group 128, benchmarked at EVERY r in {2,3,4,6,8}.
One step = five persistent launches (mq_linear_stack), one per r, each running
all 224 linears at that width from weights already packed and resident in HBM
(slice + pack are load-time steps and are reported separately).  The stacks are
1.6-6.5 GB each, far beyond the 256 MB last-level cache, so every launch
streams from HBM.

Prints ONE JSON line: effective HBM GB/s over the step (algorithmic bytes:
r/8 per weight + fp16 scale and zero per group + activations in and out), the
per-r microseconds and GB/s, the roofline object of the dominant kernel
(mq::stack_kernel<1, 1, false>, HBM-bound) measured with events on the launch stream, and
the CPU oracle timed on the host cores on a bounded sample.
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

HBM_PEAK_GBPS = 8000.0
WIDTHS = (2, 3, 4, 6, 8)
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "stack_kernel_llama2_7b_m1_hbm_traffic.txt")
# the sources that define mq::stack_kernel<1, 1, false>: a traffic figure is quoted only while they are the ones profiled
KERNEL_SOURCES = ("mq_linear.hip", "mq_device.h", "mq_layout.h", "mq_internal.h", "mq_static_for.h")


def kernel_sources_sha() -> str:
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2602_03537_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def traffic_from_profile():
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary (two machine-readable
    lines: `traffic_bytes_per_launch = N`, `kernel_sources_sha = H`).  None, with the reason, if the summary is
    missing or was taken on other kernel sources than the ones in the tree."""
    try:
        kv = {}
        for line in open(TRAFFIC_PROFILE):
            if " = " in line and line.split(" = ")[0].strip() in ("traffic_bytes_per_launch", "kernel_sources_sha"):
                k, v = line.split(" = ", 1)
                kv[k.strip()] = v.strip()
        if kv.get("kernel_sources_sha") != kernel_sources_sha():
            return None, "profile summary was taken on other kernel sources"
        return int(kv["traffic_bytes_per_launch"]), os.path.relpath(TRAFFIC_PROFILE, ROOT)
    except (OSError, KeyError, ValueError) as e:
        return None, f"no usable profile summary ({type(e).__name__})"


def algo_bytes(N, K, r, M=1, group=128):
    """Bytes the method must move for one linear: r/8 per weight, fp16 scale + zero per group, x in, y out."""
    return N * K * r / 8.0 + 4.0 * N * (K // group) + 2.0 * M * K + 2.0 * M * N


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--layers", type=int, default=32, help="decoder blocks in the stack")
    ap.add_argument("--workload", default="every-r", choices=["every-r", "mixed-7b", "mixed-70b", "mlp-70b", "parent-7b", "parent-70b", "quant-7b", "gptq-7b",
                             "decode-7b"],
                    help="every-r: Llama-2-7B linears at each r (default, the headline); mixed-7b / mixed-70b: one "
                         "mixed-width stack (mean 3.5 / 4 bits); mlp-70b: batched regime on the Llama-3-70B MLP shapes; "
                         "parent-7b / parent-70b: run-time re-slicing of a resident 8-bit parent (mq_reslice, "
                         "mq_slice_pack) and the stack computed straight from the parent; quant-7b: Algorithm 1 (cross-bit-width "
                         "choice of the parent code) on the Llama-2-7B layer shapes; gptq-7b: the MatGPTQ column loop "
                         "(Algorithm 2) on those shapes; decode-7b: shared-input fusions of a decoder block (q/k/v and gate/up "
                         "as one launch each) against one launch per linear")
    ap.add_argument("--batch", type=int, default=1, help="M for the mixed-* workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-single", action="store_true", help="skip the per-call mq_linear table")
    ap.add_argument("--no-loadtime", action="store_true", help="skip the slice/pack throughput leg")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the legs folded into the default line (achievable read, mixed Llama-2-7B stack, a cut of "
                         "the batched Llama-3-70B MLP regime, decoder-block fusions)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2602_03537_amd as mq
    from paper_2602_03537_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.workload in ("mixed-7b", "mixed-70b"):
        return bench_mixed_stack(args, mq, synth, torch, np, dev)
    if args.workload == "mlp-70b":
        return bench_mlp_batched(args, mq, synth, torch, np, dev)
    if args.workload in ("parent-7b", "parent-70b"):
        return bench_resident_parent(args, mq, synth, torch, np, dev)
    if args.workload == "quant-7b":
        return bench_quant(args, mq, synth, torch, np, dev)
    if args.workload == "gptq-7b":
        return bench_gptq(args, mq, synth, torch, np, dev)
    if args.workload == "decode-7b":
        return bench_decode_fusions(args, mq, synth, torch, np, dev)
    block = synth.LLAMA2_7B_BLOCK
    M = 1

    # ---- what a plain streaming read achieves on this device, measured before anything else is resident
    read = None if args.no_extras else measure_read_probe(mq, torch, dev)

    # ---- inputs: one seeded parent per distinct shape (host recipe), uploaded once
    host = {}
    for (name, N, K) in block:
        if (N, K) not in host:
            host[(N, K)] = synth.make_layer(N, K, M=M, seed=[0, N, K])
    devp = {nk: tuple(torch.from_numpy(L[k]).to(dev) for k in ("parent", "scales", "zeros")) for nk, L in host.items()}
    xdev = {K: torch.from_numpy(synth.make_x(M, K, [0, 77, K])).to(dev) for K in {K for (_, _, K) in block}}

    # ---- load-time steps: slice + pack + meta (timed separately, not part of `value`)
    loadtime = {}
    stacks = {}
    for r in WIDTHS:
        prepared = {}
        for nk, (p, s, z) in devp.items():
            prepared[nk] = mq.prepare_layer(p, s, z, r)
        layers, nbytes, nweights = [], 0.0, 0
        for _ in range(args.layers):
            for (name, N, K) in block:
                pl = prepared[(N, K)]
                layers.append(dict(packed_W=pl["packed_W"].clone(), scales_t=pl["scales_t"].clone(),
                                   zeros_t=pl["zeros_t"].clone(), x=xdev[K],
                                   y=torch.empty((M, N), dtype=torch.float16, device=dev), N=N, K=K, r=r))
                nbytes += algo_bytes(N, K, r, M)
                nweights += N * K
        plan = mq.mq_stack_plan(layers, M, device=dev)
        stacks[r] = dict(layers=layers, plan=plan, bytes=nbytes, weights=nweights)
    torch.cuda.synchronize()

    if not args.no_loadtime:
        N, K = 11008, 4096
        p, s, z = devp[(N, K)]
        S = torch.empty_like(p)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        for r in WIDTHS:
            out = torch.empty(mq.mq_packed_bytes(N, K, r), dtype=torch.uint8, device=dev)
            mq.mq_slice_codes(p, 8, r, out=S); mq.mq_pack(S, 8, r, out=out)
            torch.cuda.synchronize()
            ev[0].record()
            for _ in range(5):
                mq.mq_slice_codes(p, 8, r, out=S)
            ev[1].record()
            for _ in range(5):
                mq.mq_pack(S, 8, r, out=out)
            ev[2].record()
            torch.cuda.synchronize()
            ts, tp = ev[0].elapsed_time(ev[1]) / 5e3, ev[1].elapsed_time(ev[2]) / 5e3
            loadtime[str(r)] = {"slice_GBps": round(2.0 * N * K / ts / 1e9, 1),
                                "pack_GBps": round((1.0 + r / 8.0) * N * K / tp / 1e9, 1)}

    # ---- the timed region
    def step(events=None):
        for i, r in enumerate(WIDTHS):
            if events is not None:
                events[i].record()
            mq.mq_linear_stack(stacks[r]["plan"])
        if events is not None:
            events[len(WIDTHS)].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(len(WIDTHS) + 1)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(evs[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    per_r_us = {r: [] for r in WIDTHS}
    for k in range(args.steps):
        for i, r in enumerate(WIDTHS):
            per_r_us[r].append(evs[k][i].elapsed_time(evs[k][i + 1]) * 1e3)
    step_bytes = sum(stacks[r]["bytes"] for r in WIDTHS)
    n_lin = len(stacks[WIDTHS[0]]["layers"])
    per_r = {}
    for r in WIDTHS:
        us = float(np.median(per_r_us[r]))
        gbps = stacks[r]["bytes"] / us / 1e3
        per_r[str(r)] = {"us_per_stack": round(us, 1), "us_min": round(float(np.min(per_r_us[r])), 1),
                         "us_per_linear": round(us / n_lin, 3), "GBps": round(gbps, 1),
                         "frac_of_8TBps": round(gbps / HBM_PEAK_GBPS, 4), "algorithmic_MB": round(stacks[r]["bytes"] / 1e6, 1)}
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    # roofline of the dominant kernel (mq::stack_kernel<1, 1, false>): algorithmic bytes per launch / mean launch duration
    launches = [u for r in WIDTHS for u in per_r_us[r]]
    avg_launch_us = float(np.mean(launches))
    bytes_per_launch = step_bytes / len(WIDTHS)
    achieved = bytes_per_launch / avg_launch_us / 1e3
    roofline = {"bound": "hbm", "kernel": "mq::stack_kernel<1, 1, false>", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                "avg_launch_us": round(avg_launch_us, 1), "algorithmic_bytes_per_launch": int(bytes_per_launch)}
    traffic, traffic_src = traffic_from_profile() if args.layers == 32 else (None, "not the profiled workload")
    roofline["traffic"] = traffic
    roofline["traffic_source"] = traffic_src

    # ---- the same stacks as symmetric layers (zeros_t = NULL: every zero-offset 128, the paper's own setting): no
    # zero-offset array is read, the algorithmic bytes drop by 2 per group
    symmetric = None
    if not args.no_extras:
        symmetric = {}
        for r in WIDTHS:
            lay_s = [dict(L, zeros_t=None) for L in stacks[r]["layers"]]
            plan_s = mq.mq_stack_plan(lay_s, M, device=dev)
            for _ in range(2):
                mq.mq_linear_stack(plan_s)
            torch.cuda.synchronize()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
            for k in range(5):
                ev[k].record()
                mq.mq_linear_stack(plan_s)
            ev[5].record()
            torch.cuda.synchronize()
            us = float(np.median([ev[k].elapsed_time(ev[k + 1]) * 1e3 for k in range(5)]))
            b = stacks[r]["bytes"] - 2.0 * stacks[r]["weights"] / 128
            symmetric[str(r)] = {"us_per_stack": round(us, 1), "GBps": round(b / us / 1e3, 1),
                                 "frac_of_8TBps": round(b / us / 1e3 / HBM_PEAK_GBPS, 4),
                                 "algorithmic_MB": round(b / 1e6, 1),
                                 "time_vs_asymmetric": round(us / per_r[str(r)]["us_per_stack"], 4)}
            del plan_s, lay_s

    # ---- per-call table: one mq_linear launch per layer, cold (cycling distinct copies), replayed from a HIP graph
    single = None
    if not args.no_single:
        single = {}
        for (N, K) in host:
            for r in WIDTHS:
                lay = stacks[r]["layers"]
                same = [L for L in lay if L["N"] == N and L["K"] == K]
                ws = mq.new_workspace(M, N, K, r)
                y = torch.empty((M, N), dtype=torch.float16, device=dev)

                def run_all():
                    for L in same:
                        mq.mq_linear(L["x"], L["packed_W"], L["scales_t"], L["zeros_t"], N, K, r, 128, ws, y=y)

                run_all()
                torch.cuda.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    run_all()
                g.replay()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(3):
                    g.replay()
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / (3 * len(same))
                b = algo_bytes(N, K, r, M)
                del g
                # warm: the same weights again and again (cache-resident up to the last-level cache), graph replay
                L0 = same[0]

                def run_warm():
                    for _ in range(32):
                        mq.mq_linear(L0["x"], L0["packed_W"], L0["scales_t"], L0["zeros_t"], N, K, r, 128, ws, y=y)

                run_warm()
                torch.cuda.synchronize()
                gw = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gw):
                    run_warm()
                gw.replay()
                torch.cuda.synchronize()
                e0.record()
                for _ in range(3):
                    gw.replay()
                e1.record()
                torch.cuda.synchronize()
                us_warm = e0.elapsed_time(e1) * 1e3 / (3 * 32)
                del gw
                # isolated: one launch on an idle device, cold weights (another copy each time), events around it
                iso = []
                for L1 in same[1:9]:
                    torch.cuda.synchronize()
                    e0.record()
                    mq.mq_linear(L1["x"], L1["packed_W"], L1["scales_t"], L1["zeros_t"], N, K, r, 128, ws, y=y)
                    e1.record()
                    torch.cuda.synchronize()
                    iso.append(e0.elapsed_time(e1) * 1e3)
                single[f"{N}x{K}:r{r}"] = {"us": round(us, 2), "GBps": round(b / us / 1e3, 1), "copies": len(same),
                                           "us_warm": round(us_warm, 2), "us_isolated": round(float(np.median(iso)), 2)}

    # ---- CPU oracle on the host cores: whole decoder blocks (7 linears at every r) until about 12 s of work
    cpu = None
    if not args.no_cpu:
        from oracle import c_oracle
        cb, ct, cores, passes = 0.0, 0.0, 1, 0
        while ct < 12.0 and passes < 64:
            for r in WIDTHS:
                for (name, N, K) in block:
                    L = host[(N, K)]
                    ta = time.perf_counter()
                    _, cores = c_oracle.linear(L["x"], L["parent"], L["scales"], L["zeros"], 8, r, 128)
                    ct += time.perf_counter() - ta
                    cb += algo_bytes(N, K, r, M)
            passes += 1
        cpu = {"value": round(cb / ct / 1e9, 3), "unit": "GB/s", "cores": int(cores), "kind": "oracle",
               "sample": "plain-C oracle (oracle/mq_oracle.c, slice+dequant+fp64 dot per weight, OpenMP over rows) on "
                         f"{passes} Llama-2-7B decoder blocks (7 linears each, M=1) at each r in {{2,3,4,6,8}} "
                         f"= {passes}/{args.layers} of the timed workload; same algorithmic-byte accounting as the GPU value",
               "seconds": round(ct, 2)}

    # ---- legs folded into the default line so that one driver run checks every quoted configuration
    extras = {}
    if not args.no_extras:
        del stacks, prepared, layers
        torch.cuda.empty_cache()
        extras["achievable_read"] = read
        extras["symmetric"] = symmetric
        for r in WIDTHS:
            per_r[str(r)]["frac_of_achievable_read"] = round(per_r[str(r)]["GBps"] / read["GBps"], 4)
        roofline["frac_of_achievable_read"] = round(achieved / read["GBps"], 4)
        m = measure_mixed_stack(mq, synth, torch, np, dev, False, synth.LLAMA2_7B_LAYERS, 1, args.steps, args.warmup)
        gb = m["bytes"] / float(np.median(m["us"])) / 1e3
        extras["mixed_7b"] = {"workload": f"Llama-2-7B-shaped stack, 32 blocks ({m['n_linears']} linears), M=1, per-layer r by seed, "
                                          f"mean {m['mean_bits']:.3f} bits, one persistent launch",
                              "us_median": round(float(np.median(m["us"])), 1), "us_min": round(float(np.min(m["us"])), 1),
                              "GBps": round(gb, 1), "frac": round(gb / HBM_PEAK_GBPS, 4),
                              "frac_of_achievable_read": round(gb / read["GBps"], 4),
                              "algorithmic_GB": round(m["bytes"] / 1e9, 3)}
        del m
        torch.cuda.empty_cache()
        # a cut of configs[4]: the first 16 blocks of the Llama-3-70B-shaped stack (widths drawn for those blocks), at the
        # batch sizes of the three kernel families (vector ALUs, narrow and wide matrix-core kernels)
        cut70 = {}
        for Mb in (1, 8, 64):
            m = measure_mixed_stack(mq, synth, torch, np, dev, True, 16, Mb, max(4, args.steps // 4), 2)
            gb = m["bytes"] / float(np.median(m["us"])) / 1e3
            cut70["M%d" % Mb] = {"us_median": round(float(np.median(m["us"])), 1), "GBps": round(gb, 1),
                                 "frac": round(gb / HBM_PEAK_GBPS, 4), "kernel": m["kernel"],
                                 "mean_bits": round(m["mean_bits"], 3), "algorithmic_GB": round(m["bytes"] / 1e9, 3),
                                 "TFLOPs": round(2.0 * Mb * m["weights"] / float(np.median(m["us"])) / 1e6, 1)}
            del m
            torch.cuda.empty_cache()
        extras["mixed_70b_cut"] = {"workload": "Llama-3-70B-shaped stack, first 16 blocks (112 linears, 8-bit parent resident), per-layer "
                                               "r by seed, one persistent launch, M in {1, 8, 64}", "table": cut70}
        cut = measure_mlp(mq, synth, torch, dev, (("up", 28672, 8192),), (4,), (1, 4, 16, 64, 256), max(2, args.steps // 4))
        for v in cut.values():
            v.pop("bytes")
        extras["mlp_70b_cut"] = {"workload": "Llama-3-70B up-projection 28672x8192, r=4, M in {1,4,16,64,256}, one mq_linear "
                                             "launch per call, 4 weight copies cycled (cold)", "table": cut}
        torch.cuda.empty_cache()
        res, dbytes, dmean = measure_decode_fusions(mq, synth, torch, np, dev, 1, 32, max(5, args.steps // 2))
        extras["decode_7b"] = {"workload": f"Llama-2-7B decoder blocks x32, M=1, per-layer r by seed (mean {dmean:.3f} bits), "
                                           "every block its own weights, HIP-graph replay", "table": res,
                               "frac": round(res["fused_qkv_and_gate_up"]["GBps"] / HBM_PEAK_GBPS, 4)}
        del res
        torch.cuda.empty_cache()
        extras["chain_7b"] = {"workload": "three dependent 4096x4096 links (r = 3, 4, 8), M=1, 32 chains with their own weights, "
                                          "HIP-graph replay: one chained launch (MQ_X_AFTER_EARLIER) against one launch per link",
                              "table": measure_chain(mq, synth, torch, np, dev, 1, 32, max(5, args.steps // 2))}

    out = {
        "metric": "batch-1 sliced GEMV effective HBM GB/s (algorithmic bytes / time) over r in {2,3,4,6,8}",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"Llama-2-7B-shaped decoder linears x{args.layers} blocks ({n_lin} linears), M=1, "
                               "8-bit parent, group 128, every r in {2,3,4,6,8} (one persistent launch per r)",
                   "M": M, "group": 128, "c": 8, "widths": list(WIDTHS), "launches_per_step": len(WIDTHS),
                   "algorithmic_GB_per_step": round(step_bytes / 1e9, 3)},
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        "per_r": per_r,
        "roofline": roofline,
        "cpu_baseline": cpu,
        "single_call": single,
        "load_time": loadtime or None,
    }
    out.update(extras)
    print(json.dumps(out))
    return 0


def _base_line(metric, value, unit, args, ms_per_step, workload, extra_cfg):
    return {"metric": metric, "value": round(value, 1), "unit": unit, "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "f16", "data": "synthetic", "config": dict({"workload": workload}, **extra_cfg)}


def measure_mixed_stack(mq, synth, torch, np, dev, big, n_blocks, M, steps, warmup):
    """One mixed-width stack (per-layer r drawn by seed), one persistent launch per step.  Returns a dict of results."""
    block = synth.LLAMA3_70B_BLOCK if big else synth.LLAMA2_7B_BLOCK
    target = 4.0 if big else 3.5
    shapes = synth.stack_shapes(block, n_blocks)
    widths, mean = synth.draw_bitwidths([N * K for (_, _, N, K) in shapes], target, seed=0)
    layers, nbytes, keep, weights = [], 0.0, [], 0
    for i, ((_, _, N, K), r) in enumerate(zip(shapes, widths)):
        weights += N * K
        L = synth.make_layer_device(N, K, M, seed=7000 + i, device=dev)
        lay = mq.prepare_layer(L["parent"], L["scales"], L["zeros"], int(r))
        lay.update(x=L["x"], y=torch.empty((M, N), dtype=torch.float16, device=dev))
        layers.append(lay)
        if big:
            keep.append(L["parent"])          # the 8-bit parent stays resident, as the configuration states
        nbytes += algo_bytes(N, K, int(r), M)
    plan = mq.mq_stack_plan(layers, M, device=dev)
    for _ in range(warmup):
        mq.mq_linear_stack(plan)
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    for k in range(steps):
        evs[k].record()
        mq.mq_linear_stack(plan)
    evs[steps].record()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    us = [evs[k].elapsed_time(evs[k + 1]) * 1e3 for k in range(steps)]
    kernel = ("mq::stack_kernel<%d, 1, false>" % M if M <= 3 else "mq::gemm_stack_kernel" if M <= 16
              else "mq::wide_stack_kernel")
    return {"ms_wall": ms, "us": us, "bytes": nbytes, "mean_bits": mean, "n_linears": len(layers), "n_blocks": n_blocks,
            "kernel": kernel, "weights": weights}


def bench_mixed_stack(args, mq, synth, torch, np, dev):
    big = args.workload == "mixed-70b"
    n_blocks = (synth.LLAMA3_70B_LAYERS if big else synth.LLAMA2_7B_LAYERS) if args.layers == 32 else args.layers
    M = args.batch
    m = measure_mixed_stack(mq, synth, torch, np, dev, big, n_blocks, M, args.steps, args.warmup)
    ms, us, nbytes, mean = m["ms_wall"], m["us"], m["bytes"], m["mean_bits"]
    value = nbytes / (ms * 1e-3) / 1e9
    out = _base_line("mixed-precision stack, decode-step latency and aggregate effective HBM GB/s", value, "GB/s", args,
                     ms, f"{'Llama-3-70B' if big else 'Llama-2-7B'}-shaped stack, {n_blocks} blocks ({m['n_linears']} linears), "
                     f"M={M}, per-layer r from {{2,3,4,6,8}} by seed, parameter-weighted mean {mean:.3f} bits",
                     {"M": M, "mean_bits": round(mean, 4), "algorithmic_GB_per_step": round(nbytes / 1e9, 3)})
    ach = nbytes / float(np.mean(us)) / 1e3
    out["stack_us_median"] = round(float(np.median(us)), 1)
    out["stack_us_min"] = round(float(np.min(us)), 1)
    out["frac_of_hbm_peak"] = round(value / HBM_PEAK_GBPS, 4)
    out["roofline"] = {"bound": "hbm", "kernel": m["kernel"], "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                       "frac": round(ach / HBM_PEAK_GBPS, 4), "avg_launch_us": round(float(np.mean(us)), 1),
                       "algorithmic_bytes_per_launch": int(nbytes), "traffic": None}
    out["cpu_baseline"] = None
    print(json.dumps(out))
    return 0


def bench_resident_parent(args, mq, synth, torch, np, dev):
    """One resident 8-bit parent, every budget: the mixed-width stack computed from the parent (Eq. 1 in registers,
    8 bits per weight streamed whatever r is), and the rate at which resident layers are re-sliced to another width."""
    big = args.workload == "parent-70b"
    block = synth.LLAMA3_70B_BLOCK if big else synth.LLAMA2_7B_BLOCK
    n_blocks = (synth.LLAMA3_70B_LAYERS if big else synth.LLAMA2_7B_LAYERS) if args.layers == 32 else args.layers
    M = args.batch
    shapes = synth.stack_shapes(block, n_blocks)
    widths, mean = synth.draw_bitwidths([N * K for (_, _, N, K) in shapes], 4.0 if big else 3.5, seed=0)
    layers, nbytes, nweights = [], 0.0, 0
    for i, ((_, _, N, K), r) in enumerate(zip(shapes, widths)):
        L = synth.make_layer_device(N, K, M, seed=7000 + i, device=dev)
        st, zt = mq.mq_pack_meta(L["scales"], L["zeros"], K, 128)
        layers.append(dict(packed_W=mq.mq_pack(L["parent"], 8, 8), scales_t=st, zeros_t=zt, N=N, K=K, r=int(r),
                           from_parent=1, x=L["x"], y=torch.empty((M, N), dtype=torch.float16, device=dev)))
        nbytes += algo_bytes(N, K, 8, M)
        nweights += N * K
        del L
    plan = mq.mq_stack_plan(layers, M, device=dev)
    for _ in range(args.warmup):
        mq.mq_linear_stack(plan)
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        evs[k].record()
        mq.mq_linear_stack(plan)
    evs[args.steps].record()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    us = [evs[k].elapsed_time(evs[k + 1]) * 1e3 for k in range(args.steps)]
    value = nbytes / (ms * 1e-3) / 1e9
    out = _base_line("stack computed from the resident 8-bit parent (Eq. 1 in registers), effective HBM GB/s", value,
                     "GB/s", args, ms,
                     f"{'Llama-3-70B' if big else 'Llama-2-7B'}-shaped stack, {n_blocks} blocks ({len(layers)} linears), "
                     f"M={M}, per-layer r from {{2,3,4,6,8}} by seed (mean {mean:.3f} bits) applied to the resident parent",
                     {"M": M, "mean_bits": round(mean, 4), "algorithmic_GB_per_step": round(nbytes / 1e9, 3)})
    ach = nbytes / float(np.mean(us)) / 1e3
    out["stack_us_median"] = round(float(np.median(us)), 1)
    out["frac_of_hbm_peak"] = round(value / HBM_PEAK_GBPS, 4)
    out["roofline"] = {"bound": "hbm", "kernel": "mq::stack_kernel<%d, 1, true>" % M, "achieved": round(ach, 1),
                       "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4),
                       "avg_launch_us": round(float(np.mean(us)), 1), "algorithmic_bytes_per_launch": int(nbytes),
                       "traffic": None}

    # re-slicing rate: every distinct shape of the block at every width, over all resident copies of that shape (cold)
    # every layer has its own output buffer (sized for r = 8), as a real switch of budget would
    for L in layers:
        L["out"] = torch.empty(mq.mq_packed_bytes(L["N"], L["K"], 8), dtype=torch.uint8, device=dev)
    table, tot = {}, {r: [0.0, 0.0] for r in WIDTHS}
    for (N, K) in sorted({(N, K) for (_, N, K) in block}):
        same = [L for L in layers if L["N"] == N and L["K"] == K][:16]
        for r in WIDTHS:
            mq.mq_reslice(same[0]["packed_W"], N, K, 8, r, out=same[0]["out"])
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for L in same:
                mq.mq_reslice(L["packed_W"], N, K, 8, r, out=L["out"])
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) * 1e-3 / len(same)
            b = (1.0 + r / 8.0) * N * K
            table[f"reslice:{N}x{K}:r{r}"] = {"us": round(t * 1e6, 1), "GBps": round(b / t / 1e9, 1)}
            cnt = sum(1 for (_, n, k) in block if (n, k) == (N, K)) * n_blocks
            tot[r][0] += b * cnt
            tot[r][1] += t * cnt
    out["reslice"] = table
    out["reslice_whole_model"] = {str(r): {"ms": round(tot[r][1] * 1e3, 2), "GBps": round(tot[r][0] / tot[r][1] / 1e9, 1),
                                           "frac_of_8TBps": round(tot[r][0] / tot[r][1] / 1e9 / HBM_PEAK_GBPS, 4)}
                                  for r in WIDTHS}
    # the whole model switched to one width with mq_reslice_many (one launch per 16 layers), every resident layer once
    many = {}
    for r in WIDTHS:
        jobs = [dict(packed_parent=L["packed_W"], N=L["N"], K=L["K"], r=r, out=L["out"]) for L in layers]
        mq.mq_reslice_many(jobs[:16])
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        mq.mq_reslice_many(jobs)
        e1.record()
        torch.cuda.synchronize()
        t = e0.elapsed_time(e1) * 1e-3
        b = (1.0 + r / 8.0) * nweights
        many[str(r)] = {"ms": round(t * 1e3, 2), "GBps": round(b / t / 1e9, 1),
                        "frac_of_8TBps": round(b / t / 1e9 / HBM_PEAK_GBPS, 4)}
    out["reslice_many_whole_model"] = many
    # fused slice + pack from a row-major parent (load-time form of the same step), largest shape of the block
    N, K = max({(N, K) for (_, N, K) in block}, key=lambda nk: nk[0] * nk[1])
    parent = mq.mq_unpack(layers[[i for i, L in enumerate(layers) if (L["N"], L["K"]) == (N, K)][0]]["packed_W"], N, K, 8, 8)
    sp = {}
    for r in WIDTHS:
        outb = torch.empty(mq.mq_packed_bytes(N, K, r), dtype=torch.uint8, device=dev)
        mq.mq_slice_pack(parent, 8, r, out=outb)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            mq.mq_slice_pack(parent, 8, r, out=outb)
        e1.record()
        torch.cuda.synchronize()
        t = e0.elapsed_time(e1) * 1e-3 / 5
        sp[str(r)] = {"us": round(t * 1e6, 1), "GBps": round((1.0 + r / 8.0) * N * K / t / 1e9, 1)}
    out["slice_pack_%dx%d" % (N, K)] = sp
    out["cpu_baseline"] = None
    print(json.dumps(out))
    return 0


FP32_VECTOR_PEAK_TFLOPS = 157.3
# Vector lanes x clock without the factor two of a fused multiply-add: 256 CUs x 4 SIMDs x 32 lanes per clock x 2.4 GHz.
# Algorithm 1's arithmetic is defined operation by operation (nothing may be fused), so this is its ceiling.
VECTOR_LANE_OPS_PEAK_T = 78.6
# Vector instructions the compiled quant_kernel<140, 4> executes per candidate and weight (R = {3,4,8}), from the
# SQ_INSTS_VALU counter in profiles/quant_kernel_alg1_llama2_7b_shapes.txt (8117 per wave of 64 lanes x 4 weights x 256
# candidates); the definition counts 19 per candidate and weight, the kernel skips recomputing terms that cannot change.
QUANT_PROFILE = os.path.join(ROOT, "profiles", "quant_kernel_alg1_llama2_7b_shapes.txt")


def quant_executed_ops_per_weight():
    """executed vector lane-operations per weight of quant_kernel<140, 4>, read from the committed counter summary"""
    import re
    try:
        m = re.search(r"R = \{3,4,8\}, \d+ weights: SQ_INSTS_VALU [^\n]*?= ([0-9.]+) per candidate and lane \(4 weights\)",
                      open(QUANT_PROFILE).read())
        return float(m.group(1)) * 256.0 / 4.0
    except (OSError, AttributeError, ValueError):
        return None


def bench_quant(args, mq, synth, torch, np, dev):
    """Algorithm 1 over whole layers: one mq_quant_matgptq launch per (shape, R); fp32 weights resident in HBM."""
    sets = {"3,4,8": ((3, 4, 8), (1.0, 1.0, 1.0)), "2,3,4,6,8": ((2, 3, 4, 6, 8), (1.0,) * 5), "8": ((8,), (1.0,))}
    table, tot_w, tot_t, tot_fl = {}, 0.0, 0.0, 0.0
    g = torch.Generator(device=dev)
    g.manual_seed(4242)
    for (N, K) in ((4096, 4096), (11008, 4096), (4096, 11008)):
        L = synth.make_layer_device(N, K, 1, seed=8000 + N, device=dev, want_x=False)
        W = torch.randn((N, K), generator=g, device=dev, dtype=torch.float32) * 0.02
        Q = torch.empty((N, K), dtype=torch.uint8, device=dev)
        for name, (widths, lam) in sets.items():
            for _ in range(max(1, args.warmup // 2)):
                mq.mq_quant_matgptq(W, L["scales"], L["zeros"], widths, lam, out=Q)
            torch.cuda.synchronize()
            reps = max(2, args.steps // 4)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                mq.mq_quant_matgptq(W, L["scales"], L["zeros"], widths, lam, out=Q)
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) * 1e-3 / reps
            # the brute force as defined: per candidate and width sub, mul, sub, mul, mul, add; one compare per candidate
            fl = (6.0 * len(widths) + 1.0) * 256.0 * N * K
            table[f"{N}x{K}:R{{{name}}}"] = {"us": round(t * 1e6, 1), "Gweights_per_s": round(N * K / t / 1e9, 2),
                                             "TFLOPs": round(fl / t / 1e12, 1)}
            if name == "3,4,8":
                tot_w += N * K
                tot_t += t
                tot_fl += fl
        del W, Q, L
    out = _base_line("Algorithm 1 (brute-force cross-bit-width code choice) throughput, R = {3,4,8}", tot_w / tot_t / 1e9,
                     "Gweights/s", args, tot_t * 1e3,
                     "Llama-2-7B layer shapes (4096x4096, 11008x4096, 4096x11008), fp32 weights, group 128, "
                     "c = 8, R = {3,4,8} with lambda = 1 (the paper's setting); other R in `table`", {})
    out["dtype"] = "f32"
    out["table"] = table
    # roofline: the lane-operations the kernel EXECUTES per second against the unfused vector peak (the brute force as
    # defined counts 19 operations per candidate and weight; the kernel executes fewer because a width's term is only
    # recomputed where its slice changes, so the counted-work rate would exceed the peak and say nothing)
    ops_w = quant_executed_ops_per_weight()
    counted = tot_fl / tot_t / 1e12
    if ops_w is not None:
        ach = ops_w * tot_w / tot_t / 1e12
        out["roofline"] = {"bound": "alu", "kernel": "mq::quant_kernel<140, 4>", "achieved": round(ach, 1),
                           "peak": VECTOR_LANE_OPS_PEAK_T, "unit": "T lane-op/s", "frac": round(ach / VECTOR_LANE_OPS_PEAK_T, 4),
                           "avg_launch_us": round(tot_t / 3 * 1e6, 1),
                           "executed_lane_ops_per_weight": round(ops_w, 1),
                           "executed_ops_source": os.path.relpath(QUANT_PROFILE, ROOT),
                           "counted_brute_force_Tops": round(counted, 1), "traffic": None}
    else:
        out["roofline"] = {"bound": "alu", "kernel": "mq::quant_kernel<140, 4>", "achieved": None,
                           "peak": VECTOR_LANE_OPS_PEAK_T, "unit": "T lane-op/s", "frac": None,
                           "counted_brute_force_Tops": round(counted, 1), "traffic": None}
    cpu = None
    if not args.no_cpu:
        import oracle
        N, K, rows = 4096, 4096, 32
        Wh = synth.make_weights(rows, K, [4242, 1])
        _, sh, zh = synth.quantize_parent(Wh)
        done, ct = 0, 0.0
        while ct < 10.0:
            ta = time.perf_counter()
            oracle.quant_matgptq(Wh, sh, zh, 8, (3, 4, 8), (1.0, 1.0, 1.0), 128, np.float32)
            ct += time.perf_counter() - ta
            done += rows * K
        cpu = {"value": round(done / ct / 1e9, 5), "unit": "Gweights/s", "cores": 1, "kind": "oracle",
               "sample": f"numpy oracle (oracle/mq_quant_oracle.py, binary32) on {rows} rows of a 4096-column layer, "
                         f"R = {{3,4,8}}, repeated for {ct:.1f} s", "seconds": round(ct, 2)}
    out["cpu_baseline"] = cpu
    print(json.dumps(out))
    return 0


def measure_decode_fusions(mq, synth, torch, np, dev, M, n_blocks, steps):
    """Decode-shaped fusions: the linears of a decoder block that share their input (q/k/v; gate/up) as ONE
    mq_linear_stack launch each, against one mq_linear launch per linear.  Llama-2-7B shapes, per-layer widths by
    seed (mean 3.5 bits), every block its own weights (cold), replayed from a HIP graph."""
    block = synth.LLAMA2_7B_BLOCK
    shapes = synth.stack_shapes(block, n_blocks)
    widths, mean = synth.draw_bitwidths([N * K for (_, _, N, K) in shapes], 3.5, seed=0)
    proto = {}
    blocks, nbytes = [], 0.0
    it = iter(widths)
    for b in range(n_blocks):
        lays = {}
        xh = torch.randn((M, 4096), device=dev, dtype=torch.float32).to(torch.float16)       # hidden state
        xa = torch.randn((M, 4096), device=dev, dtype=torch.float32).to(torch.float16)       # attention output
        xm = torch.randn((M, 11008), device=dev, dtype=torch.float32).to(torch.float16)      # MLP activation
        for (name, N, K) in block:
            r = int(next(it))
            if (N, K, r) not in proto:
                L = synth.make_layer_device(N, K, M, seed=6000 + len(proto), device=dev, want_x=False)
                proto[(N, K, r)] = mq.prepare_layer(L["parent"], L["scales"], L["zeros"], r)
            p = proto[(N, K, r)]
            x = xm if K == 11008 else xa if name.startswith("o") else xh
            lays[name] = dict(packed_W=p["packed_W"].clone(), scales_t=p["scales_t"].clone(), zeros_t=p["zeros_t"].clone(),
                              N=N, K=K, r=r, x=x, y=torch.empty((M, N), dtype=torch.float16, device=dev))
            nbytes += algo_bytes(N, K, r, M)
        blocks.append(lays)
    names = [n for (n, _, _) in block]
    qkv, gu = names[0:3], names[4:6]
    single = [n for n in names if n not in qkv + gu]
    # one workspace for every mq_linear call: the largest any width needs (the prepared activations depend on r)
    ws = torch.empty(max(mq.mq_workspace_bytes(M, 11008, 11008, r) for r in WIDTHS), dtype=torch.uint8, device=dev)
    mq.mq_workspace_init(ws)
    for lays in blocks:
        lays["_qkv"] = mq.mq_stack_plan([lays[n] for n in qkv], M, device=dev)
        lays["_gu"] = mq.mq_stack_plan([lays[n] for n in gu], M, device=dev)

    def per_linear():
        for lays in blocks:
            for n in names:
                L = lays[n]
                mq.mq_linear(L["x"], L["packed_W"], L["scales_t"], L["zeros_t"], L["N"], L["K"], L["r"], 128, ws, y=L["y"])

    def fused():
        for lays in blocks:
            mq.mq_linear_stack(lays["_qkv"])
            L = lays[single[0]]
            mq.mq_linear(L["x"], L["packed_W"], L["scales_t"], L["zeros_t"], L["N"], L["K"], L["r"], 128, ws, y=L["y"])
            mq.mq_linear_stack(lays["_gu"])
            L = lays[single[1]]
            mq.mq_linear(L["x"], L["packed_W"], L["scales_t"], L["zeros_t"], L["N"], L["K"], L["r"], 128, ws, y=L["y"])

    res = {}
    for label, fn in (("one_launch_per_linear", per_linear), ("fused_qkv_and_gate_up", fused)):
        fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        t = e0.elapsed_time(e1) * 1e-3 / steps
        res[label] = {"us_per_block": round(t / n_blocks * 1e6, 2), "GBps": round(nbytes / t / 1e9, 1),
                      "launches_per_block": 7 if label.startswith("one") else 4}
        del g
    return res, nbytes, mean


def measure_chain(mq, synth, torch, np, dev, M, n_chains, steps, widths=(3, 4, 8)):
    """A chained small stack: three dependent 4096 x 4096 links (x -> y0 -> y1 -> y2) as ONE launch whose later layers
    wait inside the launch for the earlier ones (MQ_X_AFTER_EARLIER), against the same links as three launches in stream
    order.  Every chain has its own weights (cold), replayed from a HIP graph."""
    proto = []
    for i, r in enumerate(widths):
        L = synth.make_layer_device(4096, 4096, M, seed=6100 + i, device=dev, want_x=False)
        proto.append(mq.prepare_layer(L["parent"], L["scales"], L["zeros"], r))
    chains, nbytes = [], 0.0
    for c in range(n_chains):
        x = torch.randn((M, 4096), device=dev, dtype=torch.float32).to(torch.float16)
        lays = []
        for i, r in enumerate(widths):
            p = proto[i]
            y = torch.empty((M, 4096), dtype=torch.float16, device=dev)
            lays.append(dict(packed_W=p["packed_W"].clone(), scales_t=p["scales_t"].clone(), zeros_t=p["zeros_t"].clone(),
                             N=4096, K=4096, r=r, x=x, y=y, flags=mq.MQ_X_AFTER_EARLIER if i else 0))
            x = y
            nbytes += algo_bytes(4096, 4096, r, M)
        chains.append((lays, mq.mq_stack_plan(lays, M, device=dev)))
    ws = torch.empty(max(mq.mq_workspace_bytes(M, 4096, 4096, r) for r in widths), dtype=torch.uint8, device=dev)
    mq.mq_workspace_init(ws)

    def chained():
        for _, plan in chains:
            mq.mq_linear_stack(plan)

    def per_link():
        for lays, _ in chains:
            for L in lays:
                mq.mq_linear(L["x"], L["packed_W"], L["scales_t"], L["zeros_t"], L["N"], L["K"], L["r"], 128, ws, y=L["y"])

    res = {}
    for label, fn in (("one_launch_per_link", per_link), ("chained_one_launch", chained)):
        fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        t = e0.elapsed_time(e1) * 1e-3 / steps
        res[label] = {"us_per_chain": round(t / n_chains * 1e6, 2), "GBps": round(nbytes / t / 1e9, 1),
                      "launches_per_chain": len(widths) if label.startswith("one") else 1}
        del g
    # both ways compute the same chain (the launch shapes differ, so the sums are ordered differently: equal to rounding)
    lays = chains[0][0]
    chained()
    torch.cuda.synchronize()
    want = [L["y"].float().clone() for L in lays]
    per_link()
    torch.cuda.synchronize()
    res["max_abs_diff_between_the_two"] = max(float((L["y"].float() - w).abs().max()) for L, w in zip(lays, want))
    return res


def bench_decode_fusions(args, mq, synth, torch, np, dev):
    M, n_blocks = args.batch, args.layers
    res, nbytes, mean = measure_decode_fusions(mq, synth, torch, np, dev, M, n_blocks, args.steps)
    t_f = res["fused_qkv_and_gate_up"]["us_per_block"] * n_blocks * 1e-6
    out = _base_line("decoder-block linears with shared-input fusions, effective HBM GB/s", nbytes / t_f / 1e9, "GB/s", args,
                     t_f * 1e3, f"Llama-2-7B decoder blocks x{n_blocks}, M={M}, per-layer r by seed (mean {mean:.3f} bits): "
                     "q/k/v and gate/up as one mq_linear_stack launch each, o and down as mq_linear", {"M": M})
    out["table"] = res
    out["roofline"] = {"bound": "hbm", "kernel": "mq::stack_kernel<%d, 1, false> + mq::linear_rb_kernel" % M,
                       "achieved": res["fused_qkv_and_gate_up"]["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                       "frac": round(res["fused_qkv_and_gate_up"]["GBps"] / HBM_PEAK_GBPS, 4), "avg_launch_us": None,
                       "algorithmic_bytes_per_launch": None, "traffic": None}
    out["cpu_baseline"] = None
    print(json.dumps(out))
    return 0


def bench_gptq(args, mq, synth, torch, np, dev):
    """The MatGPTQ column loop per layer: mq_matgptq_quantize on a working copy of W, U resident."""
    widths, lam = (3, 4, 8), (1.0, 1.0, 1.0)
    g = torch.Generator(device=dev)
    g.manual_seed(777)
    table, tot_w, tot_t, tot_fl = {}, 0.0, 0.0, 0.0
    for (N, K) in ((4096, 4096), (11008, 4096), (4096, 11008)):
        L = synth.make_layer_device(N, K, 1, seed=8100 + N, device=dev, want_x=False)
        W = torch.randn((N, K), generator=g, device=dev, dtype=torch.float32) * 0.02
        # calibration statistics: H = 2 X X^T + 1 % damping on seeded features; U = chol(H^-1)^T (library calls: input creation)
        X = torch.randn((K, 2 * K), generator=g, device=dev, dtype=torch.float32)
        X *= 1.0 + 3.0 * torch.rand((K, 1), generator=g, device=dev)
        H = (2.0 * X @ X.T).double()
        del X
        H += 0.01 * H.diagonal().mean() * torch.eye(K, device=dev, dtype=torch.float64)
        U = torch.linalg.cholesky(torch.linalg.inv(H)).T.contiguous().float()
        del H
        Wc = torch.empty_like(W)
        Q = torch.empty((N, K), dtype=torch.uint8, device=dev)
        reps = max(1, args.steps // 10)
        for it in range(1 + reps):
            Wc.copy_(W)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            mq.mq_matgptq_quantize(Wc, U, L["scales"], L["zeros"], widths, lam, out=Q)
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) * 1e-3                      # the last repetition is reported
        # algorithmic flops: Algorithm 1's brute force per weight (256 x (6|R| + 1)), the error (3|R| + 1 per weight)
        # and the updates (every weight receives one multiply and one subtract from each earlier column: N K (K-1))
        fl = N * K * (256.0 * (6 * len(widths) + 1) + 3 * len(widths) + 1) + float(N) * K * (K - 1)
        table[f"{N}x{K}"] = {"ms": round(t * 1e3, 2), "Mweights_per_s": round(N * K / t / 1e6, 1),
                             "us_per_column": round(t / K * 1e6, 2), "TFLOPs": round(fl / t / 1e12, 1)}
        tot_w += N * K
        tot_t += t
        tot_fl += fl
        del W, Wc, Q, U, L
    out = _base_line("MatGPTQ column loop (Algorithm 2) throughput, R = {3,4,8}", tot_w / tot_t / 1e9, "Gweights/s", args,
                     tot_t * 1e3, "Llama-2-7B layer shapes (4096x4096, 11008x4096, 4096x11008), fp32 weights, group 128, "
                     "block 128, c = 8, R = {3,4,8}, lambda = 1; Cholesky factor of the inverse Hessian given", {})
    out["dtype"] = "f32"
    out["table"] = table
    ach = tot_fl / tot_t / 1e12
    # a dependent chain over the columns: the figure is low by construction (latency per column step x K)
    out["roofline"] = {"bound": "alu", "kernel": "mq::gptq_block_kernel<140, LPR> + mq::gptq_trailing_kernel<true>",
                       "achieved": round(ach, 1), "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                       "frac": round(ach / FP32_VECTOR_PEAK_TFLOPS, 4), "avg_launch_us": None,
                       "algorithmic_flops_per_launch": None, "traffic": None}
    out["cpu_baseline"] = None
    print(json.dumps(out))
    return 0


def measure_mlp(mq, synth, torch, dev, shapes, widths, batches, reps):
    """mq_linear per (shape, r, M) on the Llama-3-70B MLP shapes, cold (four distinct weight copies cycled)."""
    table = {}
    for (name, N, K) in shapes:
        L = synth.make_layer_device(N, K, max(batches), seed=9000 + N, device=dev)
        for r in widths:
            lay = mq.prepare_layer(L["parent"], L["scales"], L["zeros"], r)
            copies = [(lay["packed_W"].clone(), lay["scales_t"].clone(), lay["zeros_t"].clone()) for _ in range(4)]
            for M in batches:
                x = L["x"][:M].contiguous()
                ws = mq.new_workspace(M, N, K, r)
                y = torch.empty((M, N), dtype=torch.float16, device=dev)

                def run():
                    for (p, s, z) in copies:
                        mq.mq_linear(x, p, s, z, N, K, r, 128, ws, y=y)
                run()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    run()
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / (reps * len(copies))
                b, fl = algo_bytes(N, K, r, M), 2.0 * M * N * K
                table[f"{name}:{N}x{K}:r{r}:M{M}"] = {"us": round(us, 1), "GBps": round(b / us / 1e3, 1),
                                                     "hbm_frac": round(b / us / 1e3 / HBM_PEAK_GBPS, 4),
                                                     "TFLOPs": round(fl / us / 1e6, 1),
                                                     "mfma_frac": round(fl / us / 1e6 / 2500.0, 4), "bytes": b}
            del copies
        del L
    return table


def bench_mlp_batched(args, mq, synth, torch, np, dev):
    """Batched regime on the Llama-3-70B MLP shapes: mq_linear per (shape, r, M), cold (cycling copies)."""
    table = measure_mlp(mq, synth, torch, dev, (("up", 28672, 8192), ("down", 8192, 28672)), (3, 4, 8), (1, 4, 16, 64, 256),
                        max(1, args.steps // 4))
    tot_b = sum(v.pop("bytes") for v in table.values())
    tot_t = sum(v["us"] for v in table.values())
    out = _base_line("batched sliced linear, effective HBM GB/s and MFMA utilisation", tot_b / tot_t / 1e3, "GB/s", args,
                     tot_t / 1e3, "Llama-3-70B MLP shapes (28672x8192, 8192x28672), M in {1,4,16,64,256}, r in {3,4,8}, "
                     "one mq_linear launch per call, 4 distinct weight copies cycled", {})
    out["table"] = table
    # dense regime: the M = 256 calls (activation prep launch + mq::wide_stack_kernel<4>, timed together per call)
    big = [v for k, v in table.items() if k.endswith(":M256")]
    fl = float(np.mean([v["TFLOPs"] for v in big]))
    out["roofline"] = {"bound": "mfma", "kernel": "mq::wide_stack_kernel<4>", "achieved": round(fl, 1), "peak": 2500.0,
                       "unit": "TFLOP/s", "frac": round(fl / 2500.0, 4),
                       "avg_launch_us": round(float(np.mean([v["us"] for v in big])), 1),
                       "algorithmic_flops_per_launch": int(2 * 256 * 28672 * 8192), "traffic": None}
    out["cpu_baseline"] = None
    print(json.dumps(out))
    return 0


def measure_read_probe(mq, torch, dev, gib=4, reps=10):
    """What a plain streaming read achieves: mq_read_probe over a buffer far beyond the last-level cache."""
    buf = torch.empty(gib << 30, dtype=torch.uint8, device=dev)
    buf.zero_()
    out = torch.zeros(1, dtype=torch.int32, device=dev)
    for _ in range(3):
        mq.mq_read_probe(buf, out)
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    for k in range(reps):
        evs[k].record()
        mq.mq_read_probe(buf, out)
    evs[reps].record()
    torch.cuda.synchronize()
    us = sorted(evs[k].elapsed_time(evs[k + 1]) * 1e3 for k in range(reps))
    med = us[len(us) // 2]
    nbytes = buf.numel()
    del buf
    torch.cuda.empty_cache()
    return {"GBps": round(nbytes / med / 1e3, 1), "frac_of_8TBps": round(nbytes / med / 1e3 / HBM_PEAK_GBPS, 4),
            "bytes": nbytes, "us_median": round(med, 1), "us_min": round(us[0], 1),
            "kernel": "mq::read_probe_kernel (non-temporal 16-byte loads, contiguous share per wave)"}


if __name__ == "__main__":
    sys.exit(main())
