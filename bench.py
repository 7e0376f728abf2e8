#!/usr/bin/env python3
"""Benchmark of the fused rotated-W4A16 linear on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: the fused
transform + INT4 linear (paro_rotated_linear) of each of the four linears of one 8B-class
decoder layer (config 1 of paro_inputs.CONFIGS: batch-1 decode, hidden 4096, group 128, K = 8).
Inputs are resident in HBM before the timed region.  Decode streams every weight once per
token, so consecutive steps use different copies of the layer's weights from a pool larger
than the 256 MB Infinity Cache - as successive layers of a real model would.

Prints ONE JSON line (see the keys below).  `value` is the achieved algorithmic HBM bandwidth
of the step: bytes that must move (packed codes + group scales + 4-bit zeros + X + Y + rotation
parameters at 8 B per pair + channel scales) divided by the time per step.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# `bench.py --pmc-probe`, scaled by the same counters on a 256 MiB copy (profiles/ has the runs)
TRAFFIC_BYTES_PER_LAUNCH = {1: 64_800_000}
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense fp16


def algorithmic_bytes(c_in: int, c_out: int, T: int, rotated: bool = True, K: int = 8) -> int:
    g = c_in // 128
    b = c_out * c_in // 2            # INT4 codes
    b += g * c_out * 2               # fp16 group scales
    b += g * c_out // 2              # 4-bit zero points
    b += T * c_in * 2 + T * c_out * 2
    if rotated:
        b += g * K * 64 * 8 + c_in * 2   # pairs (2 x int16) + theta (fp32) per pair, channel scales
    return b


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1, help="workload config (1: 8B decode b1, 2: b16, 4: 32B b1)")
    ap.add_argument("--pool-mb", type=int, default=1200, help="minimum total size of the weight-copy pool")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-prefill", action="store_true", help="skip the prefill (config 3) side measurement")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: 3 plain 256 MiB device copies, then on the dominant linear 3 fused "
                         "launches, 3 bare launches and 3 pure-read launches over the same bytes, each on distinct "
                         "weight copies; prints nothing else")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); multi-GPU runs are not part of it", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paro_inputs as pin
    import paper_2511_10645_amd as paro

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    paro.lib()
    cfg = pin.CONFIGS[args.config]
    T = cfg.tokens[0]
    dev = "cuda"

    # ---- inputs, resident in HBM --------------------------------------------------------
    lin = []
    layer_packed_bytes = 0
    for li_idx, shp in enumerate(cfg.linears):
        li = pin.make_linear(args.config, li_idx, tokens=T, keep_codes=False)
        rot = paro.Rotation(li.pairs, li.theta, li.ch_scale)
        paro.paro_rotation_plan_build(rot)
        w = paro.W4Weight(li.qweight, li.scales, li.qzeros)
        paro.paro_w4_repack(w)
        w.drop_interchange()
        layer_packed_bytes += w.packed.numel()
        lin.append(dict(shape=shp, li=li, rot=rot, w=w, x=torch.as_tensor(li.x).to(dev),
                        y=torch.empty((T, shp.c_out), dtype=torch.float16, device=dev),
                        bytes=algorithmic_bytes(shp.c_in, shp.c_out, T),
                        bytes_bare=algorithmic_bytes(shp.c_in, shp.c_out, T, rotated=False)))
    # every linear cycles through its own pool of >= pool_mb, so that it misses the Infinity Cache
    # both inside the layer step and when it is timed alone
    for L in lin:
        copies = [L["w"]]
        L["n_copies"] = max(2, -(-args.pool_mb * (1 << 20) // L["w"].packed.numel()))
        for _ in range(L["n_copies"] - 1):
            c = paro.W4Weight.__new__(paro.W4Weight)
            c.c_in, c.c_out = L["w"].c_in, L["w"].c_out
            c.qweight = c.scales = c.qzeros = c.bias = None
            c.packed = L["w"].packed.clone()
            c.c = type(L["w"].c)(c.c_in, c.c_out, 128, None, None, None, None, c.packed.data_ptr())
            copies.append(c)
        L["copies"] = copies
        L["ws"] = paro.Workspace(paro.paro_workspace_bytes(L["rot"], L["w"], T))
    torch.cuda.synchronize()

    def step(i: int, which=None, bare: bool = False):
        for k, L in enumerate(lin):
            if which is not None and k != which:
                continue
            w = L["copies"][i % L["n_copies"]]
            if bare:
                paro.paro_w4a16_linear(w, L["x"], L["ws"], L["y"])
            else:
                paro.paro_rotated_linear(L["rot"], w, L["x"], L["ws"], L["y"])

    def timed(n_steps: int, warmup: int, which=None, bare: bool = False) -> float:
        """ms per step over exactly n_steps steps, HIP events on the launch stream."""
        stream = torch.cuda.current_stream()
        for i in range(warmup):
            step(i, which, bare)
        torch.cuda.synchronize()
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if args.no_graph:
            start.record(stream)
            for i in range(n_steps):
                step(i, which, bare)
            stop.record(stream)
            torch.cuda.synchronize()
            return start.elapsed_time(stop) / n_steps
        # capture the steps once (launch-bound loop), replay as one graph
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for i in range(n_steps):
                    step(i, which, bare)
        stream.wait_stream(side)
        g.replay()                      # untimed: first replay uploads the graph
        torch.cuda.synchronize()
        start.record(stream)
        g.replay()
        stop.record(stream)
        torch.cuda.synchronize()
        return start.elapsed_time(stop) / n_steps

    if args.pmc_probe:
        dom = max(lin, key=lambda L: L["bytes"])
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        k = lin.index(dom)
        for i in range(3):
            step(i, which=k)
        for i in range(3, 6):
            step(i, which=k, bare=True)
        for i in range(6, 9):
            c = dom["copies"][i % dom["n_copies"]]
            paro.paro_diag_read_stream(c.packed, c.packed.numel() // 16 * 16)
        torch.cuda.synchronize()
        return 0

    # ---- the timed region: exactly --steps steps of the whole layer ---------------------------
    ms_step = timed(args.steps, args.warmup)
    step_bytes = sum(L["bytes"] for L in lin)
    value = step_bytes / (ms_step * 1e-3) / 1e9

    # ---- per-linear launch durations (same pool, same launch configuration) ---------------------
    per = {}
    for k, L in enumerate(lin):
        ms_f = timed(args.steps, 5, which=k)
        ms_b = timed(args.steps, 5, which=k, bare=True)
        per[L["shape"].name] = {
            "us_fused": round(ms_f * 1e3, 3), "us_bare": round(ms_b * 1e3, 3),
            "gbs_fused": round(L["bytes"] / (ms_f * 1e-3) / 1e9, 1),
            "gbs_bare": round(L["bytes_bare"] / (ms_b * 1e-3) / 1e9, 1),
        }
    ms_bare_step = timed(args.steps, 5, bare=True)
    overhead_pct = 100.0 * (ms_step - ms_bare_step) / ms_bare_step

    dom = max(lin, key=lambda L: L["bytes"])
    dom_us = per[dom["shape"].name]["us_fused"]
    achieved = dom["bytes"] / (dom_us * 1e-6) / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": TRAFFIC_BYTES_PER_LAUNCH.get(args.config),
                "kernel": (f"decode_kernel (fused, split-K, T={T})" if T <= 4 else
                           f"rotate_planned_kernel + decode_wide_kernel (two launches, T={T})")
                          + f" on {dom['shape'].name} {dom['shape'].c_in}->{dom['shape'].c_out}",
                "algorithmic_bytes_per_launch": dom["bytes"], "avg_launch_us": dom_us}

    # ---- prefill side (config 3: 2048 tokens): rotation pass + MFMA GEMM per linear ----------------
    prefill = None
    if not args.no_prefill and args.config in (1, 4):
        pcfg = 3 if args.config == 1 else 4             # config 3 = the 8B shapes at 2048 tokens; config 4 has its own 4096
        Tp = pin.CONFIGS[pcfg].tokens[-1]
        prefill = {"tokens": Tp, "per_linear": {}}
        tot_fl = tot_us = tot_us_bare = 0.0
        for k, L in enumerate(lin):
            shp = L["shape"]
            xp = torch.as_tensor(pin.make_x(pcfg, k, Tp, shp.c_in, pin.CONFIGS[pcfg].n_outlier(shp.c_in))[0]).to(dev)
            xr = torch.empty_like(xp)
            yp = torch.empty((Tp, shp.c_out), dtype=torch.float16, device=dev)
            wsp = paro.Workspace(paro.paro_workspace_bytes(L["rot"], L["w"], Tp))

            def t_us(fn, n=10):
                # graph replay, so that host launch time does not count against the short kernels
                for _ in range(2):
                    fn()
                torch.cuda.synchronize()
                g = torch.cuda.CUDAGraph()
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    with torch.cuda.graph(g, stream=side):
                        for _ in range(n):
                            fn()
                torch.cuda.current_stream().wait_stream(side)
                g.replay()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                g.replay()
                e1.record()
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / n * 1e3

            us_rot = t_us(lambda: paro.paro_rotate_scale(L["rot"], xp, xr))
            us_gemm = t_us(lambda: paro.paro_w4a16_linear(L["w"], xr, wsp, yp))
            us_full = t_us(lambda: paro.paro_rotated_linear(L["rot"], L["w"], xp, wsp, yp))
            fl = 2.0 * Tp * shp.c_in * shp.c_out
            prefill["per_linear"][shp.name] = {
                "us_rotate": round(us_rot, 1), "rotate_gbs": round(Tp * shp.c_in * 4 / us_rot / 1e3, 1),
                "us_gemm": round(us_gemm, 1), "gemm_tflops": round(fl / us_gemm / 1e6, 1),
                "us_rotated_linear": round(us_full, 1)}
            tot_fl += fl; tot_us += us_full; tot_us_bare += us_gemm
            del xp, xr, yp, wsp
        prefill["layer_tflops"] = round(tot_fl / tot_us / 1e6, 1)
        prefill["pct_of_mfma_f16_peak"] = round(100.0 * tot_fl / tot_us / 1e6 / MFMA_F16_PEAK_TFLOPS, 2)
        prefill["overhead_pct_vs_bare_w4a16"] = round(100.0 * (tot_us - tot_us_bare) / tot_us_bare, 2)
        prefill["tokens_per_s_layer"] = round(Tp / (tot_us * 1e-6), 1)

    # ---- per-linear transforms (the method gives q / k / v and gate / up their own): one launch --------
    multi = None
    if not args.no_prefill and args.config == 1:
        multi = {}
        xm = lin[0]["x"]
        for name, outs in (("qkv", (4096, 1024, 1024)), ("gate_up", (14336, 14336))):
            rots_m, pools = [], []
            n_cp = max(2, -(-args.pool_mb * (1 << 20) // (sum(outs) * 4096 // 2)))
            for k, n_out in enumerate(outs):
                pairs, theta, chs = pin.make_rotation(1, k, 4096)
                r = paro.Rotation(pairs, theta, chs)
                paro.paro_rotation_plan_build(r)
                rots_m.append(r)
                w0 = paro.W4Weight(pin.pack_nibbles_u32(np.random.default_rng(k).integers(0, 16, (n_out, 4096), dtype=np.uint8)),
                                   np.full((32, n_out), 0.01, dtype=np.float16),
                                   np.zeros((32, n_out // 8), dtype=np.uint32))
                paro.paro_w4_repack(w0)
                w0.drop_interchange()
                cps = [w0]
                for _ in range(n_cp - 1):
                    c = paro.W4Weight.__new__(paro.W4Weight)
                    c.c_in, c.c_out = w0.c_in, w0.c_out
                    c.qweight = c.scales = c.qzeros = c.bias = None
                    c.packed = w0.packed.clone()
                    c.c = type(w0.c)(c.c_in, c.c_out, 128, None, None, None, None, c.packed.data_ptr())
                    cps.append(c)
                pools.append(cps)
            ys_m = [torch.empty((T, n_out), dtype=torch.float16, device=dev) for n_out in outs]
            ws_s = paro.Workspace(max(paro.paro_workspace_bytes(r, p[0], T) for r, p in zip(rots_m, pools)))
            ws_m = paro.Workspace(paro.paro_workspace_bytes_multi(rots_m, [p[0] for p in pools], T))

            def run_sep(i):
                for k in range(len(outs)):
                    paro.paro_rotated_linear(rots_m[k], pools[k][i % n_cp], xm, ws_s, ys_m[k])

            def run_one(i):
                paro.paro_rotated_linear_multi(rots_m, [p[i % n_cp] for p in pools], xm, ws_m, ys_m)

            res = {}
            for label, fn in (("us_separate_launches", run_sep), ("us_one_launch", run_one)):
                g = torch.cuda.CUDAGraph()
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    fn(0)
                    torch.cuda.synchronize()
                    with torch.cuda.graph(g, stream=side):
                        for i in range(args.steps):
                            fn(i)
                torch.cuda.current_stream().wait_stream(side)
                g.replay()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                g.replay()
                e1.record()
                torch.cuda.synchronize()
                res[label] = round(e0.elapsed_time(e1) / args.steps * 1e3, 3)
            res["parts"] = [f"4096->{n}" for n in outs]
            multi[name] = res
            del pools, rots_m, ys_m

    # ---- the oracle on the host cores, bounded sample ---------------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.lib()

        def oracle_step():
            for L in lin:
                li = L["li"]
                u = oracle.rotate_scale(li.x, li.pairs, li.theta, li.ch_scale)
                oracle.linear(u, li.qweight, li.scales, li.qzeros)

        oracle_step()                                   # warm-up
        reps, t0 = 0, time.perf_counter()
        while reps < 3 or (time.perf_counter() - t0 < 10.0 and reps < 50):
            oracle_step()
            reps += 1
        dt = (time.perf_counter() - t0) / reps
        cpu = {"value": round(step_bytes / dt / 1e9, 3), "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
               "sample": f"{reps} full steps (all 4 linears, T={T}) of the fp64 oracle, {dt * 1e3:.1f} ms per step",
               "ms_per_step": round(dt * 1e3, 2)}

    out = {
        "metric": "fused rotated-W4A16 linear: decode HBM GB/s",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 6), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"config {args.config} ({cfg.name}): one decoder layer's 4 linears "
                               + ", ".join(f"{s.name} {s.c_in}->{s.c_out}" for s in cfg.linears)
                               + f"; T={T}, group 128, K=8; every linear cycles through >= {args.pool_mb} MB of weight copies",
                   "launch": "eager" if args.no_graph else "hip graph replay", "tokens": T},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "tokens_per_s_layer": round(T / (ms_step * 1e-3), 1),
        "overhead_pct_vs_bare_w4a16": round(overhead_pct, 2),
        "ms_per_step_bare": round(ms_bare_step, 6),
        "per_linear": per,
        "prefill": prefill, "own_transform_per_projection": multi,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
