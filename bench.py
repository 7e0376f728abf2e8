#!/usr/bin/env python3
"""Benchmark of the fused rotated-W4A16 linear on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: the fused
transform + INT4 linear (paro_rotated_linear) of each of the four linears of one 8B-class
decoder layer (config 1 of paro_inputs.CONFIGS: batch-1 decode, hidden 4096, group 128, K = 8).
Inputs are resident in HBM before the timed region.  Decode streams every weight once per
token, so consecutive steps use different copies of the layer's weights from a pool larger
than the 256 MB Infinity Cache - as successive layers of a real model would.

Prints ONE JSON line.  `value` is the achieved algorithmic HBM bandwidth of the step: bytes that
must move (packed codes + group scales + 4-bit zeros + X + Y + rotation parameters at 8 B per
pair + channel scales) divided by the time per step.  Beside the contract's keys the line carries:
  per_linear           fused / bare launch times of config 1, each over a walk of the whole pool
  config2, config4     the same step on the 16-token and the 32B-class shapes (compact records)
  prefill              config 3 (2048 tokens): rotation pass, MFMA GEMM, fused call per linear
  rotate_vs_fwht       transform kernel against the Walsh-Hadamard yardstick over channel counts
  ceiling              what a pure-read kernel and a pure-MFMA loop reach on this machine, so that
                       every roofline fraction can also be read against the measured ceiling
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
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense fp16
MFMA_FP4_PEAK_TFLOPS = 10100.0 # dense fp4
# HBM bytes per launch of the dominant fused kernel (gate/up) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs of `bench.py --pmc-probe [--config 4]`, scaled by the same counters on a 256 MiB copy
# (profiles/decode_stream_pmc.md).  Configs 1 and 4 (one token): the streaming kernel whose waves transform their own
# K-slice (62.07 MB + 0.06 MB written; 148.45 + 0.11).  Config 2 (16 tokens) takes the two-launch route (rotation pass +
# bare kernel): the sum of both launches' counters (62.3 MB + 0.9 MB written by the linear, 0.4 MB by the pass).
TRAFFIC_BYTES_PER_LAUNCH = {1: 62_100_000, 2: 63_600_000, 4: 148_600_000}


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
    ap.add_argument("--config", type=int, default=1, help="headline workload (1: 8B decode b1, 2: b16, 4: 32B b1)")
    ap.add_argument("--pool-mb", type=int, default=1200, help="minimum total size of each linear's weight-copy pool")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-prefill", action="store_true", help="skip the prefill (config 3) side measurement")
    ap.add_argument("--no-extras", action="store_true", help="headline and per-linear figures only")
    ap.add_argument("--mxfp4-probe", action="store_true",
                    help="for rocprofv3: a few launches of the MXFP4 x MXFP4 linear on gate/up (1 token and 2048) and nothing else")
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
    dev = "cuda"

    def clone_weight(w0):
        c = paro.W4Weight.__new__(paro.W4Weight)
        c.c_in, c.c_out = w0.c_in, w0.c_out
        c.qweight = c.scales = c.qzeros = c.bias = None
        c.packed = w0.packed.clone()
        c.c = type(w0.c)(c.c_in, c.c_out, 128, None, None, None, None, c.packed.data_ptr())
        return c

    def build_layer(config: int, T: int, weights_from=None):
        """The four linears of a config at T tokens, each with its own pool of >= pool_mb of weight copies (so that it
        misses the Infinity Cache inside the layer step and when timed alone).  weights_from: reuse another layer's
        rotations and pools (config 2 has config 1's shapes)."""
        cfg = pin.CONFIGS[config]
        lin = []
        for k, shp in enumerate(cfg.linears):
            if weights_from is not None:
                src = weights_from[k]
                rot, copies, li = src["rot"], src["copies"], None
                x = torch.as_tensor(pin.make_x(config, k, T, shp.c_in, cfg.n_outlier(shp.c_in))[0]).to(dev)
            else:
                li = pin.make_linear(config, k, tokens=T, keep_codes=False)
                rot = paro.Rotation(li.pairs, li.theta, li.ch_scale)
                paro.paro_rotation_plan_build(rot)
                w = paro.W4Weight(li.qweight, li.scales, li.qzeros)
                paro.paro_w4_repack(w)
                w.drop_interchange()
                n_copies = max(2, -(-args.pool_mb * (1 << 20) // w.packed.numel()))
                copies = [w] + [clone_weight(w) for _ in range(n_copies - 1)]
                x = torch.as_tensor(li.x).to(dev)
            lin.append(dict(shape=shp, li=li, rot=rot, copies=copies, n_copies=len(copies), x=x,
                            y=torch.empty((T, shp.c_out), dtype=torch.float16, device=dev),
                            ws=paro.Workspace(max(paro.paro_workspace_bytes(rot, copies[0], T),
                                                  paro.paro_workspace_bytes(None, copies[0], T))),
                            bytes=algorithmic_bytes(shp.c_in, shp.c_out, T),
                            bytes_bare=algorithmic_bytes(shp.c_in, shp.c_out, T, rotated=False)))
        torch.cuda.synchronize()
        return lin

    def step(lin, i: int, which=None, bare: bool = False):
        for k, L in enumerate(lin):
            if which is not None and k != which:
                continue
            w = L["copies"][i % L["n_copies"]]
            if bare:
                paro.paro_w4a16_linear(w, L["x"], L["ws"], L["y"])
            else:
                paro.paro_rotated_linear(L["rot"], w, L["x"], L["ws"], L["y"])

    def graph_ms(fn, n: int, warmup: int) -> float:
        """ms per call of fn(i) over exactly n calls, HIP events on the launch stream; the n calls are
        captured once (launch-bound loop) and replayed as one graph."""
        stream = torch.cuda.current_stream()
        for i in range(warmup):
            fn(i)
        torch.cuda.synchronize()
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if args.no_graph:
            start.record(stream)
            for i in range(n):
                fn(i)
            stop.record(stream)
            torch.cuda.synchronize()
            return start.elapsed_time(stop) / n
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for i in range(n):
                    fn(i)
        stream.wait_stream(side)
        g.replay()                      # untimed: first replay uploads the graph
        torch.cuda.synchronize()
        start.record(stream)
        g.replay()
        stop.record(stream)
        torch.cuda.synchronize()
        return start.elapsed_time(stop) / n

    def time_layer(lin, n_steps: int, warmup: int):
        """Layer step fused / bare over exactly n_steps steps, and every linear alone over a walk of its WHOLE pool
        (so that no copy is reused within 1 GB, whatever n_steps is)."""
        ms_step = graph_ms(lambda i: step(lin, i), n_steps, warmup)
        ms_bare = graph_ms(lambda i: step(lin, i, bare=True), n_steps, min(warmup, 5))
        per = {}
        for k, L in enumerate(lin):
            n = max(n_steps, L["n_copies"])
            ms_f = graph_ms(lambda i: step(lin, i, which=k), n, 3)
            ms_b = graph_ms(lambda i: step(lin, i, which=k, bare=True), n, 3)
            per[L["shape"].name] = {
                "us_fused": round(ms_f * 1e3, 3), "us_bare": round(ms_b * 1e3, 3),
                "gbs_fused": round(L["bytes"] / (ms_f * 1e-3) / 1e9, 1),
                "gbs_bare": round(L["bytes_bare"] / (ms_b * 1e-3) / 1e9, 1),
                "overhead_pct": round(100.0 * (ms_f - ms_b) / ms_b, 1), "launches_timed": n,
            }
        return ms_step, ms_bare, per

    def read_ceiling_us(L) -> float:
        """A pure-read kernel over the same weight copies (same bytes, same pool walk), best of several grid sizes."""
        nbytes = L["copies"][0].packed.numel() // 16 * 16
        n = max(20, L["n_copies"])
        return min(graph_ms(lambda i: paro.paro_diag_read_stream(L["copies"][i % L["n_copies"]].packed, nbytes, blocks), n, 3)
                   for blocks in (512, 1024, 2048, 4096)) * 1e3

    def two_launches(L, T: int) -> bool:
        # the call asks for a scratch part exactly when the transform runs as a pass of its own
        w = L["copies"][0]
        return paro.paro_workspace_bytes(L["rot"], w, T) > paro.paro_workspace_exchange_bytes(L["rot"], w, T)

    def fused_kernels(L, T: int) -> str:
        # which kernels the fused call launches on this shape, read off the workspace it asks for
        w = L["copies"][0]
        if two_launches(L, T):
            return f"rotate_planned_kernel + decode_wide_kernel (two launches, T={T})"
        ex = paro.paro_workspace_exchange_bytes(L["rot"], w, T)
        if T == 1 and L["shape"].c_in > 512 and ex == max(256, paro.paro_workspace_exchange_bytes(None, w, T)):
            return "decode_wide_kernel (every wave transforms its own K-slice, T=1)"
        return f"decode_kernel (fused, split-K, T={T})"

    def roofline_of(config: int, lin, per, T: int):
        dom = max(lin, key=lambda L: L["bytes"])
        dom_us = per[dom["shape"].name]["us_fused"]
        achieved = dom["bytes"] / (dom_us * 1e-6) / 1e9
        read_us = read_ceiling_us(dom)
        read_bytes = dom["copies"][0].packed.numel()
        return {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": TRAFFIC_BYTES_PER_LAUNCH.get(config),
                "kernel": fused_kernels(dom, T) + f" on {dom['shape'].name} {dom['shape'].c_in}->{dom['shape'].c_out}",
                "algorithmic_bytes_per_launch": dom["bytes"], "avg_launch_us": dom_us,
                "pure_read_us_same_bytes": round(read_us, 3),
                "frac_of_measured": round((dom["bytes"] / dom_us) / (read_bytes / read_us), 4)}

    cfg = pin.CONFIGS[args.config]
    T = cfg.tokens[0]

    if args.mxfp4_probe:
        shp = max(cfg.linears, key=lambda q: q.c_in * q.c_out)
        N, C = shp.c_out, shp.c_in
        w0 = paro.Mxfp4Weight(torch.randint(-2 ** 31, 2 ** 31 - 1, (N, C // 8), dtype=torch.int32, device=dev),
                              torch.randint(112, 122, (N, C // 32), dtype=torch.uint8, device=dev))
        paro.paro_mxfp4_repack(w0)
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        for Tq in (1, 2048):
            xc = torch.randint(-2 ** 31, 2 ** 31 - 1, (Tq, C // 8), dtype=torch.int32, device=dev)
            xs = torch.randint(118, 126, (Tq, C // 32), dtype=torch.uint8, device=dev)
            yq = torch.empty((Tq, N), dtype=torch.float16, device=dev)
            for _ in range(5):
                paro.paro_mxfp4_linear(w0, xc, xs, yq)
        torch.cuda.synchronize()
        return 0

    lin = build_layer(args.config, T)

    if args.pmc_probe:
        dom = max(lin, key=lambda L: L["bytes"])
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        k = lin.index(dom)
        for i in range(3):
            step(lin, i, which=k)
        for i in range(3, 6):
            step(lin, i, which=k, bare=True)
        for i in range(6, 9):
            c = dom["copies"][i % dom["n_copies"]]
            paro.paro_diag_read_stream(c.packed, c.packed.numel() // 16 * 16)
        torch.cuda.synchronize()
        return 0

    # ---- the timed region: exactly --steps steps of the whole layer ---------------------------
    ms_step, ms_bare_step, per = time_layer(lin, args.steps, args.warmup)
    step_bytes = sum(L["bytes"] for L in lin)
    value = step_bytes / (ms_step * 1e-3) / 1e9
    overhead_pct = 100.0 * (ms_step - ms_bare_step) / ms_bare_step
    roofline = roofline_of(args.config, lin, per, T)

    def compact(config: int, layer, Tc: int):
        ms_f, ms_b, per_c = time_layer(layer, args.steps, 5)
        nbytes = sum(L["bytes"] for L in layer)
        return {"workload": f"config {config} ({pin.CONFIGS[config].name}), T={Tc}", "tokens": Tc,
                "us_fused_layer": round(ms_f * 1e3, 3), "us_bare_layer": round(ms_b * 1e3, 3),
                "gbs": round(nbytes / (ms_f * 1e-3) / 1e9, 1), "pct_of_hbm_peak": round(100.0 * nbytes / (ms_f * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
                "overhead_pct_vs_bare_w4a16": round(100.0 * (ms_f - ms_b) / ms_b, 2),
                "per_linear": {k: {"us_fused": v["us_fused"], "us_bare": v["us_bare"]} for k, v in per_c.items()},
                "roofline": roofline_of(config, layer, per_c, Tc)}

    extras = not args.no_extras
    config2 = config4 = None
    if extras and args.config == 1:
        lin2 = build_layer(2, 16, weights_from=lin)
        config2 = compact(2, lin2, 16)
        del lin2

    # ---- prefill side (config 3: 2048 tokens): rotation pass + MFMA GEMM per linear ----------------
    def t_us(fn, n=10):
        return graph_ms(lambda i: fn(), n, 2) * 1e3

    prefill = None
    if not args.no_prefill and args.config in (1, 4):
        pcfg = 3 if args.config == 1 else 4             # config 3 = the 8B shapes at 2048 tokens; config 4 has its own 4096
        Tp = pin.CONFIGS[pcfg].tokens[-1]
        prefill = {"tokens": Tp, "per_linear": {}}
        tot_fl = tot_us = tot_us_bare = 0.0
        for k, L in enumerate(lin):
            shp = L["shape"]
            w0 = L["copies"][0]
            xp = torch.as_tensor(pin.make_x(pcfg, k, Tp, shp.c_in, pin.CONFIGS[pcfg].n_outlier(shp.c_in))[0]).to(dev)
            xr = torch.empty_like(xp)
            yp = torch.empty((Tp, shp.c_out), dtype=torch.float16, device=dev)
            wsp = paro.Workspace(paro.paro_workspace_bytes(L["rot"], w0, Tp))
            us_rot = t_us(lambda: paro.paro_rotate_scale(L["rot"], xp, xr))
            us_gemm = t_us(lambda: paro.paro_w4a16_linear(w0, xr, wsp, yp))
            us_full = t_us(lambda: paro.paro_rotated_linear(L["rot"], w0, xp, wsp, yp))
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
    if extras and not args.no_prefill and args.config == 1:
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
                pools.append([w0] + [clone_weight(w0) for _ in range(n_cp - 1)])
            ys_m = [torch.empty((T, n_out), dtype=torch.float16, device=dev) for n_out in outs]
            ws_s = paro.Workspace(max(paro.paro_workspace_bytes(r, p[0], T) for r, p in zip(rots_m, pools)))
            ws_m = paro.Workspace(paro.paro_workspace_bytes_multi(rots_m, [p[0] for p in pools], T))

            def run_sep(i):
                for k in range(len(outs)):
                    paro.paro_rotated_linear(rots_m[k], pools[k][i % n_cp], xm, ws_s, ys_m[k])

            def run_one(i):
                paro.paro_rotated_linear_multi(rots_m, [p[i % n_cp] for p in pools], xm, ws_m, ys_m)

            multi[name] = {"us_separate_launches": round(graph_ms(run_sep, max(args.steps, n_cp), 2) * 1e3, 3),
                           "us_one_launch": round(graph_ms(run_one, max(args.steps, n_cp), 2) * 1e3, 3),
                           "parts": [f"4096->{n}" for n in outs]}
            del pools, rots_m, ys_m

    # ---- the transform kernel against the Walsh-Hadamard yardstick (Section 4.3's figure) ----------------
    fwht = None
    if extras and not args.no_prefill:
        fwht = {"tokens": 2048, "by_channels": {}}
        for C in (1024, 2048, 4096, 8192, 16384, 32768):
            pairs, theta, chs = pin.make_rotation(9, 0, C)
            r = paro.Rotation(pairs, theta, chs)
            paro.paro_rotation_plan_build(r)
            n_buf = max(2, min(8, int(600e6 // (2048 * C * 2))))
            xs = [torch.randn(2048, C, device=dev, dtype=torch.float16) for _ in range(n_buf)]
            ys = [torch.empty_like(xb) for xb in xs]
            us_r = graph_ms(lambda i: paro.paro_rotate_scale(r, xs[i % n_buf], ys[i % n_buf]), 20, 2) * 1e3
            us_h = graph_ms(lambda i: paro.paro_fwht(xs[i % n_buf], ys[i % n_buf]), 20, 2) * 1e3
            fwht["by_channels"][str(C)] = {"us_rotate_k8": round(us_r, 1), "us_fwht": round(us_h, 1),
                                           "rotate_gbs": round(2048 * C * 4 / us_r / 1e3, 1),
                                           "speedup_over_fwht": round(us_h / us_r, 2)}
            del xs, ys

    # ---- measured ceilings of this machine ---------------------------------------------------------------
    ceiling = None
    if extras:
        ceiling = {"pure_read_us": {L["shape"].name: round(read_ceiling_us(L), 3) for L in lin}}
        ceiling["pure_read_layer_us"] = round(sum(ceiling["pure_read_us"].values()), 3)
        ceiling["frac_of_measured_layer"] = round(ceiling["pure_read_layer_us"] / (ms_step * 1e3), 4)
        out_f = torch.empty(1024 * 256, dtype=torch.float32, device=dev)
        mf = {}
        for label, rnd in (("constant_operands", False), ("random_operands", True)):
            fl = paro.paro_diag_mfma_f16(out_f, 1024, 2000, rnd)      # warm-up
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fl = paro.paro_diag_mfma_f16(out_f, 1024, 2000, rnd)
            e1.record()
            torch.cuda.synchronize()
            mf[label] = round(fl / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
        ceiling["mfma_f16_tflops"] = mf
        if prefill:
            prefill["frac_of_measured_mfma_random"] = round(prefill["layer_tflops"] / mf["random_operands"], 4)

    # ---- the weight-activation form with MXFP4 operands (App. A.3) on the same shapes -----------------
    w4a4 = None
    if extras and not args.no_prefill and args.config == 1:
        w4a4 = {"decode_tokens": T, "prefill_tokens": 2048, "per_linear": {}}
        tot = {"dec": 0.0, "dec_whole": 0.0, "pre": 0.0, "pre_whole": 0.0, "bytes": 0, "flop": 0.0}
        for L in lin:
            shp = L["shape"]
            N, C = shp.c_out, shp.c_in
            nbytes = N * C // 2 + N * C // 32
            w0 = paro.Mxfp4Weight(torch.randint(-2 ** 31, 2 ** 31 - 1, (N, C // 8), dtype=torch.int32, device=dev),
                                  torch.randint(112, 122, (N, C // 32), dtype=torch.uint8, device=dev))
            paro.paro_mxfp4_repack(w0)
            n_cp = max(2, -(-args.pool_mb * (1 << 20) // nbytes))
            pool = [w0]
            for _ in range(n_cp - 1):
                wc = paro.Mxfp4Weight(w0.codes, w0.scales)
                wc.packed = w0.packed.clone()
                wc.c.packed = wc.packed.data_ptr()
                pool.append(wc)
            rec = {}
            for label, Tq in (("decode", T), ("prefill", 2048)):
                xq = torch.as_tensor(pin.make_x(1, 0, Tq, C, pin.CONFIGS[1].n_outlier(C))[0]).to(dev)
                xc, xs = paro.paro_rotate_scale_quantize_mxfp4(L["rot"], xq)
                yq = torch.empty((Tq, N), dtype=torch.float16, device=dev)
                wsq = torch.empty(paro.paro_workspace_bytes_mxfp4(C, Tq), dtype=torch.uint8, device=dev)
                n_it = max(args.steps, n_cp) if label == "decode" else 10
                us_c = graph_ms(lambda i: paro.paro_mxfp4_linear(pool[i % n_cp], xc, xs, yq), n_it, 2) * 1e3
                us_w = graph_ms(lambda i: paro.paro_rotated_linear_mxfp4(L["rot"], pool[i % n_cp], xq, wsq, yq), n_it, 2) * 1e3
                if label == "decode":
                    rec.update({"us_contraction": round(us_c, 3), "us_whole": round(us_w, 3), "weight_bytes": nbytes,
                                "contraction_gbs": round(nbytes / us_c / 1e3, 1)})
                    tot["dec"] += us_c; tot["dec_whole"] += us_w; tot["bytes"] += nbytes
                else:
                    fl = 2.0 * Tq * C * N
                    rec.update({"us_contraction_prefill": round(us_c, 1), "us_whole_prefill": round(us_w, 1),
                                "contraction_tflops": round(fl / us_c / 1e6, 1)})
                    tot["pre"] += us_c; tot["pre_whole"] += us_w; tot["flop"] += fl
                del xq, xc, xs, yq, wsq
            w4a4["per_linear"][shp.name] = rec
            del pool, w0
        w4a4["decode_layer_us"] = round(tot["dec"], 3)
        w4a4["decode_layer_us_whole"] = round(tot["dec_whole"], 3)
        w4a4["decode_layer_gbs"] = round(tot["bytes"] / tot["dec"] / 1e3, 1)
        w4a4["decode_pct_of_hbm_peak"] = round(100.0 * tot["bytes"] / tot["dec"] / 1e3 / HBM_PEAK_GBS, 2)
        w4a4["prefill_layer_tflops"] = round(tot["flop"] / tot["pre"] / 1e6, 1)
        w4a4["prefill_layer_tflops_whole"] = round(tot["flop"] / tot["pre_whole"] / 1e6, 1)
        w4a4["prefill_pct_of_mfma_fp4_peak"] = round(100.0 * tot["flop"] / tot["pre"] / 1e6 / MFMA_FP4_PEAK_TFLOPS, 2)
        out_f4 = torch.empty(1024 * 512, dtype=torch.float32, device=dev)
        mf4 = {}
        for label, rnd in (("constant_operands", False), ("random_operands", True)):
            paro.paro_diag_mfma_fp4(out_f4, 1024, 1000, rnd)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fl = paro.paro_diag_mfma_fp4(out_f4, 1024, 1000, rnd)
            e1.record()
            torch.cuda.synchronize()
            mf4[label] = round(fl / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
        w4a4["mfma_fp4_tflops_measured"] = mf4
        w4a4["prefill_frac_of_measured_mfma_random"] = round(w4a4["prefill_layer_tflops"] / mf4["random_operands"], 4)

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

    # the 32B-class layer last: its pools replace config 1's in HBM
    if extras and args.config == 1:
        del lin
        torch.cuda.empty_cache()
        lin4 = build_layer(4, 1)
        config4 = compact(4, lin4, 1)
        del lin4

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
        "config2": config2, "config4": config4,
        "prefill": prefill, "own_transform_per_projection": multi,
        "rotate_vs_fwht": fwht, "ceiling": ceiling, "w4a4_mxfp4": w4a4,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
