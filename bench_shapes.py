#!/usr/bin/env python3
"""Side measurements of the FlexiQ hot path on one MI355X: everything that is not the headline workload of
bench.py.  One JSON line per section on stdout, progress on stderr.

Sections (`--what`, comma-separated, default all):
  copy      achievable HBM bandwidth: one plain device copy of 2 GiB (read + write bytes / time)
  linear    ViT-B fc2 and ViT-L fc1 / fc2 at full size, r in {0, .5, 1}, int8 requant epilogue
  small_m   ViT-L fc1 / fc2 with M in {1, 16, 64} rows: the weight-streaming case (GB/s of weight bytes)
  conv      the 3x3 256->256 convolution at 14x14, batch 64, r in {0, .5, 1}
  resnet50  one pass over the 52 convolutions of ResNet-50 stages 1-4 at batch 128 (22 unique shapes, every layer
            packed once, inputs and outputs of every layer in buffers of their own, so that a pass touches more
            memory than the 256 MB last-level cache holds: the cold regime), with the low-bit ratio drawn per call
            from the seeded schedule, and the same pass at fixed ratios (the difference is the cost of switching)

All inputs are seeded and synthetic (module `workloads`).  Launches are captured into HIP graphs (ten launches of a
shape, or one whole pass) and the median of seven replays, after about 40 ms of untimed ones, is reported.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0
HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def emit(section, **kw):
    print(json.dumps({"section": section, **kw}), flush=True)


def median_replay_us(torch, graph, launches, repeats=7, settle_s=0.04):
    t_end = time.perf_counter() + settle_s      # the card needs tens of milliseconds of work to reach its running clocks
    while time.perf_counter() < t_end:
        graph.replay()
    torch.cuda.synchronize()
    ts = []
    for _ in range(repeats):
        a0 = torch.cuda.Event(enable_timing=True)
        a1 = torch.cuda.Event(enable_timing=True)
        a0.record()
        graph.replay()
        a1.record()
        torch.cuda.synchronize()
        ts.append(a0.elapsed_time(a1) * 1e3 / launches)
    return float(np.median(ts))


def calib(case):
    Xc = case.Xcal.reshape(-1, case.Xcal.shape[-1])
    amax = np.abs(Xc).max(0)
    return float(np.float32(amax.max()) / np.float32(127.0)), amax


def section_copy(torch, dev):
    n = 2 << 30
    src = torch.empty(n, dtype=torch.int8, device=dev)
    dst = torch.empty_like(src)
    src.fill_(1)
    dst.copy_(src)
    torch.cuda.synchronize()
    ts = []
    for _ in range(5):
        a0 = torch.cuda.Event(enable_timing=True)
        a1 = torch.cuda.Event(enable_timing=True)
        a0.record()
        dst.copy_(src)
        a1.record()
        torch.cuda.synchronize()
        ts.append(a0.elapsed_time(a1) * 1e3)
    us = float(np.median(ts))
    emit("copy", bytes_read_plus_written=2 * n, us=round(us, 1), GBs=round(2 * n / us / 1e3, 1),
         frac_hbm_peak=round(2 * n / us / 1e3 / HBM_PEAK_GBS, 3))


def time_linear(torch, fq, dev, case, ratios, M=None):
    x_scale, amax = calib(case)
    layer = fq.flexiq_quantize_pack(case.W, amax, x_scale, case.group_size, bias=case.bias)
    X = case.X if M is None else case.X[:M]
    Xq = fq.flexiq_permute_channels(layer, fq.flexiq_quantize_act(torch.from_numpy(np.ascontiguousarray(X)).to(dev), x_scale))
    fq.flexiq_set_ratio(layer, 0.0)
    y0 = fq.flexiq_mixed_gemm(layer, Xq, y=True)["y"]
    out_scale = float(y0.abs().max().item() / 127.0)
    del y0
    rows = Xq.shape[0]
    bufs = {"q": torch.empty((rows, case.N), dtype=torch.int8, device=dev)}
    res = []
    for r in ratios:
        fq.flexiq_set_ratio(layer, r)
        for _ in range(2):
            fq.flexiq_mixed_gemm(layer, Xq, q=True, out_scale=out_scale, bufs=bufs)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(10):
                fq.flexiq_mixed_gemm(layer, Xq, q=True, out_scale=out_scale, bufs=bufs)
        us = median_replay_us(torch, g, 10)
        del g
        ops = 2.0 * rows * case.N * case.K
        wbytes = case.N * case.K * (1.0 - r / 2.0)
        res.append({"r": r, "us": round(us, 2), "tops": round(ops / us / 1e6, 1),
                    "frac_int8_mfma_peak": round(ops / us / 1e6 / INT8_MFMA_PEAK_TOPS, 4),
                    "weight_stream_GBs": round(wbytes / us / 1e3, 1), "launch": fq.debug_last_launch()})
    return res


def section_linear(torch, fq, workloads, dev):
    for mk, which in ((workloads.config1, "fc2"), (workloads.config3, "fc1"), (workloads.config3, "fc2")):
        case = mk(which)
        res = time_linear(torch, fq, dev, case, (0.0, 0.5, 1.0))
        emit("linear", workload=case.name, M=case.M, K=case.K, N=case.N, group_size=case.group_size, per_r=res)
        log("linear", case.name, [(x["r"], x["us"], x["tops"]) for x in res])
        del case


def section_small_m(torch, fq, workloads, dev):
    for which in ("fc1", "fc2"):
        case = workloads.config3(which, M=64)
        for M in (1, 16, 64):
            res = time_linear(torch, fq, dev, case, (0.0, 1.0), M=M)
            emit("small_m", workload=case.name, M=M, K=case.K, N=case.N, per_r=res)
            log("small_m", case.name, M, [(x["r"], x["us"], x["weight_stream_GBs"]) for x in res])


def prepare_conv(torch, fq, dev, case):
    x_scale, amax = calib(case)
    layer = fq.flexiq_quantize_pack(case.W, amax, x_scale, case.group_size, bias=case.bias)
    Xq = fq.flexiq_permute_channels(layer, fq.flexiq_quantize_act(torch.from_numpy(case.X).to(dev), x_scale))
    fq.flexiq_set_ratio(layer, 0.0)
    y0 = fq.flexiq_mixed_conv_implicit(layer, Xq, case.stride, case.pad, y=True)["y"]
    out_scale = float(y0.abs().max().item() / 127.0)
    del y0
    return layer, Xq, out_scale


def conv_bytes(case, r):
    M = case.B * case.Ho * case.Wo
    K = case.R * case.S * case.C
    # a 1x1 filter with a stride reads only the pixels it lands on
    pixels = case.Ho * case.Wo if case.R == 1 and case.S == 1 else case.H * case.Wd
    return case.B * pixels * case.C + case.N * K * (1.0 - r / 2.0) + M * case.N


def section_conv(torch, fq, workloads, dev):
    case = workloads.config2()
    layer, Xq, out_scale = prepare_conv(torch, fq, dev, case)
    M, K = case.B * case.Ho * case.Wo, case.R * case.S * case.C
    q = torch.empty((case.B, case.Ho, case.Wo, case.N), dtype=torch.int8, device=dev)
    res = []
    for r in (0.0, 0.5, 1.0):
        fq.flexiq_set_ratio(layer, r)
        call = lambda: fq.flexiq_mixed_conv_implicit(layer, Xq, case.stride, case.pad, q=True, out_scale=out_scale, bufs={"q": q})
        for _ in range(2):
            call()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(10):
                call()
        us = median_replay_us(torch, g, 10)
        del g
        res.append({"r": r, "us": round(us, 2), "tops": round(2.0 * M * case.N * K / us / 1e6, 1),
                    "algorithmic_GBs": round(conv_bytes(case, r) / us / 1e3, 1), "launch": fq.debug_last_launch()})
    emit("conv", workload=case.name, M=M, K=K, N=case.N, per_r=res)
    log("conv", case.name, [(x["r"], x["us"], x["tops"]) for x in res])


def section_resnet50(torch, fq, workloads, dev):
    shapes = workloads.resnet50_shapes()
    layers = []
    t0 = time.time()
    for i, sh in enumerate(shapes):
        case = workloads.config4_layer(i, B=128)
        layer, Xq, out_scale = prepare_conv(torch, fq, dev, case)
        M, K = case.B * case.Ho * case.Wo, case.R * case.S * case.C
        # every occurrence of the shape writes a buffer of its own
        outs = [torch.empty((case.B, case.Ho, case.Wo, case.N), dtype=torch.int8, device=dev) for _ in range(sh.count)]
        layers.append({"name": sh.name, "count": sh.count, "layer": layer, "X": Xq, "so": out_scale, "outs": outs,
                       "stride": case.stride, "pad": case.pad, "M": M, "K": K, "N": case.N,
                       "bytes": [conv_bytes(case, r) for r in (0.0, 0.25, 0.5, 0.75, 1.0)]})
        del case
        log("resnet50: prepared %s (%.0fs)" % (sh.name, time.time() - t0))
    calls = [(L, j) for L in layers for j in range(L["count"])]     # network order: by stage, occurrences together
    sched = workloads.config4_ratio_schedule(len(calls))
    ops = sum(2.0 * L["M"] * L["N"] * L["K"] for L, _ in calls)

    def one_pass(ratio_of_call):
        for c, (L, j) in enumerate(calls):
            fq.flexiq_set_ratio(L["layer"], float(ratio_of_call(c)))
            fq.flexiq_mixed_conv_implicit(L["layer"], L["X"], L["stride"], L["pad"], q=True, out_scale=L["so"],
                                          bufs={"q": L["outs"][j]})

    def timed(ratio_of_call):
        one_pass(ratio_of_call)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            one_pass(ratio_of_call)
        us = median_replay_us(torch, g, 1)
        del g
        return us

    res = {}
    us = timed(lambda c: sched[c])
    byts = sum(L["bytes"][int(round(sched[c] * 4))] for c, (L, _) in enumerate(calls))
    res["scheduled"] = {"mean_r": round(float(sched.mean()), 3), "us_per_pass": round(us, 1), "tops": round(ops / us / 1e6, 1),
                        "algorithmic_GBs": round(byts / us / 1e3, 1)}
    for r in (0.0, 0.5, 1.0):
        us = timed(lambda c: r)
        byts = sum(L["bytes"][int(round(r * 4))] for L, _ in calls)
        res["fixed_r=%g" % r] = {"us_per_pass": round(us, 1), "tops": round(ops / us / 1e6, 1),
                                 "algorithmic_GBs": round(byts / us / 1e3, 1)}
    # per unique shape at r = 0 and 1 (ten launches per graph; the shape's own buffers, so warm in the last-level cache)
    per_shape = []
    for L in layers:
        row = {"name": L["name"], "count": L["count"], "M": L["M"], "K": L["K"], "N": L["N"]}
        for r in (0.0, 1.0):
            fq.flexiq_set_ratio(L["layer"], r)
            call = lambda: fq.flexiq_mixed_conv_implicit(L["layer"], L["X"], L["stride"], L["pad"], q=True,
                                                         out_scale=L["so"], bufs={"q": L["outs"][0]})
            call()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for _ in range(10):
                    call()
            us = median_replay_us(torch, g, 10)
            del g
            row["r=%g" % r] = {"us": round(us, 2), "tops": round(2.0 * L["M"] * L["N"] * L["K"] / us / 1e6, 1),
                               "algorithmic_GBs": round(L["bytes"][int(r * 4)] / us / 1e3, 1)}
        per_shape.append(row)
        log("resnet50", row)
    emit("resnet50", calls=len(calls), gop_per_pass=round(ops / 1e9, 1), passes=res, per_shape=per_shape)
    log("resnet50 passes", res)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--what", default="copy,linear,small_m,conv,resnet50")
    args = ap.parse_args()
    what = args.what.split(",")

    import torch

    import paper_2510_02822_amd as fq
    import workloads

    fq.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if "copy" in what:
        section_copy(torch, dev)
    if "linear" in what:
        section_linear(torch, fq, workloads, dev)
    if "small_m" in what:
        section_small_m(torch, fq, workloads, dev)
    if "conv" in what:
        section_conv(torch, fq, workloads, dev)
    if "resnet50" in what:
        section_resnet50(torch, fq, workloads, dev)


if __name__ == "__main__":
    main()
