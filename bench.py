#!/usr/bin/env python3
"""Benchmark of the FlexiQ hot path on one MI355X.

Workload (BASELINE.json `metric`: "... vs low-bit ratio r (ViT-B fc1)", configs[1]): the ViT-B/16
MLP fc1 linear at batch 32, M = 32*197 = 6304 tokens, K = 768, N = 3072, channel group size 32.
One step = one pass of the run-time hot path over the ratio sweep r in {0, .25, .5, .75, 1}: per
ratio the O(1) ratio switch, then the mixed 4/8-bit int8-MFMA GEMM with on-the-fly bit-lowering of
the activations, the weights of 4-bit groups streamed from their position-expanded int8 copy (one
byte per weight: on this route r saves no bytes), and the fused per-channel dequant + int8 requant
epilogue.  Inputs (int8 activations in stored channel order, packed layer) are resident in HBM
before the timed region; the offline steps (weight quantisation, channel order, positions, packing)
run once before it, as in the paper.

Prints ONE JSON line.  `value` = total int8 ops of the K timed steps / wall time (TOPS).
The default step and warm-up counts keep the GPU busy for a few tenths of a second: the card needs tens of
milliseconds of work to settle at its running clocks, and a short timed region after a cold start reads about 4 %
low; for the same reason about 50 ms of untimed steps run before the requested warm-up steps.
`roofline` covers the GEMM kernel (the only kernel in the timed region): algorithmic ops per launch
= 2*M*N*K, average launch duration = HIP-event time of the timed region / launches in it.  `cpu_baseline` times the
CPU oracle on a bounded row sample of the same workload.  `shapes` (after the timed region, not part of `value`)
carries the other workloads of the benchmark spec: ViT-B fc2, ViT-L fc1 / fc2 (int8 kernel and the FP6 variant of the
4-bit phase), fc1 -> fc2 chains, the 3x3 convolution, the ResNet-50 pass with the seeded ratio schedule, few-row
calls, the residual reorder operator and a plain 2 GiB device copy as the HBM ceiling.
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

METRIC = "mixed int4/int8 GEMM TOPS & % int8 MFMA peak vs low-bit ratio r (ViT-B fc1)"
INT8_MFMA_PEAK_TOPS = 5000.0     # MI355X dense int8 matrix peak, 5.0 POP/s
HBM_PEAK_GBS = 8000.0
RATIOS = (0.0, 0.25, 0.5, 0.75, 1.0)

# Bytes per launch of the GEMM kernel on the default workload (fc1, int8 output) measured with
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by the readings of a 256 MiB device copy (fetch x2.0,
# write x1.0): median fetch 25.8 MB + write 19.4 MB.  See profiles/k_mixed_vitb_fc1_hbm_traffic.txt.
MEASURED_TRAFFIC_BYTES = {("fc1", "q"): 45.2e6}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(M, N, K, r, out_bytes_per_elem=1, weight_route="w4x"):
    """Bytes one call must move: int8 activations, weights, position table and scales, output.  Weights of 4-bit
    groups: one byte each on the route that streams the position-expanded copy (`w4x`, the int8 kernel's default),
    half a byte when the packed codes are streamed (`w4`), 3/4 byte as FP6 (`w6`; activations of those groups too)."""
    wb = {"w4x": 1.0, "w4": 0.5, "w6": 0.75}[weight_route]
    xb = 0.75 if weight_route == "w6" else 1.0
    return M * K * (1.0 - r + r * xb) + N * K * (1.0 - r + r * wb) + N * (K // 32) + 8 * N + M * N * out_bytes_per_elem


def _median_graph_us(torch, fn, launches, repeats=5, settle_s=0.02):
    """Median microseconds per launch of `fn`, captured `launches` times into a HIP graph."""
    fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(launches):
            fn()
    t_end = time.perf_counter() + settle_s
    while time.perf_counter() < t_end:
        g.replay()
    torch.cuda.synchronize()
    # ... and until two replays in a row agree within 3 % (at most one second more): after seconds of host-only work
    # (packing a layer, the CPU oracle) the card takes longer than that to be back at its running clocks
    t_end = time.perf_counter() + 1.0
    prev = None
    while time.perf_counter() < t_end:
        b0 = torch.cuda.Event(enable_timing=True)
        b1 = torch.cuda.Event(enable_timing=True)
        b0.record()
        g.replay()
        b1.record()
        torch.cuda.synchronize()
        cur = b0.elapsed_time(b1)
        if prev is not None and abs(cur - prev) <= 0.03 * min(cur, prev):
            break
        prev = cur
    ts = []
    for _ in range(repeats):
        a0 = torch.cuda.Event(enable_timing=True)
        a1 = torch.cuda.Event(enable_timing=True)
        a0.record()
        g.replay()
        a1.record()
        torch.cuda.synchronize()
        ts.append(a0.elapsed_time(a1) * 1e3 / launches)
    del g
    return float(np.median(ts))


def _calib(case):
    Xc = case.Xcal.reshape(-1, case.Xcal.shape[-1])
    amax = np.abs(Xc).max(0)
    return float(np.float32(amax.max()) / np.float32(127.0)), amax


def measure_shapes(torch, fq, workloads, dev, resnet=True):
    """The other workloads of the benchmark spec (not in `value`): one compact record per (workload, variant, r)."""
    out = []

    def rec(workload, variant, r, us, ops=None, byts=None, **kw):
        e = {"workload": workload, "variant": variant, "r": r, "us": round(us, 2)}
        if ops is not None:
            e["tops"] = round(ops / us / 1e6, 1)
            e["frac_mfma_peak"] = round(ops / us / 1e6 / INT8_MFMA_PEAK_TOPS, 4)
        if byts is not None:
            e["GBs"] = round(byts / us / 1e3, 1)
            e["frac_hbm_peak"] = round(byts / us / 1e3 / HBM_PEAK_GBS, 4)
        e["bound"] = kw.pop("bound", "mfma" if ops is not None else "hbm")
        e.update(kw)
        out.append(e)
        log("shapes:", e)

    # ---- HBM ceiling: a plain 2 GiB device copy
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
    rec("device copy 2 GiB (read + write)", "copy", None, float(np.median(ts)), byts=2.0 * n)
    del src, dst

    # ---- linear layers at full size
    packed = {}
    for name, mk, which in (("vitb_fc1", workloads.config1, "fc1"), ("vitb_fc2", workloads.config1, "fc2"), ("vitl_fc1", workloads.config3, "fc1"),
                            ("vitl_fc2", workloads.config3, "fc2")):
        case = mk(which)
        M, K, N = case.M, case.K, case.N
        x_scale, amax = _calib(case)
        layer = fq.flexiq_quantize_pack(case.W, amax, x_scale, case.group_size, bias=case.bias)
        Xn = fq.flexiq_quantize_act(torch.from_numpy(case.X).to(dev), x_scale)
        Xq = fq.flexiq_permute_channels(layer, Xn)
        if name == "vitl_fc2":      # the residual reorder operator (Section 5 step 3) on the largest activation tensor
            us = _median_graph_us(torch, lambda: fq.flexiq_permute_channels(layer, Xn), 10)
            rec("channel reorder %d x %d int8" % (M, K), "permute_channels", None, us, byts=2.0 * M * K)
        del Xn
        fq.flexiq_set_ratio(layer, 0.0)
        y0 = fq.flexiq_mixed_gemm(layer, Xq, y=True)["y"]
        so = float(y0.abs().max().item() / 127.0)
        del y0
        bufs = {"q": torch.empty((M, N), dtype=torch.int8, device=dev)}
        ops = 2.0 * M * N * K
        wl = "%s M=%d K=%d N=%d gs=%d" % (name, M, K, N, case.group_size)
        for r in (0.0, 0.5, 1.0):
            fq.flexiq_set_ratio(layer, r)
            us = _median_graph_us(torch, lambda: fq.flexiq_mixed_gemm(layer, Xq, q=True, out_scale=so, bufs=bufs), 10)
            rec(wl, "int8 kernel, activations lowered on the fly", r, us, ops=ops)
            x6, xlow = fq.flexiq_lower_fp6(layer, Xq)
            us = _median_graph_us(torch, lambda: fq.flexiq_mixed_gemm_fp6(layer, xlow, x6, q=True, out_scale=so, bufs=bufs), 10)
            rec(wl, "FP6 variant of the 4-bit phase, activations packed by the producer", r, us, ops=ops,
                fp6_channels=fq.flexiq_fp6_channels(layer))
            if r > 0:
                x4 = fq.flexiq_lower_packed4(layer, Xq)
                us = _median_graph_us(torch, lambda: fq.flexiq_mixed_gemm_packed4(layer, Xq, x4, q=True, out_scale=so, bufs=bufs), 10)
                rec(wl, "int8 kernel, 4-bit activations arrive packed (two codes per byte)", r, us, ops=ops,
                    packed_channels=fq.flexiq_packed4_channels(layer))
                del x4
                us = _median_graph_us(torch, lambda: fq.flexiq_lower_fp6(layer, Xq, x6=x6, need_xlow=False), 10)
                rec(wl, "stand-alone FP6 lowering kernel (when no producer packs)", r, us,
                    byts=M * K * r * 1.75)
            del x6, xlow
        packed[name] = (case, layer, Xq, so, x_scale)
        del bufs

    # ---- ViT-L fc1 -> fc2 chain (fc1 writes fc2's input; in the model a GELU sits between them, outside this path)
    c1, l1_plain, X1, so1, xs1 = packed["vitl_fc1"]
    c2 = packed["vitl_fc2"][0]
    M = c1.M
    am2 = np.full(c2.K, 127.0 * so1, np.float32)
    l2 = fq.flexiq_quantize_pack(c2.W, am2, so1, c2.group_size, bias=c2.bias)
    l1 = fq.flexiq_quantize_pack(c1.W, _calib(c1)[1], xs1, c1.group_size, bias=c1.bias, out_perm=l2.info()["perm"])
    mid = {"q": torch.empty((M, c1.N), dtype=torch.int8, device=dev)}
    fin = {"q": torch.empty((M, c2.N), dtype=torch.int8, device=dev)}
    x6_2 = torch.empty(fq.flexiq_fp6_bytes(l2, M), dtype=torch.uint8, device=dev)
    ops2 = 2.0 * M * (c1.N * c1.K + c2.N * c2.K)
    for r in (0.0, 0.5, 1.0):
        fq.flexiq_set_ratio(l1, r)
        fq.flexiq_set_ratio(l2, r)

        def chain_plain():
            fq.flexiq_mixed_gemm(l1, X1, q=True, out_scale=so1, bufs=mid)
            fq.flexiq_mixed_gemm(l2, mid["q"], q=True, out_scale=so1, bufs=fin)

        def chain_lowered():
            fq.flexiq_mixed_gemm(l1, X1, q=True, out_scale=so1, bufs=mid, lower_for=l2)
            fq.flexiq_mixed_gemm(l2, mid["q"], q=True, out_scale=so1, bufs=fin)

        # the same chain with 16 rows (few-row kernels): consumer lowers on the fly against producer lowers for the consumer
        X16 = X1[:16].contiguous()
        mid16 = {"q": mid["q"][:16]}
        fin16 = {"q": fin["q"][:16]}

        def few_plain():
            fq.flexiq_mixed_gemm(l1, X16, q=True, out_scale=so1, bufs=mid16)
            fq.flexiq_mixed_gemm(l2, mid16["q"], q=True, out_scale=so1, bufs=fin16)

        def few_lowered():
            fq.flexiq_mixed_gemm(l1, X16, q=True, out_scale=so1, bufs=mid16, lower_for=l2)
            fq.flexiq_mixed_gemm(l2, mid16["q"], q=True, out_scale=so1, bufs=fin16)

        wl16 = "vitl fc1 -> fc2 chain, M=16 rows (few-row kernels)"
        by16 = c1.N * c1.K + c2.N * c2.K + 16 * (c1.K + 2 * c1.N + c2.N)
        rec(wl16, "int8 kernels, consumer lowers on the fly", r, _median_graph_us(torch, few_plain, 10), byts=by16)
        fq.flexiq_input_prelowered(l2, True)
        rec(wl16, "int8 kernels, producer lowers for the consumer", r, _median_graph_us(torch, few_lowered, 10), byts=by16)
        fq.flexiq_input_prelowered(l2, False)

        # the same chain on one image's tokens (197 rows: a tile per block, the reduction split over its waves)
        X197 = X1[:197].contiguous()
        mid197 = {"q": torch.empty((197, c1.N), dtype=torch.int8, device=dev)}
        fin197 = {"q": torch.empty((197, c2.N), dtype=torch.int8, device=dev)}
        x6_197 = torch.empty(fq.flexiq_fp6_bytes(l2, 197), dtype=torch.uint8, device=dev)
        x6_a, xlow_a = fq.flexiq_lower_fp6(l1, X197)

        def img_plain():
            fq.flexiq_mixed_gemm(l1, X197, q=True, out_scale=so1, bufs=mid197)
            fq.flexiq_mixed_gemm(l2, mid197["q"], q=True, out_scale=so1, bufs=fin197)

        def img_lowered():
            fq.flexiq_mixed_gemm(l1, X197, q=True, out_scale=so1, bufs=mid197, lower_for=l2)
            fq.flexiq_mixed_gemm(l2, mid197["q"], q=True, out_scale=so1, bufs=fin197)

        def img_fp6():
            fq.flexiq_mixed_gemm_fp6(l1, xlow_a, x6_a, q=True, out_scale=so1, bufs=mid197, lower_for=l2, x6_out=x6_197)
            fq.flexiq_mixed_gemm_fp6(l2, mid197["q"], x6_197, q=True, out_scale=so1, bufs=fin197)

        wl197 = "vitl fc1 -> fc2 chain, M=197 rows (one image)"
        by197 = c1.N * c1.K + c2.N * c2.K + 197 * (c1.K + 2 * c1.N + c2.N)
        rec(wl197, "int8 kernels, consumer lowers on the fly", r, _median_graph_us(torch, img_plain, 10), byts=by197)
        fq.flexiq_input_prelowered(l2, True)
        rec(wl197, "int8 kernels, producer lowers for the consumer", r, _median_graph_us(torch, img_lowered, 10), byts=by197)
        fq.flexiq_input_prelowered(l2, False)
        rec(wl197, "FP6 variant, producer packs the consumer's FP6 activations", r, _median_graph_us(torch, img_fp6, 10), byts=by197)
        del x6_a, xlow_a, x6_197

        x6_1, xlow_1 = fq.flexiq_lower_fp6(l1, X1)

        def chain_fp6():
            fq.flexiq_mixed_gemm_fp6(l1, xlow_1, x6_1, q=True, out_scale=so1, bufs=mid, lower_for=l2, x6_out=x6_2)
            fq.flexiq_mixed_gemm_fp6(l2, mid["q"], x6_2, q=True, out_scale=so1, bufs=fin)

        wl = "vitl fc1 -> fc2 chain, M=%d" % M
        rec(wl, "int8 kernels, consumer lowers on the fly", r, _median_graph_us(torch, chain_plain, 5), ops=ops2)
        fq.flexiq_input_prelowered(l2, True)
        rec(wl, "int8 kernels, producer lowers for the consumer", r, _median_graph_us(torch, chain_lowered, 5), ops=ops2)
        fq.flexiq_input_prelowered(l2, False)
        rec(wl, "FP6 variant, producer packs the consumer's FP6 activations", r, _median_graph_us(torch, chain_fp6, 5), ops=ops2)
        del x6_1, xlow_1
        if r > 0:
            # run-time extraction positions for the consumer (Section 4.1, dynamic option; the paper reports 2-5 % of
            # the layer): the OR scan as a kernel of its own between the layers, and riding in the producer's epilogue
            def chain_scan_kernel():
                fq.flexiq_mixed_gemm(l1, X1, q=True, out_scale=so1, bufs=mid)
                fq.flexiq_dynamic_positions(l2, mid["q"])
                fq.flexiq_mixed_gemm(l2, mid["q"], q=True, out_scale=so1, bufs=fin)

            def chain_scan_fused():
                fq.flexiq_mixed_gemm(l1, X1, q=True, out_scale=so1, bufs=mid, scan_for=l2)
                fq.flexiq_mixed_gemm(l2, mid["q"], q=True, out_scale=so1, bufs=fin)

            rec(wl, "int8 kernels, consumer's positions found at run time by a scan kernel", r, _median_graph_us(torch, chain_scan_kernel, 5), ops=ops2)
            rec(wl, "int8 kernels, consumer's positions found at run time in the producer's epilogue", r, _median_graph_us(torch, chain_scan_fused, 5), ops=ops2)
            fq.flexiq_static_positions(l2)
    del l1, l2, mid, fin, x6_2

    # ---- calls of few rows (weight streaming) and of one image's tokens: ViT-L layers with M in {1, 16, 64, 197}, ViT-B layers with M = 197
    for name in ("vitl_fc1", "vitl_fc2", "vitb_fc1", "vitb_fc2"):
        case, layer, Xq, so, _ = packed[name]
        for Ms in ((1, 16, 64, 197) if name.startswith("vitl") else (197,)):
            Xs = Xq[:Ms].contiguous()
            bufs = {"q": torch.empty((Ms, case.N), dtype=torch.int8, device=dev)}
            for r in (0.0, 0.5, 1.0):
                fq.flexiq_set_ratio(layer, r)
                for tag, force in (("tiled kernel", 0), ("automatic route", -1)):
                    fq.debug_force_few_rows(force)
                    fq.debug_force_tile_splitk(force)
                    us = _median_graph_us(torch, lambda: fq.flexiq_mixed_gemm(layer, Xs, q=True, out_scale=so, bufs=bufs), 20)
                    launch = fq.debug_last_launch()
                    # (of the few-row kernels only the dot-product one streams the packed 4-bit codes)
                    route = "w4" if launch["tile"] == -4 and fq.debug_force_few_rows(force) == 2 else "w4x"
                    kern = {-4: ": few-row kernel", -5: ": tile per block, reduction split over its waves"}.get(launch["tile"], "")
                    rec("%s weights %d x %d, M=%d rows" % (name, case.N, case.K, Ms), "%s call, %s%s" % ("few-row" if Ms <= 64 else "one-image", tag, kern), r, us,
                        byts=algorithmic_bytes(Ms, case.N, case.K, r, 1, route), launch=launch)
                fq.debug_force_few_rows(-1)
                fq.debug_force_tile_splitk(-1)
                if Ms >= 16:   # the FP6 variant of the 4-bit phase (activations packed by the producer)
                    x6, xlow = fq.flexiq_lower_fp6(layer, Xs)
                    us = _median_graph_us(torch, lambda: fq.flexiq_mixed_gemm_fp6(layer, xlow, x6, q=True, out_scale=so, bufs=bufs), 20)
                    k6 = fq.flexiq_fp6_channels(layer)
                    kern = "tile per block, reduction split over its waves" if fq.debug_force_tile_splitk(-1) > 0 else ("few-row kernel" if Ms <= 64 else "tiled FP6 kernel")
                    rec("%s weights %d x %d, M=%d rows" % (name, case.N, case.K, Ms), "%s call, FP6 variant of the 4-bit phase (%s)" % ("few-row" if Ms <= 64 else "one-image", kern), r, us,
                        byts=Ms * case.K + case.N * (case.K - k6 // 4) + Ms * case.N, fp6_channels=k6)
                    del x6, xlow
    packed.clear()

    # ---- the weight-streaming regime proper: one activation row against a 16384 x 4096 weight matrix (67 MB as int8, group
    # size 64), where the call is HBM-bound at r = 0 and 4-bit groups move half the bytes (dot-product kernel: v_dot8_i32_i4
    # on the packed codes); seeded like the other linear layers
    case = workloads.make_linear("stream_16384x4096", 9, 16384 + 4096, 16, 4096, 16384, 64, outlier_frac=0.02)
    x_scale, amax = _calib(case)
    layer = fq.flexiq_quantize_pack(case.W, amax, x_scale, 64, bias=case.bias)
    Xq = fq.flexiq_permute_channels(layer, fq.flexiq_quantize_act(torch.from_numpy(case.X).to(dev), x_scale))
    fq.flexiq_set_ratio(layer, 0.0)
    so = float(fq.flexiq_mixed_gemm(layer, Xq, y=True)["y"].abs().max().item() / 127.0)
    # Two cache regimes: warm (one set of weights, replayed: 67 MB fit the 256 MB Infinity Cache) and cold (ten packed copies of
    # the layer taken in turn, 671 MB of int8 weights resp. 336 MB of packed codes: every call streams from HBM).  Only the cold
    # figures are HBM-roofline fractions.
    copies = [layer] + [fq.flexiq_quantize_pack(case.W, amax, x_scale, 64, bias=case.bias) for _ in range(9)]

    def cold_calls(Xs, bufs):
        for L in copies:
            fq.flexiq_mixed_gemm(L, Xs, q=True, out_scale=so, bufs=bufs)

    for Ms in (1, 2, 4, 16):
        Xs = Xq[:Ms].contiguous()
        bufs = {"q": torch.empty((Ms, case.N), dtype=torch.int8, device=dev)}
        for r in ((0.0, 0.25, 0.5, 0.75, 1.0) if Ms == 1 else (0.0, 0.5, 1.0)):
            for L in copies:
                fq.flexiq_set_ratio(L, r)
            us = _median_graph_us(torch, lambda: fq.flexiq_mixed_gemm(layer, Xs, q=True, out_scale=so, bufs=bufs), 20)
            kern = fq.debug_force_few_rows(-1)     # 2: the dot-product kernel (packed codes), 1: the matrix-core kernel (expanded copy)
            route = "w4" if kern == 2 else "w4x"
            kname = {1: "matrix-core kernel", 2: "dot-product kernel"}.get(kern, "?")
            rec("weight streaming: 16384 x 4096 weights, M=%d rows" % Ms, "few-row kernels (automatic route), warm: one weight set", r, us,
                byts=algorithmic_bytes(Ms, case.N, case.K, r, 1, route), launch=fq.debug_last_launch(), kernel=kname)
            us = _median_graph_us(torch, lambda: cold_calls(Xs, bufs), 2) / len(copies)
            rec("weight streaming: 16384 x 4096 weights, M=%d rows" % Ms, "few-row kernels (automatic route), cold: ten weight sets in turn", r, us,
                byts=algorithmic_bytes(Ms, case.N, case.K, r, 1, route), launch=fq.debug_last_launch(), kernel=kname)
            if Ms == 16:   # the FP6 variant on the few-row kernel, cold as well (the positions of all copies are the same)
                x6, xlow = fq.flexiq_lower_fp6(layer, Xs)

                def cold_fp6():
                    for L in copies:
                        fq.flexiq_mixed_gemm_fp6(L, xlow, x6, q=True, out_scale=so, bufs=bufs)

                us = _median_graph_us(torch, cold_fp6, 2) / len(copies)
                k6 = fq.flexiq_fp6_channels(layer)
                rec("weight streaming: 16384 x 4096 weights, M=%d rows" % Ms, "FP6 variant of the 4-bit phase (few-row kernel), cold: ten weight sets in turn",
                    r, us, byts=Ms * case.K + case.N * (case.K - k6 // 4) + Ms * case.N, fp6_channels=k6)
                del x6, xlow
    del layer, copies, Xq, case

    # ---- an HBM-bound layer as a linear call: the ResNet-50 stage-1 1x1 convolution 256 -> 64 at 56 x 56, batch 128
    # (M = 401408 pixels, K = 256, N = 64): int8 activations against packed 4-bit activations, where the ratio saves
    # activation bytes (algorithmic bytes: M*K*(1 - r/2) + N*K + M*N)
    case = workloads.config4_layer(3, B=128)
    Xl = case.X.reshape(-1, case.C)
    Ml = Xl.shape[0]
    x_scale, amax = _calib(case)
    layer = fq.flexiq_quantize_pack(case.W.reshape(case.N, case.C), amax, x_scale, case.group_size, bias=case.bias)
    Xq = fq.flexiq_permute_channels(layer, fq.flexiq_quantize_act(torch.from_numpy(np.ascontiguousarray(Xl)).to(dev), x_scale))
    fq.flexiq_set_ratio(layer, 0.0)
    so = float(fq.flexiq_mixed_gemm(layer, Xq, y=True)["y"].abs().max().item() / 127.0)
    bufs = {"q": torch.empty((Ml, case.N), dtype=torch.int8, device=dev)}
    wl = "resnet50 s1 1x1 256->64 as a linear layer, M=%d K=%d N=%d" % (Ml, case.C, case.N)
    for r in (0.0, 0.5, 1.0):
        fq.flexiq_set_ratio(layer, r)
        us = _median_graph_us(torch, lambda: fq.flexiq_mixed_gemm(layer, Xq, q=True, out_scale=so, bufs=bufs), 10)
        kern = {-2: "row-streaming kernel", -3: "3x3 kernel"}.get(fq.debug_last_launch()["tile"], "tiled kernel")
        rec(wl, "int8 activations, lowered on the fly", r, us, byts=Ml * case.C + case.N * case.C + Ml * case.N, kernel=kern)
        if r > 0:
            x4 = fq.flexiq_lower_packed4(layer, Xq)
            us = _median_graph_us(torch, lambda: fq.flexiq_mixed_gemm_packed4(layer, Xq, x4, q=True, out_scale=so, bufs=bufs), 10)
            k4p = fq.flexiq_packed4_channels(layer)
            rec(wl, "4-bit activations arrive packed (two codes per byte)", r, us,
                byts=Ml * (case.C - k4p // 2) + case.N * case.C + Ml * case.N)
            del x4
    del layer, Xq, bufs, case, Xl

    # ---- configuration 2: 3x3 convolution 256 -> 256 at 14 x 14, batch 64
    def conv_bytes(case, r):
        Mo = case.B * case.Ho * case.Wo
        pixels = case.Ho * case.Wo if case.R == 1 and case.S == 1 else case.H * case.Wd   # a strided 1x1 reads only its pixels
        return case.B * pixels * case.C + case.N * case.R * case.S * case.C + Mo * case.N

    def prepare_conv(case):
        x_scale, amax = _calib(case)
        layer = fq.flexiq_quantize_pack(case.W, amax, x_scale, case.group_size, bias=case.bias)
        Xq = fq.flexiq_permute_channels(layer, fq.flexiq_quantize_act(torch.from_numpy(case.X).to(dev), x_scale))
        fq.flexiq_set_ratio(layer, 0.0)
        y0 = fq.flexiq_mixed_conv_implicit(layer, Xq, case.stride, case.pad, y=True)["y"]
        so = float(y0.abs().max().item() / 127.0)
        return layer, Xq, so

    case = workloads.config2()
    layer, Xq, so = prepare_conv(case)
    q = {"q": torch.empty((case.B, case.Ho, case.Wo, case.N), dtype=torch.int8, device=dev)}
    Mo, Kc = case.B * case.Ho * case.Wo, case.R * case.S * case.C
    for r in (0.0, 0.5, 1.0):
        fq.flexiq_set_ratio(layer, r)
        us = _median_graph_us(torch, lambda: fq.flexiq_mixed_conv_implicit(layer, Xq, case.stride, case.pad, q=True, out_scale=so, bufs=q), 10)
        rec("cfg2 conv 3x3 256->256 @14x14 batch 64 (M=%d K=%d N=%d)" % (Mo, Kc, case.N), "int8 kernel, implicit GEMM", r, us,
            ops=2.0 * Mo * case.N * Kc)
    del layer, Xq, q, case

    # ---- configuration 4: ResNet-50 stages 1-4, batch 128; every layer packed once, buffers of its own (1.3 GB per
    # pass: the cold regime), the ratio drawn per call from the seeded schedule, against passes at fixed ratios
    if resnet:
        layers = []
        for i, sh in enumerate(workloads.resnet50_shapes()):
            case = workloads.config4_layer(i, B=128)
            layer, Xq, so = prepare_conv(case)
            outs = [torch.empty((case.B, case.Ho, case.Wo, case.N), dtype=torch.int8, device=dev) for _ in range(sh.count)]
            layers.append({"count": sh.count, "layer": layer, "X": Xq, "so": so, "outs": outs, "stride": case.stride, "pad": case.pad,
                           "ops": 2.0 * case.B * case.Ho * case.Wo * case.N * case.R * case.S * case.C, "bytes": conv_bytes(case, 0)})
            del case
        calls = [(L, j) for L in layers for j in range(L["count"])]
        sched = workloads.config4_ratio_schedule(len(calls))
        ops = sum(L["ops"] for L, _ in calls)
        byts = sum(L["bytes"] for L, _ in calls)

        def one_pass(ratio_of_call):
            for c, (L, j) in enumerate(calls):
                fq.flexiq_set_ratio(L["layer"], float(ratio_of_call(c)))
                fq.flexiq_mixed_conv_implicit(L["layer"], L["X"], L["stride"], L["pad"], q=True, out_scale=L["so"], bufs={"q": L["outs"][j]})

        wl = "cfg4 ResNet-50 stages 1-4, batch 128: %d convolutions, %.0f GOP per pass, cold buffers" % (len(calls), ops / 1e9)
        for tag, fn in (("fixed r", lambda c: 0.0), ("fixed r", lambda c: 0.5), ("fixed r", lambda c: 1.0),
                        ("seeded per-call ratio schedule (mean r = %.2f)" % float(sched.mean()), lambda c: sched[c])):
            us = _median_graph_us(torch, lambda: one_pass(fn), 1, repeats=5, settle_s=0.04)
            # which kernel every call of the pass ran on (eager pass after the timing; the route depends on the ratio)
            routes = {"tiled": 0, "row-streaming": 0, "3x3 resident weights": 0}
            for c, (L, j) in enumerate(calls):
                fq.flexiq_set_ratio(L["layer"], float(fn(c)))
                fq.flexiq_mixed_conv_implicit(L["layer"], L["X"], L["stride"], L["pad"], q=True, out_scale=L["so"], bufs={"q": L["outs"][j]})
                t = fq.debug_last_launch()["tile"]
                routes["row-streaming" if t == -2 else ("3x3 resident weights" if t == -3 else "tiled")] += 1
            torch.cuda.synchronize()
            rec(wl, "int8 kernels, " + tag, float(fn(0)) if tag == "fixed r" else None, us, ops=ops, GBs=round(byts / us / 1e3, 1),
                frac_hbm_peak=round(byts / us / 1e3 / HBM_PEAK_GBS, 4), bound="mixed (mfma / hbm per layer)", calls_per_kernel=routes)
        # The same pass with the bottleneck chains fused (Section 5 steps 1-2, Section 4.1 at the producer): inside a
        # bottleneck the reducing 1x1 feeds the 3x3 and the 3x3 feeds the expanding 1x1, so those producers are packed
        # with the consumer's stored channel order as their output order and lower their int8 output for it
        # (flexiq_out.lower_for); the consumers copy their activations like 8-bit ones.  The reducing 1x1 layers and
        # the downsample layers read the output of the residual addition (not a layer of this library) and still lower
        # on the fly.  Timing only: the consumers' input buffers hold the same synthetic activations as above.
        names = [sh.name for sh in workloads.resnet50_shapes()]
        consumer_of = {"s1_1x1_64_64": "s1_3x3_64_64", "s1_3x3_64_64": "s1_1x1_64_256", "s1_1x1_256_64": "s1_3x3_64_64",
                       "s2_1x1_256_128": "s2_3x3_128_128_s2", "s2_3x3_128_128_s2": "s2_1x1_128_512", "s2_1x1_512_128": "s2_3x3_128_128",
                       "s2_3x3_128_128": "s2_1x1_128_512", "s3_1x1_512_256": "s3_3x3_256_256_s2", "s3_3x3_256_256_s2": "s3_1x1_256_1024",
                       "s3_1x1_1024_256": "s3_3x3_256_256", "s3_3x3_256_256": "s3_1x1_256_1024", "s4_1x1_1024_512": "s4_3x3_512_512_s2",
                       "s4_3x3_512_512_s2": "s4_1x1_512_2048", "s4_1x1_2048_512": "s4_3x3_512_512", "s4_3x3_512_512": "s4_1x1_512_2048"}
        fed = set(consumer_of.values())
        for i, nm in enumerate(names):
            L = layers[i]
            L["consumer"] = layers[names.index(consumer_of[nm])]["layer"] if nm in consumer_of else None
            L["chained"] = L["layer"]
            if L["consumer"] is not None:
                case = workloads.config4_layer(i, B=128)
                x_scale, amax = _calib(case)
                L["chained"] = fq.flexiq_quantize_pack(case.W, amax, x_scale, case.group_size, bias=case.bias,
                                                       out_perm=L["consumer"].info()["perm"])
                del case
            L["fed"] = nm in fed

        def chained_pass(r):
            for L, j in calls:
                fq.flexiq_mixed_conv_implicit(L["chained"], L["X"], L["stride"], L["pad"], q=True, out_scale=L["so"], bufs={"q": L["outs"][j]},
                                              lower_for=L["consumer"])

        for r in (0.5, 1.0):
            for L in layers:
                fq.flexiq_set_ratio(L["layer"], r)
                fq.flexiq_set_ratio(L["chained"], r)
                fq.flexiq_input_prelowered(L["chained"], L["fed"])
            us = _median_graph_us(torch, lambda: chained_pass(r), 1, repeats=5, settle_s=0.04)
            routes = {"tiled": 0, "row-streaming": 0, "3x3 resident weights": 0}
            for L, j in calls:
                fq.flexiq_mixed_conv_implicit(L["chained"], L["X"], L["stride"], L["pad"], q=True, out_scale=L["so"], bufs={"q": L["outs"][j]},
                                              lower_for=L["consumer"])
                t = fq.debug_last_launch()["tile"]
                routes["row-streaming" if t == -2 else ("3x3 resident weights" if t == -3 else "tiled")] += 1
            torch.cuda.synchronize()
            rec(wl, "int8 kernels, fixed r, bottleneck chains fused: %d of %d calls lower for their consumer, %d read lowered input"
                % (sum(1 for L, _ in calls if L["consumer"] is not None), len(calls), sum(1 for L, _ in calls if L["fed"])),
                r, us, ops=ops, GBs=round(byts / us / 1e3, 1), frac_hbm_peak=round(byts / us / 1e3 / HBM_PEAK_GBS, 4),
                bound="mixed (mfma / hbm per layer)", calls_per_kernel=routes)
        for L in layers:
            fq.flexiq_input_prelowered(L["chained"], False)
        del layers, calls
    return out


PROFILE_TARGETS = ("vitl_fc2", "vitl_fc2_fp6", "vitl_fc2_fp6_rows64", "vitl_fc2_fp6_rows197", "vitl_fc2_rows16", "vitl_fc2_rows197", "vitl_fc2_rows1", "stream_rows1", "reorder", "resnet_1x1_64_256", "resnet_3x3_64_64",
                   "resnet_1x1_256_64", "resnet_1x1_256_64_packed4")


def profile_only(torch, fq, workloads, dev, what, launches):
    """A short eager run of ONE side workload, for rocprofv3 (no headline, no oracle): `launches` launches per ratio in
    the order r = 0, 0.5, 1 (the kernel trace lists dispatches in launch order), one copy of `--calib-copy-mib` after."""
    res = {"profile_only": what, "launches_per_ratio": launches, "ratios": [0.0, 0.5, 1.0]}
    if what.startswith("resnet_"):
        idx = {"resnet_1x1_64_256": 2, "resnet_3x3_64_64": 1, "resnet_1x1_256_64": 3, "resnet_1x1_256_64_packed4": 3}[what]
        case = workloads.config4_layer(idx, B=128)
        x_scale, amax = _calib(case)
        layer = fq.flexiq_quantize_pack(case.W, amax, x_scale, case.group_size, bias=case.bias)
        Xq = fq.flexiq_permute_channels(layer, fq.flexiq_quantize_act(torch.from_numpy(case.X).to(dev), x_scale))
        q = {"q": torch.empty((case.B, case.Ho, case.Wo, case.N), dtype=torch.int8, device=dev)}
        res["workload"] = "%s batch 128: M=%d K=%d N=%d" % (case.name, case.B * case.Ho * case.Wo, case.R * case.S * case.C, case.N)
        call = lambda: fq.flexiq_mixed_conv_implicit(layer, Xq, case.stride, case.pad, q=True, out_scale=0.05, bufs=q)
        if what.endswith("_packed4"):   # the same pixels as rows of a linear layer (packed activations are defined for those)
            Xq = Xq.reshape(-1, case.C)
            q = {"q": q["q"].reshape(-1, case.N)}
    else:
        # (stream_rows1: the weight-streaming workload of `shapes`, one row against 16384 x 4096 weights)
        case = workloads.make_linear("stream_16384x4096", 9, 16384 + 4096, 16, 4096, 16384, 64, outlier_frac=0.02) if what == "stream_rows1" \
            else workloads.config3("fc2")
        x_scale, amax = _calib(case)
        layer = fq.flexiq_quantize_pack(case.W, amax, x_scale, case.group_size, bias=case.bias)
        Xn = fq.flexiq_quantize_act(torch.from_numpy(case.X).to(dev), x_scale)
        Xq = fq.flexiq_permute_channels(layer, Xn)
        rows = {"vitl_fc2_rows16": 16, "vitl_fc2_rows1": 1, "stream_rows1": 1, "vitl_fc2_fp6_rows64": 64, "vitl_fc2_rows197": 197, "vitl_fc2_fp6_rows197": 197}.get(what, case.M)
        Xs = Xq[:rows].contiguous()
        q = {"q": torch.empty((rows, case.N), dtype=torch.int8, device=dev)}
        res["workload"] = "%s M=%d K=%d N=%d gs=%d" % (case.name, rows, case.K, case.N, case.group_size)
        if what == "vitl_fc2":
            call = lambda: fq.flexiq_mixed_gemm(layer, Xs, q=True, out_scale=0.05, bufs=q)
        elif what in ("vitl_fc2_rows16", "vitl_fc2_rows1", "stream_rows1", "vitl_fc2_rows197"):   # few-row calls (the matrix-core resp. the dot-product kernel), one image's tokens
            call = lambda: fq.flexiq_mixed_gemm(layer, Xs, q=True, out_scale=0.05, bufs=q)
        elif what == "reorder":
            call = lambda: fq.flexiq_permute_channels(layer, Xn)
        else:
            call = None   # FP6 variant: the operands depend on the ratio
    for r in res["ratios"]:
        fq.flexiq_set_ratio(layer, r)
        if what in ("vitl_fc2_fp6", "vitl_fc2_fp6_rows64", "vitl_fc2_fp6_rows197"):
            x6, xlow = fq.flexiq_lower_fp6(layer, Xs)
            call = lambda: fq.flexiq_mixed_gemm_fp6(layer, xlow, x6, q=True, out_scale=0.05, bufs=q)
        if what.endswith("_packed4"):
            x4 = fq.flexiq_lower_packed4(layer, Xq)
            call = lambda: fq.flexiq_mixed_gemm_packed4(layer, Xq, x4, q=True, out_scale=0.05, bufs=q)
        for _ in range(launches):
            call()
        torch.cuda.synchronize()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=400)
    ap.add_argument("--layer", default="fc1", choices=["fc1", "fc2"])
    ap.add_argument("--out", default="q", choices=["q", "y", "acc"], help="epilogue output written in the timed region")
    ap.add_argument("--cpu-rows", type=int, default=4096, help="rows of the workload the CPU oracle is timed on (0: skip)")
    ap.add_argument("--eager", action="store_true", help="launch from Python instead of replaying a captured HIP graph")
    ap.add_argument("--no-shapes", action="store_true", help="skip the side measurements of the other workloads (`shapes`)")
    ap.add_argument("--no-resnet", action="store_true", help="skip the ResNet-50 pass inside `shapes`")
    ap.add_argument("--profile-only", default=None, choices=PROFILE_TARGETS,
                    help="run only this side workload, eagerly, --steps launches per ratio in {0, 0.5, 1} (for rocprofv3)")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="after the timed region run one plain device copy of this many MiB (reference for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (the method is single-device; rows of M would shard "
            "data-parallel with replicated weights).  --gpus %d is not supported." % args.gpus)
        sys.exit(2)

    import torch

    import paper_2510_02822_amd as fq
    import workloads

    fq.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.profile_only:
        res = profile_only(torch, fq, workloads, dev, args.profile_only, args.steps)
        if args.calib_copy_mib > 0:
            n = args.calib_copy_mib << 20
            src = torch.ones(n, dtype=torch.int8, device=dev)
            dst = torch.empty_like(src)
            dst.copy_(src)
            torch.cuda.synchronize()
            res["calib_copy_bytes"] = n
        print(json.dumps(res), flush=True)
        return

    t0 = time.time()
    case = workloads.config1(args.layer)
    M, K, N, gs = case.M, case.K, case.N, case.group_size
    absmax_c = np.abs(case.Xcal).max(0)
    x_scale = float(np.float32(absmax_c.max()) / np.float32(127.0))
    layer = fq.flexiq_quantize_pack(case.W, absmax_c, x_scale, gs, bias=case.bias)
    Xq_nat = fq.flexiq_quantize_act(torch.from_numpy(case.X).to(dev), x_scale)
    Xq = fq.flexiq_permute_channels(layer, Xq_nat)
    torch.cuda.synchronize()
    log("setup %.1fs: %s M=%d K=%d N=%d gs=%d" % (time.time() - t0, case.name, M, K, N, gs))

    # output scale for the requant epilogue: from one fp32 pass at r = 0
    fq.flexiq_set_ratio(layer, 0.0)
    y0 = fq.flexiq_mixed_gemm(layer, Xq, y=True)["y"]
    out_scale = float(y0.abs().max().item() / 127.0)
    del y0
    want = {"acc": args.out == "acc", "y": args.out == "y", "q": args.out == "q"}
    dt = {"acc": torch.int32, "y": torch.float32, "q": torch.int8}[args.out]
    bufs = {args.out: torch.empty((M, N), dtype=dt, device=dev)}
    out_bytes = 1 if args.out == "q" else 4

    def one_step():
        for r in RATIOS:
            fq.flexiq_set_ratio(layer, r)      # O(1) host-side switch; the value travels as a kernel argument
            fq.flexiq_mixed_gemm(layer, Xq, out_scale=out_scale, bufs=bufs, **want)

    for _ in range(2):
        one_step()
    torch.cuda.synchronize()
    # Steps (ratio sweeps) are captured into a HIP graph, several to a graph, and replayed: launch-bound Python
    # overhead and most graph-to-graph launch gaps stay out of the device timeline.  --eager launches from Python.
    chunk = 1
    if not args.eager:
        chunk = next(c for c in (20, 10, 5, 4, 2, 1) if args.steps % c == 0)
        step_graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(step_graph):
            for _ in range(chunk):
                one_step()
        run_chunk = step_graph.replay
    else:
        run_chunk = one_step

    # Untimed: about 50 ms of the same steps, so that the card has settled at its running clocks whatever warm-up and
    # step counts were asked for (a cold start reads about 4 % low), then the requested warm-up steps.
    t_settle = time.perf_counter() + 0.05
    while time.perf_counter() < t_settle:
        run_chunk()
    torch.cuda.synchronize()
    for _ in range(-(-args.warmup // chunk)):    # at least the requested warm-up steps
        run_chunk()
    torch.cuda.synchronize()

    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    e0.record()
    for _ in range(args.steps // chunk):      # exactly args.steps steps
        run_chunk()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t1
    dev_us = e0.elapsed_time(e1) * 1e3          # HIP events on the launch stream around the timed region

    # per-ratio launch times (outside the timed region): 50 launches per graph, median of 7 replays
    per_r_us = {}
    for r in RATIOS:
        fq.flexiq_set_ratio(layer, r)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(50):
                fq.flexiq_mixed_gemm(layer, Xq, out_scale=out_scale, bufs=bufs, **want)
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        ts = []
        for _ in range(7):
            a0 = torch.cuda.Event(enable_timing=True)
            a1 = torch.cuda.Event(enable_timing=True)
            a0.record()
            g.replay()
            a1.record()
            torch.cuda.synchronize()
            ts.append(a0.elapsed_time(a1) * 1e3 / 50)
        per_r_us[r] = float(np.median(ts))
        del g

    # the same GEMM when the producing layer has lowered the activations already (flexiq_out.lower_for on the
    # producer, flexiq_input_prelowered on this layer): what the fused producer epilogue buys the consumer.
    # Side measurement; the timed region above lowers on the fly.
    pre = []
    fq.flexiq_input_prelowered(layer, True)
    for r in RATIOS[1:]:
        fq.flexiq_set_ratio(layer, r)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(50):
                fq.flexiq_mixed_gemm(layer, Xq, out_scale=out_scale, bufs=bufs, **want)
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        ts = []
        for _ in range(7):
            a0 = torch.cuda.Event(enable_timing=True)
            a1 = torch.cuda.Event(enable_timing=True)
            a0.record()
            g.replay()
            a1.record()
            torch.cuda.synchronize()
            ts.append(a0.elapsed_time(a1) * 1e3 / 50)
        pre.append({"r": r, "us": round(float(np.median(ts)), 2)})
        del g
    fq.flexiq_input_prelowered(layer, False)

    # ratio switch (Section 7 "Low-bitwidth Ratio Adjustment"): host cost of one flexiq_set_ratio call through the
    # Python binding (an upper bound of the C call, which writes one integer), and the per-launch time of the
    # sweep, where every launch follows a switch, against launches at a fixed ratio
    n_sw = 20000
    t_sw = time.perf_counter()
    for i in range(n_sw):
        fq.flexiq_set_ratio(layer, RATIOS[i % len(RATIOS)])
    switch_ns = (time.perf_counter() - t_sw) / n_sw * 1e9
    ratio_switch = {"set_ratio_host_ns": round(switch_ns, 1),
                    "sweep_us_per_launch": round(dev_us / (args.steps * len(RATIOS)), 2),
                    "fixed_ratio_mean_us_per_launch": round(float(np.mean([per_r_us[r] for r in RATIOS])), 2)}

    # run-time extraction positions (Section 4.1, dynamic option): cost of the OR scan next to the GEMM it serves
    # (outside the timed region; the paper reports 2-5 % of the layer)
    dyn = []
    for r in RATIOS[1:]:
        fq.flexiq_set_ratio(layer, r)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(25):
                fq.flexiq_dynamic_positions(layer, Xq)
                fq.flexiq_mixed_gemm(layer, Xq, out_scale=out_scale, bufs=bufs, **want)
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        ts = []
        for _ in range(7):
            a0 = torch.cuda.Event(enable_timing=True)
            a1 = torch.cuda.Event(enable_timing=True)
            a0.record()
            g.replay()
            a1.record()
            torch.cuda.synchronize()
            ts.append(a0.elapsed_time(a1) * 1e3 / 25)
        both = float(np.median(ts))
        dyn.append({"r": r, "scan_plus_gemm_us": round(both, 2),
                    "overhead_frac": round(both / per_r_us[r] - 1.0, 4)})
        del g
    fq.flexiq_static_positions(layer)

    # the same scan done by the producing layer's own epilogue (flexiq_out.scan_for): this layer as the producer of
    # a small consumer with C = N input channels; the chain producer -> consumer with and without the scan (the
    # producer's last block turns the merged masks into the consumer's positions).  Side measurement.
    fused_scan = None
    if args.out == "q":
        rng2 = np.random.default_rng(7)
        W2 = (rng2.standard_normal((32, N)) * 0.02).astype(np.float32)
        # (the consumer reads its channels in the order this layer writes its columns: identity)
        cons = fq.flexiq_quantize_pack(W2, np.full(N, 127.0 * out_scale, np.float32), float(out_scale), 32,
                                       perm=np.arange(N, dtype=np.int32))
        fq.flexiq_set_ratio(cons, 1.0)
        fq.flexiq_set_ratio(layer, 0.5)
        cbufs = {"q": torch.empty((M, 32), dtype=torch.int8, device=dev)}
        res = {}
        for tag, kw in (("chain_us", {}), ("chain_with_scan_us", {"scan_for": cons})):
            fq.flexiq_static_positions(cons)
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for _ in range(25):
                    fq.flexiq_mixed_gemm(layer, Xq, out_scale=out_scale, bufs=bufs, q=True, **kw)
                    fq.flexiq_mixed_gemm(cons, bufs["q"], out_scale=out_scale, bufs=cbufs, q=True)
            for _ in range(3):
                g.replay()
            torch.cuda.synchronize()
            ts = []
            for _ in range(7):
                a0 = torch.cuda.Event(enable_timing=True)
                a1 = torch.cuda.Event(enable_timing=True)
                a0.record()
                g.replay()
                a1.record()
                torch.cuda.synchronize()
                ts.append(a0.elapsed_time(a1) * 1e3 / 25)
            res[tag] = round(float(np.median(ts)), 2)
            del g
        res["overhead_frac_of_producer"] = round((res["chain_with_scan_us"] - res["chain_us"]) / per_r_us[0.5], 4)
        fused_scan = res
        del cons

    if args.calib_copy_mib > 0:
        src = torch.empty(args.calib_copy_mib << 20, dtype=torch.int8, device=dev)
        dst = torch.empty_like(src)
        src.fill_(1)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ops_call = 2.0 * M * N * K
    ops_step = ops_call * len(RATIOS)
    value = ops_step * args.steps / wall / 1e12
    per_r = []
    for r in RATIOS:
        us = per_r_us[r]
        per_r.append({"r": r, "us": round(us, 2), "tops": round(ops_call / us / 1e6, 1),
                      "frac_int8_mfma_peak": round(ops_call / us / 1e6 / INT8_MFMA_PEAK_TOPS, 4),
                      "algorithmic_GBs": round(algorithmic_bytes(M, N, K, r, out_bytes, "w4x") / us / 1e3, 1)})
    avg_us = dev_us / (args.steps * len(RATIOS))
    achieved = ops_call / avg_us / 1e6 if avg_us else value
    roofline = {"bound": "mfma", "kernel": "flexiq::k_mixed (int8 MFMA mixed GEMM)", "achieved": round(achieved, 1),
                "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s", "frac": round(achieved / INT8_MFMA_PEAK_TOPS, 4),
                "avg_launch_us": round(avg_us, 2) if avg_us else None,
                "ops_per_launch": ops_call, "traffic": MEASURED_TRAFFIC_BYTES.get((args.layer, args.out))}

    # ---- CPU oracle on a bounded row sample (rank 0, N = 1 only), with a parity check on those rows
    cpu = None
    parity = None
    if args.cpu_rows > 0:
        import oracle
        oracle.build()
        rows = min(args.cpu_rows, M)
        ol = oracle.prepare_layer(case.W, absmax_c, x_scale, gs, bias=case.bias)
        Xs = oracle.quantize(case.X[:rows], x_scale)[:, ol.perm]
        cores = len(os.sched_getaffinity(0))
        try:
            cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
        except ValueError:
            pass
        tc = time.perf_counter()
        refs = [oracle.forward_gemm(ol, Xs, r) for r in RATIOS]
        cpu_s = time.perf_counter() - tc
        cpu_tops = 2.0 * rows * N * K * len(RATIOS) / cpu_s / 1e12
        cpu = {"value": round(cpu_tops, 6), "unit": "TOPS", "cores": cores, "kind": "oracle",
               "sample": "first %d of %d rows of the same layer, all N and K, ratio sweep %s, %.1f s"
                         % (rows, M, list(RATIOS), cpu_s)}
        ok = True
        Xd = Xq[:rows].contiguous()
        for r, ref in zip(RATIOS, refs):
            fq.flexiq_set_ratio(layer, r)
            got = fq.flexiq_mixed_gemm(layer, Xd, acc=True)["acc"].cpu().numpy()
            ok = ok and bool((got == ref).all())
        parity = "int32 accumulators bit-exact with the oracle on %d rows x %d ratios" % (rows, len(RATIOS)) if ok \
            else "MISMATCH against the oracle"

    shapes = None
    if not args.no_shapes:
        del layer, Xq, bufs
        torch.cuda.empty_cache()
        t_sh = time.time()
        shapes = measure_shapes(torch, fq, workloads, dev, resnet=not args.no_resnet)
        log("shapes: %.0f s" % (time.time() - t_sh))

    line = {
        "metric": METRIC, "value": round(value, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(wall / args.steps * 1e3, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "i8", "data": "synthetic",
        "config": {"workload": "ViT-B/16 MLP %s, batch 32 @224px: M=%d K=%d N=%d, group size %d, ratio sweep %s "
                               "per step, epilogue=%s" % (args.layer, M, K, N, gs, list(RATIOS),
                                                          {"q": "int8 requant", "y": "fp32 dequant", "acc": "int32 dump"}[args.out]),
                   "M": M, "K": K, "N": N, "group_size": gs, "ratios": list(RATIOS), "steps_per_graph": chunk},
        "roofline": roofline, "cpu_baseline": cpu, "per_r": per_r, "prelowered_input": pre, "dynamic_positions": dyn, "fused_scan": fused_scan, "ratio_switch": ratio_switch, "parity": parity,
        "shapes": shapes,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
