#!/usr/bin/env python3
"""Benchmark of the FlexiQ hot path on one MI355X.

Workload (BASELINE.json `metric`: "... vs low-bit ratio r (ViT-B fc1)", configs[1]): the ViT-B/16
MLP fc1 linear at batch 32, M = 32*197 = 6304 tokens, K = 768, N = 3072, channel group size 32.
One step = one pass of the run-time hot path over the ratio sweep r in {0, .25, .5, .75, 1}: per
ratio the O(1) ratio switch, then the mixed 4/8-bit MFMA GEMM with on-the-fly bit-lowering of
the activations, in-register expansion of the packed 4-bit weights and the fused per-channel
dequant + int8 requant epilogue.  Inputs (int8 activations in stored channel order, packed layer)
are resident in HBM before the timed region; the offline steps (weight quantisation, channel
order, positions, packing) run once before it, as in the paper.

Prints ONE JSON line.  `value` = total int8 ops of the K timed steps / wall time (TOPS).
The default step and warm-up counts keep the GPU busy for a few tenths of a second: the card needs tens of
milliseconds of work to settle at its running clocks, and a short timed region after a cold start reads about 4 %
low; for the same reason about 50 ms of untimed steps run before the requested warm-up steps.
`roofline` covers the GEMM kernel (the only kernel in the timed region): algorithmic ops per launch
= 2*M*N*K, average launch duration = HIP-event time of the timed region / launches in it.  `cpu_baseline` times the CPU oracle on a bounded row sample of the same workload.
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


def algorithmic_bytes(M, N, K, r, out_bytes_per_elem=1):
    """Bytes one call must move: int8 activations, weights (1 B per 8-bit channel, 1/2 B per 4-bit
    channel when the packed codes are streamed), position table and scales, output."""
    return M * K + N * K * (1.0 - r / 2.0) + N * (K // 32) + 8 * N + M * N * out_bytes_per_elem


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=400)
    ap.add_argument("--layer", default="fc1", choices=["fc1", "fc2"])
    ap.add_argument("--out", default="q", choices=["q", "y", "acc"], help="epilogue output written in the timed region")
    ap.add_argument("--cpu-rows", type=int, default=4096, help="rows of the workload the CPU oracle is timed on (0: skip)")
    ap.add_argument("--eager", action="store_true", help="launch from Python instead of replaying a captured HIP graph")
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
    # consumer turns the masks into positions in its prologue and clears the other mask set).  Side measurement.
    fused_scan = None
    if args.out == "q":
        rng2 = np.random.default_rng(7)
        W2 = (rng2.standard_normal((32, N)) * 0.02).astype(np.float32)
        cons = fq.flexiq_quantize_pack(W2, np.full(N, 127.0 * out_scale, np.float32), float(out_scale), 32)
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
                      "algorithmic_GBs": round(algorithmic_bytes(M, N, K, r, out_bytes) / us / 1e3, 1)})
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

    line = {
        "metric": METRIC, "value": round(value, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(wall / args.steps * 1e3, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "i8", "data": "synthetic",
        "config": {"workload": "ViT-B/16 MLP %s, batch 32 @224px: M=%d K=%d N=%d, group size %d, ratio sweep %s "
                               "per step, epilogue=%s" % (args.layer, M, K, N, gs, list(RATIOS),
                                                          {"q": "int8 requant", "y": "fp32 dequant", "acc": "int32 dump"}[args.out]),
                   "M": M, "K": K, "N": N, "group_size": gs, "ratios": list(RATIOS), "steps_per_graph": chunk},
        "roofline": roofline, "cpu_baseline": cpu, "per_r": per_r, "prelowered_input": pre, "dynamic_positions": dyn, "fused_scan": fused_scan, "ratio_switch": ratio_switch, "parity": parity,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
