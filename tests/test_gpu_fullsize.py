"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
uses (automatic tile choice, int8 / fp32 / int32 outputs).  The oracle is too slow for whole outputs
at these sizes, so it computes sampled output rows (first and last tile rows, the ragged tail, a
seeded strided sample) or sampled images one by one; each sampled value is compared bit for bit."""
import numpy as np
import pytest

import workloads
from helpers import calib, check_q, check_y, requant_fp32_sequence

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


@pytest.fixture(scope="module")
def env():
    import torch
    import oracle
    import paper_2510_02822_amd as fq
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    fq.load()
    oracle.build()
    fq.debug_force_tile(-1)
    return torch, oracle, fq, torch.device("cuda:0")


def _sample_rows(M, seed, n_random=48):
    rng = np.random.default_rng(seed)
    rows = set(range(min(24, M))) | set(range(max(0, M - 40), M)) | set(rng.integers(0, M, n_random).tolist())
    return np.array(sorted(rows))


def _linear_fullsize(env, case, ratios):
    torch, oracle, fq, dev = env
    x_scale, amax = calib(case)
    ol = oracle.prepare_layer(case.W, amax, x_scale, case.group_size, bias=case.bias)
    hl = fq.flexiq_quantize_pack(case.W, amax, x_scale, case.group_size, bias=case.bias)
    info = hl.info()
    assert (info["perm"] == ol.perm).all() and (info["w_shift"] == ol.w_shift).all() and (info["a_shift"] == ol.a_shift).all()
    Xq_nat = fq.flexiq_quantize_act(torch.from_numpy(case.X).to(dev), x_scale)
    Xq = fq.flexiq_permute_channels(hl, Xq_nat)
    rows = _sample_rows(case.M, case.M + case.N)
    Xs = oracle.quantize(case.X[rows], x_scale)[:, ol.perm]
    assert (Xq[torch.from_numpy(rows).to(dev)].cpu().numpy() == Xs).all()          # producer-side quantiser + reorder
    for r in ratios:
        fq.flexiq_set_ratio(hl, r)
        ref = oracle.forward_gemm(ol, Xs, r)
        so = float(np.abs(oracle.dequant_f64(ref, x_scale, ol.w_scale, ol.bias)).max() / 127 * 0.9)
        out = fq.flexiq_mixed_gemm(hl, Xq, acc=True)                                # int32 dump
        assert (out["acc"][torch.from_numpy(rows).to(dev)].cpu().numpy() == ref).all(), (case.name, r)
        del out
        out = fq.flexiq_mixed_gemm(hl, Xq, q=True, out_scale=so)                    # the configuration bench.py times
        got_q = out["q"][torch.from_numpy(rows).to(dev)].cpu().numpy()
        used = check_q(got_q, ref, ol, so)          # float64 definition, tie window
        print("%s r=%g: %d of %d sampled codes inside the tie window" % (case.name, r, used, got_q.size))
        assert (got_q == requant_fp32_sequence(ref, ol, so)).all()
        del out
        out = fq.flexiq_mixed_gemm(hl, Xq, y=True)
        check_y(out["y"][torch.from_numpy(rows).to(dev)].cpu().numpy(), ref, ol)
        del out


@pytest.mark.parametrize("which", ["fc1", "fc2"])
def test_vitb_mlp_fullsize(env, which):
    _linear_fullsize(env, workloads.config1(which), (0.0, 0.25, 0.5, 0.75, 1.0))


@pytest.mark.parametrize("which", ["fc1", "fc2"])
def test_vitl_mlp_fullsize(env, which):
    _linear_fullsize(env, workloads.config3(which), (0.0, 0.5, 1.0))


def _conv_fullsize(env, case, ratios, images):
    torch, oracle, fq, dev = env
    x_scale, amax = calib(case)
    ol = oracle.prepare_layer(case.W, amax, x_scale, case.group_size, bias=case.bias)
    hl = fq.flexiq_quantize_pack(case.W, amax, x_scale, case.group_size, bias=case.bias)
    Xq_nat = fq.flexiq_quantize_act(torch.from_numpy(case.X).to(dev), x_scale)
    Xq = fq.flexiq_permute_channels(hl, Xq_nat)
    del Xq_nat
    Xs = np.ascontiguousarray(oracle.quantize(case.X[images], x_scale)[..., ol.perm])
    idx = torch.from_numpy(np.array(images)).to(dev)
    assert (Xq[idx].cpu().numpy() == Xs).all()
    for r in ratios:
        fq.flexiq_set_ratio(hl, float(r))
        ref = oracle.forward_conv(ol, Xs, case.stride, case.pad, float(r))
        so = float(np.abs(oracle.dequant_f64(ref, x_scale, ol.w_scale, ol.bias)).max() / 127 * 0.9)
        out = fq.flexiq_mixed_conv_implicit(hl, Xq, case.stride, case.pad, acc=True, q=True, out_scale=so)
        assert (out["acc"][idx].cpu().numpy() == ref).all(), (case.name, r)
        got_q = out["q"][idx].cpu().numpy()
        check_q(got_q, ref, ol, so)
        assert (got_q == requant_fp32_sequence(ref, ol, so)).all()
        del out


def test_resnet_3x3_conv_fullsize(env):
    # configuration 2: NHWC [64,14,14,256] -> 256 channels, 3x3, stride 1, pad 1
    _conv_fullsize(env, workloads.config2(), (0.0, 0.5, 1.0), [0, 31, 63])


@pytest.mark.parametrize("lo,hi", [(0, 6), (6, 12), (12, 17), (17, 22)])
def test_resnet50_stack_ratio_schedule(env, lo, hi):
    # configuration 4: every conv shape of ResNet-50 stages 1-4 at batch 128, one handle per layer packed
    # once, the low-bit ratio drawn per call from the seeded schedule
    sched = workloads.config4_ratio_schedule(3 * 22)
    for i in range(lo, hi):
        case = workloads.config4_layer(i, B=128)
        _conv_fullsize(env, case, sched[3 * i:3 * i + 3], [0, 127])
        del case


def test_weight_streaming_few_rows(env):
    # bench.py's weight-streaming workload (16384 x 4096 weights, group size 64) in the launch configuration it times: 1, 2, 4
    # and 16 rows through the automatic few-row route (dot-product kernel with four column groups per block for 1 and 2 rows
    # and, from r = 0.5 on, 4 rows; the matrix-core kernel otherwise), whole outputs against the oracle
    torch, oracle, fq, dev = env
    case = workloads.make_linear("stream_16384x4096", 9, 16384 + 4096, 16, 4096, 16384, 64, outlier_frac=0.02)
    x_scale, amax = calib(case)
    ol = oracle.prepare_layer(case.W, amax, x_scale, 64, bias=case.bias)
    hl = fq.flexiq_quantize_pack(case.W, amax, x_scale, 64, bias=case.bias)
    assert (hl.info()["perm"] == ol.perm).all()
    Xq = np.ascontiguousarray(oracle.quantize(case.X, x_scale)[:, ol.perm])
    for r in (0.0, 0.25, 0.5, 1.0):
        fq.flexiq_set_ratio(hl, r)
        ref = oracle.forward_gemm(ol, Xq, r)
        so = float(np.abs(oracle.dequant_f64(ref, x_scale, ol.w_scale, ol.bias)).max() / 127 * 0.9)
        for M in (1, 2, 4, 16):
            out = fq.flexiq_mixed_gemm(hl, torch.from_numpy(Xq[:M]).to(dev), acc=True, q=True, out_scale=so)
            torch.cuda.synchronize()
            assert fq.debug_last_launch()["tile"] == -4
            assert fq.debug_force_few_rows(-1) == (2 if M <= 2 or (M == 4 and r >= 0.5) else 1), (M, r)   # which kernel ran
            assert (out["acc"].cpu().numpy() == ref[:M]).all(), (M, r)
            check_q(out["q"].cpu().numpy(), ref[:M], ol, so)


@pytest.mark.parametrize("which", ["fc1", "fc2"])
def test_one_image_vitl(env, which):
    # bench.py's one-image calls (the 197 tokens of one image on the ViT-L linear layers) in the launch configuration it times: the
    # automatic route (a tile per block, the reduction split over its waves), int8 and FP6 builds, whole outputs against the oracle
    torch, oracle, fq, dev = env
    case = workloads.config3(which)
    x_scale, amax = calib(case)
    ol = oracle.prepare_layer(case.W, amax, x_scale, case.group_size, bias=case.bias)
    hl = fq.flexiq_quantize_pack(case.W, amax, x_scale, case.group_size, bias=case.bias)
    assert (hl.info()["perm"] == ol.perm).all()
    Xq = np.ascontiguousarray(oracle.quantize(case.X[:197], x_scale)[:, ol.perm])
    Xd = torch.from_numpy(Xq).to(dev)
    for r in (0.0, 0.5, 1.0):
        fq.flexiq_set_ratio(hl, r)
        ref = oracle.forward_gemm(ol, Xq, r)
        so = float(np.abs(oracle.dequant_f64(ref, x_scale, ol.w_scale, ol.bias)).max() / 127 * 0.9)
        out = fq.flexiq_mixed_gemm(hl, Xd, acc=True, q=True, out_scale=so)
        torch.cuda.synchronize()
        assert fq.debug_last_launch()["tile"] == -5, r
        assert (out["acc"].cpu().numpy() == ref).all(), r
        got_q = out["q"].cpu().numpy()
        check_q(got_q, ref, ol, so)
        assert (got_q == requant_fp32_sequence(ref, ol, so)).all()
        x6, xlow = fq.flexiq_lower_fp6(hl, Xd)
        out = fq.flexiq_mixed_gemm_fp6(hl, xlow, x6, acc=True, q=True, out_scale=so)
        torch.cuda.synchronize()
        assert fq.debug_force_tile_splitk(-1) > 0, r
        assert (out["acc"].cpu().numpy() == ref).all(), r
        assert (out["q"].cpu().numpy() == got_q).all(), r
