"""GPU parity of the row-streaming kernel (layers with 64, 128 or 256 input channels) against the CPU oracle, through the
same entry points as the tiled kernel: int32 accumulators and int8 codes bit for bit, fp32 within 1e-5."""
import numpy as np
import pytest

import workloads
from helpers import both_layers, check_q, check_y, requant_fp32_sequence

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import oracle
    import paper_2510_02822_amd as fq
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    fq.load()
    oracle.build()
    return torch, oracle, fq, torch.device("cuda:0")


def _dev(torch, a, dev):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev)


@pytest.mark.parametrize("M,K,N,gs", [(1000, 64, 64, 32), (777, 64, 256, 32), (129, 128, 16, 32), (2000, 128, 520, 64),
                                      (513, 256, 72, 32), (300, 256, 128, 64), (1, 256, 40, 32), (4099, 64, 300, 32)])
@pytest.mark.parametrize("kernel", [1, 2])   # 1: blocks walk tiles of 128 rows together; 2: every wave walks groups of 32 rows on its own
def test_linear_forced(env, M, K, N, gs, kernel):
    torch, oracle, fq, dev = env
    case = workloads.make_linear("st", 12, M + K + N, M, K, N, gs, outlier_frac=0.02)
    case.X *= 2.0   # some rows saturate under the calibrated positions
    ol, hl, x_scale = both_layers(case)
    Xq = oracle.quantize(case.X, x_scale)[:, ol.perm]
    Xd = _dev(torch, Xq, dev)
    G = K // gs
    fq.debug_force_stream(kernel)
    try:
        for r in (0.0, 1.0 / G, 0.5, 1.0):
            fq.flexiq_set_ratio(hl, r)
            ref = oracle.forward_gemm(ol, Xq, r)
            so = float(np.abs(oracle.dequant_f64(ref, x_scale, ol.w_scale, ol.bias)).max() / 127 * 0.9) or 1.0
            out = fq.flexiq_mixed_gemm(hl, Xd, acc=True, y=True, q=True, out_scale=so)
            torch.cuda.synchronize()
            assert fq.debug_force_stream(kernel) == kernel          # the call ran on that kernel
            assert fq.debug_last_launch()["tile"] == -2
            assert (out["acc"].cpu().numpy() == ref).all(), r
            check_y(out["y"].cpu().numpy(), ref, ol)
            got_q = out["q"].cpu().numpy()
            check_q(got_q, ref, ol, so)
            assert (got_q == requant_fp32_sequence(ref, ol, so)).all()
            only_q = fq.flexiq_mixed_gemm(hl, Xd, q=True, out_scale=so)["q"]   # the variant with pre-multiplied scales
            assert (only_q.cpu().numpy() == got_q).all(), r
            # the tiled kernel gives the same bytes
            fq.debug_force_stream(0)
            fq.debug_force_few_rows(0)
            tiled = fq.flexiq_mixed_gemm(hl, Xd, q=True, out_scale=so)["q"]
            assert fq.debug_last_launch()["tile"] >= 0
            fq.debug_force_few_rows(-1)
            fq.debug_force_stream(kernel)
            assert (tiled.cpu().numpy() == got_q).all(), r
    finally:
        fq.debug_force_stream(-1)
        fq.debug_force_few_rows(-1)


def test_run_time_positions_and_prelowered_input(env):
    torch, oracle, fq, dev = env
    M, K, N, gs = 3000, 256, 96, 32
    case = workloads.make_linear("stdyn", 12, 3, M, K, N, gs, outlier_frac=0.02)
    case.X *= 3.0
    ol, hl, x_scale = both_layers(case)
    Xq = oracle.quantize(case.X, x_scale)[:, ol.perm]
    Xd = _dev(torch, Xq, dev)
    fq.debug_force_stream(1)
    try:
        k4 = fq.flexiq_set_ratio(hl, 0.75)
        G4 = k4 // gs
        fq.flexiq_dynamic_positions(hl, Xd)
        dyn = oracle.dynamic_act_shifts(Xq, gs, G4, ol.a_shift)
        got = fq.flexiq_mixed_gemm(hl, Xd, acc=True)["acc"].cpu().numpy()
        assert fq.debug_force_stream(1) == 1
        assert (got == oracle.mixed_gemm(Xq, ol.Wq.reshape(N, K), gs, G4, dyn, ol.w_shift)).all()
        fq.flexiq_static_positions(hl)
        # activations that arrive lowered: the kernel must not lower again with other positions, only copy
        sh = np.repeat(ol.a_shift.astype(np.int32), gs)[None, :]
        Xl = Xq.astype(np.int32).copy()
        Xl[:, :k4] = np.clip(Xl[:, :k4] >> sh[:, :k4], -8, 7) << sh[:, :k4]
        fq.flexiq_input_prelowered(hl, True)
        got = fq.flexiq_mixed_gemm(hl, _dev(torch, Xl.astype(np.int8), dev), acc=True)["acc"].cpu().numpy()
        fq.flexiq_input_prelowered(hl, False)
        assert (got == oracle.forward_gemm(ol, Xq, 0.75)).all()
    finally:
        fq.debug_force_stream(-1)
        fq.flexiq_input_prelowered(hl, False)


def test_conv_1x1_and_automatic_route(env):
    torch, oracle, fq, dev = env
    # a 1x1 convolution with stride 1 and no padding is a linear layer over the pixels
    case = workloads.make_conv("st1x1", 12, 7, 3, 20, 20, 128, 48, 1, 1, 1, 0, 32)
    ol, hl, x_scale = both_layers(case)
    Xq = np.ascontiguousarray(oracle.quantize(case.X, x_scale)[..., ol.perm])
    Xd = _dev(torch, Xq, dev)
    fq.debug_force_stream(1)
    try:
        for r in (0.0, 0.5, 1.0):
            fq.flexiq_set_ratio(hl, r)
            ref = oracle.forward_conv(ol, Xq, 1, 0, r)
            got = fq.flexiq_mixed_conv_implicit(hl, Xd, 1, 0, acc=True)["acc"].cpu().numpy()
            assert fq.debug_force_stream(1) == 1
            assert (got == ref).all(), r
        # a strided 1x1 convolution does not qualify
        fq.flexiq_mixed_conv_implicit(hl, Xd, 2, 0, acc=True)
        assert fq.debug_force_stream(1) == 0
    finally:
        fq.debug_force_stream(-1)
    # automatic: taken with many rows, not with few
    M, K, N = 200000, 64, 64
    rng = np.random.default_rng(5)
    case = workloads.make_linear("stauto", 12, 9, 4096, K, N, 32, outlier_frac=0.02)
    ol, hl, x_scale = both_layers(case)
    Xbig = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
    rows = np.r_[0:300, M - 300:M]
    for r, kernel in ((0.0, 1), (0.5, 2)):   # nothing to lower: blocks walk tiles; else (64 x 64): every wave on its own
        fq.flexiq_set_ratio(hl, r)
        got = fq.flexiq_mixed_gemm(hl, _dev(torch, Xbig, dev), acc=True)["acc"].cpu().numpy()
        assert fq.debug_force_stream(-1) == kernel
        assert (got[rows] == oracle.forward_gemm(ol, Xbig[rows], r)).all()
    fq.flexiq_mixed_gemm(hl, _dev(torch, Xbig[:5000], dev), acc=True)
    assert fq.debug_force_stream(-1) == 0


@pytest.mark.parametrize("K,N", [(64, 256), (64, 64), (128, 128), (256, 64)])
@pytest.mark.parametrize("kernel", [1, 2])
def test_blocks_walk_many_tiles(env, K, N, kernel):
    """More row tiles than resident blocks: every block (or wave, second kernel) goes round its ring of slots several times (each wave-count
    and ring-depth configuration of the kernels), int32 and int8 outputs together."""
    torch, oracle, fq, dev = env
    M = 150001
    case = workloads.make_linear("stwalk", 12, K + N, 2048, K, N, 32, outlier_frac=0.02)
    ol, hl, x_scale = both_layers(case)
    rng = np.random.default_rng(K * 1000 + N)
    Xq = rng.integers(-128, 128, size=(M, K)).astype(np.int8)
    Xd = _dev(torch, Xq, dev)
    rows = np.r_[0:200, 70000:70300, M - 400:M]
    fq.debug_force_stream(kernel)
    try:
        for r in (1.0, 0.5, 0.0):
            fq.flexiq_set_ratio(hl, r)
            ref = oracle.forward_gemm(ol, Xq[rows], r)
            so = float(np.abs(oracle.dequant_f64(ref, x_scale, ol.w_scale, ol.bias)).max() / 127 * 0.9) or 1.0
            out = fq.flexiq_mixed_gemm(hl, Xd, acc=True, q=True, out_scale=so)
            torch.cuda.synchronize()
            assert fq.debug_force_stream(kernel) == kernel
            assert (out["acc"].cpu().numpy()[rows] == ref).all(), r
            assert (out["q"].cpu().numpy()[rows] == requant_fp32_sequence(ref, ol, so)).all(), r
            # the whole int8 output against the tiled kernel's
            fq.debug_force_stream(0)
            tiled = fq.flexiq_mixed_gemm(hl, Xd, q=True, out_scale=so)["q"]
            fq.debug_force_stream(kernel)
            only_q = fq.flexiq_mixed_gemm(hl, Xd, q=True, out_scale=so)["q"]
            assert bool((tiled == only_q).all()) and bool((only_q == out["q"]).all()), r
    finally:
        fq.debug_force_stream(-1)


@pytest.mark.parametrize("M,K1,N1,N2,gs2", [(1000, 64, 256, 40, 32), (777, 128, 576, 64, 64), (513, 256, 96, 24, 32), (300, 256, 128, 128, 64),
                                           (2100, 64, 64, 256, 32)])
@pytest.mark.parametrize("kernel", [1, 2])
def test_producer_lowers_for_consumer(env, M, K1, N1, N2, gs2, kernel):
    # the fused producer (Section 4.1 applied where the tensor is produced; Section 5 steps 1-2) on the row-streaming kernels:
    # int8 rows in the consumer's stored channel order, its 4-bit channels clamped and masked at the consumer's positions;
    # the consumer, told so, then copies them like 8-bit ones and gets the accumulators of lowering on the fly
    torch, oracle, fq, dev = env
    helpers = __import__("helpers")
    c1 = workloads.make_linear("slow1", 12, 300 + M + N1, M, K1, N1, 32, outlier_frac=0.02)
    c2 = workloads.make_linear("slow2", 12, 301 + M + N1, M, N1, N2, gs2, outlier_frac=0.02)
    xs1, am1 = helpers.calib(c1)
    o1 = oracle.prepare_layer(c1.W, am1, xs1, 32, bias=c1.bias)
    Xq = np.ascontiguousarray(oracle.quantize(c1.X, xs1)[:, o1.perm])
    acc1 = oracle.forward_gemm(o1, Xq, 0.5)
    s_mid = float(np.abs(oracle.dequant_f64(acc1, xs1, o1.w_scale, o1.bias)).max() / 127.0 * 0.8)   # some codes clip
    q1 = requant_fp32_sequence(acc1, o1, s_mid)
    check_q(q1, acc1, o1, s_mid)
    am2 = np.abs(q1).max(0).astype(np.float32) * np.float32(s_mid) * np.float32(0.5)   # calibrated too narrow: the clamp bites
    o2 = oracle.prepare_layer(c2.W, am2, s_mid, gs2, bias=c2.bias)
    h2 = fq.flexiq_quantize_pack(c2.W, am2, s_mid, gs2, bias=c2.bias)
    h1 = fq.flexiq_quantize_pack(c1.W, am1, xs1, 32, bias=c1.bias, out_perm=o2.perm)
    X2 = np.ascontiguousarray(q1[:, o2.perm])
    fq.flexiq_set_ratio(h1, 0.5)
    Xd = _dev(torch, Xq, dev)
    sh = np.repeat(o2.a_shift.astype(np.int32), gs2)
    G2 = N1 // gs2
    fq.debug_force_stream(kernel)
    try:
        for r2 in sorted({0.0, 1.0 / G2, 0.5, 1.0}):
            k4 = fq.flexiq_set_ratio(h2, r2)
            want = X2.astype(np.int32).copy()
            want[:, :k4] = np.clip(want[:, :k4] >> sh[:k4], -8, 7) << sh[:k4]
            assert all(oracle.bitlower(int(X2[i, j]), int(sh[j])) << int(sh[j]) == want[i, j] for i in (0, M // 2, M - 1) for j in range(0, k4, 7))
            low = fq.flexiq_mixed_gemm(h1, Xd, q=True, out_scale=s_mid, lower_for=h2)["q"]
            torch.cuda.synchronize()
            assert fq.debug_force_stream(kernel) == kernel and fq.debug_last_launch()["tile"] == -2   # ran on that kernel
            assert (low.cpu().numpy().astype(np.int32) == want).all(), r2
            fq.debug_force_stream(0)
            tiled = fq.flexiq_mixed_gemm(h1, Xd, q=True, out_scale=s_mid, lower_for=h2)["q"]       # the tiled kernel lowers alike
            assert fq.debug_last_launch()["tile"] >= 0
            assert (tiled.cpu().numpy() == low.cpu().numpy()).all(), r2
            fq.flexiq_input_prelowered(h2, True)
            got = fq.flexiq_mixed_gemm(h2, low, acc=True)["acc"].cpu().numpy()
            fq.flexiq_input_prelowered(h2, False)
            fq.debug_force_stream(kernel)
            assert (got == oracle.forward_gemm(o2, X2, r2)).all(), r2
        # an output that is not int8 alone next to lower_for is served by the tiled kernel, with the same int8 rows
        both = fq.flexiq_mixed_gemm(h1, Xd, acc=True, q=True, out_scale=s_mid, lower_for=h2)
        assert fq.debug_last_launch()["tile"] >= 0
        assert (both["q"].cpu().numpy() == low.cpu().numpy()).all() and (both["acc"].cpu().numpy() == acc1[:, o2.perm]).all()
    finally:
        fq.debug_force_stream(-1)
        fq.flexiq_input_prelowered(h2, False)
