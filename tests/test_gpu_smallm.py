"""GPU parity of the few-row kernel (linear calls with at most 64 rows) against the CPU oracle, through the same
entry point as every other linear call: int32 accumulators bit-exact, fp32 within 1e-5, int8 codes by the float64
definition with the tie window."""
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


@pytest.mark.parametrize("K,N,gs", [(256, 256, 32), (1024, 520, 64), (192, 72, 32), (4096, 1024, 64), (64, 7, 32), (96, 30, 32), (2112, 48, 64), (128, 8200, 32)])
# 1: matrix-core kernel (up to 64 rows); 2: dot-product kernel (up to 4 rows); 14: the same with 4 column groups per block
@pytest.mark.parametrize("kernel", [1, 2, 14])
def test_few_rows_kernel(env, K, N, gs, kernel):
    # the few-row kernels (a block per 16 resp. 8 output columns, its waves split the reduction and meet in LDS): every
    # fragment / row count, reductions with an odd unit count, a half 4-bit K-step, N below / not a multiple of 16
    torch, oracle, fq, dev = env
    case = workloads.make_linear("fewrows", 8, 700 + K + N, 64, K, N, gs, outlier_frac=0.02)
    case.X *= 2.0                                    # some saturation in the lowering
    ol, hl, x_scale = both_layers(case)
    Xq_all = oracle.quantize(case.X, x_scale)[:, ol.perm]
    G = K // gs
    fq.debug_force_few_rows(kernel)
    try:
        for M in ((1, 7, 16, 17, 33, 48, 64) if kernel == 1 else ((1, 2, 3, 4) if kernel == 2 else (1, 2, 4))):
            Xq = np.ascontiguousarray(Xq_all[:M])
            Xd = torch.from_numpy(Xq).to(dev)
            for r in sorted({0.0, 1.0 / G, 0.5, 1.0}):
                fq.flexiq_set_ratio(hl, r)
                ref = oracle.forward_gemm(ol, Xq, r)
                so = float(np.abs(oracle.dequant_f64(ref, x_scale, ol.w_scale, ol.bias)).max() / 127 * 0.9) or 1.0
                out = fq.flexiq_mixed_gemm(hl, Xd, acc=True, y=True, q=True, out_scale=so)
                torch.cuda.synchronize()
                assert fq.debug_force_few_rows(kernel) == min(kernel, 2) and fq.debug_last_launch()["tile"] == -4   # ran on this kernel
                assert (out["acc"].cpu().numpy() == ref).all(), (M, r)
                check_y(out["y"].cpu().numpy(), ref, ol)
                got_q = out["q"].cpu().numpy()
                check_q(got_q, ref, ol, so)
                assert (got_q == requant_fp32_sequence(ref, ol, so)).all()
                only_q = fq.flexiq_mixed_gemm(hl, Xd, q=True, out_scale=so)["q"]
                assert (only_q.cpu().numpy() == got_q).all(), (M, r)
        # more rows: the other kernels serve the call
        X65 = torch.from_numpy(np.ascontiguousarray(np.concatenate([Xq_all, Xq_all[:1]]))).to(dev)
        fq.flexiq_mixed_gemm(hl, X65, acc=True)
        assert fq.debug_last_launch()["tile"] != -4
    finally:
        fq.debug_force_few_rows(-1)


@pytest.mark.parametrize("kernel,M", [(1, 48), (1, 5), (2, 3)])
def test_few_rows_prelowered_and_dynamic(env, kernel, M):
    torch, oracle, fq, dev = env
    case = workloads.make_linear("fewrows_dyn", 8, 760, M, 1024, 256, 32, outlier_frac=0.02)
    case.X *= 0.4
    ol, hl, x_scale = both_layers(case)
    Xq = oracle.quantize(case.X, x_scale)[:, ol.perm]
    Xd = torch.from_numpy(np.ascontiguousarray(Xq)).to(dev)
    k4 = fq.flexiq_set_ratio(hl, 0.75)
    G4 = k4 // 32
    fq.debug_force_few_rows(kernel)
    try:
        fq.flexiq_dynamic_positions(hl, Xd)      # run-time positions
        dyn = oracle.dynamic_act_shifts(Xq, 32, G4, ol.a_shift)
        got = fq.flexiq_mixed_gemm(hl, Xd, acc=True)["acc"].cpu().numpy()
        assert fq.debug_last_launch()["tile"] == -4
        assert (got == oracle.mixed_gemm(Xq, ol.Wq.reshape(256, 1024), 32, G4, dyn, ol.w_shift)).all()
        fq.flexiq_static_positions(hl)
        sh = np.repeat(ol.a_shift.astype(np.int32), 32)[None, :k4]     # activations that arrive lowered
        Xl = Xq.astype(np.int32).copy()
        Xl[:, :k4] = np.clip(Xl[:, :k4] >> sh, -8, 7) << sh
        fq.flexiq_input_prelowered(hl, True)
        got = fq.flexiq_mixed_gemm(hl, torch.from_numpy(Xl.astype(np.int8)).to(dev), acc=True)["acc"].cpu().numpy()
        assert fq.debug_last_launch()["tile"] == -4
        assert (got == oracle.forward_gemm(ol, Xq, 0.75)).all()
    finally:
        fq.flexiq_input_prelowered(hl, False)
        fq.debug_force_few_rows(-1)


@pytest.mark.parametrize("M,K1,N1,N2,gs2,kernel", [(1, 256, 256, 40, 32, 2), (2, 192, 136, 64, 32, 14), (4, 128, 8200, 16, 64, -1), (5, 1024, 96, 24, 32, 1),
                                                  (40, 256, 520, 128, 32, 1), (64, 64, 72, 256, 32, -1), (3, 512, 64, 64, 64, 2)])
def test_few_rows_lower_for_consumer(env, M, K1, N1, N2, gs2, kernel):
    # the fused producer (Section 4.1 applied where the tensor is produced) on the few-row kernels: int8 rows in the consumer's
    # stored channel order with its 4-bit channels clamped and masked at its positions; the consumer, told so, runs as a
    # few-row call on the lowered rows and gets the accumulators of lowering on the fly
    torch, oracle, fq, dev = env
    helpers = __import__("helpers")
    if N1 % gs2:
        N1 = (N1 // gs2) * gs2
    c1 = workloads.make_linear("fewlow1", 8, 900 + M + N1, M, K1, N1, 32, outlier_frac=0.02)
    c2 = workloads.make_linear("fewlow2", 8, 901 + M + N1, M, N1, N2, gs2, outlier_frac=0.02)
    xs1, am1 = helpers.calib(c1)
    o1 = oracle.prepare_layer(c1.W, am1, xs1, 32, bias=c1.bias)
    Xq = np.ascontiguousarray(oracle.quantize(c1.X, xs1)[:, o1.perm])
    acc1 = oracle.forward_gemm(o1, Xq, 0.5)
    s_mid = float(np.abs(oracle.dequant_f64(acc1, xs1, o1.w_scale, o1.bias)).max() / 127.0 * 0.8) or 1.0   # some codes clip
    q1 = requant_fp32_sequence(acc1, o1, s_mid)
    check_q(q1, acc1, o1, s_mid)
    am2 = np.abs(q1).max(0).astype(np.float32) * np.float32(s_mid) * np.float32(0.5) + np.float32(1e-6)   # too narrow: the clamp bites
    o2 = oracle.prepare_layer(c2.W, am2, s_mid, gs2, bias=c2.bias)
    h2 = fq.flexiq_quantize_pack(c2.W, am2, s_mid, gs2, bias=c2.bias)
    h1 = fq.flexiq_quantize_pack(c1.W, am1, xs1, 32, bias=c1.bias, out_perm=o2.perm)
    X2 = np.ascontiguousarray(q1[:, o2.perm])
    fq.flexiq_set_ratio(h1, 0.5)
    Xd = torch.from_numpy(Xq).to(dev)
    sh = np.repeat(o2.a_shift.astype(np.int32), gs2)
    G2 = N1 // gs2
    fq.debug_force_few_rows(kernel)
    try:
        for r2 in sorted({0.0, 1.0 / G2, 0.5, 1.0}):
            k4 = fq.flexiq_set_ratio(h2, r2)
            want = X2.astype(np.int32).copy()
            want[:, :k4] = np.clip(want[:, :k4] >> sh[:k4], -8, 7) << sh[:k4]
            low = fq.flexiq_mixed_gemm(h1, Xd, q=True, out_scale=s_mid, lower_for=h2)["q"]
            torch.cuda.synchronize()
            assert fq.debug_last_launch()["tile"] == -4 and fq.debug_force_few_rows(kernel) in (1, 2)   # a few-row kernel ran
            assert (low.cpu().numpy().astype(np.int32) == want).all(), r2
            fq.flexiq_input_prelowered(h2, True)
            got = fq.flexiq_mixed_gemm(h2, low, acc=True)["acc"].cpu().numpy()
            fq.flexiq_input_prelowered(h2, False)
            assert (got == oracle.forward_gemm(o2, X2, r2)).all(), r2
    finally:
        fq.debug_force_few_rows(-1)
        fq.flexiq_input_prelowered(h2, False)


@pytest.mark.parametrize("M,K,N,gs", [(65, 1024, 72, 64), (197, 2112, 520, 64), (130, 96, 64, 32), (300, 1024, 1030, 32), (64 * 3, 256, 7, 32)])
@pytest.mark.parametrize("shape", [2, 3, 4])
def test_tile_splitk_kernel(env, M, K, N, gs, shape):
    # more than 64 rows on a layer with few output tiles: a tile per block (64 x 64, 32 x 64, 32 x 32), the reduction split over
    # its waves (ragged last row and column tiles, an odd unit count, a half 4-bit K-step, fewer K-steps than waves)
    torch, oracle, fq, dev = env
    case = workloads.make_linear("tilesplit", 8, 1000 + M + K + N, M, K, N, gs, outlier_frac=0.02)
    case.X *= 2.0
    ol, hl, x_scale = both_layers(case)
    Xq = np.ascontiguousarray(oracle.quantize(case.X, x_scale)[:, ol.perm])
    Xd = torch.from_numpy(Xq).to(dev)
    G = K // gs
    fq.debug_force_tile_splitk(shape)
    try:
        for r in sorted({0.0, 1.0 / G, 0.5, 1.0}):
            fq.flexiq_set_ratio(hl, r)
            ref = oracle.forward_gemm(ol, Xq, r)
            so = float(np.abs(oracle.dequant_f64(ref, x_scale, ol.w_scale, ol.bias)).max() / 127 * 0.9) or 1.0
            out = fq.flexiq_mixed_gemm(hl, Xd, acc=True, y=True, q=True, out_scale=so)
            torch.cuda.synchronize()
            assert fq.debug_force_tile_splitk(shape) == shape - 1 and fq.debug_last_launch()["tile"] == -5   # ran on this kernel, this tile
            assert (out["acc"].cpu().numpy() == ref).all(), r
            check_y(out["y"].cpu().numpy(), ref, ol)
            got_q = out["q"].cpu().numpy()
            check_q(got_q, ref, ol, so)
            assert (got_q == requant_fp32_sequence(ref, ol, so)).all()
            fq.debug_force_tile_splitk(0)
            tiled = fq.flexiq_mixed_gemm(hl, Xd, q=True, out_scale=so)["q"]       # the tiled kernel gives the same bytes
            assert fq.debug_last_launch()["tile"] >= 0 or fq.debug_last_launch()["tile"] == -2
            fq.debug_force_tile_splitk(shape)
            assert (tiled.cpu().numpy() == got_q).all(), r
        # activations that arrive lowered
        k4 = fq.flexiq_set_ratio(hl, 0.5)
        sh = np.repeat(ol.a_shift.astype(np.int32), gs)[None, :k4]
        Xl = Xq.astype(np.int32).copy()
        Xl[:, :k4] = np.clip(Xl[:, :k4] >> sh, -8, 7) << sh
        fq.flexiq_input_prelowered(hl, True)
        got = fq.flexiq_mixed_gemm(hl, torch.from_numpy(Xl.astype(np.int8)).to(dev), acc=True)["acc"].cpu().numpy()
        assert fq.debug_last_launch()["tile"] == -5
        assert (got == oracle.forward_gemm(ol, Xq, 0.5)).all()
    finally:
        fq.flexiq_input_prelowered(hl, False)
        fq.debug_force_tile_splitk(-1)


@pytest.mark.parametrize("M,K1,N1,N2,gs2", [(100, 1024, 520, 128, 32), (197, 256, 136, 64, 32), (33, 2048, 256, 24, 64)])
@pytest.mark.parametrize("shape", [2, 3, 4])
def test_tile_splitk_lower_for_consumer(env, M, K1, N1, N2, gs2, shape):
    # the fused producer on the tile-per-block kernel: int8 rows in the consumer's stored channel order with its 4-bit channels
    # clamped and masked at its positions (ragged column tiles; a consumer group size of 64); the consumer, told so, reads them
    torch, oracle, fq, dev = env
    helpers = __import__("helpers")
    N1 = (N1 // gs2) * gs2
    c1 = workloads.make_linear("tilelow1", 8, 950 + M + N1, M, K1, N1, 32, outlier_frac=0.02)
    c2 = workloads.make_linear("tilelow2", 8, 951 + M + N1, M, N1, N2, gs2, outlier_frac=0.02)
    xs1, am1 = helpers.calib(c1)
    o1 = oracle.prepare_layer(c1.W, am1, xs1, 32, bias=c1.bias)
    Xq = np.ascontiguousarray(oracle.quantize(c1.X, xs1)[:, o1.perm])
    acc1 = oracle.forward_gemm(o1, Xq, 0.5)
    s_mid = float(np.abs(oracle.dequant_f64(acc1, xs1, o1.w_scale, o1.bias)).max() / 127.0 * 0.8) or 1.0   # some codes clip
    q1 = requant_fp32_sequence(acc1, o1, s_mid)
    check_q(q1, acc1, o1, s_mid)
    am2 = np.abs(q1).max(0).astype(np.float32) * np.float32(s_mid) * np.float32(0.5) + np.float32(1e-6)   # too narrow: the clamp bites
    o2 = oracle.prepare_layer(c2.W, am2, s_mid, gs2, bias=c2.bias)
    h2 = fq.flexiq_quantize_pack(c2.W, am2, s_mid, gs2, bias=c2.bias)
    h1 = fq.flexiq_quantize_pack(c1.W, am1, xs1, 32, bias=c1.bias, out_perm=o2.perm)
    X2 = np.ascontiguousarray(q1[:, o2.perm])
    fq.flexiq_set_ratio(h1, 0.5)
    Xd = torch.from_numpy(Xq).to(dev)
    sh = np.repeat(o2.a_shift.astype(np.int32), gs2)
    G2 = N1 // gs2
    try:
        for r2 in sorted({0.0, 1.0 / G2, 0.5, 1.0}):
            k4 = fq.flexiq_set_ratio(h2, r2)
            want = X2.astype(np.int32).copy()
            want[:, :k4] = np.clip(want[:, :k4] >> sh[:k4], -8, 7) << sh[:k4]
            fq.debug_force_tile_splitk(shape)
            low = fq.flexiq_mixed_gemm(h1, Xd, q=True, out_scale=s_mid, lower_for=h2)["q"]
            torch.cuda.synchronize()
            assert fq.debug_last_launch()["tile"] == -5 and fq.debug_force_tile_splitk(-1) == shape - 1, r2
            assert (low.cpu().numpy().astype(np.int32) == want).all(), r2
            fq.flexiq_input_prelowered(h2, True)
            got = fq.flexiq_mixed_gemm(h2, low, acc=True)["acc"].cpu().numpy()
            fq.flexiq_input_prelowered(h2, False)
            assert (got == oracle.forward_gemm(o2, X2, r2)).all(), r2
    finally:
        fq.debug_force_tile_splitk(-1)
        fq.flexiq_input_prelowered(h2, False)
