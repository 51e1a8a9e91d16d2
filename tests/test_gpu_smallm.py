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
