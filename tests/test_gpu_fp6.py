"""GPU parity of the FP6 variant of the 4-bit phase (flexiq_lower_fp6, flexiq_mixed_gemm_fp6) against the same CPU
oracle as the int8 path: the variant must produce the identical int32 accumulators, so no new oracle arithmetic is
involved.  The packed FP6 activation buffer is an encoding; it is decoded here with numpy and compared with the
oracle's bit-lowering."""
import numpy as np
import pytest

import workloads
from helpers import both_layers, calib, check_q, check_y, requant_fp32_sequence

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


def _decode_x6(buf, M, C, k6):
    """FP6 activation buffer (layout of include/flexiq.h) -> int codes [M][k6] in stored channel order."""
    S = C // 64
    blocks = buf.reshape(-1, S, 3, 64, 16)
    out = np.zeros((M, k6), np.int32)
    e = np.arange(32)
    chan = 8 * ((e % 16) // 4) + 4 * (e // 16) + e % 4
    for m in range(M):
        rr = m % 64
        for u in range(k6 // 32):
            t, h = u // 2, u % 2
            half = h ^ ((rr >> 4) & 1)
            raw = np.concatenate([blocks[m // 64, t, h, rr], blocks[m // 64, t, 2, rr, 8 * half:8 * half + 8]])
            bits = int.from_bytes(raw.tobytes(), "little")
            for el in range(32):
                pat = (bits >> (6 * el)) & 63
                mag = pat & 31
                assert mag <= 8
                out[m, u * 32 + chan[el]] = -mag if pat & 32 else mag
    return out


def test_lower_fp6_encoding(env):
    torch, oracle, fq, dev = env
    case = workloads.make_linear("fp6enc", 8, 401, 150, 256, 64, 32, outlier_frac=0.02)
    case.X *= 2.0
    ol, hl, x_scale = both_layers(case)
    Xq = oracle.quantize(case.X, x_scale)[:, ol.perm]
    Xd = _dev(torch, Xq, dev)
    for r in (1.0, 0.5, 0.375):            # 8, 4 and 3 groups of 32: the last leaves one 4-bit group outside the FP6 prefix
        k4 = fq.flexiq_set_ratio(hl, r)
        k6 = fq.flexiq_fp6_channels(hl)
        assert k6 == (k4 // 64) * 64
        x6, xlow = fq.flexiq_lower_fp6(hl, Xd)
        torch.cuda.synchronize()
        assert x6.numel() == fq.flexiq_fp6_bytes(hl, 150) == 3 * 4 * 3072
        codes = _decode_x6(x6.cpu().numpy(), 150, 256, k6)
        sh = np.repeat(ol.a_shift.astype(np.int32), 32)[None, :k6]
        want = np.clip(Xq[:, :k6].astype(np.int32) >> sh, -8, 7)
        assert all(oracle.bitlower(int(Xq[i, j]), int(sh[0, j])) == want[i, j] for i in (0, 77, 149) for j in range(0, k6, 7))
        assert (codes == want).all(), r
        # the int8 copy: 4-bit channels outside the FP6 prefix lowered at their position, everything else unchanged
        xl = xlow.cpu().numpy().astype(np.int32)
        want_l = Xq.astype(np.int32).copy()
        sh4 = np.repeat(ol.a_shift.astype(np.int32), 32)[None, k6:k4]
        want_l[:, k6:k4] = np.clip(want_l[:, k6:k4] >> sh4, -8, 7) << sh4
        assert (xl[:, k6:] == want_l[:, k6:]).all(), r


def _run_fp6_case(env, case, ratios, with_q=True, scale=1.0):
    torch, oracle, fq, dev = env
    case.X *= scale
    ol, hl, x_scale = both_layers(case)
    Xq = oracle.quantize(case.X, x_scale)[:, ol.perm]
    Xd = _dev(torch, Xq, dev)
    n_shapes = fq.debug_force_fp6_tile(-1)
    try:
        for r in ratios:
            fq.flexiq_set_ratio(hl, r)
            ref = oracle.forward_gemm(ol, Xq, r)
            so = float(np.abs(oracle.dequant_f64(ref, x_scale, ol.w_scale, ol.bias)).max() / 127 * 0.9) or 1.0
            x6, xlow = fq.flexiq_lower_fp6(hl, Xd)
            for t in list(range(n_shapes)) + [-1]:
                fq.debug_force_fp6_tile(t)
                out = fq.flexiq_mixed_gemm_fp6(hl, xlow, x6, acc=True, y=True, q=with_q, out_scale=so)
                torch.cuda.synchronize()
                assert (out["acc"].cpu().numpy() == ref).all(), (case.name, r, t)
                check_y(out["y"].cpu().numpy(), ref, ol)
                if with_q:
                    got_q = out["q"].cpu().numpy()
                    check_q(got_q, ref, ol, so)
                    assert (got_q == requant_fp32_sequence(ref, ol, so)).all()
                    only_q = fq.flexiq_mixed_gemm_fp6(hl, xlow, x6, q=True, out_scale=so)["q"]
                    assert (only_q.cpu().numpy() == got_q).all(), (case.name, r, t)
    finally:
        fq.debug_force_fp6_tile(-1)
    return hl


def test_fp6_gemm_config0_all_ratios(env):
    _run_fp6_case(env, workloads.config0(), (0.0, 0.25, 0.5, 0.75, 1.0))


@pytest.mark.parametrize("M,K,N,gs", [(1, 64, 16, 32), (333, 192, 72, 32), (300, 320, 520, 64), (700, 128, 260, 32),
                                      (65, 448, 7, 64), (531, 576, 328, 32)])
def test_fp6_gemm_ragged_shapes(env, M, K, N, gs):
    # several tiles plus ragged tails in M and N; ratios that leave a 4-bit group outside the FP6 prefix included
    case = workloads.make_linear("fp6ragged", 8, 410 + M + N, M, K, N, gs, outlier_frac=0.02)
    G = K // gs
    _run_fp6_case(env, case, sorted({0.0, 1.0, 0.5, 1.0 / G, 3.0 / G if G >= 3 else 1.0}))


def test_fp6_gemm_saturating_inputs(env):
    # activations far beyond the calibrated range: the clamp of the lowering is active everywhere
    case = workloads.make_linear("fp6sat", 8, 420, 96, 128, 64, 32)
    _run_fp6_case(env, case, (0.5, 1.0), scale=6.0)


def test_fp6_exactness_at_the_certified_bound(env):
    # Extreme operands (every code -8 at position 4, i.e. products of 2^14, all of one sign; then alternating signs):
    # the host may only take as many leading channels as keep every partial sum below 2^24, and within that prefix
    # the fp32 accumulation of the matrix instruction must give the exact integers.
    torch, oracle, fq, dev = env
    M, K, N, gs = 70, 2048, 64, 64
    perm = np.arange(K, dtype=np.int32)
    for name, wsign, xsign in (("same", np.ones(K), np.ones(K)), ("alt", np.where(np.arange(K) % 2, -1.0, 1.0), np.ones(K)),
                               ("altx", np.ones(K), np.where(np.arange(K) % 3 == 0, -1.0, 1.0))):
        W = (-np.ones((N, K)) * wsign[None, :]).astype(np.float32)          # quantises to -+127: code -8 / 7 at position 4
        X = (-np.ones((M, K)) * xsign[None, :]).astype(np.float32) * 128.0
        amax = np.full(K, 127.0, np.float32)
        x_scale = 1.0
        ol = oracle.prepare_layer(W, amax, x_scale, gs, perm=perm)
        hl = fq.flexiq_quantize_pack(W, amax, x_scale, gs, perm=perm)
        Xq = oracle.quantize(X, x_scale)                                     # clips to -+127
        assert (ol.a_shift == 4).all() and (ol.w_shift == 4).all()
        fq.flexiq_set_ratio(hl, 1.0)
        k6 = fq.flexiq_fp6_channels(hl)
        # bound per channel: (8 << 4) * |L(w) << 4| = 128 * 128 (w = -127) or 128 * 112 (w = +127)
        per = np.where(wsign > 0, 128 * 128, 128 * 112)
        cum = np.cumsum(per)
        want_limit = int((cum < 2 ** 24).sum()) // 64 * 64
        assert k6 == want_limit and 0 < k6 < K, (name, k6, want_limit)
        Xd = _dev(torch, Xq, dev)
        x6, xlow = fq.flexiq_lower_fp6(hl, Xd)
        got = fq.flexiq_mixed_gemm_fp6(hl, xlow, x6, acc=True)["acc"].cpu().numpy()
        ref = oracle.forward_gemm(ol, Xq, 1.0)
        assert (got == ref).all(), name
        assert np.abs(ref).max() > 2 ** 22 or name != "same"
        # with run-time positions nothing is known about the activations: the prefix is certified for position 4
        fq.flexiq_dynamic_positions(hl, Xd)
        assert fq.flexiq_fp6_channels(hl) <= k6
        x6, xlow = fq.flexiq_lower_fp6(hl, Xd)
        got = fq.flexiq_mixed_gemm_fp6(hl, xlow, x6, acc=True)["acc"].cpu().numpy()
        dyn = oracle.dynamic_act_shifts(Xq, gs, K // gs, ol.a_shift)
        assert (got == oracle.mixed_gemm(Xq, ol.Wq.reshape(N, K), gs, K // gs, dyn, ol.w_shift)).all(), name
        fq.flexiq_static_positions(hl)


def test_fp6_two_layer_chain(env):
    # fc1 (FP6-variant kernel) writes fc2's input directly: FP6 codes for fc2's FP6 channels, lowered int8 for its other
    # 4-bit channels, plain int8 beyond, all in fc2's stored channel order; fc2 consumes both buffers.
    torch, oracle, fq, dev = env
    M, K1, N1, N2, gs = 300, 192, 256, 96, 32
    c1 = workloads.make_linear("fp6chain1", 8, 431, M, K1, N1, gs, outlier_frac=0.02)
    c2 = workloads.make_linear("fp6chain2", 8, 432, M, N1, N2, gs, outlier_frac=0.02)
    xs1, am1 = calib(c1)
    o1 = oracle.prepare_layer(c1.W, am1, xs1, gs, bias=c1.bias)
    Xq = oracle.quantize(c1.X, xs1)[:, o1.perm]
    r1 = 0.5
    acc1 = oracle.forward_gemm(o1, Xq, r1)
    s_mid = float(np.abs(oracle.dequant_f64(acc1, xs1, o1.w_scale, o1.bias)).max() / 127.0)
    q1 = requant_fp32_sequence(acc1, o1, s_mid)
    check_q(q1, acc1, o1, s_mid)
    am2 = np.abs(q1).max(0).astype(np.float32) * np.float32(s_mid)
    o2 = oracle.prepare_layer(c2.W, am2, s_mid, gs, bias=c2.bias)
    X2 = np.ascontiguousarray(q1[:, o2.perm])
    h2 = fq.flexiq_quantize_pack(c2.W, am2, s_mid, gs, bias=c2.bias)
    h1 = fq.flexiq_quantize_pack(c1.W, am1, xs1, gs, bias=c1.bias, out_perm=o2.perm)
    fq.flexiq_set_ratio(h1, r1)
    Xd = _dev(torch, Xq, dev)
    x6_1, xlow_1 = fq.flexiq_lower_fp6(h1, Xd)
    n_shapes = fq.debug_force_fp6_tile(-1)
    try:
        for r2 in (1.0, 0.625, 0.25, 0.0):      # 8, 5, 2, 0 of fc2's 8 groups at 4 bits
            k4 = fq.flexiq_set_ratio(h2, r2)
            k6 = fq.flexiq_fp6_channels(h2)
            assert k6 == (k4 // 64) * 64
            sh = np.repeat(o2.a_shift.astype(np.int32), gs)[None, :]
            for t in range(n_shapes):
                fq.debug_force_fp6_tile(t)
                x6_2 = torch.zeros(fq.flexiq_fp6_bytes(h2, M), dtype=torch.uint8, device=dev)
                mid = fq.flexiq_mixed_gemm_fp6(h1, xlow_1, x6_1, q=True, out_scale=s_mid, lower_for=h2, x6_out=x6_2)["q"]
                torch.cuda.synchronize()
                got_mid = mid.cpu().numpy().astype(np.int32)
                want_mid = X2.astype(np.int32).copy()
                want_mid[:, :k4] = np.clip(want_mid[:, :k4] >> sh[:, :k4], -8, 7) << sh[:, :k4]
                assert (got_mid[:, k6:] == want_mid[:, k6:]).all(), (r2, t)
                codes = _decode_x6(x6_2.cpu().numpy(), M, N1, k6)
                assert (codes == np.clip(X2[:, :k6].astype(np.int32) >> sh[:, :k6], -8, 7)).all(), (r2, t)
                fq.debug_force_fp6_tile(-1)
                got = fq.flexiq_mixed_gemm_fp6(h2, mid, x6_2, acc=True)["acc"].cpu().numpy()
                assert (got == oracle.forward_gemm(o2, X2, r2)).all(), (r2, t)
            # the same from the kernel that gives a block one tile and splits the reduction over its waves (three tile shapes)
            for shape in (2, 3, 4):
                fq.debug_force_tile_splitk(shape)
                x6_2 = torch.zeros(fq.flexiq_fp6_bytes(h2, M), dtype=torch.uint8, device=dev)
                mid = fq.flexiq_mixed_gemm_fp6(h1, xlow_1, x6_1, q=True, out_scale=s_mid, lower_for=h2, x6_out=x6_2)["q"]
                torch.cuda.synchronize()
                assert fq.debug_force_tile_splitk(-1) == shape - 1, (r2, shape)
                got_mid = mid.cpu().numpy().astype(np.int32)
                assert (got_mid[:, k6:] == want_mid[:, k6:]).all(), (r2, shape)
                codes = _decode_x6(x6_2.cpu().numpy(), M, N1, k6)
                assert (codes == np.clip(X2[:, :k6].astype(np.int32) >> sh[:, :k6], -8, 7)).all(), (r2, shape)
                got = fq.flexiq_mixed_gemm_fp6(h2, mid, x6_2, acc=True)["acc"].cpu().numpy()
                assert (got == oracle.forward_gemm(o2, X2, r2)).all(), (r2, shape)
    finally:
        fq.debug_force_fp6_tile(-1)
        fq.debug_force_tile_splitk(-1)
    # refused: a consumer whose order the producer does not write; FP6 output without a consumer; C not a multiple of 64
    h1_plain = fq.flexiq_quantize_pack(c1.W, am1, xs1, gs, bias=c1.bias)
    fq.flexiq_set_ratio(h1_plain, r1)
    with pytest.raises(fq.FlexiqError):
        fq.flexiq_mixed_gemm_fp6(h1_plain, xlow_1, x6_1, q=True, out_scale=s_mid, lower_for=h2, x6_out=x6_2)
    with pytest.raises(fq.FlexiqError):
        fq.flexiq_mixed_gemm_fp6(h1, xlow_1, x6_1, q=True, out_scale=s_mid, x6_out=x6_2)
    odd = both_layers(workloads.make_linear("fp6odd", 8, 433, 8, 96, 16, 32))[1]
    with pytest.raises(fq.FlexiqError):
        fq.flexiq_fp6_bytes(odd, 8)


@pytest.mark.parametrize("K,N,gs", [(256, 256, 32), (1024, 520, 64), (192, 72, 32), (4096, 1024, 64), (64, 7, 32), (2112, 48, 64)])
def test_fp6_few_rows(env, K, N, gs):
    # calls of at most 64 rows: the few-row kernel with the FP6 K-steps on v_mfma_scale_f32_16x16x128_f8f6f4 (chunks of two
    # K-steps; an odd number of FP6 K-steps leaves half a chunk), every fragment count, ratios that leave 4-bit groups outside
    # the FP6 prefix; the tiled FP6 kernel gives the same bytes
    torch, oracle, fq, dev = env
    case = workloads.make_linear("fp6few", 8, 800 + K + N, 64, K, N, gs, outlier_frac=0.02)
    case.X *= 2.0
    ol, hl, x_scale = both_layers(case)
    Xq_all = oracle.quantize(case.X, x_scale)[:, ol.perm]
    G = K // gs
    fq.debug_force_few_rows(1)   # (beyond 32 rows the automatic route may prefer the kernel that gives a block a whole tile)
    try:
        for M in (1, 7, 16, 17, 33, 48, 64):
            Xq = np.ascontiguousarray(Xq_all[:M])
            Xd = _dev(torch, Xq, dev)
            for r in sorted({0.0, 1.0 / G, 0.5, 3.0 / G if G >= 3 else 1.0, 1.0}):
                fq.flexiq_set_ratio(hl, r)
                ref = oracle.forward_gemm(ol, Xq, r)
                so = float(np.abs(oracle.dequant_f64(ref, x_scale, ol.w_scale, ol.bias)).max() / 127 * 0.9) or 1.0
                x6, xlow = fq.flexiq_lower_fp6(hl, Xd)
                fq.debug_force_fp6_tile(-1)
                out = fq.flexiq_mixed_gemm_fp6(hl, xlow, x6, acc=True, y=True, q=True, out_scale=so)
                torch.cuda.synchronize()
                # the few-row kernel's FP6 build ran (with no 4-bit channel at all the call is an ordinary int8 call)
                assert fq.debug_force_few_rows(1) == (3 if r > 0 else 1), (M, r)
                assert (out["acc"].cpu().numpy() == ref).all(), (M, r)
                check_y(out["y"].cpu().numpy(), ref, ol)
                got_q = out["q"].cpu().numpy()
                check_q(got_q, ref, ol, so)
                assert (got_q == requant_fp32_sequence(ref, ol, so)).all()
                fq.debug_force_fp6_tile(0)                                    # a forced tile shape: the tiled FP6 kernel
                tiled = fq.flexiq_mixed_gemm_fp6(hl, xlow, x6, q=True, out_scale=so)["q"]
                assert (tiled.cpu().numpy() == got_q).all(), (M, r)
    finally:
        fq.debug_force_fp6_tile(-1)
        fq.debug_force_few_rows(-1)


@pytest.mark.parametrize("shape", [2, 3, 4])
@pytest.mark.parametrize("K,N,gs", [(1024, 520, 64), (192, 72, 32), (4096, 100, 64), (2112, 48, 64)])
def test_fp6_tile_splitk(env, K, N, gs, shape):
    # tens to hundreds of rows on a layer with few output tiles: a tile per block (64 x 64, 32 x 64, 32 x 32), the reduction
    # split over its waves, the FP6 K-steps first (an odd number of them leaves half a chunk; fewer chunks than waves), ratios
    # that leave 4-bit groups outside the FP6 prefix; ragged last row and column tiles
    torch, oracle, fq, dev = env
    case = workloads.make_linear("fp6tile", 8, 900 + K + N, 197, K, N, gs, outlier_frac=0.02)
    case.X *= 2.0
    ol, hl, x_scale = both_layers(case)
    Xq_all = oracle.quantize(case.X, x_scale)[:, ol.perm]
    G = K // gs
    fq.debug_force_tile_splitk(shape)
    try:
        for M in (33, 65, 197):
            Xq = np.ascontiguousarray(Xq_all[:M])
            Xd = _dev(torch, Xq, dev)
            for r in sorted({1.0 / G, 0.5, 3.0 / G if G >= 3 else 1.0, 1.0}):
                fq.flexiq_set_ratio(hl, r)
                ref = oracle.forward_gemm(ol, Xq, r)
                so = float(np.abs(oracle.dequant_f64(ref, x_scale, ol.w_scale, ol.bias)).max() / 127 * 0.9) or 1.0
                x6, xlow = fq.flexiq_lower_fp6(hl, Xd)
                out = fq.flexiq_mixed_gemm_fp6(hl, xlow, x6, acc=True, y=True, q=True, out_scale=so)
                torch.cuda.synchronize()
                assert fq.debug_force_tile_splitk(shape) == shape - 1, (M, r)     # ran on this kernel, this tile
                assert (out["acc"].cpu().numpy() == ref).all(), (M, r)
                check_y(out["y"].cpu().numpy(), ref, ol)
                got_q = out["q"].cpu().numpy()
                check_q(got_q, ref, ol, so)
                assert (got_q == requant_fp32_sequence(ref, ol, so)).all()
    finally:
        fq.debug_force_tile_splitk(-1)


@pytest.mark.parametrize("M", [1, 5, 20, 48])
def test_fp6_chain_few_rows(env, M):
    # the two-layer FP6 chain on a few rows, automatic route: the producer (long reduction, few tiles) runs on the kernel that gives
    # a block one tile and writes the consumer's FP6 codes and lowered int8 rows; the consumer reads both on a few-row kernel
    torch, oracle, fq, dev = env
    K1, N1, N2, gs = 1024, 256, 96, 32
    c1 = workloads.make_linear("fp6few1", 8, 441 + M, M, K1, N1, gs, outlier_frac=0.02)
    c2 = workloads.make_linear("fp6few2", 8, 442 + M, M, N1, N2, gs, outlier_frac=0.02)
    xs1, am1 = calib(c1)
    o1 = oracle.prepare_layer(c1.W, am1, xs1, gs, bias=c1.bias)
    Xq = np.ascontiguousarray(oracle.quantize(c1.X, xs1)[:, o1.perm])
    acc1 = oracle.forward_gemm(o1, Xq, 0.5)
    s_mid = float(np.abs(oracle.dequant_f64(acc1, xs1, o1.w_scale, o1.bias)).max() / 127.0) or 1.0
    q1 = requant_fp32_sequence(acc1, o1, s_mid)
    am2 = np.abs(q1).max(0).astype(np.float32) * np.float32(s_mid) + np.float32(1e-6)
    o2 = oracle.prepare_layer(c2.W, am2, s_mid, gs, bias=c2.bias)
    X2 = np.ascontiguousarray(q1[:, o2.perm])
    h2 = fq.flexiq_quantize_pack(c2.W, am2, s_mid, gs, bias=c2.bias)
    h1 = fq.flexiq_quantize_pack(c1.W, am1, xs1, gs, bias=c1.bias, out_perm=o2.perm)
    fq.flexiq_set_ratio(h1, 0.5)
    x6_1, xlow_1 = fq.flexiq_lower_fp6(h1, _dev(torch, Xq, dev))
    sh = np.repeat(o2.a_shift.astype(np.int32), gs)[None, :]
    for r2 in (1.0, 0.625, 0.25):
        k4 = fq.flexiq_set_ratio(h2, r2)
        k6 = fq.flexiq_fp6_channels(h2)
        x6_2 = torch.zeros(fq.flexiq_fp6_bytes(h2, M), dtype=torch.uint8, device=dev)
        mid = fq.flexiq_mixed_gemm_fp6(h1, xlow_1, x6_1, q=True, out_scale=s_mid, lower_for=h2, x6_out=x6_2)["q"]
        torch.cuda.synchronize()
        assert fq.debug_force_tile_splitk(-1) > 0, (M, r2)
        want_mid = X2.astype(np.int32).copy()
        want_mid[:, :k4] = np.clip(want_mid[:, :k4] >> sh[:, :k4], -8, 7) << sh[:, :k4]
        assert (mid.cpu().numpy().astype(np.int32)[:, k6:] == want_mid[:, k6:]).all(), (M, r2)
        codes = _decode_x6(x6_2.cpu().numpy(), M, N1, k6)
        assert (codes == np.clip(X2[:, :k6].astype(np.int32) >> sh[:, :k6], -8, 7)).all(), (M, r2)
        got = fq.flexiq_mixed_gemm_fp6(h2, mid, x6_2, acc=True)["acc"].cpu().numpy()
        assert (got == oracle.forward_gemm(o2, X2, r2)).all(), (M, r2)
