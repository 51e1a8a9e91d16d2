"""GPU parity: the HIP library through its C ABI against the CPU oracle, element by element.
int32 accumulators, int8 codes, indices and packed bytes must match bit for bit; fp32 outputs
within 1e-5 relative."""
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


def test_pack_matches_oracle(env):
    torch, oracle, fq, dev = env
    for case in (workloads.config0(), workloads.make_linear("odd", 9, 1, 8, 192, 72, 64, outlier_frac=0.02),
                 workloads.make_conv("c", 9, 2, 1, 5, 5, 96, 40, 3, 3, 1, 1, 32)):
        ol, hl, _ = both_layers(case)
        info = hl.info()
        assert (info["perm"] == ol.perm).all()
        assert (info["w_scale"] == ol.w_scale).all()
        assert (info["a_shift"] == ol.a_shift).all()
        assert (info["w_shift"] == ol.w_shift).all()
        assert info["G"] == ol.G and info["max_4bit_ch"] == 0
        w8, w4, w4x = fq.flexiq_layer_dump(hl)
        T = ol.R * ol.S
        Wq = ol.Wq.reshape(ol.N, T, ol.C)
        assert (w8 == Wq).all()
        # the cached 4-bit copy of ALL groups is the oracle's bit-lowering of the stored 8-bit weights
        for t in range(T):
            ref4 = oracle.bitlower_pack(Wq[:, t, :], ol.group_size, ol.w_shift, per_row=True)
            assert (w4[:, t, :] == ref4).all()
            # ... and the expanded copy holds every code at its position: L(w, s) << s
            sh = np.repeat(ol.w_shift.astype(np.int32), ol.group_size, axis=1)
            lowered = np.clip(Wq[:, t, :].astype(np.int32) >> sh, -8, 7)
            assert (np.vectorize(oracle.bitlower)(Wq[:5, t, :17].astype(int), sh[:5, :17]) == lowered[:5, :17]).all()
            assert (w4x[:, t, :].astype(np.int32) == lowered << sh).all()


def test_pack_with_given_perm(env):
    torch, oracle, fq, dev = env
    case = workloads.config0()
    perm = np.random.default_rng(5).permutation(case.K).astype(np.int32)
    ol, hl, _ = both_layers(case, perm=perm)
    assert (hl.info()["perm"] == perm).all()
    w8, _, _ = fq.flexiq_layer_dump(hl)
    assert (w8[:, 0, :] == ol.Wq.reshape(ol.N, ol.C)).all()


def test_quantize_act(env):
    torch, oracle, fq, dev = env
    rng = np.random.default_rng(1)
    for n in (0, 1, 3, 4, 5, 1023, 4096, 100003):
        x = (rng.standard_normal(n) * 3).astype(np.float32)
        if n > 8:
            x[:8] = np.array([0.5, 1.5, 2.5, -0.5, -1.5, 1e9, -1e9, 0.0], np.float32) * np.float32(0.05)
        S = 0.05
        xd = torch.empty(max(n, 4), dtype=torch.float32, device=dev)[:n]
        xd.copy_(torch.from_numpy(x))
        q = fq.flexiq_quantize_act(xd, S)
        torch.cuda.synchronize()
        assert (q.cpu().numpy() == oracle.quantize(x, S)).all()


def test_bitlower_exhaustive(env):
    torch, oracle, fq, dev = env
    # all 256 values x 5 positions x both modes
    vals = np.arange(-128, 128, dtype=np.int16).astype(np.int8)
    src = np.tile(vals, (5, 1))                                 # rows: one per position, C = 256
    for mode in (0, 1):
        for gs in (32, 64):
            G = 256 // gs
            shifts = np.repeat(np.arange(5, dtype=np.uint8)[:, None], G, axis=1)   # per row
            got = fq.flexiq_bitlower(_dev(torch, src, dev), gs, _dev(torch, shifts, dev), per_row=True, mode=mode)
            torch.cuda.synchronize()
            assert (got.cpu().numpy() == oracle.bitlower_pack(src, gs, shifts, per_row=True, mode=mode)).all()
    rng = np.random.default_rng(2)
    src = rng.integers(-128, 128, size=(37, 192)).astype(np.int8)
    sh = rng.integers(0, 5, size=6).astype(np.uint8)
    got = fq.flexiq_bitlower(_dev(torch, src, dev), 32, _dev(torch, sh, dev), per_row=False)
    assert (got.cpu().numpy() == oracle.bitlower_pack(src, 32, sh, per_row=False)).all()


def test_permute_channels(env):
    torch, oracle, fq, dev = env
    case = workloads.config0()
    ol, hl, x_scale = both_layers(case)
    Xq = oracle.quantize(case.X, x_scale)
    got = fq.flexiq_permute_channels(hl, _dev(torch, Xq, dev))
    assert (got.cpu().numpy() == Xq[:, ol.perm]).all()


@pytest.mark.parametrize("C,gs,rows", [(32, 32, 1), (96, 32, 1000), (768, 32, 333), (4096, 64, 37), (4128, 32, 9),
                                       (8192, 64, 6), (10176, 64, 5), (64, 32, 3000)])
def test_permute_channels_row_lengths(env, C, gs, rows):
    """Row lengths on every route of the reorder operator: several rows per staged run, one, long rows dealt out over
    the block (up to the 159 groups of 64 channels a layer may have)."""
    torch, oracle, fq, dev = env
    rng = np.random.default_rng(7000 + C)
    W = rng.normal(0, 0.02, size=(8, C)).astype(np.float32)
    amax = np.abs(rng.normal(0, 1, size=C)).astype(np.float32) + 0.01
    x_scale = float(np.float32(amax.max()) / np.float32(127.0))
    ol = oracle.prepare_layer(W, amax, x_scale, gs)
    hl = fq.flexiq_quantize_pack(W, amax, x_scale, gs)
    assert (hl.info()["perm"] == ol.perm).all()
    X = rng.integers(-128, 128, size=(rows, C)).astype(np.int8)
    got = fq.flexiq_permute_channels(hl, _dev(torch, X, dev))
    assert (got.cpu().numpy() == X[:, ol.perm]).all()


_Q_WINDOW = [0, 0]   # int8 codes that needed the tie window / codes compared (printed by the last test)


def _run_gemm_case(env, case, ratios, rows=None, with_q=True):
    torch, oracle, fq, dev = env
    ol, hl, x_scale = both_layers(case)
    Xq = oracle.quantize(case.X, x_scale)[:, ol.perm]
    if rows is not None:
        Xq = np.ascontiguousarray(Xq[:rows])
    Xd = _dev(torch, Xq, dev)
    for r in ratios:
        k4 = fq.flexiq_set_ratio(hl, r)
        assert k4 == oracle.groups_for_ratio(r, ol.G) * ol.group_size
        ref = oracle.forward_gemm(ol, Xq, r)
        so = float(np.abs(oracle.dequant_f64(ref, x_scale, ol.w_scale, ol.bias)).max() / 127 * 0.9) or 1.0
        try:
            for packed in (0, 1):   # 4-bit weights from the expanded copy, then from the packed codes
                fq.debug_force_packed4(packed)
                out = fq.flexiq_mixed_gemm(hl, Xd, acc=True, y=True, q=with_q, out_scale=so)
                torch.cuda.synchronize()
                assert (out["acc"].cpu().numpy() == ref).all(), (case.name, r, packed)
                check_y(out["y"].cpu().numpy(), ref, ol)
                if with_q:
                    # against the float64 definition (ties within fp32 rounding may take either neighbour) ...
                    got_q = out["q"].cpu().numpy()
                    _Q_WINDOW[0] += check_q(got_q, ref, ol, so)
                    _Q_WINDOW[1] += got_q.size
                    # ... and, as a second assertion, bit for bit against the documented fp32 operation sequence
                    assert (got_q == requant_fp32_sequence(ref, ol, so)).all()
                    # int8 as the only output: the epilogue variants that take the requantisation constants
                    # from the tile's table (row-contiguous stores when N is a multiple of 16, the general form else)
                    only_q = fq.flexiq_mixed_gemm(hl, Xd, q=True, out_scale=so)["q"]
                    assert (only_q.cpu().numpy() == got_q).all(), (case.name, r, packed)
        finally:
            fq.debug_force_packed4(-1)


def test_gemm_config0_all_ratios_all_tiles(env):
    torch, oracle, fq, dev = env
    n = fq.debug_force_tile(-1)
    try:
        for t in range(n):
            fq.debug_force_tile(t)
            _run_gemm_case(env, workloads.config0(), (0.0, 0.25, 0.5, 0.75, 1.0))
    finally:
        fq.debug_force_tile(-1)


@pytest.mark.parametrize("M,K,N,gs", [(1, 64, 16, 32), (17, 64, 4, 64), (333, 192, 72, 32), (300, 320, 520, 64),
                                      (700, 96, 260, 32), (5, 128, 7, 32)])
def test_gemm_ragged_shapes(env, M, K, N, gs):
    # several tiles plus a ragged tail in M and N; N = 7 exercises the scalar store path
    case = workloads.make_linear("ragged", 8, M + N, M, K, N, gs, outlier_frac=0.02)
    G = K // gs
    ratios = sorted({0.0, 1.0, 0.5, 1.0 / G})
    _run_gemm_case(env, case, ratios)


def test_gemm_ragged_all_tiles(env):
    torch, oracle, fq, dev = env
    n = fq.debug_force_tile(-1)
    case = workloads.make_linear("ragged_tiles", 8, 77, 531, 160, 328, 32, outlier_frac=0.02)
    try:
        for t in range(n):
            fq.debug_force_tile(t)
            _run_gemm_case(env, case, (0.0, 0.6, 1.0))
    finally:
        fq.debug_force_tile(-1)


def test_gemm_blocks_walk_several_tiles(env):
    # few blocks, many output tiles: every block computes a sequence of tiles with its load pipeline running
    # across the tile boundaries (ragged last tile row and column included); compared with one block per tile
    torch, oracle, fq, dev = env
    n = fq.debug_force_tile(-1)
    case = workloads.make_linear("walk", 8, 78, 531, 320, 592, 32, outlier_frac=0.02)
    try:
        for t in range(n):
            fq.debug_force_tile(t)
            for nb in (1, 3, 7, -1):
                fq.debug_max_blocks(nb)
                _run_gemm_case(env, case, (0.0, 0.3, 0.5, 1.0))
    finally:
        fq.debug_force_tile(-1)
        fq.debug_max_blocks(0)


@pytest.mark.parametrize("M,K,N,gs,scale", [(300, 256, 96, 32, 1.0), (1000, 192, 72, 32, 4.0), (77, 512, 64, 64, 0.25),
                                            (2500, 96, 40, 32, 2.0), (1, 64, 16, 32, 1.0),
                                            # more than 4096 scanned channels (two column slabs of blocks), and many
                                            # row blocks (one row of partial masks each)
                                            (900, 8192, 16, 64, 1.0), (40000, 128, 16, 32, 0.5)])
def test_dynamic_positions(env, M, K, N, gs, scale):
    # positions found by the run-time OR scan == the oracle's scan, and the GEMM that uses them == the oracle's
    # GEMM with those positions; `scale` moves the run-time range above / below the calibrated one
    torch, oracle, fq, dev = env
    case = workloads.make_linear("dyn", 8, M + K + N, M, K, N, gs, outlier_frac=0.02)
    case.X *= scale
    ol, hl, x_scale = both_layers(case)
    Xq = oracle.quantize(case.X, x_scale)[:, ol.perm]
    Xd = _dev(torch, Xq, dev)
    G = K // gs
    for r in (1.0, 0.5, 1.0 / G, 0.0):
        k4 = fq.flexiq_set_ratio(hl, r)
        G4 = k4 // gs
        fq.flexiq_dynamic_positions(hl, Xd)
        want = oracle.dynamic_act_shifts(Xq, gs, G4, ol.a_shift)
        assert (fq.flexiq_layer_positions(hl) == want).all(), (r, fq.flexiq_layer_positions(hl), want)
        ref = oracle.mixed_gemm(Xq, ol.Wq.reshape(N, K), gs, G4, want, ol.w_shift)
        got = fq.flexiq_mixed_gemm(hl, Xd, acc=True)["acc"].cpu().numpy()
        assert (got == ref).all(), r
        # twice in a row: the scan leaves its scratch clean
        fq.flexiq_dynamic_positions(hl, Xd)
        assert (fq.flexiq_layer_positions(hl) == want).all()
        # and back to the calibrated positions
        fq.flexiq_static_positions(hl)
        assert (fq.flexiq_layer_positions(hl) == ol.a_shift).all()
        assert (fq.flexiq_mixed_gemm(hl, Xd, acc=True)["acc"].cpu().numpy() == oracle.forward_gemm(ol, Xq, r)).all()
    # empty input: scanned groups get position 0
    fq.flexiq_set_ratio(hl, 1.0)
    fq.flexiq_dynamic_positions(hl, Xd[:0])
    assert (fq.flexiq_layer_positions(hl) == 0).all()
    fq.flexiq_static_positions(hl)


def test_dynamic_positions_conv(env):
    torch, oracle, fq, dev = env
    case = workloads.make_conv("dynconv", 7, 41, 3, 9, 9, 64, 48, 3, 3, 1, 1, 32)
    case.X *= 3.0
    ol, hl, x_scale = both_layers(case)
    Xq = np.ascontiguousarray(oracle.quantize(case.X, x_scale)[..., ol.perm])
    Xd = _dev(torch, Xq, dev)
    fq.flexiq_set_ratio(hl, 0.5)
    G4 = oracle.groups_for_ratio(0.5, ol.G)
    fq.flexiq_dynamic_positions(hl, Xd)
    want = oracle.dynamic_act_shifts(Xq, 32, G4, ol.a_shift)
    assert (fq.flexiq_layer_positions(hl) == want).all()
    ref = oracle.mixed_conv(Xq, ol.Wq, 1, 1, 32, G4, want, ol.w_shift)
    got = fq.flexiq_mixed_conv_implicit(hl, Xd, 1, 1, acc=True)["acc"].cpu().numpy()
    assert (got == ref).all()
    fq.flexiq_static_positions(hl)


def test_two_layer_chain_static_reorder(env):
    # Section 5, steps 1-2: fc1 is packed so that it writes its int8 outputs in the stored channel order of fc2;
    # the chain fc1 -> int8 requant -> fc2 then needs no run-time reorder and equals the oracle's chain, in which
    # the oracle permutes explicitly.  Run once with calibrated and once with run-time positions for fc2.
    torch, oracle, fq, dev = env
    M, K1, N1, N2, gs = 300, 192, 256, 96, 32
    c1 = workloads.make_linear("chain1", 8, 201, M, K1, N1, gs, outlier_frac=0.02)
    c2 = workloads.make_linear("chain2", 8, 202, M, N1, N2, gs, outlier_frac=0.02)
    xs1, am1 = __import__("helpers").calib(c1)
    o1 = oracle.prepare_layer(c1.W, am1, xs1, gs, bias=c1.bias)
    Xq = oracle.quantize(c1.X, xs1)[:, o1.perm]
    r1, r2 = 0.5, 0.75
    acc1 = oracle.forward_gemm(o1, Xq, r1)
    y1 = oracle.dequant_f64(acc1, xs1, o1.w_scale, o1.bias)
    s_mid = float(np.abs(y1).max() / 127.0)                       # scale of the intermediate int8 tensor
    # The intermediate int8 tensor.  Its definition is oracle.requant_i8 (float64); an element within fp32 rounding
    # of a tie may take either neighbour, so the tensor fed to the second layer's oracle is the CPU emulation of
    # the documented fp32 sequence, itself checked against the definition with the tie window.
    q1 = requant_fp32_sequence(acc1, o1, s_mid)                     # original output-channel order
    check_q(q1, acc1, o1, s_mid)
    o2 = oracle.prepare_layer(c2.W, np.abs(q1).max(0).astype(np.float32) * np.float32(s_mid), s_mid, gs, bias=c2.bias)
    X2 = np.ascontiguousarray(q1[:, o2.perm])                     # what fc2 reads: its stored order
    # HIP side: fc2 first (its order is what fc1 must produce), then fc1 with that output order
    h2 = fq.flexiq_quantize_pack(c2.W, np.abs(q1).max(0).astype(np.float32) * np.float32(s_mid), s_mid, gs, bias=c2.bias)
    assert (h2.info()["perm"] == o2.perm).all()
    h1 = fq.flexiq_quantize_pack(c1.W, am1, xs1, gs, bias=c1.bias, out_perm=o2.perm)
    assert (h1.info()["w_scale"] == o1.w_scale[o2.perm]).all()
    fq.flexiq_set_ratio(h1, r1)
    fq.flexiq_set_ratio(h2, r2)
    mid = fq.flexiq_mixed_gemm(h1, _dev(torch, Xq, dev), q=True, out_scale=s_mid)["q"]
    assert (mid.cpu().numpy() == X2).all()
    got = fq.flexiq_mixed_gemm(h2, mid, acc=True)["acc"].cpu().numpy()
    assert (got == oracle.forward_gemm(o2, X2, r2)).all()
    G4 = oracle.groups_for_ratio(r2, o2.G)
    fq.flexiq_dynamic_positions(h2, mid)
    dyn = oracle.dynamic_act_shifts(X2, gs, G4, o2.a_shift)
    got = fq.flexiq_mixed_gemm(h2, mid, acc=True)["acc"].cpu().numpy()
    assert (got == oracle.mixed_gemm(X2, o2.Wq.reshape(N2, N1), gs, G4, dyn, o2.w_shift)).all()
    fq.flexiq_static_positions(h2)
    # Fused producer: fc1's epilogue also bit-lowers the columns that are 4-bit channels of fc2 (fc2's ratio and
    # positions); fc2, told so, copies its activations like 8-bit ones.  Same accumulators as lowering on the fly.
    for r2b in (0.75, 1.0, 0.25, 0.0):
        k4 = fq.flexiq_set_ratio(h2, r2b)
        mid_l = fq.flexiq_mixed_gemm(h1, _dev(torch, Xq, dev), q=True, out_scale=s_mid, lower_for=h2)["q"]
        sh = np.repeat(o2.a_shift.astype(np.int32), gs)[None, :]
        want_mid = X2.astype(np.int32).copy()
        want_mid[:, :k4] = (np.clip(want_mid[:, :k4] >> sh[:, :k4], -8, 7)) << sh[:, :k4]
        assert all(oracle.bitlower(int(X2[i, j]), int(sh[0, j])) << int(sh[0, j]) == want_mid[i, j]
                   for i in (0, 7, 299) for j in range(0, k4, 5))
        assert (mid_l.cpu().numpy().astype(np.int32) == want_mid).all(), r2b
        if r2b == 0.75:   # every tile shape of the producer lowers alike
            n_tiles = fq.debug_force_tile(-1)
            try:
                for t in range(n_tiles):
                    fq.debug_force_tile(t)
                    got_t = fq.flexiq_mixed_gemm(h1, _dev(torch, Xq, dev), q=True, out_scale=s_mid, lower_for=h2)["q"]
                    assert (got_t.cpu().numpy().astype(np.int32) == want_mid).all(), t
            finally:
                fq.debug_force_tile(-1)
        fq.flexiq_input_prelowered(h2, True)
        got = fq.flexiq_mixed_gemm(h2, mid_l, acc=True)["acc"].cpu().numpy()
        fq.flexiq_input_prelowered(h2, False)
        assert (got == oracle.forward_gemm(o2, X2, r2b)).all(), r2b
    with pytest.raises(fq.FlexiqError):
        fq.flexiq_quantize_pack(c1.W, am1, xs1, gs, out_perm=np.zeros(N1, np.int32))   # not a permutation
    with pytest.raises(fq.FlexiqError):
        fq.flexiq_mixed_gemm(h2, mid, q=True, out_scale=1.0, lower_for=h2)             # consumer width mismatch


def test_producer_scans_for_consumer(env):
    # Section 4.1 / Section 9 "Finding extraction positions at runtime", done where the tensor is produced: fc1's
    # epilogue ORs the magnitude bits of its int8 output per channel group of fc2 and the last block leaves fc2's
    # run-time positions (and the scan scratch clean: the second of two calls in a row is as good as the first).  Checked for every tile shape of the producer (all reduction paths over the wave), on a
    # ragged row count (rows of the last tile beyond M carry the bias and must not count), for several ratios of the
    # consumer in a row (the scan words must be clean again after every call) and two output scales.
    torch, oracle, fq, dev = env
    M, K1, N1, N2, gs = 300, 192, 256, 96, 32
    c1 = workloads.make_linear("scan1", 8, 211, M, K1, N1, gs, outlier_frac=0.02)
    c2 = workloads.make_linear("scan2", 8, 212, M, N1, N2, gs, outlier_frac=0.02)
    xs1, am1 = __import__("helpers").calib(c1)
    o1 = oracle.prepare_layer(c1.W, am1, xs1, gs, bias=c1.bias)
    Xq = oracle.quantize(c1.X, xs1)[:, o1.perm]
    acc1 = oracle.forward_gemm(o1, Xq, 0.5)
    y1 = oracle.dequant_f64(acc1, xs1, o1.w_scale, o1.bias)
    s0 = float(np.abs(y1).max() / 127.0)
    n_tiles = fq.debug_force_tile(-1)
    seen_dynamic = False   # the scan changed something against the calibrated positions
    try:
        for s_mid in (s0, 6.0 * s0):
            q1 = requant_fp32_sequence(acc1, o1, s_mid)      # checked against the float64 definition, tie window
            check_q(q1, acc1, o1, s_mid)
            am2 = np.abs(q1).max(0).astype(np.float32) * np.float32(s_mid) * np.float32(3.0)   # calibrated too wide
            o2 = oracle.prepare_layer(c2.W, am2, s_mid, gs, bias=c2.bias)
            X2 = np.ascontiguousarray(q1[:, o2.perm])
            h2 = fq.flexiq_quantize_pack(c2.W, am2, s_mid, gs, bias=c2.bias)
            h1 = fq.flexiq_quantize_pack(c1.W, am1, xs1, gs, bias=c1.bias, out_perm=o2.perm)
            fq.flexiq_set_ratio(h1, 0.5)
            for t in range(n_tiles):
                for r2 in (0.75, 0.25, 1.0):
                    fq.flexiq_set_ratio(h2, r2)
                    G4 = oracle.groups_for_ratio(r2, o2.G)
                    fq.debug_force_tile(t)
                    mid = fq.flexiq_mixed_gemm(h1, _dev(torch, Xq, dev), q=True, out_scale=s_mid, scan_for=h2)["q"]
                    fq.debug_force_tile(-1)
                    assert (mid.cpu().numpy() == X2).all(), (t, r2)
                    dyn = oracle.dynamic_act_shifts(X2, gs, G4, o2.a_shift)
                    assert (fq.flexiq_layer_positions(h2) == dyn).all(), (t, r2, s_mid)
                    seen_dynamic |= bool((dyn != o2.a_shift).any())
                    got = fq.flexiq_mixed_gemm(h2, mid, acc=True)["acc"].cpu().numpy()
                    assert (got == oracle.mixed_gemm(X2, o2.Wq.reshape(N2, N1), gs, G4, dyn, o2.w_shift)).all(), (t, r2)
            # two producer calls in a row (the first on other data): only the last one counts
            fq.flexiq_set_ratio(h2, 0.75)
            fq.flexiq_mixed_gemm(h1, _dev(torch, (Xq // 2).astype(np.int8), dev), q=True, out_scale=s_mid / 4, scan_for=h2)
            mid = fq.flexiq_mixed_gemm(h1, _dev(torch, Xq, dev), q=True, out_scale=s_mid, scan_for=h2)["q"]
            G4 = oracle.groups_for_ratio(0.75, o2.G)
            assert (fq.flexiq_layer_positions(h2) == oracle.dynamic_act_shifts(X2, gs, G4, o2.a_shift)).all()
            # same result as the stand-alone scan kernel
            fq.flexiq_set_ratio(h2, 1.0)
            fq.flexiq_dynamic_positions(h2, mid)
            assert (fq.flexiq_layer_positions(h2) == oracle.dynamic_act_shifts(X2, gs, o2.G, o2.a_shift)).all()
            with pytest.raises(fq.FlexiqError):
                fq.flexiq_mixed_gemm(h1, _dev(torch, Xq, dev), q=True, out_scale=s_mid, lower_for=h2, scan_for=h2)
            with pytest.raises(fq.FlexiqError):
                fq.flexiq_mixed_gemm(h1, _dev(torch, Xq, dev), acc=True, scan_for=h2)   # needs the int8 output
    finally:
        fq.debug_force_tile(-1)
    assert seen_dynamic


def test_producer_scan_graph_replay(env):
    # The chain producer (scan for the consumer) -> consumer captured once in a HIP graph and replayed on changing
    # inputs, with eager work and synchronisations in between: every replay must see positions scanned from ITS
    # data (the scan scratch is cleaned by the kernel itself, nothing is frozen at capture time).
    torch, oracle, fq, dev = env
    M, K1, N1, N2, gs = 200, 128, 128, 64, 32
    c1 = workloads.make_linear("gscan1", 8, 221, M, K1, N1, gs, outlier_frac=0.02)
    c2 = workloads.make_linear("gscan2", 8, 222, M, N1, N2, gs, outlier_frac=0.02)
    xs1, am1 = __import__("helpers").calib(c1)
    o1 = oracle.prepare_layer(c1.W, am1, xs1, gs, bias=c1.bias)
    Xq0 = oracle.quantize(c1.X, xs1)[:, o1.perm]
    acc0 = oracle.forward_gemm(o1, Xq0, 0.5)
    s_mid = float(np.abs(oracle.dequant_f64(acc0, xs1, o1.w_scale, o1.bias)).max() / 127.0)
    am2 = np.full(N1, 127.0 * s_mid, np.float32)
    o2 = oracle.prepare_layer(c2.W, am2, s_mid, gs, bias=c2.bias)
    h2 = fq.flexiq_quantize_pack(c2.W, am2, s_mid, gs, bias=c2.bias)
    h1 = fq.flexiq_quantize_pack(c1.W, am1, xs1, gs, bias=c1.bias, out_perm=o2.perm)
    fq.flexiq_set_ratio(h1, 0.5)
    fq.flexiq_set_ratio(h2, 1.0)
    x_in = torch.empty((M, K1), dtype=torch.int8, device=dev)
    bufs1 = {"q": torch.empty((M, N1), dtype=torch.int8, device=dev)}
    bufs2 = {"acc": torch.empty((M, N2), dtype=torch.int32, device=dev)}

    def chain():
        fq.flexiq_mixed_gemm(h1, x_in, q=True, out_scale=s_mid, bufs=bufs1, scan_for=h2)
        fq.flexiq_mixed_gemm(h2, bufs1["q"], acc=True, bufs=bufs2)

    x_in.copy_(_dev(torch, Xq0, dev))
    chain()                                   # warm-up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        chain()
    for div in (1, 3, 9, 2):                  # smaller and smaller activations, then larger again
        Xq = (Xq0.astype(np.int32) // div).astype(np.int8)
        x_in.copy_(_dev(torch, Xq, dev))
        g.replay()
        torch.cuda.synchronize()
        acc1 = oracle.forward_gemm(o1, Xq, 0.5)
        q1 = requant_fp32_sequence(acc1, o1, s_mid)
        check_q(q1, acc1, o1, s_mid)
        X2 = np.ascontiguousarray(q1[:, o2.perm])
        assert (bufs1["q"].cpu().numpy() == X2).all(), div
        dyn = oracle.dynamic_act_shifts(X2, gs, o2.G, o2.a_shift)
        assert (fq.flexiq_layer_positions(h2) == dyn).all(), div
        want = oracle.mixed_gemm(X2, o2.Wq.reshape(N2, N1), gs, o2.G, dyn, o2.w_shift)
        assert (bufs2["acc"].cpu().numpy() == want).all(), div
        _ = (x_in.float().sum().item())        # eager work between replays


def test_gemm_saturating_inputs(env):
    # activations far beyond the calibrated range: the clamp of the lowering is active everywhere
    torch, oracle, fq, dev = env
    case = workloads.make_linear("sat", 8, 3, 96, 128, 64, 32)
    case.X *= 6.0
    _run_gemm_case(env, case, (0.0, 0.5, 1.0))
    case.X[:] = 1e9
    _run_gemm_case(env, case, (1.0,))
    case.X[:] = -1e9
    _run_gemm_case(env, case, (1.0,))


def test_gemm_empty_and_errors(env):
    torch, oracle, fq, dev = env
    case = workloads.config0()
    ol, hl, x_scale = both_layers(case)
    X0 = torch.empty((0, case.K), dtype=torch.int8, device=dev)
    out = fq.flexiq_mixed_gemm(hl, X0, acc=True)
    assert out["acc"].shape == (0, case.N)
    with pytest.raises(fq.FlexiqError):
        fq.flexiq_set_ratio(hl, 1.5)
    with pytest.raises(fq.FlexiqError):
        fq.flexiq_set_ratio(hl, -0.1)
    X = torch.zeros((8, case.K), dtype=torch.int8, device=dev)
    with pytest.raises(fq.FlexiqError):
        fq.flexiq_mixed_gemm(hl, X)                      # no output requested
    with pytest.raises(fq.FlexiqError):
        fq.flexiq_mixed_gemm(hl, X, q=True, out_scale=0.0)
    Xmis = torch.zeros(8 * case.K + 16, dtype=torch.int8, device=dev)[1:1 + 8 * case.K].view(8, case.K)
    with pytest.raises(fq.FlexiqError):
        fq.flexiq_mixed_gemm(hl, Xmis.contiguous() if False else Xmis, acc=True)   # misaligned pointer


def test_ratio_switch_needs_no_repack(env):
    # one handle, packed once, serves every ratio: device buffers identical before and after
    torch, oracle, fq, dev = env
    case = workloads.config0()
    ol, hl, x_scale = both_layers(case)
    w8a, w4a, w4xa = fq.flexiq_layer_dump(hl)
    Xq = oracle.quantize(case.X, x_scale)[:, ol.perm]
    Xd = _dev(torch, Xq, dev)
    sched = workloads.config4_ratio_schedule(12)
    for r in sched:
        fq.flexiq_set_ratio(hl, float(r))
        got = fq.flexiq_mixed_gemm(hl, Xd, acc=True)["acc"].cpu().numpy()
        fresh = both_layers(case)[1]
        fq.flexiq_set_ratio(fresh, float(r))
        assert (got == fq.flexiq_mixed_gemm(fresh, Xd, acc=True)["acc"].cpu().numpy()).all()
        assert (got == oracle.forward_gemm(ol, Xq, float(r))).all()
    w8b, w4b, w4xb = fq.flexiq_layer_dump(hl)
    assert (w8a == w8b).all() and (w4a == w4b).all() and (w4xa == w4xb).all()


@pytest.mark.parametrize("B,H,C,N,R,stride,pad,gs", [(2, 7, 64, 24, 3, 1, 1, 32), (3, 9, 128, 72, 3, 2, 1, 64),
                                                     (2, 6, 96, 130, 1, 1, 0, 32), (2, 8, 64, 64, 1, 2, 0, 32),
                                                     (1, 5, 32, 16, 3, 1, 1, 32), (5, 14, 64, 96, 3, 1, 1, 32)])
def test_conv_small(env, B, H, C, N, R, stride, pad, gs):
    torch, oracle, fq, dev = env
    case = workloads.make_conv("conv", 7, B * H + C + N + R, B, H, H, C, N, R, R, stride, pad, gs)
    ol, hl, x_scale = both_layers(case)
    Xq = np.ascontiguousarray(oracle.quantize(case.X, x_scale)[..., ol.perm])
    Xd = _dev(torch, Xq, dev)
    G = C // gs
    for r in sorted({0.0, 1.0 / G, 1.0}):
        fq.flexiq_set_ratio(hl, r)
        ref = oracle.forward_conv(ol, Xq, stride, pad, r)
        so = float(np.abs(oracle.dequant_f64(ref, x_scale, ol.w_scale, ol.bias)).max() / 127 * 0.9) or 1.0
        out = fq.flexiq_mixed_conv_implicit(hl, Xd, stride, pad, acc=True, y=True, q=True, out_scale=so)
        torch.cuda.synchronize()
        assert (out["acc"].cpu().numpy() == ref).all(), r
        check_y(out["y"].cpu().numpy(), ref, ol)
        check_q(out["q"].cpu().numpy(), ref, ol, so)
        assert (out["q"].cpu().numpy() == requant_fp32_sequence(ref, ol, so)).all()


def test_conv_all_tiles(env):
    torch, oracle, fq, dev = env
    case = workloads.make_conv("conv_tiles", 7, 99, 3, 10, 10, 64, 80, 3, 3, 1, 1, 32)
    ol, hl, x_scale = both_layers(case)
    Xq = np.ascontiguousarray(oracle.quantize(case.X, x_scale)[..., ol.perm])
    Xd = _dev(torch, Xq, dev)
    n = fq.debug_force_tile(-1)
    try:
        for t in range(n):
            fq.debug_force_tile(t)
            for r in (0.0, 0.5, 1.0):
                fq.flexiq_set_ratio(hl, r)
                ref = oracle.forward_conv(ol, Xq, 1, 1, r)
                for packed in (0, 1):
                    fq.debug_force_packed4(packed)
                    got = fq.flexiq_mixed_conv_implicit(hl, Xd, 1, 1, acc=True)["acc"].cpu().numpy()
                    assert (got == ref).all(), (t, r, packed)
                # int8 as the only output (NHWC in, NHWC out)
                so = float(np.abs(oracle.dequant_f64(ref, x_scale, ol.w_scale, ol.bias)).max() / 127 * 0.9) or 1.0
                fq.debug_force_packed4(0)
                q = fq.flexiq_mixed_conv_implicit(hl, Xd, 1, 1, q=True, out_scale=so)["q"].cpu().numpy()
                check_q(q, ref, ol, so)
                assert (q == requant_fp32_sequence(ref, ol, so)).all(), (t, r)
    finally:
        fq.debug_force_tile(-1)
        fq.debug_force_packed4(-1)


def test_conv_blocks_walk_several_tiles(env):
    # the convolution form with few blocks and many output tiles (tile rows that straddle images, ragged last
    # tile), every tile shape, compared in full with the oracle
    torch, oracle, fq, dev = env
    case = workloads.make_conv("conv_walk", 7, 123, 5, 12, 12, 64, 136, 3, 3, 1, 1, 32)
    ol, hl, x_scale = both_layers(case)
    Xq = np.ascontiguousarray(oracle.quantize(case.X, x_scale)[..., ol.perm])
    Xd = _dev(torch, Xq, dev)
    refs = {r: oracle.forward_conv(ol, Xq, 1, 1, r) for r in (0.0, 0.5, 1.0)}
    n = fq.debug_force_tile(-1)
    try:
        for t in range(n):
            fq.debug_force_tile(t)
            for nb in (1, 3, 7):
                fq.debug_max_blocks(nb)
                for r, ref in refs.items():
                    fq.flexiq_set_ratio(hl, r)
                    got = fq.flexiq_mixed_conv_implicit(hl, Xd, 1, 1, acc=True)["acc"].cpu().numpy()
                    assert (got == ref).all(), (t, nb, r)
    finally:
        fq.debug_force_tile(-1)
        fq.debug_max_blocks(0)


def test_conv_producer_lowers_and_scans_for_consumer(env):
    # the fused producer (Section 5 steps 1-2, Section 4.1) with a convolution as the producing layer: its NHWC int8
    # output, in the consumer's stored channel order, lowered for the consumer (lower_for) or scanned for the
    # consumer's run-time positions (scan_for); the consumer is a 1x1 convolution over the same pixels
    torch, oracle, fq, dev = env
    helpers = __import__("helpers")
    c1 = workloads.make_conv("cprod", 7, 131, 3, 9, 9, 64, 96, 3, 3, 1, 1, 32)
    xs1, am1 = helpers.calib(c1)
    o1 = oracle.prepare_layer(c1.W, am1, xs1, 32, bias=c1.bias)
    X1 = np.ascontiguousarray(oracle.quantize(c1.X, xs1)[..., o1.perm])
    acc1 = oracle.forward_conv(o1, X1, 1, 1, 0.5)
    s_mid = float(np.abs(oracle.dequant_f64(acc1, xs1, o1.w_scale, o1.bias)).max() / 127.0)
    q1 = requant_fp32_sequence(acc1, o1, s_mid)          # [B][Ho][Wo][N1], original output-channel order
    check_q(q1, acc1, o1, s_mid)
    c2 = workloads.make_conv("ccons", 7, 132, 3, 9, 9, 96, 40, 1, 1, 1, 0, 32)
    am2 = np.abs(q1).reshape(-1, 96).max(0).astype(np.float32) * np.float32(s_mid) * np.float32(2.0)   # calibrated too wide
    o2 = oracle.prepare_layer(c2.W, am2, s_mid, 32, bias=c2.bias)
    h2 = fq.flexiq_quantize_pack(c2.W, am2, s_mid, 32, bias=c2.bias)
    h1 = fq.flexiq_quantize_pack(c1.W, am1, xs1, 32, bias=c1.bias, out_perm=o2.perm)
    X2 = np.ascontiguousarray(q1[..., o2.perm])
    fq.flexiq_set_ratio(h1, 0.5)
    X1d = _dev(torch, X1, dev)
    n_tiles = fq.debug_force_tile(-1)
    try:
        for r2 in (1.0, 1.0 / 3.0):
            k4 = fq.flexiq_set_ratio(h2, r2)
            G4 = k4 // 32
            sh = np.repeat(o2.a_shift.astype(np.int32), 32)
            want_low = X2.astype(np.int32).copy()
            want_low[..., :k4] = np.clip(want_low[..., :k4] >> sh[:k4], -8, 7) << sh[:k4]
            dyn = oracle.dynamic_act_shifts(X2, 32, G4, o2.a_shift)
            for t in range(n_tiles):
                fq.debug_force_tile(t)
                fq.flexiq_static_positions(h2)
                low = fq.flexiq_mixed_conv_implicit(h1, X1d, 1, 1, q=True, out_scale=s_mid, lower_for=h2)["q"]
                assert (low.cpu().numpy().astype(np.int32) == want_low).all(), (t, r2)
                mid = fq.flexiq_mixed_conv_implicit(h1, X1d, 1, 1, q=True, out_scale=s_mid, scan_for=h2)["q"]
                assert (mid.cpu().numpy() == X2).all(), (t, r2)
                assert (fq.flexiq_layer_positions(h2) == dyn).all(), (t, r2)
            fq.debug_force_tile(-1)
            # the consumer on the lowered tensor (static positions) and on the scanned one (run-time positions)
            fq.flexiq_static_positions(h2)
            fq.flexiq_input_prelowered(h2, True)
            got = fq.flexiq_mixed_conv_implicit(h2, low, 1, 0, acc=True)["acc"].cpu().numpy()
            fq.flexiq_input_prelowered(h2, False)
            assert (got == oracle.forward_conv(o2, X2, 1, 0, r2)).all(), r2
            fq.flexiq_mixed_conv_implicit(h1, X1d, 1, 1, q=True, out_scale=s_mid, scan_for=h2)
            got = fq.flexiq_mixed_conv_implicit(h2, mid, 1, 0, acc=True)["acc"].cpu().numpy()
            assert (got == oracle.mixed_conv(X2, o2.Wq, 1, 0, 32, G4, dyn, o2.w_shift)).all(), r2
    finally:
        fq.debug_force_tile(-1)
        fq.flexiq_static_positions(h2)
    # a producer whose output order is not the consumer's stored order is refused
    h1_plain = fq.flexiq_quantize_pack(c1.W, am1, xs1, 32, bias=c1.bias)
    assert not (o2.perm == np.arange(96)).all()
    with pytest.raises(fq.FlexiqError):
        fq.flexiq_mixed_conv_implicit(h1_plain, X1d, 1, 1, q=True, out_scale=s_mid, lower_for=h2)
    with pytest.raises(fq.FlexiqError):
        fq.flexiq_mixed_conv_implicit(h1_plain, X1d, 1, 1, q=True, out_scale=s_mid, scan_for=h2)


def test_launch_limits_are_refused_without_a_launch(env):
    # include/flexiq.h, limits of the run-time entry points: checked on the host, nothing is launched
    torch, oracle, fq, dev = env
    import ctypes as C
    lib = fq.load()
    case = workloads.make_conv("limits", 7, 140, 1, 4, 4, 32, 16, 3, 3, 1, 1, 32)
    ol, hl, x_scale = both_layers(case)
    x = torch.zeros(64, dtype=torch.int8, device=dev)
    out_buf = torch.zeros(64, dtype=torch.int32, device=dev)
    o = fq.binding._Out(out_buf.data_ptr(), None, None, 1.0, None, None)
    # the 2 GiB activation window of the convolution form: H * W * C * (320 / (Ho * Wo) + 2) >= 2^31
    assert lib.flexiq_mixed_conv_implicit(hl._h, x.data_ptr(), 1, 8192, 8192, 1, 1, C.byref(o), None) == -1
    assert lib.flexiq_mixed_conv_implicit(hl._h, x.data_ptr(), 1, 4, 4, 0, 1, C.byref(o), None) == -1     # stride 0
    assert lib.flexiq_mixed_conv_implicit(hl._h, x.data_ptr(), 1, 1, 1, 1, 0, C.byref(o), None) == -1     # filter larger than image
    assert lib.flexiq_mixed_gemm(hl._h, x.data_ptr(), 4, C.byref(o), None) == -1                          # not a linear layer
    lin = both_layers(workloads.make_linear("limits_lin", 8, 141, 4, 64, 16, 32))[1]
    assert lib.flexiq_mixed_gemm(lin._h, x.data_ptr(), (1 << 31) - 512, C.byref(o), None) == -1           # 32-bit row indices
    assert lib.flexiq_mixed_gemm(lin._h, x.data_ptr() + 4, 4, C.byref(o), None) == -2                     # alignment
    torch.cuda.synchronize()
    assert int(out_buf.abs().sum().item()) == 0                                                          # nothing ran


def test_determinism(env):
    # integer accumulation is order independent: two runs must be identical (a mismatch = race / stray read)
    torch, oracle, fq, dev = env
    case = workloads.make_linear("det", 8, 5, 1000, 256, 512, 32, outlier_frac=0.02)
    ol, hl, x_scale = both_layers(case)
    Xd = _dev(torch, oracle.quantize(case.X, x_scale)[:, ol.perm], dev)
    fq.flexiq_set_ratio(hl, 0.5)
    a = fq.flexiq_mixed_gemm(hl, Xd, acc=True)["acc"].clone()
    for _ in range(3):
        b = fq.flexiq_mixed_gemm(hl, Xd, acc=True)["acc"]
        assert torch.equal(a, b)


def test_zz_requant_window_statistics(env):
    # how many of the int8 codes compared above needed the tie window of the float64 definition
    used, total = _Q_WINDOW
    print("requantised codes compared with the float64 definition: %d, inside the tie window and on the other "
          "neighbour: %d (%.4f %%)" % (total, used, 100.0 * used / max(total, 1)))
    assert total == 0 or used <= 1e-3 * total
