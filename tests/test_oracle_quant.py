"""Pins for the oracle's quantiser (Eq. 1), channel scores and order (Sections 4.2, 5), extraction
positions of a prepared layer, and the dequant / requant epilogue."""
import numpy as np

import workloads


def test_quantize_textbook(oracle):
    # Eq. 1: clip(round(x / S)); ties to even; symmetric clip
    S = 0.5
    x = np.array([0.0, 0.24, 0.25, 0.26, 0.75, 1.25, -0.25, -0.75, 63.4, 63.5, 100.0, -100.0], np.float32)
    want = np.array([0, 0, 0, 1, 2, 2, 0, -2, 127, 127, 127, -127], np.int8)
    assert (oracle.quantize(x, S) == want).all()
    rng = np.random.default_rng(41)
    x = rng.standard_normal(5000).astype(np.float32) * 3
    S = oracle.absmax_scale(x)
    assert S == np.float32(np.abs(x).max()) / np.float32(127)
    q = oracle.quantize(x, S)
    ref = np.clip(np.rint(x / np.float32(S)), -127, 127)
    assert (q == ref).all()
    assert np.abs(q).max() == 127
    assert np.abs(q.astype(np.float64) * S - x).max() <= S / 2 * (1 + 1e-6)
    # the paper's worked example: step 0.0330 maps 0.957 -> 29 and -0.297 -> -9
    assert (oracle.quantize(np.array([0.957, -0.297], np.float32), 0.0330) == np.array([29, -9])).all()


def test_quantize_rows_is_per_output_channel(oracle):
    rng = np.random.default_rng(42)
    W = rng.standard_normal((6, 50)).astype(np.float32) * np.array([1, 10, 0.1, 3, 0.01, 100], np.float32)[:, None]
    q, s = oracle.quantize_rows(W)
    for n in range(6):
        assert s[n] == oracle.absmax_scale(W[n])
        assert (q[n] == oracle.quantize(W[n], s[n])).all()
        assert np.abs(q[n]).max() == 127
    z, sz = oracle.quantize_rows(np.zeros((2, 8), np.float32))
    assert (z == 0).all() and (sz == 1).all()


def test_scores_and_order(oracle):
    # score = (largest weight magnitude of the channel over outputs and taps) x (activation range)
    rng = np.random.default_rng(43)
    Wq = rng.integers(-127, 128, size=(5, 3, 12)).astype(np.int8)
    ar = rng.integers(0, 128, size=12).astype(np.int32)
    sc = oracle.channel_scores(Wq, ar)
    assert (sc == np.abs(Wq.astype(np.int64)).max(axis=(0, 1)) * ar).all()
    # ascending, stable
    sc2 = np.array([5, 1, 5, 0, 1, 9, 0], np.int64)
    assert (oracle.order_by_score(sc2) == np.argsort(sc2, kind="stable")).all()
    assert list(oracle.order_by_score(sc2)) == [3, 6, 1, 4, 0, 2, 5]
    big = rng.integers(0, 50, size=3000).astype(np.int64)
    assert (oracle.order_by_score(big) == np.argsort(big, kind="stable")).all()


def test_prepared_layer_properties(oracle):
    case = workloads.config0()
    x_scale = oracle.absmax_scale(case.Xcal)
    amax = np.abs(case.Xcal).max(0)
    layer = oracle.prepare_layer(case.W, amax, x_scale, 32)
    C, gs, G = layer.C, 32, layer.G
    assert sorted(layer.perm.tolist()) == list(range(C))
    # the stored order is ascending in score, hence nested: the 25 % prefix is inside the 50 % prefix
    Wq_nat, _ = oracle.quantize_rows(case.W)
    rq = np.clip(np.rint(amax / np.float32(x_scale)), 0, 127).astype(np.int64)
    score = np.abs(Wq_nat.astype(np.int64)).max(0) * rq
    assert (np.diff(score[layer.perm]) >= 0).all()
    assert (layer.Wq.reshape(layer.N, C) == Wq_nat[:, layer.perm]).all()
    # every position fits its group: lowering the calibration data and the weights never saturates
    Xc = oracle.quantize(case.Xcal, x_scale)[:, layer.perm].astype(np.int64)
    for g in range(G):
        s = int(layer.a_shift[g])
        blk = Xc[:, g * gs:(g + 1) * gs]
        assert -8 * 2 ** s <= blk.min() and blk.max() <= 8 * 2 ** s - 1
        assert s == 0 or max(abs(int(blk.min())), int(blk.max())) > 8 * 2 ** (s - 1) - 1   # and is minimal
        for n in range(layer.N):
            sw = int(layer.w_shift[n, g])
            wb = layer.Wq.reshape(layer.N, C)[n, g * gs:(g + 1) * gs].astype(np.int64)
            assert -8 * 2 ** sw <= wb.min() and wb.max() <= 8 * 2 ** sw - 1
            assert sw == 0 or not (-8 * 2 ** (sw - 1) <= wb.min() and wb.max() <= 8 * 2 ** (sw - 1) - 1)
    # explicit perm override is honoured
    ident = np.arange(C, dtype=np.int32)
    l2 = oracle.prepare_layer(case.W, amax, x_scale, 32, perm=ident)
    assert (l2.Wq.reshape(layer.N, C) == Wq_nat).all()


def test_library_perm_equals_pre_permuted(oracle):
    # a layer prepared on unsorted tensors, fed activations gathered by its perm, equals the layer
    # prepared on tensors that were permuted beforehand with the identity order
    case = workloads.config0()
    x_scale = oracle.absmax_scale(case.Xcal)
    amax = np.abs(case.Xcal).max(0)
    layer = oracle.prepare_layer(case.W, amax, x_scale, 32)
    p = layer.perm
    l2 = oracle.prepare_layer(case.W[:, p], amax[p], x_scale, 32, perm=np.arange(layer.C, dtype=np.int32))
    Xq = oracle.quantize(case.X, x_scale)
    for r in (0.0, 0.5, 1.0):
        assert (oracle.forward_gemm(layer, Xq[:, p], r) == oracle.forward_gemm(l2, Xq[:, p], r)).all()


def test_dequant_and_requant(oracle):
    rng = np.random.default_rng(44)
    acc = rng.integers(-2 ** 26, 2 ** 26, size=(9, 7)).astype(np.int32)
    ws = (rng.random(7).astype(np.float32) + 0.5) * 1e-3
    bias = rng.standard_normal(7).astype(np.float32)
    xs = np.float32(0.031)
    y = oracle.dequant_f64(acc, xs, ws, bias)
    ref = acc.astype(np.float64) * np.float64(xs) * ws.astype(np.float64)[None, :] + bias.astype(np.float64)[None, :]
    assert np.allclose(y, ref, rtol=1e-15, atol=0)
    assert (oracle.dequant_f64(acc, xs, ws) == acc.astype(np.float64) * np.float64(xs) * ws.astype(np.float64)).all()
    # requantised code = clip(round_half_even(y / S_out), -128, 127), checked against numpy in float64
    so = np.float32(np.abs(y).max() / 127 * 0.8)          # 0.8: some outputs clip
    q, t = oracle.requant_i8(acc, xs, ws, so, bias, return_arg=True)
    assert np.allclose(t, ref / np.float64(so), rtol=1e-15, atol=0)
    assert (q == np.clip(np.rint(ref / np.float64(so)), -128, 127)).all()
    assert q.min() == -128 or q.max() == 127


def test_requant_ties_and_clip_edges(oracle):
    # Hand-placed arguments: S_x = 1, S_w = 0.5, S_out = 1 make t = acc / 2 + bias exact, so every expected code
    # below is Eq. 1 worked by hand: ties go to the even code, the range is [-128, 127].
    acc = np.array([[1, 3, 5, -1, -3, -5, 0, 2, 254, 255, 256, 257, 1000, -255, -256, -257, -258, -259, -1000, 7]],
                   np.int32).T.copy()                    # one output channel, 20 rows
    ws = np.array([0.5], np.float32)
    q, t = oracle.requant_i8(acc, 1.0, ws, 1.0, None, return_arg=True)
    want_t = [0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 0.0, 1.0, 127.0, 127.5, 128.0, 128.5, 500.0, -127.5, -128.0, -128.5,
              -129.0, -129.5, -500.0, 3.5]
    want_q = [0, 2, 2, 0, -2, -2, 0, 1, 127, 127, 127, 127, 127, -128, -128, -128, -128, -128, -128, 4]
    assert t[:, 0].tolist() == want_t
    assert q[:, 0].tolist() == want_q
    # a bias moves the tie: t = acc / 2 + 0.25 is never a tie, t = acc / 2 + 0.5 turns even acc into ties
    q2 = oracle.requant_i8(acc[:8], 1.0, ws, 1.0, np.array([0.25], np.float32))
    assert q2[:, 0].tolist() == [1, 2, 3, 0, -1, -2, 0, 1]
    q3 = oracle.requant_i8(np.array([[0], [2], [4], [-2], [-4]], np.int32), 1.0, ws, 1.0, np.array([0.5], np.float32))
    assert q3[:, 0].tolist() == [0, 2, 2, 0, -2]
    # the output scale divides: S_out = 0.25 -> t = 4 * (acc / 2) ; per-channel weight scales apply per column
    q4 = oracle.requant_i8(np.array([[1, 1], [-3, -3]], np.int32), 1.0, np.array([0.5, 0.0625], np.float32), 0.25)
    assert q4.tolist() == [[2, 0], [-6, -1]]    # columns: 4 * 0.5 = 2, 4 * 0.0625 = 0.25 -> 0; -6, -0.75 -> -1
