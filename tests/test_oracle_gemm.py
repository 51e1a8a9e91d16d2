"""Pins for the oracle's mixed 4-/8-bit GEMM (paper Sections 2.3 and 7).

None of these re-types the oracle's formula: they use numpy int64 matmul on the special cases where
the method reduces to a plain GEMM, Python-integer brute force on tiny shapes, and invariants that a
dropped term, wrong sign, wrong index or transposed operand would break."""
import numpy as np
import pytest

import workloads


def _rand_case(rng, M, N, K, gs, spread=None):
    """int8 operands whose channel ranges grow along K (like a sorted layer) + fitted positions."""
    G = K // gs
    if spread is None:
        spread = np.minimum(127, 3 + 4 * np.arange(K) * 127 // (4 * K) + rng.integers(0, 6, K))
    X = np.stack([rng.integers(-s, s + 1, size=M) for s in spread], axis=1).astype(np.int8)
    W = np.stack([rng.integers(-max(1, s // 2), max(1, s // 2) + 1, size=N) for s in spread], axis=1).astype(np.int8)
    return X, W, G


def _fitted_shifts(oracle, X, W, gs):
    M, K = X.shape
    N = W.shape[0]
    G = K // gs
    a = np.array([oracle.shift_for_range(int(X[:, g * gs:(g + 1) * gs].min()), int(X[:, g * gs:(g + 1) * gs].max()))
                  for g in range(G)], np.uint8)
    w = oracle.weight_shifts(W.reshape(N, 1, K), gs)
    return a, w


def _brute(X, W, gs, G4, a_shift, w_shift):
    """Triple loop with Python integers, written from the problem statement."""
    M, K = X.shape
    N = W.shape[0]
    out = [[0] * N for _ in range(M)]
    for m in range(M):
        for n in range(N):
            tot = 0
            for k in range(K):
                g = k // gs
                x, w = int(X[m, k]), int(W[n, k])
                if g < G4:
                    sa, sw = int(a_shift[g]), int(w_shift[n, g])
                    x4 = max(-8, min(7, x >> sa))
                    w4 = max(-8, min(7, w >> sw))
                    tot += (x4 * w4) << (sa + sw)
                else:
                    tot += x * w
            out[m][n] = tot
    return np.array(out, np.int64)


def test_ratio_zero_is_plain_int8_gemm(oracle):
    # Table 2 caption: a 0 % 4-bit ratio is the 8-bit model
    rng = np.random.default_rng(11)
    X = rng.integers(-128, 128, size=(37, 96)).astype(np.int8)
    W = rng.integers(-128, 128, size=(29, 96)).astype(np.int8)
    a = rng.integers(0, 5, size=3).astype(np.uint8)
    w = rng.integers(0, 5, size=(29, 3)).astype(np.uint8)
    acc = oracle.mixed_gemm(X, W, 32, 0, a, w)
    assert (acc == X.astype(np.int64) @ W.astype(np.int64).T).all()


def test_ratio_one_naive_top_four_bits_is_plain_int4_gemm(oracle):
    # all positions forced to 4: both operands keep their top four bits (the paper's "naive
    # conversion"), and the method is a 4-bit GEMM scaled by 2^8
    rng = np.random.default_rng(12)
    X = rng.integers(-128, 128, size=(21, 128)).astype(np.int8)
    W = rng.integers(-128, 128, size=(17, 128)).astype(np.int8)
    G = 4
    a = np.full(G, 4, np.uint8)
    w = np.full((17, G), 4, np.uint8)
    acc = oracle.mixed_gemm(X, W, 32, G, a, w)
    x4 = np.floor_divide(X.astype(np.int64), 16)
    w4 = np.floor_divide(W.astype(np.int64), 16)
    assert (acc == 256 * (x4 @ w4.T)).all()


def test_full_four_bit_gemm_with_uniform_positions(oracle):
    # r = 1 with one common position pair: Sum L(x,sa) L(w,sw) 2^(sa+sw) = 2^(sa+sw) (L(X) @ L(W)^T)
    rng = np.random.default_rng(13)
    X = rng.integers(-128, 128, size=(9, 64)).astype(np.int8)
    W = rng.integers(-128, 128, size=(7, 64)).astype(np.int8)
    for sa in range(5):
        for sw in range(5):
            a = np.full(2, sa, np.uint8)
            w = np.full((7, 2), sw, np.uint8)
            acc = oracle.mixed_gemm(X, W, 32, 2, a, w)
            lx = np.clip(np.floor_divide(X.astype(np.int64), 2 ** sa), -8, 7)
            lw = np.clip(np.floor_divide(W.astype(np.int64), 2 ** sw), -8, 7)
            assert (acc == (lx @ lw.T) * 2 ** (sa + sw)).all()


def test_lossless_when_low_groups_fit_four_bits(oracle):
    # if every value of the 4-bit groups already lies in [-8, 7], positions are 0 and any ratio
    # gives the 8-bit result
    rng = np.random.default_rng(14)
    K, gs = 128, 32
    X = rng.integers(-128, 128, size=(13, K)).astype(np.int8)
    W = rng.integers(-128, 128, size=(11, K)).astype(np.int8)
    X[:, :96] = rng.integers(-8, 8, size=(13, 96))
    W[:, :96] = rng.integers(-8, 8, size=(11, 96))
    a, w = _fitted_shifts(oracle, X, W, gs)
    assert (a[:3] == 0).all() and (w[:, :3] == 0).all()
    ref = X.astype(np.int64) @ W.astype(np.int64).T
    for G4 in range(4):
        assert (oracle.mixed_gemm(X, W, gs, G4, a, w) == ref).all()


@pytest.mark.parametrize("gs", [32, 64])
def test_brute_force_tiny(oracle, gs):
    rng = np.random.default_rng(15 + gs)
    K = 2 * gs
    X, W, G = _rand_case(rng, 6, 5, K, gs)
    a, w = _fitted_shifts(oracle, X, W, gs)
    # also exercise saturation: positions one too small for some groups
    a2 = np.maximum(a.astype(int) - 1, 0).astype(np.uint8)
    w2 = np.maximum(w.astype(int) - 1, 0).astype(np.uint8)
    for G4 in range(G + 1):
        for (aa, ww) in ((a, w), (a2, w2)):
            got = oracle.mixed_gemm(X, W, gs, G4, aa, ww)
            assert (got == _brute(X, W, gs, G4, aa, ww)).all()


def test_group_partial_fits_sixteen_bits(oracle):
    # Section 7 (NPU): the 4-bit products of a 64-channel group are summed into a 16-bit value.
    # int4 x int4 products lie in [-56, 64], so |partial| <= 64 * gs
    rng = np.random.default_rng(16)
    for gs in (32, 64):
        X = rng.integers(-128, 128, size=(40, 4 * gs)).astype(np.int8)
        W = rng.integers(-128, 128, size=(30, 4 * gs)).astype(np.int8)
        X[0, :] = -128
        W[0, :] = -128
        a = rng.integers(0, 5, size=4).astype(np.uint8)
        w = rng.integers(0, 5, size=(30, 4)).astype(np.uint8)
        _, gp = oracle.mixed_gemm(X, W, gs, 4, a, w, return_partial=True)
        assert gp <= 64 * gs <= 32767
        assert gp == 64 * gs  # the all -8 x -8 row reaches the bound


def test_permutation_invariance(oracle):
    rng = np.random.default_rng(17)
    gs, G = 32, 6
    K = gs * G
    X, W, _ = _rand_case(rng, 10, 9, K, gs)
    a, w = _fitted_shifts(oracle, X, W, gs)
    N = W.shape[0]
    # (i) at r = 0 any common permutation of the input channels leaves the result unchanged
    p = rng.permutation(K)
    assert (oracle.mixed_gemm(X, W, gs, 0, a, w) == oracle.mixed_gemm(X[:, p], W[:, p], gs, 0, a, w)).all()
    G4 = 4
    ref = oracle.mixed_gemm(X, W, gs, G4, a, w)
    # (ii-a) permutation inside each group
    p = np.concatenate([g * gs + rng.permutation(gs) for g in range(G)])
    assert (oracle.mixed_gemm(X[:, p], W[:, p], gs, G4, a, w) == ref).all()
    # (ii-b) whole groups reordered within the 4-bit prefix (positions travel with them) and within the 8-bit suffix
    go = np.concatenate([rng.permutation(G4), G4 + rng.permutation(G - G4)])
    p = np.concatenate([g * gs + np.arange(gs) for g in go])
    assert (oracle.mixed_gemm(X[:, p], W[:, p], gs, G4, a[go], w[:, go]) == ref).all()
    # (ii-c) any permutation of single channels inside the 8-bit suffix
    p = np.concatenate([np.arange(G4 * gs), G4 * gs + rng.permutation(K - G4 * gs)])
    assert (oracle.mixed_gemm(X[:, p], W[:, p], gs, G4, a, w) == ref).all()
    # a transposed-operand or wrong-index bug: output rows follow X rows, columns follow W rows
    assert (oracle.mixed_gemm(X[::-1], W, gs, G4, a, w) == ref[::-1]).all()
    assert (oracle.mixed_gemm(X, W[::-1], gs, G4, a, w[::-1]) == ref[:, ::-1]).all()


def test_additivity_over_groups_and_error_bound(oracle):
    # acc(G4) - acc(0) is the sum over the 4-bit groups of (lowered - exact) group partials, and
    # without saturation |error| <= sum |x|(2^sw - 1) + |w|(2^sa - 1) + (2^sa - 1)(2^sw - 1)
    rng = np.random.default_rng(18)
    gs, G = 32, 5
    K = gs * G
    X, W, _ = _rand_case(rng, 12, 8, K, gs)
    a, w = _fitted_shifts(oracle, X, W, gs)
    X64, W64 = X.astype(np.int64), W.astype(np.int64)
    acc0 = oracle.mixed_gemm(X, W, gs, 0, a, w).astype(np.int64)
    prev = acc0
    for G4 in range(1, G + 1):
        cur = oracle.mixed_gemm(X, W, gs, G4, a, w).astype(np.int64)
        g = G4 - 1
        sl = slice(g * gs, (g + 1) * gs)
        exact = X64[:, sl] @ W64[:, sl].T
        only_g = oracle.mixed_gemm(X[:, sl], W[:, sl], gs, 1, a[g:g + 1], w[:, g:g + 1]).astype(np.int64)
        assert (cur - prev == only_g - exact).all()
        ea = 2 ** a[g].astype(np.int64) - 1
        ew = 2 ** w[:, g].astype(np.int64) - 1              # [N]
        bound = (np.abs(X64[:, sl]).sum(1)[:, None] * ew[None, :] + np.abs(W64[:, sl]).sum(1)[None, :] * ea
                 + gs * ea * ew[None, :])
        assert (np.abs(only_g - exact) <= bound).all()
        prev = cur


def test_config0_reductions(oracle):
    # the benchmark's small configuration through the whole offline chain
    case = workloads.config0()
    x_scale = oracle.absmax_scale(case.Xcal)
    layer = oracle.prepare_layer(case.W, np.abs(case.Xcal).max(0), x_scale, case.group_size)
    Xq = oracle.quantize(case.X, x_scale)[:, layer.perm]
    Wq = layer.Wq.reshape(layer.N, layer.C)
    plain = Xq.astype(np.int64) @ Wq.astype(np.int64).T
    assert (oracle.forward_gemm(layer, Xq, 0.0) == plain).all()
    errs = []
    for r in (0.25, 0.5, 0.75, 1.0):
        acc = oracle.forward_gemm(layer, Xq, r)
        errs.append(np.linalg.norm(acc - plain) / np.linalg.norm(plain))
    # lowering the small-range prefix perturbs the layer output only slightly (Fig. 1b / Fig. 14)
    assert 0 < errs[0] < 0.05 and errs == sorted(errs)
    # tiny corner through brute force at r = 0.5
    G4 = oracle.groups_for_ratio(0.5, layer.G)
    got = oracle.mixed_gemm(Xq[:4], Wq[:6], 32, G4, layer.a_shift, layer.w_shift[:6])
    assert (got == _brute(Xq[:4], Wq[:6], 32, G4, layer.a_shift, layer.w_shift[:6])).all()
    # sorted order: the small-range channels come first, so the lowered prefix has small positions
    assert layer.a_shift[0] <= layer.a_shift[-1]


def test_groups_for_ratio(oracle):
    # the count of low-bit groups is the smallest whose share reaches the target (Section 2.3)
    for G in (1, 2, 3, 8, 16, 24, 64, 96):
        for r in (0.0, 0.25, 0.5, 0.75, 1.0, 0.1, 0.33, 0.999):
            g4 = oracle.groups_for_ratio(r, G)
            assert 0 <= g4 <= G
            assert g4 / G >= r - 1e-9
            assert g4 == 0 or (g4 - 1) / G < r
    assert oracle.groups_for_ratio(0.25, 2) == 1 and oracle.groups_for_ratio(0.75, 2) == 2
    assert oracle.groups_for_ratio(0.5, 8) == 4
