"""Pins for the oracle's mixed-precision convolution: it must equal the (separately pinned) mixed
GEMM on an explicit im2col matrix built here, a 1x1 conv must be the GEMM itself, and a tiny case
is checked against a Python-integer loop nest."""
import numpy as np
import pytest


def _im2col(X, R, S, stride, pad):
    B, H, Wd, C = X.shape
    Ho = (H + 2 * pad - R) // stride + 1
    Wo = (Wd + 2 * pad - S) // stride + 1
    Xp = np.zeros((B, H + 2 * pad, Wd + 2 * pad, C), X.dtype)
    Xp[:, pad:pad + H, pad:pad + Wd] = X
    cols = np.empty((B, Ho, Wo, R, S, C), X.dtype)
    for dy in range(R):
        for dx in range(S):
            cols[:, :, :, dy, dx] = Xp[:, dy:dy + stride * Ho:stride, dx:dx + stride * Wo:stride]
    return cols.reshape(B * Ho * Wo, R * S * C), Ho, Wo


@pytest.mark.parametrize("R,stride,pad,H", [(1, 1, 0, 6), (3, 1, 1, 7), (3, 2, 1, 8), (1, 2, 0, 8), (3, 1, 0, 5)])
def test_conv_equals_gemm_on_im2col(oracle, R, stride, pad, H):
    rng = np.random.default_rng(21 + R + stride)
    B, C, N, gs = 2, 64, 10, 32
    G = C // gs
    X = rng.integers(-128, 128, size=(B, H, H, C)).astype(np.int8)
    W = rng.integers(-128, 128, size=(N, R, R, C)).astype(np.int8)
    a = rng.integers(0, 5, size=G).astype(np.uint8)
    w = rng.integers(0, 5, size=(N, G)).astype(np.uint8)
    cols, Ho, Wo = _im2col(X, R, R, stride, pad)
    T = R * R
    # in the im2col matrix the reduction index is (tap, channel): tap t's group g is GEMM group t*G+g
    a_g = np.tile(a, T)
    w_g = np.tile(w, (1, T))
    for G4 in range(G + 1):
        got = oracle.mixed_conv(X, W, stride, pad, gs, G4, a, w)
        assert got.shape == (B, Ho, Wo, N)
        # GEMM with "first G4 groups of every tap lowered": reorder the columns so those come first
        low = np.concatenate([t * C + np.arange(G4 * gs) for t in range(T)]).astype(int)
        high = np.concatenate([t * C + np.arange(G4 * gs, C) for t in range(T)]).astype(int)
        order = np.concatenate([low, high])
        gorder = order[::gs] // gs
        ref = oracle.mixed_gemm(cols[:, order], W.reshape(N, -1)[:, order], gs, G4 * T, a_g[gorder], w_g[:, gorder])
        assert (got.reshape(-1, N) == ref).all()


def test_conv_1x1_is_gemm(oracle):
    rng = np.random.default_rng(31)
    X = rng.integers(-128, 128, size=(3, 4, 5, 96)).astype(np.int8)
    W = rng.integers(-128, 128, size=(7, 1, 1, 96)).astype(np.int8)
    a = rng.integers(0, 5, size=3).astype(np.uint8)
    w = rng.integers(0, 5, size=(7, 3)).astype(np.uint8)
    for G4 in range(4):
        got = oracle.mixed_conv(X, W, 1, 0, 32, G4, a, w)
        ref = oracle.mixed_gemm(X.reshape(-1, 96), W.reshape(7, 96), 32, G4, a, w)
        assert (got.reshape(-1, 7) == ref).all()


def test_conv_brute_force_tiny(oracle):
    rng = np.random.default_rng(32)
    B, H, Wd, C, N, R, S, stride, pad, gs = 1, 4, 3, 64, 3, 3, 3, 1, 1, 32
    X = rng.integers(-40, 41, size=(B, H, Wd, C)).astype(np.int8)
    W = rng.integers(-128, 128, size=(N, R, S, C)).astype(np.int8)
    a = np.array([1, 2], np.uint8)
    w = rng.integers(0, 5, size=(N, 2)).astype(np.uint8)
    G4 = 1
    got = oracle.mixed_conv(X, W, stride, pad, gs, G4, a, w)
    for ho in range(H):
        for wo in range(Wd):
            for n in range(N):
                tot = 0
                for dy in range(R):
                    for dx in range(S):
                        hi, wi = ho + dy - pad, wo + dx - pad
                        if not (0 <= hi < H and 0 <= wi < Wd):
                            continue
                        for c in range(C):
                            x, ww = int(X[0, hi, wi, c]), int(W[n, dy, dx, c])
                            g = c // gs
                            if g < G4:
                                sa, sw = int(a[g]), int(w[n, g])
                                tot += (max(-8, min(7, x >> sa)) * max(-8, min(7, ww >> sw))) << (sa + sw)
                            else:
                                tot += x * ww
                assert got[0, ho, wo, n] == tot
