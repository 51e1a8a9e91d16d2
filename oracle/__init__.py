"""FlexiQ CPU oracle -- TEST INFRASTRUCTURE ONLY.

ctypes access to ``flexiq_oracle.c`` (plain C, 64-bit integer sums) plus the few
lines of glue that chain its functions into "prepare a layer" and "run a layer".
Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package; the HIP library never does, and this
package never imports the HIP library.

Nothing here computes: every arithmetic step is a call into the C file; the
Python code only allocates numpy arrays, permutes channel axes and passes
pointers.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "flexiq_oracle.c")
_LIB = os.path.join(_HERE, "libflexiq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over output rows, no FP contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct)) if a is not None else None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        i8p, u8p, i32p, i64p, f32p, f64p = (C.POINTER(t) for t in
                                            (C.c_int8, C.c_uint8, C.c_int32, C.c_int64, C.c_float, C.c_double))
        L.fq_o_absmax_scale.restype = C.c_float
        L.fq_o_absmax_scale.argtypes = [f32p, C.c_int64]
        L.fq_o_quantize.restype = None
        L.fq_o_quantize.argtypes = [f32p, C.c_int64, C.c_float, C.c_int32, C.c_int32, i8p]
        L.fq_o_quantize_rows.restype = None
        L.fq_o_quantize_rows.argtypes = [f32p, C.c_int64, C.c_int64, f32p, i8p]
        L.fq_o_shift_for_range.restype = C.c_int32
        L.fq_o_shift_for_range.argtypes = [C.c_int32, C.c_int32]
        L.fq_o_shift_from_values.restype = C.c_int32
        L.fq_o_shift_from_values.argtypes = [i8p, C.c_int64, C.c_int64]
        L.fq_o_bitlower.restype = C.c_int32
        L.fq_o_bitlower.argtypes = [C.c_int32, C.c_int32, C.c_int32]
        L.fq_o_bitlower_pack.restype = None
        L.fq_o_bitlower_pack.argtypes = [i8p, u8p, C.c_int64, C.c_int32, C.c_int32, u8p, C.c_int32, C.c_int32]
        L.fq_o_channel_scores.restype = None
        L.fq_o_channel_scores.argtypes = [i8p, C.c_int64, C.c_int32, C.c_int32, i32p, i64p]
        L.fq_o_order_by_score.restype = None
        L.fq_o_order_by_score.argtypes = [i64p, C.c_int32, i32p]
        L.fq_o_range_code.restype = C.c_int32
        L.fq_o_range_code.argtypes = [C.c_float, C.c_float]
        L.fq_o_act_shifts.restype = None
        L.fq_o_act_shifts.argtypes = [i32p, C.c_int32, C.c_int32, u8p]
        L.fq_o_weight_shifts.restype = None
        L.fq_o_weight_shifts.argtypes = [i8p, C.c_int64, C.c_int32, C.c_int32, C.c_int32, u8p]
        L.fq_o_groups_for_ratio.restype = C.c_int32
        L.fq_o_groups_for_ratio.argtypes = [C.c_double, C.c_int32]
        L.fq_o_mixed_gemm.restype = C.c_int64
        L.fq_o_mixed_gemm.argtypes = [i8p, i8p, C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.c_int32, u8p, u8p,
                                      C.c_int32, i32p, i64p]
        L.fq_o_mixed_conv.restype = C.c_int64
        L.fq_o_mixed_conv.argtypes = [i8p, i8p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_int32,
                                      C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, u8p, u8p, C.c_int32,
                                      i32p]
        L.fq_o_dequant_f64.restype = None
        L.fq_o_dequant_f64.argtypes = [i32p, C.c_int64, C.c_int64, C.c_float, f32p, f32p, f64p]
        L.fq_o_requant_i8.restype = None
        L.fq_o_requant_i8.argtypes = [i32p, C.c_int64, C.c_int64, C.c_float, f32p, f32p, C.c_float, i8p, f64p]
        _lib = L
    return _lib


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


# ---- thin wrappers -----------------------------------------------------------------------------

def absmax_scale(x) -> float:
    x = _c(x, np.float32)
    return float(lib().fq_o_absmax_scale(_p(x, C.c_float), x.size))


def quantize(x, S: float, qmin: int = -127, qmax: int = 127) -> np.ndarray:
    x = _c(x, np.float32)
    q = np.empty(x.shape, np.int8)
    lib().fq_o_quantize(_p(x, C.c_float), x.size, np.float32(S), qmin, qmax, _p(q, C.c_int8))
    return q


def quantize_rows(W):
    W = _c(W, np.float32)
    N = W.shape[0]
    K = W.size // N
    scale = np.empty(N, np.float32)
    q = np.empty(W.shape, np.int8)
    lib().fq_o_quantize_rows(_p(W, C.c_float), N, K, _p(scale, C.c_float), _p(q, C.c_int8))
    return q, scale


def shift_for_range(vmin: int, vmax: int) -> int:
    return int(lib().fq_o_shift_for_range(int(vmin), int(vmax)))


def shift_from_values(v) -> int:
    v = _c(v, np.int8).ravel()
    return int(lib().fq_o_shift_from_values(_p(v, C.c_int8), v.size, 1))


def bitlower(q: int, s: int, mode: int = 0) -> int:
    return int(lib().fq_o_bitlower(int(q), int(s), int(mode)))


def bitlower_pack(src, group_size: int, shifts, per_row: bool, mode: int = 0) -> np.ndarray:
    src = _c(src, np.int8)
    rows, Cc = src.shape
    shifts = _c(shifts, np.uint8)
    dst = np.empty((rows, Cc // 2), np.uint8)
    lib().fq_o_bitlower_pack(_p(src, C.c_int8), _p(dst, C.c_uint8), rows, Cc, group_size, _p(shifts, C.c_uint8),
                             1 if per_row else 0, mode)
    return dst


def channel_scores(Wq_ntc, act_range_q) -> np.ndarray:
    Wq = _c(Wq_ntc, np.int8)
    N, T, Cc = Wq.shape
    ar = _c(act_range_q, np.int32)
    score = np.empty(Cc, np.int64)
    lib().fq_o_channel_scores(_p(Wq, C.c_int8), N, T, Cc, _p(ar, C.c_int32), _p(score, C.c_int64))
    return score


def order_by_score(score) -> np.ndarray:
    score = _c(score, np.int64)
    perm = np.empty(score.size, np.int32)
    lib().fq_o_order_by_score(_p(score, C.c_int64), score.size, _p(perm, C.c_int32))
    return perm


def range_codes(act_absmax, x_scale: float) -> np.ndarray:
    a = _c(act_absmax, np.float32)
    return np.array([lib().fq_o_range_code(np.float32(v), np.float32(x_scale)) for v in a], np.int32)


def act_shifts(range_q_perm, group_size: int) -> np.ndarray:
    rq = _c(range_q_perm, np.int32)
    out = np.empty(rq.size // group_size, np.uint8)
    lib().fq_o_act_shifts(_p(rq, C.c_int32), rq.size, group_size, _p(out, C.c_uint8))
    return out


def dynamic_act_shifts(Xq_perm, group_size: int, G4: int, a_shift_static) -> np.ndarray:
    """Activation positions found at run time (Section 4.1, dynamic option): for each of the first G4 groups the
    OR scan of shift_from_values over every value of the group in Xq_perm ([..., C], stored order); the other
    groups keep the calibrated position."""
    X = _c(Xq_perm, np.int8).reshape(-1, np.shape(Xq_perm)[-1])
    out = np.array(a_shift_static, np.uint8).copy()
    for g in range(G4):
        out[g] = shift_from_values(X[:, g * group_size:(g + 1) * group_size]) if X.shape[0] else 0
    return out


def weight_shifts(Wq_ntc, group_size: int) -> np.ndarray:
    Wq = _c(Wq_ntc, np.int8)
    N, T, Cc = Wq.shape
    out = np.empty((N, Cc // group_size), np.uint8)
    lib().fq_o_weight_shifts(_p(Wq, C.c_int8), N, T, Cc, group_size, _p(out, C.c_uint8))
    return out


def groups_for_ratio(r: float, G: int) -> int:
    return int(lib().fq_o_groups_for_ratio(float(r), int(G)))


def mixed_gemm(Xq, Wq, group_size: int, G4: int, a_shift, w_shift, mode: int = 0, return_partial=False):
    Xq = _c(Xq, np.int8)
    Wq = _c(Wq, np.int8)
    M, K = Xq.shape
    N = Wq.shape[0]
    assert Wq.shape[1] == K and K % group_size == 0
    a_shift = _c(a_shift, np.uint8)
    w_shift = _c(w_shift, np.uint8)
    assert a_shift.size == K // group_size and w_shift.size == N * (K // group_size)
    acc = np.empty((M, N), np.int32)
    gp = C.c_int64(0)
    ovf = lib().fq_o_mixed_gemm(_p(Xq, C.c_int8), _p(Wq, C.c_int8), M, N, K, group_size, G4,
                                _p(a_shift, C.c_uint8), _p(w_shift, C.c_uint8), mode, _p(acc, C.c_int32),
                                C.byref(gp))
    assert ovf == 0, "int32 accumulator overflow in oracle"
    return (acc, gp.value) if return_partial else acc


def mixed_conv(Xq_nhwc, Wq_nrsc, stride: int, pad: int, group_size: int, G4: int, a_shift, w_shift, mode: int = 0):
    Xq = _c(Xq_nhwc, np.int8)
    Wq = _c(Wq_nrsc, np.int8)
    B, H, Wd, Cc = Xq.shape
    N, R, S, C2 = Wq.shape
    assert C2 == Cc and Cc % group_size == 0
    Ho = (H + 2 * pad - R) // stride + 1
    Wo = (Wd + 2 * pad - S) // stride + 1
    a_shift = _c(a_shift, np.uint8)
    w_shift = _c(w_shift, np.uint8)
    acc = np.empty((B, Ho, Wo, N), np.int32)
    ovf = lib().fq_o_mixed_conv(_p(Xq, C.c_int8), _p(Wq, C.c_int8), B, H, Wd, Cc, N, R, S, stride, pad,
                                group_size, G4, _p(a_shift, C.c_uint8), _p(w_shift, C.c_uint8), mode,
                                _p(acc, C.c_int32))
    assert ovf == 0, "int32 accumulator overflow in oracle"
    return acc


def dequant_f64(acc, x_scale: float, w_scale, bias=None) -> np.ndarray:
    acc = _c(acc, np.int32)
    N = acc.shape[-1]
    M = acc.size // N
    w_scale = _c(w_scale, np.float32)
    b = _c(bias, np.float32) if bias is not None else None
    y = np.empty(acc.shape, np.float64)
    lib().fq_o_dequant_f64(_p(acc, C.c_int32), M, N, np.float32(x_scale), _p(w_scale, C.c_float),
                           _p(b, C.c_float), _p(y, C.c_double))
    return y


def requant_i8(acc, x_scale: float, w_scale, out_scale: float, bias=None, return_arg: bool = False):
    """Eq. 1 applied to the dequantised output: clip(round_half_even(y / out_scale), -128, 127), in float64.
    With return_arg also the float64 argument y / out_scale of every element."""
    acc = _c(acc, np.int32)
    N = acc.shape[-1]
    M = acc.size // N
    w_scale = _c(w_scale, np.float32)
    b = _c(bias, np.float32) if bias is not None else None
    q = np.empty(acc.shape, np.int8)
    t = np.empty(acc.shape, np.float64) if return_arg else None
    lib().fq_o_requant_i8(_p(acc, C.c_int32), M, N, np.float32(x_scale), _p(w_scale, C.c_float),
                          _p(b, C.c_float), np.float32(out_scale), _p(q, C.c_int8), _p(t, C.c_double))
    return (q, t) if return_arg else q


# ---- glue: one layer, offline preparation then forward ------------------------------------------

@dataclass
class OracleLayer:
    """Everything the offline steps of the method produce for one layer (stored channel order)."""
    N: int
    C: int
    R: int
    S: int
    group_size: int
    perm: np.ndarray        # int32 [C]  stored position -> original channel
    Wq: np.ndarray          # int8 [N][R][S][C], channels in stored order
    w_scale: np.ndarray     # fp32 [N]
    a_shift: np.ndarray     # uint8 [G]
    w_shift: np.ndarray     # uint8 [N][G]
    x_scale: float
    bias: Optional[np.ndarray]

    @property
    def G(self):
        return self.C // self.group_size


def prepare_layer(W_nrsc, act_absmax, x_scale: float, group_size: int, perm=None, bias=None) -> OracleLayer:
    """Offline steps: quantise weights per output channel, score and order the input channels,
    lay them out in that order, choose the extraction positions."""
    W = _c(W_nrsc, np.float32)
    if W.ndim == 2:
        W = W[:, None, None, :]
    N, R, S, Cc = W.shape
    Wq, w_scale = quantize_rows(W)
    rq = range_codes(act_absmax, x_scale)
    if perm is None:
        perm = order_by_score(channel_scores(Wq.reshape(N, R * S, Cc), rq))
    perm = _c(perm, np.int32)
    Wq_p = np.ascontiguousarray(Wq[..., perm])
    a_sh = act_shifts(rq[perm], group_size)
    w_sh = weight_shifts(Wq_p.reshape(N, R * S, Cc), group_size)
    return OracleLayer(N, Cc, R, S, group_size, perm, Wq_p, w_scale, a_sh, w_sh, float(np.float32(x_scale)),
                       None if bias is None else _c(bias, np.float32))


def forward_gemm(layer: OracleLayer, Xq_perm, r: float, mode: int = 0) -> np.ndarray:
    assert layer.R == 1 and layer.S == 1
    G4 = groups_for_ratio(r, layer.G)
    return mixed_gemm(Xq_perm, layer.Wq.reshape(layer.N, layer.C), layer.group_size, G4, layer.a_shift,
                      layer.w_shift, mode)


def forward_conv(layer: OracleLayer, Xq_nhwc_perm, stride: int, pad: int, r: float, mode: int = 0) -> np.ndarray:
    G4 = groups_for_ratio(r, layer.G)
    return mixed_conv(Xq_nhwc_perm, layer.Wq, stride, pad, layer.group_size, G4, layer.a_shift, layer.w_shift, mode)
