"""ctypes binding of libflexiq.so.  Same names as the C entry points; tensors in, tensors out."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflexiq.so")   # built in-tree; there is no non-HIP path
_lib = None


class FlexiqError(RuntimeError):
    pass


class _PackDesc(C.Structure):
    _fields_ = [("N", C.c_int32), ("C", C.c_int32), ("R", C.c_int32), ("S", C.c_int32),
                ("group_size", C.c_int32), ("W", C.c_void_p), ("act_absmax", C.c_void_p),
                ("x_scale", C.c_float), ("perm", C.c_void_p), ("bias", C.c_void_p), ("out_perm", C.c_void_p)]


class _Out(C.Structure):
    _fields_ = [("acc", C.c_void_p), ("y", C.c_void_p), ("q", C.c_void_p), ("out_scale", C.c_float),
                ("lower_for", C.c_void_p), ("scan_for", C.c_void_p), ("x6", C.c_void_p), ("x4", C.c_void_p)]


def exported_symbols():
    """Names include/flexiq.h declares."""
    return ["flexiq_packed4_channels", "flexiq_packed4_bytes", "flexiq_lower_packed4", "flexiq_mixed_gemm_packed4",
            "flexiq_dynamic_positions_static", "flexiq_fp6_channels", "flexiq_fp6_bytes", "flexiq_lower_fp6",
            "flexiq_mixed_gemm_fp6", "flexiq_strerror", "flexiq_last_hip_error", "flexiq_quantize_pack", "flexiq_layer_free",
            "flexiq_layer_info", "flexiq_layer_dump", "flexiq_set_ratio", "flexiq_quantize_act",
            "flexiq_bitlower", "flexiq_dynamic_positions", "flexiq_static_positions", "flexiq_layer_positions",
            "flexiq_input_prelowered", "flexiq_permute_channels", "flexiq_mixed_gemm", "flexiq_mixed_conv_implicit"]


def load():
    """Load libflexiq.so; raise if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FlexiqError("libflexiq.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(hipcc --offload-arch=gfx950).  There is no CPU fallback.")
    L = C.CDLL(LIB_PATH)
    L.flexiq_strerror.restype = C.c_char_p
    L.flexiq_strerror.argtypes = [C.c_int]
    L.flexiq_last_hip_error.restype = C.c_char_p
    L.flexiq_quantize_pack.argtypes = [C.POINTER(_PackDesc), C.POINTER(C.c_void_p)]
    L.flexiq_layer_free.argtypes = [C.c_void_p]
    L.flexiq_layer_info.argtypes = [C.c_void_p] + [C.POINTER(C.c_void_p)] * 4 + [C.POINTER(C.c_int32)] * 2
    L.flexiq_layer_dump.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.flexiq_set_ratio.argtypes = [C.c_void_p, C.c_float, C.POINTER(C.c_int32)]
    L.flexiq_quantize_act.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_float, C.c_void_p]
    L.flexiq_bitlower.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_int,
                                  C.c_int, C.c_void_p]
    L.flexiq_dynamic_positions.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
    L.flexiq_dynamic_positions_static.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
    L.flexiq_static_positions.argtypes = [C.c_void_p]
    L.flexiq_input_prelowered.argtypes = [C.c_void_p, C.c_int]
    L.flexiq_layer_positions.argtypes = [C.c_void_p, C.c_void_p]
    L.flexiq_permute_channels.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
    L.flexiq_mixed_gemm.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.POINTER(_Out), C.c_void_p]
    L.flexiq_mixed_conv_implicit.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                             C.c_int32, C.POINTER(_Out), C.c_void_p]
    L.flexiq_fp6_channels.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
    L.flexiq_fp6_bytes.argtypes = [C.c_void_p, C.c_int64]
    L.flexiq_fp6_bytes.restype = C.c_int64
    L.flexiq_lower_fp6.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
    L.flexiq_mixed_gemm_fp6.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.POINTER(_Out), C.c_void_p]
    L.flexiq_packed4_channels.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
    L.flexiq_packed4_bytes.argtypes = [C.c_void_p, C.c_int64]
    L.flexiq_packed4_bytes.restype = C.c_int64
    L.flexiq_lower_packed4.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
    L.flexiq_mixed_gemm_packed4.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.POINTER(_Out), C.c_void_p]
    L.flexiq_debug_force_fp6_tile.argtypes = [C.c_int]
    L.flexiq_debug_force_stream.argtypes = [C.c_int]
    L.flexiq_debug_force_few_rows.argtypes = [C.c_int]
    L.flexiq_debug_force_tile_splitk.argtypes = [C.c_int]
    L.flexiq_debug_force_conv3.argtypes = [C.c_int, C.c_int]
    L.flexiq_debug_force_tile.argtypes = [C.c_int]
    L.flexiq_debug_force_packed4.argtypes = [C.c_int]
    L.flexiq_debug_max_blocks.argtypes = [C.c_int]
    L.flexiq_debug_last_launch.argtypes = [C.c_int]
    for name in exported_symbols():
        getattr(L, name)
    _lib = L
    return L


def _check(rc: int):
    if rc != 0:
        L = load()
        msg = L.flexiq_strerror(rc).decode()
        if rc == -4:
            msg += " (" + L.flexiq_last_hip_error().decode() + ")"
        raise FlexiqError("flexiq status %d: %s" % (rc, msg))


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


class Layer:
    """Owns a flexiq_layer handle; frees it on garbage collection."""

    def __init__(self, handle: int, N: int, Cc: int, R: int, S: int, group_size: int):
        self._h = C.c_void_p(handle)
        self.N, self.C, self.R, self.S, self.group_size = N, Cc, R, S, group_size

    def __del__(self):
        try:
            if self._h and _lib is not None:
                _lib.flexiq_layer_free(self._h)
                self._h = None
        except Exception:
            pass

    def info(self):
        """Host tables of the handle as numpy copies."""
        L = load()
        ps = [C.c_void_p() for _ in range(4)]
        G = C.c_int32()
        k4 = C.c_int32()
        _check(L.flexiq_layer_info(self._h, *[C.byref(p) for p in ps], C.byref(G), C.byref(k4)))
        g = G.value

        def arr(p, ct, n):
            return np.ctypeslib.as_array(C.cast(p, C.POINTER(ct)), shape=(n,)).copy()
        return {"perm": arr(ps[0], C.c_int32, self.C), "a_shift": arr(ps[1], C.c_uint8, g),
                "w_shift": arr(ps[2], C.c_uint8, self.N * g).reshape(self.N, g),
                "w_scale": arr(ps[3], C.c_float, self.N), "G": g, "max_4bit_ch": k4.value}


def flexiq_quantize_pack(W, act_absmax, x_scale: float, group_size: int, perm=None, bias=None, out_perm=None) -> Layer:
    """W: fp32 [N][C] or [N][R][S][C] (numpy, original channel order).  out_perm: output column j = original
    output channel out_perm[j] (e.g. the next layer's stored channel order)."""
    L = load()
    W = _f32(W)
    if W.ndim == 2:
        W = W[:, None, None, :]
    N, R, S, Cc = W.shape
    W = np.ascontiguousarray(W)
    am = _f32(act_absmax)
    assert am.shape == (Cc,)
    pm = None if perm is None else np.ascontiguousarray(perm, dtype=np.int32)
    bs = None if bias is None else _f32(bias)
    op = None if out_perm is None else np.ascontiguousarray(out_perm, dtype=np.int32)
    assert op is None or op.shape == (N,)
    d = _PackDesc(N, Cc, R, S, group_size, W.ctypes.data, am.ctypes.data, float(x_scale),
                  None if pm is None else pm.ctypes.data, None if bs is None else bs.ctypes.data,
                  None if op is None else op.ctypes.data)
    h = C.c_void_p()
    _check(L.flexiq_quantize_pack(C.byref(d), C.byref(h)))
    return Layer(h.value, N, Cc, R, S, group_size)


def flexiq_layer_dump(layer: Layer):
    L = load()
    T = layer.R * layer.S
    w8 = np.empty((layer.N, T, layer.C), np.int8)
    w4 = np.empty((layer.N, T, layer.C // 2), np.uint8)
    w4x = np.empty((layer.N, T, layer.C), np.int8)
    _check(L.flexiq_layer_dump(layer._h, w8.ctypes.data, w4.ctypes.data, w4x.ctypes.data))
    return w8, w4, w4x


def flexiq_set_ratio(layer: Layer, r: float) -> int:
    k4 = C.c_int32()
    _check(load().flexiq_set_ratio(layer._h, float(r), C.byref(k4)))
    return k4.value


def flexiq_quantize_act(x, scale: float, out=None):
    import torch
    assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()
    q = out if out is not None else torch.empty(x.shape, dtype=torch.int8, device=x.device)
    _check(load().flexiq_quantize_act(x.data_ptr(), q.data_ptr(), x.numel(), float(scale), _stream()))
    return q


def flexiq_bitlower(src, group_size: int, shifts, per_row: bool, mode: int = 0):
    import torch
    assert src.is_cuda and src.dtype == torch.int8 and src.is_contiguous() and src.dim() == 2
    rows, Cc = src.shape
    dst = torch.empty((rows, Cc // 2), dtype=torch.uint8, device=src.device)
    _check(load().flexiq_bitlower(src.data_ptr(), dst.data_ptr(), rows, Cc, group_size, shifts.data_ptr(),
                                  1 if per_row else 0, mode, _stream()))
    return dst


def flexiq_dynamic_positions(layer: Layer, X) -> None:
    """Scan X (int8, [..., C] contiguous, stored channel order) for the run-time extraction positions of the
    groups that are 4-bit under the current ratio; later GEMM / conv calls on the handle use them."""
    import torch
    assert X.dtype == torch.int8 and X.is_cuda and X.is_contiguous() and X.shape[-1] == layer.C
    rows = X.numel() // layer.C
    _check(load().flexiq_dynamic_positions(layer._h, X.data_ptr(), rows, _stream()))


def flexiq_dynamic_positions_static(layer: Layer, X) -> None:
    """flexiq_dynamic_positions with the scan scratch in the library's file-scope device array (allocates nothing)."""
    import torch
    assert X.dtype == torch.int8 and X.is_cuda and X.is_contiguous() and X.shape[-1] == layer.C
    rows = X.numel() // layer.C
    _check(load().flexiq_dynamic_positions_static(layer._h, X.data_ptr(), rows, _stream()))


def flexiq_input_prelowered(layer: Layer, on: bool) -> None:
    """The activations given to this layer's GEMM / conv calls are lowered already (flexiq_out.lower_for)."""
    _check(load().flexiq_input_prelowered(layer._h, 1 if on else 0))


def flexiq_static_positions(layer: Layer) -> None:
    _check(load().flexiq_static_positions(layer._h))


def flexiq_layer_positions(layer: Layer) -> np.ndarray:
    out = np.empty(layer.C // layer.group_size, np.uint8)
    _check(load().flexiq_layer_positions(layer._h, out.ctypes.data))
    return out


def flexiq_permute_channels(layer: Layer, src):
    import torch
    assert src.is_cuda and src.dtype == torch.int8 and src.is_contiguous()
    dst = torch.empty_like(src)
    _check(load().flexiq_permute_channels(layer._h, src.data_ptr(), dst.data_ptr(), src.numel() // layer.C, _stream()))
    return dst


def flexiq_fp6_channels(layer: Layer) -> int:
    """Leading stored channels that run on the FP6 matrix path under the current ratio and positions."""
    k6 = C.c_int32()
    _check(load().flexiq_fp6_channels(layer._h, C.byref(k6)))
    return k6.value


def flexiq_fp6_bytes(layer: Layer, M: int) -> int:
    n = load().flexiq_fp6_bytes(layer._h, int(M))
    if n < 0:
        _check(int(n))
    return int(n)


def flexiq_packed4_channels(layer: Layer) -> int:
    k = C.c_int32(0)
    _check(load().flexiq_packed4_channels(layer._h, C.byref(k)))
    return int(k.value)


def flexiq_packed4_bytes(layer: Layer, M: int) -> int:
    n = int(load().flexiq_packed4_bytes(layer._h, M))
    if n < 0:
        _check(n)
    return n


def flexiq_lower_packed4(layer: Layer, X, x4=None):
    """Stand-alone producer of the packed 4-bit activations (uint8 cuda [M][C/2])."""
    import torch
    assert X.is_cuda and X.dtype == torch.int8 and X.is_contiguous() and X.dim() == 2 and X.shape[1] == layer.C
    M = X.shape[0]
    if x4 is None:
        x4 = torch.empty((max(M, 1), layer.C // 2), dtype=torch.uint8, device=X.device)
    _check(load().flexiq_lower_packed4(layer._h, X.data_ptr(), M, x4.data_ptr(), _stream()))
    return x4


def flexiq_mixed_gemm_packed4(layer: Layer, X, x4, acc: bool = False, y: bool = False, q: bool = False, out_scale: float = 1.0,
                              bufs: Optional[dict] = None, lower_for: Optional[Layer] = None, x4_out=None):
    """flexiq_mixed_gemm with the leading 4-bit channels read from packed codes.  x4_out: with lower_for, the consumer's
    packed buffer (flexiq_out.x4)."""
    import torch
    assert X.is_cuda and X.dtype == torch.int8 and X.is_contiguous() and X.dim() == 2 and X.shape[1] == layer.C
    M = X.shape[0]
    o, res = _outs((M, layer.N), X.device, acc, y, q, out_scale, bufs, lower_for, None)
    if x4_out is not None:
        o.x4 = x4_out.data_ptr()
    _check(load().flexiq_mixed_gemm_packed4(layer._h, X.data_ptr(), x4.data_ptr(), M, C.byref(o), _stream()))
    return res


def flexiq_lower_fp6(layer: Layer, X, x6=None, need_xlow: Optional[bool] = None):
    """Stand-alone producer of the FP6 activations: returns (x6, xlow).  xlow is X itself unless some 4-bit channels
    lie outside the FP6 prefix (then a copy with those channels lowered)."""
    import torch
    assert X.is_cuda and X.dtype == torch.int8 and X.is_contiguous() and X.dim() == 2 and X.shape[1] == layer.C
    M = X.shape[0]
    if x6 is None:
        x6 = torch.empty(max(flexiq_fp6_bytes(layer, M), 16), dtype=torch.uint8, device=X.device)
    k6 = flexiq_fp6_channels(layer)
    k4 = layer.info()["max_4bit_ch"]
    if need_xlow is None:
        need_xlow = k6 < k4
    xlow = torch.empty_like(X) if need_xlow else None
    _check(load().flexiq_lower_fp6(layer._h, X.data_ptr(), M, x6.data_ptr(), xlow.data_ptr() if xlow is not None else None,
                                   _stream()))
    return x6, (xlow if xlow is not None else X)


def flexiq_mixed_gemm_fp6(layer: Layer, X, x6, acc: bool = False, y: bool = False, q: bool = False,
                          out_scale: float = 1.0, bufs: Optional[dict] = None, lower_for: Optional[Layer] = None,
                          x6_out=None):
    """The FP6-variant GEMM.  X: int8 cuda [M][C] (4-bit channels outside the FP6 prefix lowered), x6: FP6 activations.
    x6_out: with lower_for, the consumer's FP6 activation buffer (flexiq_out.x6)."""
    import torch
    assert X.is_cuda and X.dtype == torch.int8 and X.is_contiguous() and X.dim() == 2 and X.shape[1] == layer.C
    M = X.shape[0]
    o, res = _outs((M, layer.N), X.device, acc, y, q, out_scale, bufs, lower_for, None)
    if x6_out is not None:
        o.x6 = x6_out.data_ptr()
    _check(load().flexiq_mixed_gemm_fp6(layer._h, X.data_ptr(), x6.data_ptr() if x6 is not None else None, M, C.byref(o),
                                        _stream()))
    return res


def debug_force_fp6_tile(index: int) -> int:
    rc = load().flexiq_debug_force_fp6_tile(index)
    if rc < 0:
        _check(rc)
    return rc


def _outs(shape, device, want_acc, want_y, want_q, out_scale, bufs, lower_for=None, scan_for=None):
    import torch
    acc = y = q = None
    if want_acc:
        acc = bufs.get("acc") if bufs and "acc" in bufs else torch.empty(shape, dtype=torch.int32, device=device)
    if want_y:
        y = bufs.get("y") if bufs and "y" in bufs else torch.empty(shape, dtype=torch.float32, device=device)
    if want_q:
        q = bufs.get("q") if bufs and "q" in bufs else torch.empty(shape, dtype=torch.int8, device=device)
    o = _Out(acc.data_ptr() if acc is not None else None, y.data_ptr() if y is not None else None,
             q.data_ptr() if q is not None else None, float(out_scale),
             lower_for._h if lower_for is not None else None, scan_for._h if scan_for is not None else None, None, None)
    return o, {"acc": acc, "y": y, "q": q}


def flexiq_mixed_gemm(layer: Layer, X, acc: bool = False, y: bool = False, q: bool = False,
                      out_scale: float = 1.0, bufs: Optional[dict] = None, lower_for: Optional[Layer] = None,
                      scan_for: Optional[Layer] = None, x4_out=None):
    """X: int8 cuda [M][C] in stored channel order.  Returns a dict of the requested outputs.
    lower_for / scan_for: the layer that consumes q (flexiq_out.lower_for, flexiq_out.scan_for).
    x4_out: with lower_for, the consumer's packed 4-bit activation buffer (flexiq_out.x4)."""
    import torch
    assert X.is_cuda and X.dtype == torch.int8 and X.is_contiguous() and X.dim() == 2 and X.shape[1] == layer.C
    M = X.shape[0]
    o, res = _outs((M, layer.N), X.device, acc, y, q, out_scale, bufs, lower_for, scan_for)
    if x4_out is not None:
        o.x4 = x4_out.data_ptr()
    _check(load().flexiq_mixed_gemm(layer._h, X.data_ptr(), M, C.byref(o), _stream()))
    return res


def flexiq_mixed_conv_implicit(layer: Layer, X, stride: int, pad: int, acc: bool = False, y: bool = False,
                               q: bool = False, out_scale: float = 1.0, bufs: Optional[dict] = None,
                               lower_for: Optional[Layer] = None, scan_for: Optional[Layer] = None):
    """X: int8 cuda NHWC [B][H][W][C] in stored channel order."""
    import torch
    assert X.is_cuda and X.dtype == torch.int8 and X.is_contiguous() and X.dim() == 4 and X.shape[3] == layer.C
    B, H, Wd, _ = X.shape
    Ho = (H + 2 * pad - layer.R) // stride + 1
    Wo = (Wd + 2 * pad - layer.S) // stride + 1
    o, res = _outs((B, Ho, Wo, layer.N), X.device, acc, y, q, out_scale, bufs, lower_for, scan_for)
    _check(load().flexiq_mixed_conv_implicit(layer._h, X.data_ptr(), B, H, Wd, stride, pad, C.byref(o), _stream()))
    return res


def debug_force_tile(index: int) -> int:
    """Force a tile shape of the GEMM kernel table (-1: automatic).  Returns the table size."""
    rc = load().flexiq_debug_force_tile(index)
    if rc < 0:
        _check(rc)
    return rc


def debug_force_packed4(mode: int) -> None:
    """Where the GEMM kernel takes the weights of 4-bit units from: 1 = packed codes, 0 = expanded copy, -1 = automatic."""
    _check(load().flexiq_debug_force_packed4(mode))


def debug_max_blocks(n: int) -> None:
    """Blocks of a linear GEMM call: 0 = automatic (a resident wave of blocks, each walking several output tiles),
    n > 0 = at most n blocks, n < 0 = one block per output tile."""
    _check(load().flexiq_debug_max_blocks(int(n)))


def debug_last_launch() -> dict:
    """Tile shape index, block count and resident blocks per CU of the last GEMM / convolution launch."""
    L = load()
    return {"tile": L.flexiq_debug_last_launch(0), "blocks": L.flexiq_debug_last_launch(1),
            "resident": L.flexiq_debug_last_launch(2)}


def debug_force_conv3(mode: int, rows_per_tile: int = 0) -> int:
    """3x3 kernel with resident weights: 1 = whenever the layer form qualifies, 0 = never, -1 = automatic; rows_per_tile > 0
    forces the output rows of an image tile; returns whether the last convolution call used it."""
    rc = load().flexiq_debug_force_conv3(int(mode), int(rows_per_tile))
    if rc < 0:
        _check(rc)
    return rc


def debug_force_stream(mode: int) -> int:
    """Row-streaming kernels: 1 / 2 = the one whose blocks walk tiles / whose waves walk row groups, whenever the layer form
    qualifies; 0 = never; -1 = automatic.  Returns which of them the last call ran on (0: neither)."""
    rc = load().flexiq_debug_force_stream(int(mode))
    if rc < 0:
        _check(rc)
    return rc


def debug_force_tile_splitk(mode: int) -> int:
    """The 64 x 64 tile kernel whose waves split the reduction: 1 = whenever the call qualifies, 0 = never, -1 = automatic.
    Returns whether the last call it was offered ran on it."""
    rc = load().flexiq_debug_force_tile_splitk(int(mode))
    if rc < 0:
        _check(rc)
    return rc


def debug_force_few_rows(mode: int) -> int:
    """Few-row kernels: 1 / 2 = the matrix-core kernel / the dot-product kernel (at most 4 rows) whenever the call qualifies,
    14 = the dot-product kernel with 4 column groups per block, 0 = never, -1 = automatic.  Returns which of them the
    last call they were offered ran on (0: neither)."""
    rc = load().flexiq_debug_force_few_rows(int(mode))
    if rc < 0:
        _check(rc)
    return rc


