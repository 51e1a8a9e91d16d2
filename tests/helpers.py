"""Shared set-up for the GPU parity tests: prepare one layer on both sides from the same fp32 inputs."""
import numpy as np


def calib(case):
    """Per-tensor activation scale and per-channel ranges from the calibration draw."""
    import oracle
    Xc = case.Xcal.reshape(-1, case.Xcal.shape[-1])
    return oracle.absmax_scale(Xc), np.abs(Xc).max(0)


def both_layers(case, perm=None, bias=True, group_size=None):
    import oracle
    import paper_2510_02822_amd as fq
    x_scale, amax = calib(case)
    gs = group_size or case.group_size
    b = case.bias if bias else None
    ol = oracle.prepare_layer(case.W, amax, x_scale, gs, perm=perm, bias=b)
    hl = fq.flexiq_quantize_pack(case.W, amax, x_scale, gs, perm=perm, bias=b)
    return ol, hl, x_scale


def check_y(y_gpu, acc_ref, ol, rtol=1e-5):
    """fp32 dequantised output against the float64 definition, relative to |acc*scale| + |bias|."""
    import oracle
    yref = oracle.dequant_f64(acc_ref, ol.x_scale, ol.w_scale, ol.bias)
    mag = np.abs(oracle.dequant_f64(acc_ref, ol.x_scale, ol.w_scale, None))
    if ol.bias is not None:
        mag = mag + np.abs(ol.bias.astype(np.float64))
    err = np.abs(y_gpu.astype(np.float64) - yref)
    assert (err <= rtol * mag + 1e-30).all(), float((err / (mag + 1e-30)).max())


# ---- int8 requantised output -------------------------------------------------------------------------------
# The checker is the real-number definition (oracle.requant_i8, float64).  The library decides the code with a
# handful of correctly rounded single-precision operations, so its argument differs from the exact one by at most
#     eps = 2^-21 * (|acc * S_x * S_w| + |bias|) / S_out + 2^-14
# (products of scales: 3 roundings of 2^-24 each, int32 -> fp32 one more, the bias product two, i.e. below
# 8 * 2^-24 relative; the +128 offset and the fused multiply-add round at magnitude <= 512: 2 * 2^-15 absolute).
# A code may therefore differ from the definition only where the exact argument lies within eps of a rounding tie
# k + 1/2, and then only by taking the other neighbour.  check_q() enforces exactly that and returns how many
# elements needed the window.

def requant_window(acc_ref, ol, out_scale):
    import oracle
    q_def, t = oracle.requant_i8(acc_ref, ol.x_scale, ol.w_scale, out_scale, ol.bias, return_arg=True)
    mag = np.abs(oracle.dequant_f64(acc_ref, ol.x_scale, ol.w_scale, None))
    if ol.bias is not None:
        mag = mag + np.abs(ol.bias.astype(np.float64))
    eps = 2.0 ** -21 * mag / float(np.float32(out_scale)) + 2.0 ** -14
    near_tie = np.abs(t - np.floor(t) - 0.5) <= eps
    return q_def, t, near_tie


def check_q(q_gpu, acc_ref, ol, out_scale, max_window_frac=1e-3):
    """int8 codes against clip(round_half_even(y / S_out), -128, 127) in float64: equal, or the other neighbour of
    a tie that lies within single-precision rounding of the exact argument."""
    q_def, t, near_tie = requant_window(acc_ref, ol, out_scale)
    got = np.asarray(q_gpu).astype(np.int32)
    diff = got != q_def
    lo = np.clip(np.floor(t), -128, 127).astype(np.int32)
    hi = np.clip(np.floor(t) + 1, -128, 127).astype(np.int32)
    neighbour = (got == lo) | (got == hi)
    bad = diff & ~(near_tie & neighbour)
    assert not bad.any(), ("requantised codes differ from the definition outside the tie window",
                           int(bad.sum()), got[bad][:5], q_def[bad][:5], t[bad][:5])
    used = int(diff.sum())
    if got.size >= 10000:
        assert used <= max_window_frac * got.size, (used, got.size)
    return used


def requant_fp32_sequence(acc, ol, out_scale):
    """The single-precision operation sequence the library's epilogue documents in include/flexiq.h, emulated on
    the CPU (test-side second assertion; not the oracle): m = (S_x * S_w) * (1 / S_out), b = bias * (1 / S_out)
    + 128, code = clip(round_half_even(fma(float(acc), m, b)), 0, 255) - 128.  The fused multiply-add is formed
    exactly in rational arithmetic where float64 could round twice."""
    from fractions import Fraction
    f32 = np.float32
    acc = np.asarray(acc, np.int32)
    r = f32(1.0) / f32(out_scale)
    c = f32(ol.x_scale) * ol.w_scale.astype(f32)
    mul = (c * r).astype(f32)
    bias = ol.bias.astype(f32) if ol.bias is not None else np.zeros_like(mul)
    add = ((bias * r).astype(f32) + f32(128.0)).astype(f32)
    a = acc.astype(f32).astype(np.float64)                 # int32 -> fp32, round to nearest even
    prod = a * mul.astype(np.float64)                      # exact: 24 x 24 significant bits
    s64 = prod + add.astype(np.float64)                    # may round (to 53 bits)
    t = s64.astype(f32)
    # float64 -> float32 can double-round only if the float64 sum was inexact and sits on a float32 midpoint
    bits = s64.view(np.int64) & ((1 << 29) - 1)
    sus = (bits == (1 << 28)) & ((s64 - add.astype(np.float64)) != prod)
    for idx in zip(*np.nonzero(sus)):
        n = idx[-1]
        exact = Fraction(float(a[idx])) * Fraction(float(mul[n])) + Fraction(float(add[n]))
        lo_, hi_ = np.nextafter(t[idx], f32(-np.inf)), np.nextafter(t[idx], f32(np.inf))
        cands = sorted({float(lo_), float(t[idx]), float(hi_)}, key=lambda v: abs(Fraction(v) - exact))
        t[idx] = f32(cands[0])
    code = np.clip(np.rint(t), 0, 255).astype(np.int32) - 128
    return code.astype(np.int8)
