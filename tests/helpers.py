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
