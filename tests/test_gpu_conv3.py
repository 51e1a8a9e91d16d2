"""GPU parity of the 3x3 convolution kernel with resident weights (64 or 128 input channels, stride 1, padding 1) against the
CPU oracle, through flexiq_mixed_conv_implicit: int32 accumulators and int8 codes bit for bit, fp32 within 1e-5."""
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


# (B, H, W, C, N, gs, forced rows per tile or 0): image rows that split unevenly over tiles, fragments that straddle image
# rows, a last fragment with few pixels, N below / above / not a multiple of the 64 columns of a block
CASES = [(2, 8, 8, 64, 64, 32, 0), (3, 7, 9, 64, 48, 32, 2), (2, 10, 12, 128, 128, 64, 3), (1, 5, 5, 128, 80, 32, 0),
         (2, 13, 56, 64, 64, 32, 4), (2, 9, 28, 128, 136, 32, 8), (1, 3, 40, 64, 200, 64, 1), (4, 6, 6, 64, 16, 32, 5),
         (1, 1, 1, 64, 64, 32, 0), (2, 17, 20, 128, 64, 64, 0)]


@pytest.mark.parametrize("B,H,W,C,N,gs,rows", CASES)
def test_conv3_forced(env, B, H, W, C, N, gs, rows):
    torch, oracle, fq, dev = env
    case = workloads.make_conv("c3", 13, B * H + W + C + N, B, H, W, C, N, 3, 3, 1, 1, gs)
    case.X *= 2.0   # some pixels saturate under the calibrated positions
    ol, hl, x_scale = both_layers(case)
    Xq = np.ascontiguousarray(oracle.quantize(case.X, x_scale)[..., ol.perm])
    Xd = _dev(torch, Xq, dev)
    G = C // gs
    fq.debug_force_conv3(1, rows)
    try:
        for r in sorted({0.0, 1.0 / G, 0.5, 1.0}):
            fq.flexiq_set_ratio(hl, r)
            ref = oracle.forward_conv(ol, Xq, 1, 1, r)
            so = float(np.abs(oracle.dequant_f64(ref, x_scale, ol.w_scale, ol.bias)).max() / 127 * 0.9) or 1.0
            out = fq.flexiq_mixed_conv_implicit(hl, Xd, 1, 1, acc=True, y=True, q=True, out_scale=so)
            torch.cuda.synchronize()
            assert fq.debug_force_conv3(1, rows) == 1          # the call ran on this kernel
            assert fq.debug_last_launch()["tile"] == -3
            assert (out["acc"].cpu().numpy() == ref).all(), r
            check_y(out["y"].cpu().numpy(), ref, ol)
            got_q = out["q"].cpu().numpy()
            check_q(got_q, ref, ol, so)
            assert (got_q == requant_fp32_sequence(ref, ol, so)).all()
            # int8 alone: the int8-only build when rows are whole 16-byte pieces, else the general one with pre-multiplied scales
            only_q = fq.flexiq_mixed_conv_implicit(hl, Xd, 1, 1, q=True, out_scale=so)["q"]
            assert fq.debug_force_conv3(1, rows) == 1
            assert (only_q.cpu().numpy() == got_q).all(), r
            # the tiled kernel gives the same bytes
            fq.debug_force_conv3(0, 0)
            tiled = fq.flexiq_mixed_conv_implicit(hl, Xd, 1, 1, q=True, out_scale=so)["q"]
            assert fq.debug_last_launch()["tile"] >= 0
            fq.debug_force_conv3(1, rows)
            assert (tiled.cpu().numpy() == got_q).all(), r
    finally:
        fq.debug_force_conv3(-1, 0)


def test_conv3_blocks_walk_many_tiles_and_buffers(env):
    """More tiles than blocks (every block walks its buffers round several times), run-time positions and inputs that
    arrive lowered; compared in full with the oracle."""
    torch, oracle, fq, dev = env
    B, H, W, C, N, gs = 300, 12, 12, 64, 64, 32
    case = workloads.make_conv("c3walk", 13, 7, B, H, W, C, N, 3, 3, 1, 1, gs)
    case.X *= 3.0
    ol, hl, x_scale = both_layers(case)
    Xq = np.ascontiguousarray(oracle.quantize(case.X, x_scale)[..., ol.perm])
    Xd = _dev(torch, Xq, dev)
    fq.debug_force_conv3(1, 2)   # 1800 tiles
    try:
        for r in (0.0, 0.5, 1.0):
            k4 = fq.flexiq_set_ratio(hl, r)
            ref = oracle.forward_conv(ol, Xq, 1, 1, r)
            got = fq.flexiq_mixed_conv_implicit(hl, Xd, 1, 1, acc=True)["acc"].cpu().numpy()
            assert fq.debug_force_conv3(1, 2) == 1
            assert (got == ref).all(), r
        k4 = fq.flexiq_set_ratio(hl, 1.0)
        G4 = k4 // gs
        fq.flexiq_dynamic_positions(hl, Xd.reshape(-1, C))
        dyn = oracle.dynamic_act_shifts(Xq.reshape(-1, C), gs, G4, ol.a_shift)
        got = fq.flexiq_mixed_conv_implicit(hl, Xd, 1, 1, acc=True)["acc"].cpu().numpy()
        assert fq.debug_force_conv3(1, 2) == 1
        want = oracle.mixed_conv(Xq, ol.Wq.reshape(N, 3, 3, C), 1, 1, gs, G4, dyn, ol.w_shift)
        assert (got == want).all()
        fq.flexiq_static_positions(hl)
        # activations lowered by the producer: the kernel copies them as they are
        sh = np.repeat(ol.a_shift.astype(np.int32), gs)[None, None, None, :]
        Xl = (np.clip(Xq.astype(np.int32) >> sh, -8, 7) << sh).astype(np.int8)
        fq.flexiq_input_prelowered(hl, True)
        got = fq.flexiq_mixed_conv_implicit(hl, _dev(torch, Xl, dev), 1, 1, acc=True)["acc"].cpu().numpy()
        assert fq.debug_force_conv3(1, 2) == 1
        assert (got == oracle.forward_conv(ol, Xq, 1, 1, 1.0)).all()
        fq.flexiq_input_prelowered(hl, False)
    finally:
        fq.debug_force_conv3(-1, 0)


def test_conv3_automatic_route(env):
    """A stage-1-like layer at a batch that fills the chip takes this kernel by itself; strided, padded-differently and
    wide-channel layers do not."""
    torch, oracle, fq, dev = env
    case = workloads.make_conv("c3auto", 13, 3, 100, 28, 28, 64, 64, 3, 3, 1, 1, 32)
    ol, hl, x_scale = both_layers(case)
    Xq = np.ascontiguousarray(oracle.quantize(case.X, x_scale)[..., ol.perm])
    Xd = _dev(torch, Xq, dev)
    fq.flexiq_set_ratio(hl, 0.5)
    ref = oracle.forward_conv(ol, Xq, 1, 1, 0.5)
    so = float(np.abs(oracle.dequant_f64(ref, x_scale, ol.w_scale, ol.bias)).max() / 127 * 0.9)
    got = fq.flexiq_mixed_conv_implicit(hl, Xd, 1, 1, q=True, out_scale=so)["q"].cpu().numpy()
    assert fq.debug_last_launch()["tile"] == -3
    check_q(got, ref, ol, so)
    assert (got == requant_fp32_sequence(ref, ol, so)).all()
    got = fq.flexiq_mixed_conv_implicit(hl, Xd, 2, 1, acc=True)["acc"].cpu().numpy()   # stride 2: the tiled kernel
    assert fq.debug_last_launch()["tile"] >= 0
    assert (got == oracle.forward_conv(ol, Xq, 2, 1, 0.5)).all()


@pytest.mark.parametrize("B,H,W,C,N1,gs2,rows", [(2, 9, 12, 64, 64, 32, 0), (3, 7, 9, 128, 96, 32, 2), (1, 14, 14, 64, 128, 64, 3)])
def test_conv3_lowers_for_consumer(env, B, H, W, C, N1, gs2, rows):
    # the fused producer (Section 4.1 applied where the tensor is produced) on the 3x3 kernel: the NHWC int8 output in the
    # consumer's stored channel order with the consumer's 4-bit channels clamped and masked at its positions; the consumer
    # is a 1x1 convolution over the same pixels
    torch, oracle, fq, dev = env
    helpers = __import__("helpers")
    c1 = workloads.make_conv("c3low1", 13, 400 + C + N1, B, H, W, C, N1, 3, 3, 1, 1, 32)
    xs1, am1 = helpers.calib(c1)
    o1 = oracle.prepare_layer(c1.W, am1, xs1, 32, bias=c1.bias)
    X1 = np.ascontiguousarray(oracle.quantize(c1.X, xs1)[..., o1.perm])
    acc1 = oracle.forward_conv(o1, X1, 1, 1, 0.5)
    s_mid = float(np.abs(oracle.dequant_f64(acc1, xs1, o1.w_scale, o1.bias)).max() / 127.0 * 0.8)
    q1 = requant_fp32_sequence(acc1, o1, s_mid)
    check_q(q1, acc1, o1, s_mid)
    c2 = workloads.make_conv("c3low2", 13, 401 + C + N1, B, H, W, N1, 48, 1, 1, 1, 0, gs2)
    am2 = np.abs(q1).reshape(-1, N1).max(0).astype(np.float32) * np.float32(s_mid) * np.float32(0.5)   # too narrow: the clamp bites
    o2 = oracle.prepare_layer(c2.W, am2, s_mid, gs2, bias=c2.bias)
    h2 = fq.flexiq_quantize_pack(c2.W, am2, s_mid, gs2, bias=c2.bias)
    h1 = fq.flexiq_quantize_pack(c1.W, am1, xs1, 32, bias=c1.bias, out_perm=o2.perm)
    X2 = np.ascontiguousarray(q1[..., o2.perm])
    fq.flexiq_set_ratio(h1, 0.5)
    X1d = _dev(torch, X1, dev)
    sh = np.repeat(o2.a_shift.astype(np.int32), gs2)
    G2 = N1 // gs2
    fq.debug_force_conv3(1, rows)
    try:
        for r2 in sorted({0.0, 1.0 / G2, 1.0}):
            k4 = fq.flexiq_set_ratio(h2, r2)
            want = X2.astype(np.int32).copy()
            want[..., :k4] = np.clip(want[..., :k4] >> sh[:k4], -8, 7) << sh[:k4]
            low = fq.flexiq_mixed_conv_implicit(h1, X1d, 1, 1, q=True, out_scale=s_mid, lower_for=h2)["q"]
            torch.cuda.synchronize()
            assert fq.debug_force_conv3(1, rows) == 1 and fq.debug_last_launch()["tile"] == -3   # ran on this kernel
            assert (low.cpu().numpy().astype(np.int32) == want).all(), r2
            fq.debug_force_conv3(0, 0)
            tiled = fq.flexiq_mixed_conv_implicit(h1, X1d, 1, 1, q=True, out_scale=s_mid, lower_for=h2)["q"]
            assert fq.debug_last_launch()["tile"] >= 0
            assert (tiled.cpu().numpy() == low.cpu().numpy()).all(), r2
            fq.flexiq_input_prelowered(h2, True)
            got = fq.flexiq_mixed_conv_implicit(h2, low, 1, 0, acc=True)["acc"].cpu().numpy()
            fq.flexiq_input_prelowered(h2, False)
            fq.debug_force_conv3(1, rows)
            assert (got == oracle.forward_conv(o2, X2, 1, 0, r2)).all(), r2
    finally:
        fq.debug_force_conv3(-1, 0)
        fq.flexiq_input_prelowered(h2, False)
    # a producer whose output order is not the consumer's stored order is refused on this route too
    if not (o2.perm == np.arange(N1)).all():
        h1_plain = fq.flexiq_quantize_pack(c1.W, am1, xs1, 32, bias=c1.bias)
        fq.debug_force_conv3(1, rows)
        try:
            with pytest.raises(fq.FlexiqError):
                fq.flexiq_mixed_conv_implicit(h1_plain, X1d, 1, 1, q=True, out_scale=s_mid, lower_for=h2)
        finally:
            fq.debug_force_conv3(-1, 0)
