"""The entry point that allocates nothing: flexiq_dynamic_positions_static keeps its scan scratch in a file-scope
device array of the library.  Its positions must equal those of flexiq_dynamic_positions (and the oracle's scan) on
two calls in a row, the second on a smaller input, and a GEMM that uses them must match the oracle bit for bit."""
import numpy as np
import pytest

import workloads
from helpers import both_layers

pytestmark = pytest.mark.gpu


def test_static_scratch_scan_matches_allocating_scan():
    import torch
    import oracle
    import paper_2510_02822_amd as fq
    fq.load()
    oracle.build()
    dev = torch.device("cuda:0")
    # first a large layer (24 groups, 2500 rows), then a smaller one (4 groups, 77 rows): the second call finds the
    # shared array as the first left it
    calls = [("big", 2500, 768, 96, 32, 2.0, 0.75), ("small", 77, 256, 40, 64, 0.5, 1.0), ("tiny", 1, 64, 16, 32, 1.0, 1.0)]
    for name, M, K, N, gs, scale, r in calls:
        case = workloads.make_linear("noalloc_" + name, 8, 300 + M, M, K, N, gs, outlier_frac=0.02)
        case.X *= scale
        ol, hl, x_scale = both_layers(case)
        Xq = oracle.quantize(case.X, x_scale)[:, ol.perm]
        Xd = torch.from_numpy(np.ascontiguousarray(Xq)).to(dev)
        k4 = fq.flexiq_set_ratio(hl, r)
        G4 = k4 // gs
        want = oracle.dynamic_act_shifts(Xq, gs, G4, ol.a_shift)
        fq.flexiq_dynamic_positions(hl, Xd)                       # the existing entry point
        ref_pos = fq.flexiq_layer_positions(hl).copy()
        fq.flexiq_static_positions(hl)
        fq.flexiq_dynamic_positions_static(hl, Xd)                # the one that allocates nothing
        got_pos = fq.flexiq_layer_positions(hl).copy()
        assert (got_pos == ref_pos).all(), (name, got_pos, ref_pos)
        assert (got_pos == want).all(), (name, got_pos, want)
        ref = oracle.mixed_gemm(Xq, ol.Wq.reshape(N, K), gs, G4, want, ol.w_shift)
        got = fq.flexiq_mixed_gemm(hl, Xd, acc=True)["acc"].cpu().numpy()
        assert (got == ref).all(), name
        # twice in a row on a smaller slice of the same input
        half = Xd[: max(1, M // 3)].contiguous()
        fq.flexiq_dynamic_positions_static(hl, half)
        want_half = oracle.dynamic_act_shifts(Xq[: max(1, M // 3)], gs, G4, ol.a_shift)
        assert (fq.flexiq_layer_positions(hl) == want_half).all(), name
        fq.flexiq_dynamic_positions(hl, half)
        assert (fq.flexiq_layer_positions(hl) == want_half).all(), name
        fq.flexiq_static_positions(hl)
