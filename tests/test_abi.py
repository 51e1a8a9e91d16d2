"""CPU-only checks of the boundary: the shared library loads, exports every function the header
declares, and its host-side argument checks return error codes without touching a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2510_02822_amd as fq
    if not os.path.exists(fq.binding.LIB_PATH):
        from paper_2510_02822_amd import build
        build.build()
    return fq.load()


def _declared(header):
    hdr = open(os.path.join(ROOT, "include", header)).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    return set(re.findall(r"\b(flexiq_[a-z0-9_]+)\s*\(", hdr))


def _dynamic_exports():
    """flexiq_* functions in the library's real dynamic symbol table (nm -D), not a hand-written list."""
    import subprocess
    import paper_2510_02822_amd as fq
    out = subprocess.check_output(["nm", "-D", "--defined-only", fq.binding.LIB_PATH], text=True)
    names = set()
    for line in out.splitlines():
        parts = line.split()
        if len(parts) >= 3 and parts[1] in ("T", "W") and parts[2].startswith("flexiq_"):
            names.add(parts[2])
    return names


def test_exports_every_declared_symbol(lib):
    import paper_2510_02822_amd as fq
    api = _declared("flexiq.h")
    test_aids = _declared("flexiq_test.h")
    assert {"flexiq_quantize_pack", "flexiq_bitlower", "flexiq_mixed_gemm", "flexiq_mixed_conv_implicit",
            "flexiq_set_ratio"} <= api
    assert all(n.startswith("flexiq_debug_") for n in test_aids) and not (api & test_aids)
    # the export table holds exactly what the two headers declare: nothing undeclared, nothing missing
    assert _dynamic_exports() == api | test_aids
    assert api == set(fq.exported_symbols())
    for name in api | test_aids:
        assert getattr(lib, name) is not None


def test_strerror(lib):
    assert lib.flexiq_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4):
        assert len(lib.flexiq_strerror(code)) > 0
    assert b"unknown" in lib.flexiq_strerror(-99)


def test_host_argument_checks(lib):
    EINVAL = -1
    assert lib.flexiq_set_ratio(None, C.c_float(0.5), None) == EINVAL
    assert lib.flexiq_layer_free(None) == 0
    assert lib.flexiq_layer_info(None, None, None, None, None, None, None) == EINVAL
    assert lib.flexiq_quantize_pack(None, None) == EINVAL
    assert lib.flexiq_mixed_gemm(None, None, 4, None, None) == EINVAL
    assert lib.flexiq_mixed_conv_implicit(None, None, 1, 4, 4, 1, 1, None, None) == EINVAL
    assert lib.flexiq_bitlower(None, None, 4, 48, 32, None, 0, 0, None) == EINVAL     # C % group_size != 0
    assert lib.flexiq_bitlower(None, None, -1, 64, 32, None, 0, 0, None) == EINVAL
    assert lib.flexiq_bitlower(None, None, 0, 64, 32, None, 0, 0, None) == 0          # empty input: no-op
    assert lib.flexiq_quantize_act(None, None, 0, C.c_float(1.0), None) == 0
    assert lib.flexiq_quantize_act(None, None, 8, C.c_float(0.0), None) == EINVAL
    # a pack description with a bad group size / shape is rejected before any device work
    import numpy as np
    import paper_2510_02822_amd.binding as b
    W = np.zeros((4, 64), np.float32)
    am = np.ones(64, np.float32)
    h = C.c_void_p()
    for gs, cc in ((16, 64), (48, 64), (32, 48)):
        d = b._PackDesc(4, cc, 1, 1, gs, W.ctypes.data, am.ctypes.data, 1.0, None, None)
        assert lib.flexiq_quantize_pack(C.byref(d), C.byref(h)) == EINVAL
    bad_perm = np.zeros(64, np.int32)
    d = b._PackDesc(4, 64, 1, 1, 32, W.ctypes.data, am.ctypes.data, 1.0, bad_perm.ctypes.data, None)
    assert lib.flexiq_quantize_pack(C.byref(d), C.byref(h)) == EINVAL
    d = b._PackDesc(4, 64, 1, 1, 32, W.ctypes.data, am.ctypes.data, 0.0, None, None)
    assert lib.flexiq_quantize_pack(C.byref(d), C.byref(h)) == EINVAL


def test_documented_layer_limits_are_refused_when_packing(lib):
    # include/flexiq.h: more than 159 channel groups, or a padded weight matrix of 1 GiB or more, can never be
    # launched; flexiq_quantize_pack refuses both before any device work (so this runs without a GPU; W is never read)
    import numpy as np
    import paper_2510_02822_amd.binding as b
    EINVAL = -1
    h = C.c_void_p()
    W = np.zeros(16, np.float32)
    for gs, cc in ((32, 160 * 32), (64, 160 * 64), (32, 200 * 32)):         # G = 160, 160, 200
        am = np.ones(cc, np.float32)
        d = b._PackDesc(8, cc, 1, 1, gs, W.ctypes.data, am.ctypes.data, 1.0, None, None, None)
        assert lib.flexiq_quantize_pack(C.byref(d), C.byref(h)) == EINVAL
    # weights: units of 32 channels (even per tap) x 32 bytes x N padded to 256 x two int8 copies >= 2^31 bytes
    am = np.ones(8192, np.float32)
    for n, cc, r in ((32768, 8192, 2), (16384, 8192, 3)):                   # exactly 2^31 bytes; 2.4e9 bytes
        d = b._PackDesc(n, cc, r, r, 64, W.ctypes.data, am.ctypes.data, 1.0, None, None, None)
        assert lib.flexiq_quantize_pack(C.byref(d), C.byref(h)) == EINVAL


def test_missing_library_is_loud(monkeypatch):
    import paper_2510_02822_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", "/nonexistent/libflexiq.so")
    with pytest.raises(b.FlexiqError):
        b.load()
