"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header
declares, and its host-only entry points behave (no GPU, no compute calls)."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2511_20834_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "spc.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(spc_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    assert os.path.exists(B.LIB_PATH), "build the library first: python -m paper_2511_20834_amd.build"
    L = ctypes.CDLL(B.LIB_PATH)
    names = _declared()
    assert len(names) >= 19
    for n in names:
        assert hasattr(L, n), n
    assert sorted(B.EXPORTS) == names


def test_pack_desc_fit_guard_band_and_alignment():
    d = B.spc_pack_desc_fit([-512, -512, 0], [511, 511, 40], 1, 16, 16)
    assert d.key_bits == 32 and d.pad == 16 and list(d.origin) == [-512, -512, 0]
    assert (d.bits_b, d.bits_x, d.bits_y, d.bits_z) == (0, 11, 11, 7)
    # origin is floored to a multiple of the largest stride; pad is rounded up to one
    d = B.spc_pack_desc_fit([-5, 3, 17], [5, 9, 20], 4, 8, 3)
    assert list(d.origin) == [-8, 0, 16] and d.pad == 8 and d.bits_b == 2
    for a, (lo, hi) in enumerate(zip([-5, 3, 17], [5, 9, 20])):
        bits = (d.bits_x, d.bits_y, d.bits_z)[a]
        assert hi - d.origin[a] + 2 * d.pad < (1 << bits) <= 2 * (hi - d.origin[a] + 2 * d.pad + 1)
    # the paper's example extents (4000 x 4000 x 200 voxels) fit 12/12/8 bits without a guard band
    d = B.spc_pack_desc_fit([0, 0, 0], [3999, 3999, 199], 1, 1, 0)
    assert (d.bits_x, d.bits_y, d.bits_z, d.key_bits) == (12, 12, 8, 32)
    d = B.spc_pack_desc_fit([0, 0, 0], [100000, 100000, 5000], 8, 16, 48)
    assert d.key_bits == 64


def test_pack_desc_fit_errors():
    with pytest.raises(B.SpcError) as e:
        B.spc_pack_desc_fit([0, 0, 0], [1, 1, 1], 1, 3, 1)
    assert e.value.code == B.ERR_ARG
    with pytest.raises(B.SpcError) as e:
        B.spc_pack_desc_fit([0, 0, 0], [100000, 100000, 5000], 8, 16, 48, 32)
    assert e.value.code == B.ERR_RANGE
    with pytest.raises(B.SpcError) as e:
        B.spc_pack_desc_fit([5, 0, 0], [1, 1, 1])
    assert e.value.code == B.ERR_ARG
    assert "hi < lo" in str(e.value)


def test_workspace_query_needs_no_gpu():
    d = B.spc_pack_desc_fit([0, 0, 0], [100, 100, 100])
    assert B.spc_pack_workspace_bytes(1000, d) >= 1000 * 8
    assert B.spc_version().startswith("spc-gfx950")


def test_builders_reject_descriptors_that_do_not_suit_the_layer():
    """Section 5.3: packed additivity needs a guard band of at least the layer's reach, and masking
    equals floor() only if origin - pad is a multiple of the output stride.  Both are checked on the
    host before anything touches the GPU (so this runs without one)."""
    L = B.lib()
    h = ctypes.c_void_p()

    def build(desc, K, s_p, s_l, transposed=0):
        l = B.LayerDesc(K, s_p, s_l, transposed, B.LAYOUT_OS)
        return L.spc_build_kmap(None, 0, ctypes.byref(desc), ctypes.byref(l), ctypes.byref(h), None)

    d = B.spc_pack_desc_fit([0, 0, 0], [100, 100, 100], 1, 2, 1)  # pad 2, origin 0
    assert d.pad == 2
    assert build(d, 5, 2, 1) == B.ERR_ARG and b"reach" in L.spc_last_error()      # reach 4 > pad 2
    assert build(d, 2, 4, 2) == B.ERR_ARG and b"reach" in L.spc_last_error()      # even K: (K-1) * in_stride = 4
    assert build(d, 3, 4, 1) == B.ERR_ARG                                         # reach 4
    assert build(d, 3, 1, 4) == B.ERR_ARG and b"multiple" in L.spc_last_error()   # origin - pad = -2, stride 4
    d2 = B.spc_pack_desc_fit([0, 0, 0], [100, 100, 100], 1, 4, 4)
    d2.origin[1] += 1
    assert build(d2, 3, 1, 2) == B.ERR_ARG and b"origin[1]" in L.spc_last_error()
    # the network builder applies the same rule to every layer
    layers = (B.LayerDesc * 2)(B.LayerDesc(3, 1, 1, 0, 1), B.LayerDesc(3, 4, 1, 0, 1))
    out = (ctypes.c_void_p * 2)()
    streams = (ctypes.c_void_p * 1)(None)
    assert L.spc_build_kmaps_network(None, 0, ctypes.byref(d), layers, 2, out, streams, 1, 0) == B.ERR_ARG
