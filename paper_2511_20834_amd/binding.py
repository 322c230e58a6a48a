"""Thin ctypes binding of libspc.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in
``include/spc.h``; PyTorch is used for device memory and streams.  There is no CPU
fallback: loading fails loudly when the library has not been built.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspc.so")

OK = 0
DTYPE_F16, DTYPE_BF16, DTYPE_F32 = 0, 1, 2
LAYOUT_OS, LAYOUT_WS, LAYOUT_BOTH = 1, 2, 3
LAYOUT_WS_SYM = 4  # with LAYOUT_WS: symmetric half-map of a submanifold layer


def LAYOUT_HYBRID_T(t: int) -> int:
    """with LAYOUT_BOTH: build for the hybrid dual dataflow with threshold t (dense offsets in the OS matrix only,
    sparse ones in the WS lists only)."""
    return int(t) << 8


DATAFLOW_OS, DATAFLOW_WS = 0, 1
PACK_VALIDATE = 1
CONV_RELU = 1
CONV_PACKED_WEIGHTS = 2
CONV_OS_PHASE = 4
CONV_OS_SPLITK = 8
NET_SEQUENTIAL = 1
NET_PHASE_BARRIER = 2
NET_PIPELINED = 4
ERR_ARG, ERR_RANGE, ERR_DUP, ERR_UNSUPPORTED, ERR_HIP, ERR_NOMEM = -1, -2, -3, -4, -5, -6

EXPORTS = [
    "spc_pack_desc_fit", "spc_pack_coords", "spc_pack_coords_noalloc", "spc_build_kmap", "spc_build_kmap_perm", "spc_build_kmaps_network", "spc_kmap_n_in",
    "spc_kmap_n_out", "spc_kmap_kvol", "spc_kmap_copy_out_keys", "spc_kmap_out_keys", "spc_kmap_in_keys", "spc_kmap_os_map",
    "spc_kmap_ws_lists", "spc_kmap_nnz", "spc_kmap_search_info", "spc_search_count", "spc_kmap_export_triples", "spc_kmap_set_size_hint", "spc_kmap_destroy",
    "spc_conv_forward", "spc_conv_forward_hybrid", "spc_conv_tune_threshold",
    "spc_conv_prepare_weights", "spc_permute_rows",
    "spc_probe_copy", "spc_probe_mfma",
    "spc_release_cache", "spc_last_error", "spc_version",
]


class SpcError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("spc error %d: %s" % (code, msg))
        self.code = code


class PackDesc(ctypes.Structure):
    _fields_ = [("key_bits", ctypes.c_int32), ("bits_b", ctypes.c_int32), ("bits_x", ctypes.c_int32),
                ("bits_y", ctypes.c_int32), ("bits_z", ctypes.c_int32), ("origin", ctypes.c_int32 * 3),
                ("pad", ctypes.c_int32)]

    def as_dict(self):
        return dict(key_bits=self.key_bits, bits_b=self.bits_b, bits_x=self.bits_x, bits_y=self.bits_y,
                    bits_z=self.bits_z, origin=list(self.origin), pad=self.pad)


class LayerDesc(ctypes.Structure):
    _fields_ = [("K", ctypes.c_int32), ("in_stride", ctypes.c_int32), ("layer_stride", ctypes.c_int32),
                ("transposed", ctypes.c_int32), ("layout", ctypes.c_int32)]


_lib = None


def lib():
    """The loaded C library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is missing: run `python -m paper_2511_20834_amd.build` (or __graft_entry__.build())"
                               % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        L.spc_pack_desc_fit.argtypes = [ctypes.POINTER(i32), ctypes.POINTER(i32), i32, i32, i32, i32, ctypes.POINTER(PackDesc)]
        L.spc_pack_coords.argtypes = [vp, i64, ctypes.POINTER(PackDesc), vp, vp, vp, ctypes.POINTER(ctypes.c_size_t), i32, vp]
        L.spc_pack_coords_noalloc.argtypes = [vp, i64, ctypes.POINTER(PackDesc), vp, vp, i32, vp]
        L.spc_build_kmap.argtypes = [vp, i64, ctypes.POINTER(PackDesc), ctypes.POINTER(LayerDesc), ctypes.POINTER(vp), vp]
        L.spc_build_kmap_perm.argtypes = [vp, i64, vp, ctypes.POINTER(PackDesc), ctypes.POINTER(LayerDesc), ctypes.POINTER(vp), vp]
        L.spc_build_kmaps_network.argtypes = [vp, i64, ctypes.POINTER(PackDesc), ctypes.POINTER(LayerDesc), i32,
                                              ctypes.POINTER(vp), ctypes.POINTER(vp), i32, i32]
        for f in ("spc_kmap_n_in", "spc_kmap_n_out"):
            getattr(L, f).argtypes = [vp]
            getattr(L, f).restype = i64
        L.spc_kmap_kvol.argtypes = [vp]
        for f in ("spc_kmap_out_keys", "spc_kmap_in_keys", "spc_kmap_os_map"):
            getattr(L, f).argtypes = [vp]
            getattr(L, f).restype = vp
        L.spc_kmap_copy_out_keys.argtypes = [vp, vp, i64]
        L.spc_kmap_ws_lists.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(i64)]
        L.spc_kmap_nnz.argtypes = [vp, ctypes.POINTER(i64)]
        L.spc_kmap_search_info.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.spc_search_count.restype = i64
        L.spc_kmap_export_triples.argtypes = [vp, i32, vp, i64, ctypes.POINTER(i64)]
        L.spc_kmap_set_size_hint.argtypes = [vp, i64]
        L.spc_kmap_destroy.argtypes = [vp]
        L.spc_kmap_destroy.restype = None
        L.spc_conv_forward.argtypes = [vp, vp, i64, vp, vp, i64, i32, i32, i32, i32, i32, vp]
        L.spc_conv_forward_hybrid.argtypes = [vp, vp, i64, vp, vp, i64, i32, i32, i32, i32, i32, vp]
        L.spc_conv_prepare_weights.argtypes = [vp, i32, i32, i32, i32, vp, vp]
        L.spc_conv_tune_threshold.argtypes = [vp, vp, i64, vp, vp, vp, i64, i32, i32, i32, i32, i32, ctypes.c_float,
                                              ctypes.POINTER(ctypes.c_float), i32, ctypes.POINTER(i32), ctypes.POINTER(i32), vp]
        L.spc_permute_rows.argtypes = [vp, i64, vp, i64, i64, vp, i64, vp]
        L.spc_probe_copy.argtypes = [vp, vp, i64, vp]
        L.spc_probe_mfma.argtypes = [i32, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.spc_last_error.restype = ctypes.c_char_p
        L.spc_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != OK:
        raise SpcError(rc, lib().spc_last_error().decode())


def _stream(stream=None) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream) if hasattr(s, "cuda_stream") else int(s)


def _dev_ptr(t: torch.Tensor) -> int:
    assert t.is_cuda and t.is_contiguous()
    return t.data_ptr()


_TORCH_DTYPE = {torch.float16: DTYPE_F16, torch.bfloat16: DTYPE_BF16, torch.float32: DTYPE_F32}


def spc_version() -> str:
    return lib().spc_version().decode()


def spc_pack_desc_fit(lo, hi, n_batch: int = 1, max_stride: int = 1, max_reach: int = 1, key_bits: int = 0) -> PackDesc:
    d = PackDesc()
    a = (ctypes.c_int32 * 3)(*[int(v) for v in lo])
    b = (ctypes.c_int32 * 3)(*[int(v) for v in hi])
    _check(lib().spc_pack_desc_fit(a, b, n_batch, max_stride, max_reach, key_bits, ctypes.byref(d)))
    return d


def spc_pack_workspace_bytes(n: int, desc: PackDesc) -> int:
    need = ctypes.c_size_t(0)
    _check(lib().spc_pack_coords(None, n, ctypes.byref(desc), None, None, None, ctypes.byref(need), 0, None))
    return int(need.value)


def spc_pack_coords(coords: torch.Tensor, desc: PackDesc, want_perm: bool = True, flags: int = 0, stream=None,
                    workspace: torch.Tensor | None = None, keys_out: torch.Tensor | None = None,
                    perm_out: torch.Tensor | None = None):
    """coords: int32 [N,4] device tensor (b,x,y,z).  Returns (keys, perm): sorted packed keys
    (int32/int64 tensors holding the unsigned bit patterns) and the permutation (or None)."""
    assert coords.dtype == torch.int32 and coords.dim() == 2 and coords.shape[1] == 4
    n = coords.shape[0]
    if workspace is None:
        workspace = torch.empty(spc_pack_workspace_bytes(n, desc), dtype=torch.uint8, device=coords.device)
    kdt = torch.int32 if desc.key_bits == 32 else torch.int64
    keys = keys_out if keys_out is not None else torch.empty(n, dtype=kdt, device=coords.device)
    assert keys.dtype == kdt and keys.numel() == n
    perm = None
    if want_perm:
        perm = perm_out if perm_out is not None else torch.empty(n, dtype=torch.int32, device=coords.device)
        assert perm.dtype == torch.int32 and perm.numel() == n
    size = ctypes.c_size_t(workspace.numel())
    _check(lib().spc_pack_coords(_dev_ptr(coords), n, ctypes.byref(desc), _dev_ptr(keys),
                                 _dev_ptr(perm) if want_perm else None, _dev_ptr(workspace), ctypes.byref(size), flags,
                                 _stream(stream)))
    return keys, perm


NOALLOC_MAX_N = 262144


def spc_pack_coords_noalloc(coords: torch.Tensor, desc: PackDesc, keys_out: torch.Tensor, perm_out: torch.Tensor | None,
                            flags: int = 0, stream=None) -> None:
    """spc_pack_coords on the library's static scratch buffer: the caller passes inputs and outputs only."""
    assert coords.dtype == torch.int32 and coords.dim() == 2 and coords.shape[1] == 4
    n = coords.shape[0]
    assert keys_out.dtype == (torch.int32 if desc.key_bits == 32 else torch.int64) and keys_out.numel() == n
    assert perm_out is None or (perm_out.dtype == torch.int32 and perm_out.numel() == n)
    _check(lib().spc_pack_coords_noalloc(_dev_ptr(coords), n, ctypes.byref(desc), _dev_ptr(keys_out),
                                         _dev_ptr(perm_out) if perm_out is not None else None, flags, _stream(stream)))


class KMap:
    """Owner of one spc_kmap handle (keeps the key tensor it points into alive)."""

    def __init__(self, handle: int, keep=(), desc: PackDesc | None = None):
        self.handle = ctypes.c_void_p(handle)
        self._keep = keep
        self.desc = desc

    def destroy(self):
        if self.handle:
            lib().spc_kmap_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    @property
    def n_in(self) -> int:
        v = lib().spc_kmap_n_in(self.handle)
        if v < 0:
            _check(int(v))
        return int(v)

    @property
    def n_out(self) -> int:
        v = lib().spc_kmap_n_out(self.handle)
        if v < 0:
            _check(int(v))
        return int(v)

    def set_size_hint(self, n_out_hint: int) -> None:
        _check(lib().spc_kmap_set_size_hint(self.handle, int(n_out_hint)))

    @property
    def kvol(self) -> int:
        return int(lib().spc_kmap_kvol(self.handle))

    def nnz(self):
        import numpy as np
        out = np.zeros(self.kvol, dtype=np.int64)
        _check(lib().spc_kmap_nnz(self.handle, out.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))))
        return out

    def export_triples(self, which: int = LAYOUT_OS):
        import numpy as np
        nnz = ctypes.c_int64(0)
        _check(lib().spc_kmap_export_triples(self.handle, which, None, 0, ctypes.byref(nnz)))
        t = np.empty((nnz.value, 3), dtype=np.int32)
        _check(lib().spc_kmap_export_triples(self.handle, which, t.ctypes.data_as(ctypes.c_void_p), nnz.value,
                                             ctypes.byref(nnz)))
        return t

    def out_keys(self):
        """Host copy of the layer's sorted output keys (as uint64)."""
        import numpy as np
        n = self.n_out
        a = np.empty(n, dtype=np.uint32 if self.desc.key_bits == 32 else np.uint64)
        _check(lib().spc_kmap_copy_out_keys(self.handle, a.ctypes.data_as(ctypes.c_void_p), n))
        return a.astype(np.uint64)


def spc_search_count() -> int:
    """Kernel-map searches enqueued by this process so far."""
    return int(lib().spc_search_count())


def spc_kmap_search_info(kmap: KMap):
    """(rows per search tile, input keys the tile's windows may occupy in LDS)."""
    t, w = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().spc_kmap_search_info(kmap.handle, ctypes.byref(t), ctypes.byref(w)))
    return int(t.value), int(w.value)


def spc_build_kmap(in_keys: torch.Tensor, desc: PackDesc, K: int, in_stride: int = 1, layer_stride: int = 1,
                   transposed: int = 0, layout: int = LAYOUT_BOTH, stream=None, in_perm: torch.Tensor | None = None) -> KMap:
    """in_perm: the permutation returned by spc_pack_coords; the map then addresses the caller's unsorted
    feature rows (spc_build_kmap_perm)."""
    l = LayerDesc(K, in_stride, layer_stride, transposed, layout)
    h = ctypes.c_void_p()
    if in_perm is None:
        _check(lib().spc_build_kmap(_dev_ptr(in_keys), in_keys.shape[0], ctypes.byref(desc), ctypes.byref(l), ctypes.byref(h),
                                    _stream(stream)))
        return KMap(h.value, keep=(in_keys,), desc=desc)
    assert in_perm.dtype == torch.int32 and in_perm.shape[0] == in_keys.shape[0]
    _check(lib().spc_build_kmap_perm(_dev_ptr(in_keys), in_keys.shape[0], _dev_ptr(in_perm), ctypes.byref(desc), ctypes.byref(l),
                                     ctypes.byref(h), _stream(stream)))
    return KMap(h.value, keep=(in_keys, in_perm), desc=desc)


def spc_build_kmaps_network(v0_keys: torch.Tensor, desc: PackDesc, layers, streams=None, flags: int = 0):
    """layers: sequence of (K, in_stride, layer_stride, transposed, layout).  Returns one KMap per layer
    (layers with equal (K, in_stride, layer_stride, transposed) share the underlying map)."""
    n = len(layers)
    arr = (LayerDesc * n)(*[LayerDesc(*[int(v) for v in l]) for l in layers])
    out = (ctypes.c_void_p * n)()
    if streams is None:
        streams = [torch.cuda.current_stream()]
    sarr = (ctypes.c_void_p * len(streams))(*[_stream(s) for s in streams])
    _check(lib().spc_build_kmaps_network(_dev_ptr(v0_keys), v0_keys.shape[0], ctypes.byref(desc), arr, n, out, sarr,
                                         len(streams), flags))
    return [KMap(out[i], keep=(v0_keys,), desc=desc) for i in range(n)]


def spc_conv_forward(kmap: KMap, feats_in: torch.Tensor, weights: torch.Tensor, dataflow: int = DATAFLOW_OS,
                     flags: int = 0, out: torch.Tensor | None = None, n_out: int | None = None, stream=None,
                     hybrid_t: int | None = None) -> torch.Tensor:
    """feats_in [n_in, cin] (row pitch = stride(0)), weights [K^3, cin, cout] contiguous.  ``out`` may be a
    column slice of a wider buffer (row pitch = stride(0)); it is allocated when None.  hybrid_t: threshold of the
    hybrid dual dataflow (spc_conv_forward_hybrid); `dataflow` is ignored then."""
    assert feats_in.is_cuda and weights.is_cuda and weights.is_contiguous()
    assert feats_in.dim() == 2 and feats_in.stride(1) == 1 and weights.dim() == 3
    assert feats_in.dtype == weights.dtype and feats_in.dtype in _TORCH_DTYPE
    cin, cout = feats_in.shape[1], weights.shape[2]
    # (prepacked weights hold their input channels padded to a multiple of 16)
    assert weights.shape[1] == ((cin + 15) // 16 * 16 if flags & CONV_PACKED_WEIGHTS else cin) and weights.shape[0] == kmap.kvol
    if out is None:
        out = torch.empty((n_out if n_out is not None else kmap.n_out, cout), dtype=feats_in.dtype, device=feats_in.device)
    assert out.dim() == 2 and out.stride(1) == 1 and out.shape[1] == cout and out.dtype == feats_in.dtype
    if hybrid_t is not None:
        _check(lib().spc_conv_forward_hybrid(kmap.handle, feats_in.data_ptr(), feats_in.stride(0), weights.data_ptr(),
                                             out.data_ptr(), out.stride(0), cin, cout, _TORCH_DTYPE[feats_in.dtype], int(hybrid_t),
                                             flags, _stream(stream)))
        return out
    _check(lib().spc_conv_forward(kmap.handle, feats_in.data_ptr(), feats_in.stride(0), weights.data_ptr(), out.data_ptr(),
                                  out.stride(0), cin, cout, _TORCH_DTYPE[feats_in.dtype], dataflow, flags, _stream(stream)))
    return out


def spc_conv_tune_threshold(kmap: KMap, feats_in: torch.Tensor, weights: torch.Tensor, packed: torch.Tensor | None = None,
                            flags: int = 0, reps: int = 5, ws_build_us: float = 0.0, out: torch.Tensor | None = None,
                            stream=None):
    """One-time tuning of a layer's hybrid threshold (spc_conv_tune_threshold).  Returns (best t, [microseconds for
    t = 0 .. L1max + 1], output computed with the best t)."""
    assert feats_in.is_cuda and weights.is_cuda and weights.is_contiguous() and weights.dim() == 3
    assert feats_in.dim() == 2 and feats_in.stride(1) == 1 and feats_in.dtype == weights.dtype and feats_in.dtype in _TORCH_DTYPE
    cin, cout = weights.shape[1], weights.shape[2]
    assert feats_in.shape[1] == cin and weights.shape[0] == kmap.kvol
    assert packed is None or (packed.is_cuda and packed.is_contiguous() and packed.dtype == weights.dtype
                              and packed.numel() == weights.shape[0] * ((weights.shape[1] + 15) // 16 * 16) * weights.shape[2])
    if out is None:
        out = torch.empty((kmap.n_out, cout), dtype=feats_in.dtype, device=feats_in.device)
    assert out.dim() == 2 and out.stride(1) == 1 and out.shape[1] == cout and out.dtype == feats_in.dtype
    cap = 64
    us = (ctypes.c_float * cap)()
    n_t, best = ctypes.c_int32(0), ctypes.c_int32(-1)
    _check(lib().spc_conv_tune_threshold(kmap.handle, feats_in.data_ptr(), feats_in.stride(0), weights.data_ptr(),
                                         packed.data_ptr() if packed is not None else None, out.data_ptr(), out.stride(0), cin,
                                         cout, _TORCH_DTYPE[feats_in.dtype], flags, int(reps), float(ws_build_us), us, cap,
                                         ctypes.byref(n_t), ctypes.byref(best), _stream(stream)))
    return int(best.value), [float(us[i]) for i in range(n_t.value)], out


def spc_conv_prepare_weights(weights: torch.Tensor, out: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """weights [K^3, cin, cout] fp16/bf16 -> the MFMA operand layout expected with CONV_PACKED_WEIGHTS."""
    assert weights.is_cuda and weights.is_contiguous() and weights.dim() == 3 and weights.dtype in _TORCH_DTYPE
    cin16 = (weights.shape[1] + 15) // 16 * 16  # input channels are padded with zeros to a multiple of 16
    if out is None:
        out = torch.empty((weights.shape[0], cin16, weights.shape[2]), dtype=weights.dtype, device=weights.device)
    assert out.is_contiguous() and out.dtype == weights.dtype and out.numel() == weights.shape[0] * cin16 * weights.shape[2]
    _check(lib().spc_conv_prepare_weights(weights.data_ptr(), weights.shape[0], weights.shape[1], weights.shape[2],
                                          _TORCH_DTYPE[weights.dtype], out.data_ptr(), _stream(stream)))
    return out


def spc_permute_rows(src: torch.Tensor, perm: torch.Tensor, out: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """out[r] = src[perm[r]] (feature rows into sorted-voxel order)."""
    assert src.is_cuda and src.dim() == 2 and src.stride(1) == 1 and perm.dtype == torch.int32
    if out is None:
        out = torch.empty((perm.shape[0], src.shape[1]), dtype=src.dtype, device=src.device)
    es = src.element_size()
    _check(lib().spc_permute_rows(src.data_ptr(), src.stride(0) * es, perm.data_ptr(), perm.shape[0], src.shape[1] * es,
                                  out.data_ptr(), out.stride(0) * es, _stream(stream)))
    return out


def spc_probe_copy(src: torch.Tensor, dst: torch.Tensor, stream=None) -> int:
    """dst = src by the library's plain copy kernel; returns the bytes moved one way."""
    assert src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size()
    _check(lib().spc_probe_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream(stream)))
    return nbytes


def spc_probe_mfma(iters: int, sink: torch.Tensor, stream=None) -> float:
    """Enqueues the register-resident MFMA loop; returns the floating-point operations of the launch."""
    flops = ctypes.c_double(0.0)
    _check(lib().spc_probe_mfma(int(iters), sink.data_ptr(), ctypes.byref(flops), _stream(stream)))
    return float(flops.value)


def spc_release_cache() -> None:
    _check(lib().spc_release_cache())
