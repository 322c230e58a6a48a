"""CPU oracle of the sparse-convolution layer — TEST INFRASTRUCTURE ONLY.

Only the tests, ``__graft_entry__.smoke()`` and the benchmark's ``cpu_baseline``
leg may import this package.  It never imports the HIP package and shares no
code with it.  The arithmetic lives in ``spc_oracle.cpp`` (plain C++, hash-map
lookup, fp64 accumulation); this file marshals numpy arrays and strings the
per-layer functions into the layer stack of a network.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spc_oracle.cpp")
_LIB = os.path.join(_HERE, "libspc_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C++ oracle with g++ (OpenMP on) into ``oracle/libspc_oracle.so``."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-fopenmp", "-shared", "-fPIC", _SRC, "-o", tmp])
        os.replace(tmp, _LIB)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_downsample.restype = ctypes.c_int64
        _lib.orc_triples.restype = ctypes.c_int64
        _lib.orc_pack_keys.restype = ctypes.c_int64
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    return int(lib().orc_num_threads())


def set_threads(n: int) -> None:
    lib().orc_set_threads(int(n))


def sort_coords(coords) -> tuple[np.ndarray, np.ndarray]:
    """Rows of ``coords`` [N,4] in lexicographic (b,x,y,z) order and the permutation
    ``perm`` with ``sorted = coords[perm]``.  Raises on duplicate rows."""
    c = _i32(coords)
    perm = np.empty(c.shape[0], dtype=np.int64)
    if lib().orc_sort_coords(_p(c), ctypes.c_int64(c.shape[0]), _p(perm)):
        raise ValueError("duplicate voxel coordinates")
    return c[perm], perm


def downsample(coords, s_q: int) -> np.ndarray:
    c = _i32(coords)
    out = np.empty_like(c)
    n = lib().orc_downsample(_p(c), ctypes.c_int64(c.shape[0]), ctypes.c_int32(s_q), _p(out))
    return out[:n].copy()


def offsets(K: int, s_p: int) -> np.ndarray:
    off = np.empty((K ** 3, 3), dtype=np.int32)
    lib().orc_offsets(ctypes.c_int32(K), ctypes.c_int32(s_p), _p(off))
    return off


def kernel_map(in_coords, out_coords, K: int, s_p: int) -> np.ndarray:
    a, b = _i32(in_coords), _i32(out_coords)
    M = np.empty((b.shape[0], K ** 3), dtype=np.int32)
    lib().orc_kernel_map(_p(a), ctypes.c_int64(a.shape[0]), _p(b), ctypes.c_int64(b.shape[0]),
                         ctypes.c_int32(K), ctypes.c_int32(s_p), _p(M))
    return M


def kernel_map_transposed(coarse_coords, fine_coords, K: int, s_fine: int) -> np.ndarray:
    a, b = _i32(coarse_coords), _i32(fine_coords)
    M = np.empty((b.shape[0], K ** 3), dtype=np.int32)
    lib().orc_kernel_map_transposed(_p(a), ctypes.c_int64(a.shape[0]), _p(b), ctypes.c_int64(b.shape[0]),
                                    ctypes.c_int32(K), ctypes.c_int32(s_fine), _p(M))
    return M


def triples(M) -> np.ndarray:
    """Canonical sorted (offset, in, out) triples of a kernel map."""
    M = _i32(M)
    t = np.empty((M.size, 3), dtype=np.int32)
    nnz = lib().orc_triples(_p(M), ctypes.c_int64(M.shape[0]), ctypes.c_int32(M.shape[1]), _p(t))
    return t[:nnz].copy()


def conv(M, F, W) -> np.ndarray:
    """Eq. (2) in fp64.  ``F`` [N,Cin] and ``W`` [K^3,Cin,Cout] are converted exactly."""
    M = _i32(M)
    F = np.ascontiguousarray(F, dtype=np.float64)
    W = np.ascontiguousarray(W, dtype=np.float64)
    assert W.shape[0] == M.shape[1] and W.shape[1] == F.shape[1]
    assert M.size == 0 or M.max() < F.shape[0]
    out = np.empty((M.shape[0], W.shape[2]), dtype=np.float64)
    lib().orc_conv(_p(M), ctypes.c_int64(M.shape[0]), ctypes.c_int32(M.shape[1]), _p(F), _p(W),
                   ctypes.c_int32(W.shape[1]), ctypes.c_int32(W.shape[2]), _p(out))
    return out


def pack_keys(coords, bits_b: int, bits_x: int, bits_y: int, bits_z: int, origin, pad: int):
    """Packed keys (uint64) of ``coords``; second value = rows that do not fit."""
    c = _i32(coords)
    o = _i32(origin)
    keys = np.empty(c.shape[0], dtype=np.uint64)
    bad = lib().orc_pack_keys(_p(c), ctypes.c_int64(c.shape[0]), ctypes.c_int32(bits_b), ctypes.c_int32(bits_x),
                              ctypes.c_int32(bits_y), ctypes.c_int32(bits_z), _p(o), ctypes.c_int32(pad), _p(keys))
    return keys, int(bad)


def layer(coords_sorted, K: int, s_p: int, s_l: int):
    """Output coordinates and kernel map of one layer on sorted input coordinates."""
    out = coords_sorted if s_l == 1 else downsample(coords_sorted, s_p * s_l)
    return out, kernel_map(coords_sorted, out, K, s_p)


def network_forward(coords_sorted, F0, layers, weights, act_dtype=np.float16, inputs_override=None):
    """Layer stack on the CPU: every layer is Eq. (2) in fp64, followed by ReLU (where the
    layer says so) and rounding of the activations to ``act_dtype`` (round to nearest
    even), because activations are stored in that type between layers.  ``layers`` is a
    list of dicts (K, in_stride, layer_stride, transposed, src, skip, save, relu).
    Returns (dict of saved tensors as float64 arrays holding act_dtype values, list of
    per-layer kernel maps)."""
    levels = {1: coords_sorted}

    def level(s):
        if s not in levels:
            levels[s] = downsample(coords_sorted, s)
        return levels[s]

    T = {"input": np.asarray(F0, dtype=np.float64)}
    maps = []
    for j, l in enumerate(layers):
        K, sp, sl = l["K"], l["in_stride"], l["layer_stride"]
        fine = level(sp)
        if sl == 1:
            M = kernel_map(fine, fine, K, sp)
        elif not l["transposed"]:
            M = kernel_map(fine, level(sp * sl), K, sp)
        else:
            M = kernel_map_transposed(level(sp * sl), fine, K, sp)
        maps.append(M)
        if inputs_override is not None:
            x = inputs_override[j]
        else:
            x = T[l["src"]] if l["skip"] is None else np.concatenate([T[l["src"]], T[l["skip"]]], axis=1)
        y = conv(M, x, np.asarray(weights[j], dtype=np.float64))
        if l["relu"]:
            y = np.maximum(y, 0.0)
        T[l["save"]] = y.astype(act_dtype).astype(np.float64)
        T["_raw_%d" % j] = y
    return T, maps
