"""Helpers shared by the GPU parity tests: run the HIP path through the C-ABI binding
and the CPU oracle on the same seeded inputs."""
import numpy as np
import torch

import oracle
from paper_2511_20834_amd import binding as B


def reach_of(K, in_stride):
    return ((K - 1) // 2 if K % 2 else (K - 1)) * in_stride


def fit_desc(coords, layers, key_bits=0):
    """layers: iterable of (K, in_stride, layer_stride)."""
    lo, hi = coords[:, 1:].min(0), coords[:, 1:].max(0)
    n_batch = int(coords[:, 0].max()) + 1
    max_stride = max(s * l for _, s, l in layers)
    max_reach = max(reach_of(K, s) for K, s, _ in layers)
    return B.spc_pack_desc_fit(lo, hi, n_batch, max_stride, max_reach, key_bits)


def gpu_pack(coords, desc, flags=0):
    c = torch.from_numpy(np.ascontiguousarray(coords, dtype=np.int32)).cuda()
    keys, perm = B.spc_pack_coords(c, desc, True, flags)
    return keys, perm


def keys_to_u64(keys_t):
    a = keys_t.cpu().numpy()
    return a.view(np.uint32).astype(np.uint64) if a.dtype == np.int32 else a.view(np.uint64)


def oracle_keys(coords_sorted, desc):
    k, bad = oracle.pack_keys(coords_sorted, desc.bits_b, desc.bits_x, desc.bits_y, desc.bits_z, list(desc.origin), desc.pad)
    assert bad == 0
    return k


def oracle_level(coords_sorted, stride):
    return coords_sorted if stride == 1 else oracle.downsample(coords_sorted, stride)


def oracle_layer(c0_sorted, K, in_stride, layer_stride, transposed=0):
    """(in coords, out coords, M) of a layer whose levels derive from the stride-1 cloud."""
    fine = oracle_level(c0_sorted, in_stride)
    if layer_stride == 1:
        return fine, fine, oracle.kernel_map(fine, fine, K, in_stride)
    coarse = oracle.downsample(fine, in_stride * layer_stride)
    if not transposed:
        return fine, coarse, oracle.kernel_map(fine, coarse, K, in_stride)
    return coarse, fine, oracle.kernel_map_transposed(coarse, fine, K, in_stride)


def rel_err(got, ref):
    """max |y - yhat| / max |yhat| (the tolerance reading stated in the design notes)."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    den = np.abs(ref).max() if ref.size else 1.0
    return float(np.abs(got - ref).max() / max(den, 1e-30)) if ref.size else 0.0


def assert_close(got, ref, tol, what=None):
    """Both forms of the tolerance: max|y - yhat| / max|yhat| <= tol, and element by element
    |y - yhat| <= tol * (|yhat| + rms(yhat)), so that small-magnitude outputs cannot be
    arbitrarily wrong under a global bound set by the largest one."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), what
    err = rel_err(got, ref)
    assert err <= tol, (what, err)
    rms = np.sqrt((ref ** 2).mean())
    excess = np.abs(got - ref) - tol * (np.abs(ref) + rms)
    assert excess.max() <= 0, (what, "element-wise bound exceeded by", float(excess.max()), "at", int(excess.argmax()))
    return err


def to_torch(a, dtype):
    """numpy (fp16/fp32 values) -> device tensor of the given torch dtype; also returns the
    exact fp64 values the device tensor holds (what the oracle must be fed)."""
    t = torch.from_numpy(np.ascontiguousarray(a)).to(dtype).cuda()
    return t, t.cpu().to(torch.float64).numpy()
