"""Pins of the CPU oracle against things other than itself: values printed in the
paper, hand-worked cases, brute force, closed forms on full grids, dense
convolutions from PyTorch's CPU library, and algebraic invariants."""
import os

import numpy as np
import pytest
import torch

from paper_2511_20834_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _lines(name):
    with open(os.path.join(GOLD, name)) as f:
        return [l.split() for l in f if l.strip() and not l.startswith("#")]


def _bxyz(xyz, b=0):
    xyz = np.asarray(xyz, dtype=np.int32).reshape(-1, 3)
    return np.concatenate([np.full((len(xyz), 1), b, np.int32), xyz], 1)


# ----------------------------------------------------------------------------- offsets
def test_offsets_delta_5_2_matches_paper(orc):
    vals = [int(v) for v in _lines("offsets_delta_5_2.txt")[0]]
    off = orc.offsets(5, 2)
    assert off.shape == (125, 3)
    expect = {(a, b, c) for a in vals for b in vals for c in vals}
    assert {tuple(r) for r in off.tolist()} == expect and len(expect) == 125
    # z fastest, then y, then x
    assert off[0].tolist() == [-4, -4, -4] and off[1].tolist() == [-4, -4, -2] and off[5].tolist() == [-4, -2, -4]


def test_offsets_group0_and_queries_match_paper(orc):
    rows = [[int(v) for v in r] for r in _lines("query_group0.txt")]
    q, group0, queries = np.array(rows[0]), np.array(rows[1:4]), np.array(rows[4:7])
    off = orc.offsets(3, 1)
    assert np.array_equal(off[:3], group0)
    assert np.array_equal(q + off[:3], queries)
    # an input cloud holding exactly those three queries is hit by offsets 0,1,2 of that output voxel
    cin, _ = orc.sort_coords(_bxyz(np.concatenate([queries, q[None]])))
    M = orc.kernel_map(cin, _bxyz(q[None]), 3, 1)
    assert M[0, :3].tolist() == [0, 1, 2] and M[0, 13] == 3 and (M[0] >= 0).sum() == 4


def test_offsets_even_kernel(orc):
    off = orc.offsets(2, 4)
    assert off.tolist() == [[0, 0, 0], [0, 0, 4], [0, 4, 0], [0, 4, 4], [4, 0, 0], [4, 0, 4], [4, 4, 0], [4, 4, 4]]


# ----------------------------------------------------------------------------- sort / downsample
def test_sort_matches_numpy_lexsort(orc):
    c = synth.random_cloud(3000, (40, 30, 20), seed=5, batch=3)
    c[:, 1:] -= 10  # negative coordinates too
    s, perm = orc.sort_coords(c)
    ref = np.lexsort((c[:, 3], c[:, 2], c[:, 1], c[:, 0]))
    assert np.array_equal(perm, ref) and np.array_equal(s, c[ref])
    with pytest.raises(ValueError):
        orc.sort_coords(np.concatenate([c, c[:1]]))


def test_downsample_floor_unique_sorted(orc):
    c = synth.random_cloud(4000, (50, 50, 50), seed=6, batch=2)
    c[:, 1:] -= 25
    for s_q in (2, 4, 8):
        got = orc.downsample(c, s_q)
        ref = c.copy()
        ref[:, 1:] = np.floor(c[:, 1:].astype(np.float64) / s_q).astype(np.int32) * s_q
        ref = np.unique(ref, axis=0)  # numpy's row-unique sorts lexicographically
        assert np.array_equal(got, ref)
    # floor, not truncation: -1 -> -2 at stride 2
    assert orc.downsample(_bxyz([[-1, -3, 5]]), 2).tolist() == [[0, -2, -4, 4]]


def test_downsample_closed_form_equals_recursion(orc):
    """Section 5.5: V_i = floor(V_0 / 2^i) 2^i equals level-by-level downsampling."""
    c, _ = orc.sort_coords(synth.tiny_cloud())
    c[:, 1:] -= 20
    level = c
    for i in range(1, 5):
        level = orc.downsample(level, 2 ** i)
        assert np.array_equal(level, orc.downsample(c, 2 ** i))


# ----------------------------------------------------------------------------- kernel map
def _brute_map(cin, cout, off):
    M = np.full((len(cout), len(off)), -1, np.int32)
    for i, q in enumerate(cout):
        for k, d in enumerate(off):
            tgt = q + np.array([0, d[0], d[1], d[2]])
            hit = np.nonzero((cin == tgt).all(1))[0]
            if hit.size:
                assert hit.size == 1
                M[i, k] = hit[0]
    return M


@pytest.mark.parametrize("K,s_p,s_l", [(3, 1, 1), (3, 1, 2), (5, 1, 1), (2, 1, 2), (3, 2, 1), (3, 2, 2), (2, 2, 2)])
def test_kernel_map_brute_force(orc, K, s_p, s_l):
    c = synth.random_cloud(150, (9, 8, 7), seed=11 + K, batch=2)
    c[:, 1:] -= 3
    c, _ = orc.sort_coords(c)
    if s_p > 1:
        c = orc.downsample(c, s_p)
    out, M = orc.layer(c, K, s_p, s_l)
    # written-out offsets, not the oracle's
    if K % 2:
        ax = [(i - (K - 1) // 2) * s_p for i in range(K)]
    else:
        ax = [i * s_p for i in range(K)]
    off = [(a, b, d) for a in ax for b in ax for d in ax]
    assert np.array_equal(M, _brute_map(c, out, off))


def test_kernel_map_handworked(orc):
    cases, cur = [], None
    for t in _lines("handworked_maps.txt"):
        if t[0] == "case":
            cur = dict(name=t[1], K=int(t[2]), s_p=int(t[3]), s_l=int(t[4]), i=[], o=[], t=[])
            cases.append(cur)
        else:
            cur[t[0][0]].append([int(v) for v in t[1:]])
    assert len(cases) == 4
    for c in cases:
        cin = _bxyz(c["i"])
        s, _ = orc.sort_coords(cin)
        assert np.array_equal(s, cin), "fixture inputs are listed in sorted order"
        out, M = orc.layer(cin, c["K"], c["s_p"], c["s_l"])
        assert np.array_equal(out, _bxyz(c["o"])), c["name"]
        assert orc.triples(M).tolist() == c["t"], c["name"]


def test_kernel_map_full_grid_closed_form(orc):
    n, K = 6, 3
    g = synth.full_grid(n)
    M = orc.kernel_map(g, g, K, 1)
    i = np.arange(n ** 3)
    x, y, z = i // (n * n), (i // n) % n, i % n
    for k in range(27):
        dx, dy, dz = k // 9 - 1, (k // 3) % 3 - 1, k % 3 - 1
        ok = (x + dx >= 0) & (x + dx < n) & (y + dy >= 0) & (y + dy < n) & (z + dz >= 0) & (z + dz < n)
        assert np.array_equal(M[:, k], np.where(ok, i + dx * n * n + dy * n + dz, -1))
        assert (M[:, k] >= 0).sum() == (n - abs(dx)) * (n - abs(dy)) * (n - abs(dz))


def test_kernel_map_invariants_submanifold(orc):
    c, _ = orc.sort_coords(synth.tiny_cloud())
    for K in (3, 5):
        M = orc.kernel_map(c, c, K, 1)
        K3 = K ** 3
        assert np.array_equal(M[:, K3 // 2], np.arange(len(c)))  # centre offset maps i -> i (Section 4)
        for k in range(K3):  # symmetry (Section 5.4): (i,j) at k  <=>  (j,i) at K^3-1-k
            i = np.nonzero(M[:, k] >= 0)[0]
            j = M[i, k]
            assert np.array_equal(M[j, K3 - 1 - k], i)
            assert np.all(np.diff(j) > 0)  # per-offset lists are monotone in both indices
        nnz = (M >= 0).sum(0)
        assert np.array_equal(nnz, nnz[::-1])


def test_kernel_map_downsample_k2_partitions_inputs(orc):
    """K=2 at layer stride 2: every input voxel lies in exactly one output cell."""
    c, _ = orc.sort_coords(synth.tiny_cloud())
    out, M = orc.layer(c, 2, 1, 2)
    hit = M[M >= 0]
    assert hit.size == len(c) and np.array_equal(np.sort(hit), np.arange(len(c)))
    # and the transposed map is the same set of pairs with the roles swapped
    Mt = orc.kernel_map_transposed(out, c, 2, 1)
    t, tt = orc.triples(M), orc.triples(Mt)
    assert np.array_equal(np.array(sorted(map(tuple, tt[:, [0, 2, 1]].tolist()))), t)


def test_kernel_map_batches_do_not_mix(orc):
    a = _bxyz([[0, 0, 0], [0, 0, 1]], 0)
    b = _bxyz([[0, 0, 2]], 1)
    c = np.concatenate([a, b])
    M = orc.kernel_map(c, c, 3, 1)
    assert (M[2] >= 0).sum() == 1 and M[2, 13] == 2 and M[1, 14] == -1


# ----------------------------------------------------------------------------- features
def _dense_from_sparse(c, F, lo, shape):
    g = torch.zeros((1, F.shape[1]) + tuple(shape), dtype=torch.float64)
    idx = c[:, 1:] - lo
    g[0, :, idx[:, 0], idx[:, 1], idx[:, 2]] = torch.from_numpy(F.T.copy())
    return g


def test_conv_k1_is_gemm(orc):
    rng = np.random.default_rng(0)
    F, W = rng.normal(size=(50, 7)), rng.normal(size=(1, 7, 5))
    M = np.arange(50, dtype=np.int32)[:, None]
    assert np.allclose(orc.conv(M, F, W), F @ W[0], rtol=1e-13, atol=1e-13)


def test_conv_selector_weights(orc):
    c, _ = orc.sort_coords(synth.tiny_cloud())
    M = orc.kernel_map(c, c, 3, 1)
    rng = np.random.default_rng(1)
    F = rng.normal(size=(len(c), 4))
    for k in (0, 13, 20):
        W = np.zeros((27, 4, 4))
        W[k] = np.eye(4)
        ref = np.where(M[:, k:k + 1] >= 0, F[np.maximum(M[:, k], 0)], 0.0)
        assert np.array_equal(orc.conv(M, F, W), ref)


def test_conv_linearity(orc):
    c, _ = orc.sort_coords(synth.tiny_cloud())
    M = orc.kernel_map(c, c, 3, 1)
    rng = np.random.default_rng(2)
    F1, F2 = rng.normal(size=(2, len(c), 3))
    W1, W2 = rng.normal(size=(2, 27, 3, 6))
    assert np.allclose(orc.conv(M, F1 + 2 * F2, W1), orc.conv(M, F1, W1) + 2 * orc.conv(M, F2, W1), atol=1e-12)
    assert np.allclose(orc.conv(M, F1, W1 - W2), orc.conv(M, F1, W1) - orc.conv(M, F1, W2), atol=1e-12)


@pytest.mark.parametrize("K,s_l", [(3, 1), (5, 1), (3, 2), (2, 2)])
def test_conv_equals_dense_convolution(orc, K, s_l):
    """Scatter the cloud into a zero grid, run PyTorch's dense fp64 3-D
    cross-correlation, read back at the active output sites."""
    c, _ = orc.sort_coords(synth.tiny_cloud())
    c = c[(c[:, 1] < 40) & (c[:, 2] < 40)]  # 40 x 40 x 64 crop keeps the dense run small
    cin_ch, cout_ch = 3, 4
    rng = np.random.default_rng(3)
    F = rng.normal(size=(len(c), cin_ch))
    W = rng.normal(size=(K ** 3, cin_ch, cout_ch))
    out_c, M = orc.layer(c, K, 1, s_l)
    got = orc.conv(M, F, W)
    dense = _dense_from_sparse(c, F, np.zeros(3, np.int64), (40, 40, 64))
    wt = torch.from_numpy(W.reshape(K, K, K, cin_ch, cout_ch)).permute(4, 3, 0, 1, 2).contiguous()
    pad = (K - 1) // 2 if K % 2 else 0
    res = torch.nn.functional.conv3d(dense, wt, stride=s_l, padding=pad)[0]
    # with padding r (odd K) dense output site o is centred on input s_l*o; even K starts at s_l*o
    idx = out_c[:, 1:] // s_l
    ref = res[:, idx[:, 0], idx[:, 1], idx[:, 2]].T.numpy()
    assert np.allclose(got, ref, rtol=1e-11, atol=1e-11)


def test_transposed_conv_equals_dense_conv_transpose(orc):
    c, _ = orc.sort_coords(synth.tiny_cloud())
    c = c[(c[:, 1] < 40) & (c[:, 2] < 40)]
    coarse = orc.downsample(c, 2)
    Mt = orc.kernel_map_transposed(coarse, c, 2, 1)
    rng = np.random.default_rng(4)
    Fc = rng.normal(size=(len(coarse), 3))
    W = rng.normal(size=(8, 3, 5))
    got = orc.conv(Mt, Fc, W)
    cc = coarse.copy()
    cc[:, 1:] //= 2
    dense = _dense_from_sparse(cc, Fc, np.zeros(3, np.int64), (20, 20, 32))
    wt = torch.from_numpy(W.reshape(2, 2, 2, 3, 5)).permute(3, 4, 0, 1, 2).contiguous()  # [Cin, Cout, kx, ky, kz]
    res = torch.nn.functional.conv_transpose3d(dense, wt, stride=2)[0]
    ref = res[:, c[:, 1], c[:, 2], c[:, 3]].T.numpy()
    assert np.allclose(got, ref, rtol=1e-11, atol=1e-11)


# ----------------------------------------------------------------------------- packing
def test_pack_layout_12_12_8(orc):
    """Section 5.3: 12/12/8 bits, x in the top bits: key = x<<20 | y<<8 | z."""
    c = _bxyz([[1, 2, 3], [4095, 0, 255], [17, 4000, 9]])
    keys, bad = orc.pack_keys(c, 0, 12, 12, 8, [0, 0, 0], 0)
    assert bad == 0
    assert keys.tolist() == [(1 << 20) | (2 << 8) | 3, (4095 << 20) | 255, (17 << 20) | (4000 << 8) | 9]
    _, bad = orc.pack_keys(_bxyz([[4096, 0, 0], [0, 0, 256], [0, -1, 0]]), 0, 12, 12, 8, [0, 0, 0], 0)
    assert bad == 3


def test_pack_order_and_additivity(orc):
    """Section 5.3: packing preserves lexicographic order, and
    packed(q) + packed(delta) = packed(q + delta) while no field over- or underflows."""
    c = synth.random_cloud(2000, (60, 50, 40), seed=9, batch=3)
    c[:, 1:] -= 20
    origin, pad, bits = [-20, -20, -20], 4, (2, 7, 7, 6)
    keys, bad = orc.pack_keys(c, *bits, origin, pad)
    assert bad == 0
    s, perm = orc.sort_coords(c)
    assert np.array_equal(np.argsort(keys, kind="stable"), perm)
    # round trip
    k = keys.astype(np.int64)
    z = (k & 63) - pad + origin[2]
    y = ((k >> 6) & 127) - pad + origin[1]
    x = ((k >> 13) & 127) - pad + origin[0]
    b = k >> 20
    assert np.array_equal(np.stack([b, x, y, z], 1), c)
    for d in orc.offsets(5, 2):
        pd = int(d[0]) * (1 << 13) + int(d[1]) * (1 << 6) + int(d[2])  # signed packed offset
        # the sum is the key of the shifted voxel: its fields decode to q + delta (the shifted voxel itself
        # may lie in the guard band, where the packer accepts no input rows)
        kd = k + pd
        dec = np.stack([kd >> 20, ((kd >> 13) & 127) - pad + origin[0], ((kd >> 6) & 127) - pad + origin[1],
                        (kd & 63) - pad + origin[2]], 1)
        shifted = c.copy()
        shifted[:, 1:] += d
        assert np.array_equal(dec, shifted)


def test_pack_guard_band_rule(orc):
    """Section 5.3 (reading of the silent point): a field stores v - origin + pad and a row is accepted
    only if the guard band fits on both sides, 0 <= v - origin and v - origin + 2 pad < 2^bits, which is
    exactly the condition under which adding any packed offset with |component| <= pad stays inside the
    field.  Hand-worked edge rows: 7-bit fields, pad 4, origin -20: v - origin in [0, 119] is accepted."""
    bits, origin, pad = (0, 7, 7, 7), [-20, -20, -20], 4
    edge = _bxyz([[-20, -20, -20], [99, 99, 99], [-20, 99, -20]])
    keys, bad = orc.pack_keys(edge, *bits, origin, pad)
    assert bad == 0
    assert keys.tolist() == [(4 << 14) | (4 << 7) | 4, (123 << 14) | (123 << 7) | 123, (4 << 14) | (123 << 7) | 4]
    # one step into either guard band is rejected although the biased value would still fit the field
    for row in ([-21, 0, 0], [0, 100, 0], [0, 0, -21], [100, 0, 0], [0, 0, 103]):
        k, bad = orc.pack_keys(_bxyz([row]), *bits, origin, pad)
        assert bad == 1 and k[0] == np.uint64(0xFFFFFFFFFFFFFFFF), row
    # accepted extremes plus any offset of reach <= pad decode to the shifted voxel (no borrow, no carry)
    k = keys.astype(np.int64)
    for d in ([-4, -4, -4], [4, 4, 4], [-4, 4, 0]):
        kd = k + d[0] * (1 << 14) + d[1] * (1 << 7) + d[2]
        dec = np.stack([(kd >> 14) & 127, (kd >> 7) & 127, kd & 127], 1) - pad + np.array(origin)
        assert np.array_equal(dec, edge[:, 1:] + np.array(d))


# ----------------------------------------------------------------------------- transposed maps
def _axis_offsets(K, s):
    return [(i - (K - 1) // 2) * s for i in range(K)] if K % 2 else [i * s for i in range(K)]


@pytest.mark.parametrize("K,s_fine", [(2, 1), (3, 1), (3, 2), (2, 2), (5, 1)])
def test_kernel_map_transposed_brute_force(orc, K, s_fine):
    """Reading for transposed layers: pair (coarse j, fine i, k) iff fine_i = coarse_j + delta_k with
    delta_k from Delta(K, s_fine); checked against an O(N^2) scan with written-out offsets, and
    against the strided layer's triples with the roles swapped."""
    c = synth.random_cloud(160, (9, 8, 7), seed=31 + K, batch=2)
    c[:, 1:] -= 3
    c, _ = orc.sort_coords(c)
    fine = orc.downsample(c, s_fine) if s_fine > 1 else c
    coarse = orc.downsample(fine, 2 * s_fine)
    Mt = orc.kernel_map_transposed(coarse, fine, K, s_fine)
    ax = _axis_offsets(K, s_fine)
    off = [(a, b, d) for a in ax for b in ax for d in ax]
    ref = np.full((len(fine), K ** 3), -1, np.int32)
    for i, f in enumerate(fine):
        for k, d in enumerate(off):
            src = f - np.array([0, d[0], d[1], d[2]])
            hit = np.nonzero((coarse == src).all(1))[0]
            if hit.size:
                assert hit.size == 1
                ref[i, k] = hit[0]
    assert np.array_equal(Mt, ref)
    M = orc.kernel_map(fine, coarse, K, s_fine)  # the strided twin
    t, tt = orc.triples(M), orc.triples(Mt)
    assert np.array_equal(np.array(sorted(map(tuple, tt[:, [0, 2, 1]].tolist()))).reshape(-1, 3), t)


@pytest.mark.parametrize("s_fine", [1, 2])
def test_transposed_conv_k3_equals_dense_conv_transpose(orc, s_fine):
    """K=3 transposed layer at layer stride 2 = dense conv_transpose3d(kernel 3, stride 2, padding 1)
    sampled at the active fine voxels (the strided twin is conv3d(kernel 3, stride 2, padding 1))."""
    c, _ = orc.sort_coords(synth.tiny_cloud())
    c = c[(c[:, 1] < 40) & (c[:, 2] < 40)]
    fine = orc.downsample(c, s_fine) if s_fine > 1 else c
    coarse = orc.downsample(fine, 2 * s_fine)
    Mt = orc.kernel_map_transposed(coarse, fine, 3, s_fine)
    rng = np.random.default_rng(14)
    Fc = rng.normal(size=(len(coarse), 3))
    W = rng.normal(size=(27, 3, 5))
    got = orc.conv(Mt, Fc, W)
    cc = coarse.copy()
    cc[:, 1:] //= 2 * s_fine
    dims = (40 // (2 * s_fine), 40 // (2 * s_fine), 64 // (2 * s_fine))
    dense = _dense_from_sparse(cc, Fc, np.zeros(3, np.int64), dims)
    wt = torch.from_numpy(W.reshape(3, 3, 3, 3, 5)).permute(3, 4, 0, 1, 2).contiguous()  # [Cin, Cout, kx, ky, kz]
    res = torch.nn.functional.conv_transpose3d(dense, wt, stride=2, padding=1, output_padding=1)[0]
    fi = fine[:, 1:] // s_fine
    ref = res[:, fi[:, 0], fi[:, 1], fi[:, 2]].T.numpy()
    assert np.allclose(got, ref, rtol=1e-11, atol=1e-11)


# ----------------------------------------------------------------------------- layer stack
def _chain_layers():
    """Two-level UNet-style chain with unequal widths everywhere, so that a swapped concat order, a
    transposed layer reading the wrong level or a misplaced ReLU / rounding changes the result."""
    L = [
        dict(name="stem", K=3, in_stride=1, layer_stride=1, transposed=0, cin=3, cout=4, src="input", skip=None, save="enc0"),
        dict(name="down1", K=2, in_stride=1, layer_stride=2, transposed=0, cin=4, cout=6, src="enc0", skip=None, save="d1"),
        dict(name="enc1", K=3, in_stride=2, layer_stride=1, transposed=0, cin=6, cout=7, src="d1", skip=None, save="enc1"),
        dict(name="down2", K=2, in_stride=2, layer_stride=2, transposed=0, cin=7, cout=8, src="enc1", skip=None, save="d2"),
        dict(name="enc2", K=3, in_stride=4, layer_stride=1, transposed=0, cin=8, cout=8, src="d2", skip=None, save="enc2"),
        dict(name="up2", K=2, in_stride=2, layer_stride=2, transposed=1, cin=8, cout=5, src="enc2", skip=None, save="u2"),
        dict(name="dec2", K=3, in_stride=2, layer_stride=1, transposed=0, cin=12, cout=6, src="u2", skip="enc1", save="dec2"),
        dict(name="up1", K=2, in_stride=1, layer_stride=2, transposed=1, cin=6, cout=5, src="dec2", skip=None, save="u1"),
        dict(name="dec1", K=3, in_stride=1, layer_stride=1, transposed=0, cin=9, cout=3, src="u1", skip="enc0", save="dec1"),
    ]
    for j, l in enumerate(L):
        l["relu"] = j != len(L) - 1
    return L


def test_network_forward_equals_dense_chain(orc):
    """The layer stack (ReLU after every layer but the last, activations rounded to fp16 with round to
    nearest even between layers, skip concatenation [up | skip], transposed layers writing the finer
    level) against the same chain of dense fp64 convolutions from PyTorch's CPU library on the
    zero-filled grid, masked to the active voxels of every level."""
    lo = np.array([-8, -8, -8])
    c, _ = orc.sort_coords(synth.tiny_cloud())
    c = c[(c[:, 1] < 24) & (c[:, 2] < 24) & (c[:, 3] < 32)]
    c[:, 1:] += lo  # negative coordinates: floor, not truncation, in the level derivation
    c, _ = orc.sort_coords(c)
    dims = np.array([24, 24, 32])
    layers = _chain_layers()
    rng = np.random.default_rng(21)
    F0 = rng.normal(size=(len(c), 3)).astype(np.float16).astype(np.float64)
    Ws = [rng.normal(size=(l["K"] ** 3, l["cin"], l["cout"])) * np.sqrt(2.0 / (l["K"] ** 3 * l["cin"])) for l in layers]
    Ws = [w.astype(np.float16).astype(np.float64) for w in Ws]
    T, maps = orc.network_forward(c, F0, layers, Ws)

    # dense side: level s lives on the grid dims / s; mask[s] marks its active voxels
    level = {1: c}
    for s in (2, 4):
        lv = c.copy()
        lv[:, 1:] = np.floor(c[:, 1:].astype(np.float64) / s).astype(np.int32) * s
        level[s] = np.unique(lv, axis=0)

    def cells(s):
        return ((level[s][:, 1:] - lo) // s).T

    mask = {}
    for s in (1, 2, 4):
        m = torch.zeros((1, 1) + tuple(dims // s), dtype=torch.float64)
        ix = cells(s)
        m[0, 0, ix[0], ix[1], ix[2]] = 1.0
        mask[s] = m
    D = {"input": _dense_from_sparse(c, F0, lo, dims)}
    conv3d, convT = torch.nn.functional.conv3d, torch.nn.functional.conv_transpose3d
    for l, W in zip(layers, Ws):
        K, s = l["K"], l["in_stride"]
        x = D[l["src"]] if l["skip"] is None else torch.cat([D[l["src"]], D[l["skip"]]], dim=1)
        w5 = torch.from_numpy(W.reshape(K, K, K, l["cin"], l["cout"]))
        if l["layer_stride"] == 1:
            y, so = conv3d(x, w5.permute(4, 3, 0, 1, 2).contiguous(), padding=1), s
        elif not l["transposed"]:
            y, so = conv3d(x, w5.permute(4, 3, 0, 1, 2).contiguous(), stride=2), 2 * s
        else:
            y, so = convT(x, w5.permute(3, 4, 0, 1, 2).contiguous(), stride=2), s
        y = y * mask[so]
        if l["relu"]:
            y = torch.relu(y)
        D[l["save"]] = y.to(torch.float16).to(torch.float64)
        ix = cells(so)
        ref = D[l["save"]][0][:, ix[0], ix[1], ix[2]].T.numpy()
        got = T[l["save"]]
        assert got.shape == ref.shape, l["name"]
        assert np.allclose(got, ref, rtol=1e-9, atol=1e-9), l["name"]
    # the stack's result is not trivially zero anywhere along the way
    assert all(np.abs(T[l["save"]]).max() > 1e-3 for l in layers)
