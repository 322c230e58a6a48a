"""Randomised parity of the whole map path (pack + sort, levels, kernel map, layouts, features) against the
oracle: each seed draws a cloud shape (dense box, sparse box, slabs with few x values, clusters, long z columns,
negative coordinates), the layer's K, strides and direction, the layouts, the key width and whether the sort
permutation is folded into the map.  The seeds are fixed; what they draw is printed with a failure."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_20834_amd import binding as B, synth
from gpu_common import fit_desc, gpu_pack, keys_to_u64, oracle_keys, oracle_layer, assert_close

pytestmark = pytest.mark.gpu


def _random_cloud(rng):
    kind = int(rng.integers(0, 6))
    nb = int(rng.integers(1, 4))
    if kind == 0:  # dense small box
        d = rng.integers(4, 24, 3)
        n = int(rng.integers(1, int(np.prod(d)) * nb // 2 + 2))
        c = np.stack([rng.integers(0, nb, n), rng.integers(0, d[0], n), rng.integers(0, d[1], n), rng.integers(0, d[2], n)], 1)
    elif kind == 1:  # sparse large box
        n = int(rng.integers(100, 60000))
        d = rng.integers(50, 2000, 3)
        c = np.stack([rng.integers(0, nb, n), rng.integers(0, d[0], n), rng.integers(0, d[1], n),
                      rng.integers(0, min(d[2], 300), n)], 1)
    elif kind == 2:  # slabs: few x values with many voxels each (large sort bins, large search windows)
        n = int(rng.integers(2000, 40000))
        nx = int(rng.integers(1, 6))
        c = np.stack([np.zeros(n, int), rng.integers(0, nx, n) * int(rng.integers(1, 50)), rng.integers(0, 400, n),
                      rng.integers(0, 200, n)], 1)
    elif kind == 3:  # clusters
        n = int(rng.integers(500, 30000))
        k = int(rng.integers(1, 8))
        centres = rng.integers(0, 800, (k, 3))
        c = np.concatenate([rng.integers(0, nb, (n, 1)),
                            centres[rng.integers(0, k, n)] + rng.normal(0, rng.uniform(1, 12), (n, 3)).astype(int)], 1)
    elif kind == 4:  # columns along z (long z runs)
        m, L = int(rng.integers(5, 300)), int(rng.integers(2, 120))
        xy = rng.integers(0, 60, (m, 2))
        z = np.arange(L)[:, None]
        c = np.concatenate([np.concatenate([np.zeros((L, 1), int), np.repeat(xy[i:i + 1], L, 0), z + rng.integers(-3, 3)], 1)
                            for i in range(m)])
    else:  # a few voxels around the origin, negative coordinates included
        n = int(rng.integers(1, 200))
        c = np.concatenate([np.zeros((n, 1), int), rng.integers(-40, 40, (n, 3))], 1)
    c = np.unique(c.astype(np.int32), axis=0)
    rng.shuffle(c, axis=0)
    return c


def _canon(t):
    return t[np.lexsort((t[:, 2], t[:, 1], t[:, 0]))]


@pytest.mark.parametrize("seed", range(48))
def test_random_layer(seed):
    rng = np.random.default_rng(7000021 + seed)
    c = _random_cloud(rng)
    K = int(rng.choice([1, 2, 3, 3, 3, 5, 7]))
    s_p = int(rng.choice([1, 1, 2, 4]))
    s_l = int(rng.choice([1, 1, 2])) if K != 2 else 2
    tr = int(rng.integers(0, 2)) if (s_l == 2 and K in (2, 3)) else 0
    key_bits = int(rng.choice([0, 0, 64]))
    lname, layout = (("os", B.LAYOUT_OS), ("ws", B.LAYOUT_WS), ("both", B.LAYOUT_BOTH))[int(rng.integers(0, 3))]
    submanifold_odd = K % 2 == 1 and K > 1 and s_l == 1
    hyb = None
    if lname == "both" and submanifold_odd and rng.integers(0, 2):
        hyb = int(rng.integers(1, 3 * (K - 1) // 2 + 1))
        layout |= B.LAYOUT_HYBRID_T(hyb)
    sym = bool(lname == "ws" and submanifold_odd and rng.integers(0, 2))
    if sym:
        layout |= B.LAYOUT_WS_SYM
    with_perm = bool(lname != "ws" and s_p == 1 and not tr and rng.integers(0, 2))
    tag = dict(seed=seed, n=len(c), K=K, s_p=s_p, s_l=s_l, tr=tr, key_bits=key_bits, layout=lname, hybrid_t=hyb, sym=sym,
               perm=with_perm)

    desc = fit_desc(c, [(K, s_p, s_l)], key_bits)
    keys, perm = gpu_pack(c, desc)
    cs, operm = oracle.sort_coords(c)
    assert np.array_equal(perm.cpu().numpy(), operm), tag
    assert np.array_equal(keys_to_u64(keys), oracle_keys(cs, desc)), tag
    cin, cout, M = oracle_layer(cs, K, s_p, s_l, tr)
    if s_p == 1 and not tr:
        km = B.spc_build_kmap(keys, desc, K, 1, s_l, 0, layout, in_perm=perm if with_perm else None)
    else:  # the layer's levels come from the stride-1 cloud
        km = B.spc_build_kmaps_network(keys, desc, [(K, s_p, s_l, tr, layout)])[0]
    ref_t = oracle.triples(M)
    if with_perm:
        ref_t[:, 1] = operm[ref_t[:, 1]]
    ref_t = _canon(ref_t)
    assert km.n_out == len(cout), tag
    assert np.array_equal(km.out_keys(), oracle_keys(cout, desc)), tag
    if hyb is None:
        for which in (B.LAYOUT_OS, B.LAYOUT_WS):
            if layout & which:
                assert np.array_equal(_canon(km.export_triples(which)), ref_t), (tag, which)
    else:  # each offset is held by one of the two layouts
        both = np.concatenate([km.export_triples(B.LAYOUT_OS), km.export_triples(B.LAYOUT_WS)])
        assert np.array_equal(_canon(both), ref_t), tag
    assert np.array_equal(km.nnz(), np.bincount(ref_t[:, 0], minlength=K ** 3)), tag

    if len(cin) <= 20000 and K <= 5:
        c_in, c_out = int(rng.choice([16, 32, 40])), int(rng.choice([16, 32, 64]))
        F = synth.features(len(c) if with_perm else len(cin), c_in, np.float16, seed=seed)
        W = synth.weights(K ** 3, c_in, c_out, np.float16, seed=seed + 1)
        ref = oracle.conv(M, (F[operm] if with_perm else F).astype(np.float64), W.astype(np.float64))
        Ft, Wt = torch.from_numpy(F).cuda(), torch.from_numpy(W).cuda()
        if hyb is not None:
            runs = [dict(hybrid_t=hyb)]
        else:
            runs = [dict(dataflow=d) for d, which in ((B.DATAFLOW_OS, B.LAYOUT_OS), (B.DATAFLOW_WS, B.LAYOUT_WS)) if layout & which]
        for kw in runs:
            y = B.spc_conv_forward(km, Ft, Wt, **kw)
            assert_close(y.cpu().double().numpy(), ref, 1e-2, (tag, kw))
    km.destroy()
