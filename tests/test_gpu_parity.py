"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.
Kernel maps must be bit-exact (sorted (offset, in, out) triples); features within
max|y - yhat| / max|yhat| <= 1e-2 for fp16/bf16 inputs with fp32 accumulation and
1e-5 in fp32 mode."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_20834_amd import binding as B
from paper_2511_20834_amd import synth

from gpu_common import (assert_close, fit_desc, gpu_pack, keys_to_u64, oracle_keys, oracle_layer, rel_err, to_torch)

pytestmark = pytest.mark.gpu

TOL = {torch.float16: 1e-2, torch.bfloat16: 1e-2, torch.float32: 1e-5}


def _cloud(name):
    if name == "tiny":
        return synth.tiny_cloud()
    if name == "tiny_neg":
        c = synth.tiny_cloud()
        c[:, 1:] -= 33
        return c
    if name == "rand_b3":
        c = synth.random_cloud(5000, (37, 29, 23), seed=3, batch=3)
        c[:, 1:] -= 7
        return c
    if name == "grid":
        return synth.full_grid(12, batch=2)
    if name == "ragged":
        return synth.random_cloud(128 * 5 + 1, (30, 30, 30), seed=4)
    if name == "one":
        return np.array([[0, 5, 6, 7]], np.int32)
    if name.startswith("rand_n"):  # sizes around the switch between the library sort and the bucket sort
        n = int(name[6:])
        c = synth.random_cloud(n, (300, 280, 40), seed=40 + n % 7, batch=2)[:n]
        c[:, 1:] -= 100
        return c
    if name == "skew_60k":  # half of the voxels in 3 of 400 x-planes: bins of very different sizes
        a = synth.random_cloud(30000, (400, 200, 60), seed=51)
        b = synth.random_cloud(30000, (3, 200, 60), seed=52)
        b[:, 1] += 197
        c = np.unique(np.concatenate([a, b]), axis=0)
        np.random.default_rng(53).shuffle(c, axis=0)
        return c
    if name in ("slab_3k", "slab_12k"):
        # a dense two-voxel-thick slab in a wide scene: thousands of keys share the sort's top bits
        ny = 25 if name == "slab_3k" else 100
        g = np.stack(np.meshgrid(np.arange(500, 502), np.arange(ny), np.arange(60), indexing="ij"), -1).reshape(-1, 3)
        far = np.array([[0, 0, 0], [1000, 3, 7], [250, 90, 59]])
        c = np.concatenate([g, far]).astype(np.int32)
        c = np.concatenate([np.zeros((len(c), 1), np.int32), c], 1)
        np.random.default_rng(12).shuffle(c, axis=0)
        return c
    raise KeyError(name)


def _check_map(c0_sorted, keys_t, desc, K, s_p, s_l, transposed, kmap):
    cin, cout, M = oracle_layer(c0_sorted, K, s_p, s_l, transposed)
    assert kmap.n_in == len(cin) and kmap.n_out == len(cout)
    assert np.array_equal(kmap.out_keys(), oracle_keys(cout, desc))
    ref = oracle.triples(M)
    got_os = kmap.export_triples(B.LAYOUT_OS)
    got_ws = kmap.export_triples(B.LAYOUT_WS)
    assert np.array_equal(got_os, ref)
    assert np.array_equal(got_ws, ref)
    assert np.array_equal(kmap.nnz(), np.bincount(ref[:, 0], minlength=K ** 3))
    return cin, cout, M


# ----------------------------------------------------------------------------- pack + sort
@pytest.mark.parametrize("name,key_bits", [("tiny", 0), ("tiny_neg", 0), ("rand_b3", 0), ("rand_b3", 64), ("one", 0),
                                           ("slab_3k", 0), ("slab_12k", 0), ("slab_12k", 64), ("ragged", 64),
                                           ("rand_n4095", 0), ("rand_n4096", 0), ("rand_n4097", 64), ("rand_n70001", 0),
                                           ("rand_n70001", 64), ("skew_60k", 0), ("skew_60k", 64),
                                           ("rand_n600001", 0)])  # 64 count/scatter workgroups, ten thousand rank workgroups
def test_pack_sort_matches_oracle(name, key_bits):
    c = _cloud(name)
    desc = fit_desc(c, [(3, 1, 2)], key_bits)
    keys, perm = gpu_pack(c, desc, B.PACK_VALIDATE)
    cs, operm = oracle.sort_coords(c)
    assert np.array_equal(keys_to_u64(keys), oracle_keys(cs, desc))
    assert np.array_equal(perm.cpu().numpy().astype(np.int64), operm)


@pytest.mark.parametrize("key_bits", [0, 64])
def test_pack_sort_repeated_voxels_still_give_a_permutation(key_bits):
    """Repeated voxels are not a valid cloud, but unless validation is asked for they are sorted like any
    other input: the keys come out in order and the permutation is complete (runs of equal keys longer
    than a rank workgroup's 64 positions, across several of them, and a run of three)."""
    base = synth.random_cloud(9000, (120, 90, 40), seed=81)
    rng = np.random.default_rng(82)
    c = np.concatenate([base, np.repeat(base[100:101], 700, axis=0), np.repeat(base[4000:4001], 2, axis=0),
                        base[rng.integers(0, len(base), 1500)]])
    rng.shuffle(c, axis=0)
    desc = fit_desc(c, [(3, 1, 1)], key_bits)
    keys, perm = gpu_pack(c, desc)
    k_ref, bad = oracle.pack_keys(c, desc.bits_b, desc.bits_x, desc.bits_y, desc.bits_z, list(desc.origin), desc.pad)
    assert bad == 0
    got = keys_to_u64(keys)
    pm = perm.cpu().numpy().astype(np.int64)
    assert np.array_equal(np.sort(pm), np.arange(len(c)))
    assert np.array_equal(got, np.sort(k_ref))
    assert np.array_equal(k_ref[pm], got)


def test_pack_validate_errors():
    c = _cloud("tiny")
    desc = fit_desc(c, [(3, 1, 1)])
    bad = c.copy()
    bad[5, 1] = 10_000
    with pytest.raises(B.SpcError) as e:
        gpu_pack(bad, desc, B.PACK_VALIDATE)
    assert e.value.code == B.ERR_RANGE
    dup = np.concatenate([c, c[7:8]])
    with pytest.raises(B.SpcError) as e:
        gpu_pack(dup, desc, B.PACK_VALIDATE)
    assert e.value.code == B.ERR_DUP
    # the same two errors on a cloud large enough for the bucket sort
    big = _cloud("rand_n70001")
    dbig = fit_desc(big, [(3, 1, 1)])
    bad = big.copy()
    bad[12345, 2] = -20_000
    with pytest.raises(B.SpcError) as e:
        gpu_pack(bad, dbig, B.PACK_VALIDATE)
    assert e.value.code == B.ERR_RANGE
    with pytest.raises(B.SpcError) as e:
        gpu_pack(np.concatenate([big, big[777:778]]), dbig, B.PACK_VALIDATE)
    assert e.value.code == B.ERR_DUP
    desc.bits_x = 31
    with pytest.raises(B.SpcError) as e:
        gpu_pack(c, desc)
    assert e.value.code == B.ERR_ARG


# ----------------------------------------------------------------------------- kernel maps
@pytest.mark.parametrize("name,K,s_l,transposed,key_bits", [
    ("tiny", 3, 1, 0, 0), ("tiny_neg", 3, 1, 0, 0), ("tiny", 5, 1, 0, 0), ("tiny", 7, 1, 0, 0), ("tiny", 1, 1, 0, 0),
    ("tiny", 3, 2, 0, 0), ("tiny_neg", 2, 2, 0, 0), ("tiny_neg", 2, 2, 1, 0), ("tiny", 3, 2, 1, 0),
    ("rand_b3", 3, 1, 0, 0), ("rand_b3", 3, 2, 0, 64), ("rand_b3", 5, 1, 0, 64), ("rand_b3", 2, 2, 1, 64),
    ("grid", 3, 1, 0, 0), ("ragged", 3, 1, 0, 0), ("ragged", 5, 1, 0, 0), ("one", 3, 1, 0, 0), ("one", 2, 2, 1, 0),
])
def test_kmap_bit_exact(name, K, s_l, transposed, key_bits):
    c = _cloud(name)
    desc = fit_desc(c, [(K, 1, s_l)], key_bits)
    keys, _ = gpu_pack(c, desc)
    cs, _ = oracle.sort_coords(c)
    km = B.spc_build_kmap(keys, desc, K, 1, s_l, transposed, B.LAYOUT_BOTH)
    _check_map(cs, keys, desc, K, 1, s_l, transposed, km)
    km.destroy()


def test_kmap_on_coarse_level():
    """A layer whose input is already a strided level (s_p = 2 and 4)."""
    c = _cloud("tiny_neg")
    desc = fit_desc(c, [(3, 4, 2)])
    keys, _ = gpu_pack(c, desc)
    cs, _ = oracle.sort_coords(c)
    down = B.spc_build_kmap(keys, desc, 2, 1, 2, 0, B.LAYOUT_OS)
    k2 = torch.from_numpy(down.out_keys().astype(np.uint32).view(np.int32)).cuda()
    for K, s_l in ((3, 1), (3, 2), (2, 2)):
        km = B.spc_build_kmap(k2, desc, K, 2, s_l, 0, B.LAYOUT_BOTH)
        _check_map(cs, k2, desc, K, 2, s_l, 0, km)
        km.destroy()
    down.destroy()


@pytest.mark.parametrize("name,key_bits", [("rand_n70001", 0), ("rand_n70001", 64), ("skew_60k", 0), ("slab_12k", 0),
                                           ("slab_12k", 64), ("rand_n4097", 0), ("rand_n600001", 0)])
def test_downsampled_levels_match_oracle(name, key_bits):
    """Levels 2, 4 and 8 straight from V_0 (Section 5.5) on clouds large enough for the library's own
    sort path: dense slabs (thousands of keys in one bin), skewed densities, both key widths."""
    c = _cloud(name)
    desc = fit_desc(c, [(2, 4, 2)], key_bits)
    keys, _ = gpu_pack(c, desc)
    cs, _ = oracle.sort_coords(c)
    maps = B.spc_build_kmaps_network(keys, desc, [(2, s, 2, 0, B.LAYOUT_OS) for s in (1, 2, 4)])
    for m, stride in zip(maps, (2, 4, 8)):
        ref = oracle_keys(oracle.downsample(cs, stride), desc)
        assert m.n_out == len(ref)
        assert np.array_equal(m.out_keys(), ref), stride
    for m in maps:
        m.destroy()


def test_kmap_empty_input():
    desc = B.spc_pack_desc_fit([0, 0, 0], [10, 10, 10], 1, 2, 1)
    keys = torch.empty(0, dtype=torch.int32, device="cuda")
    for s_l in (1, 2):
        km = B.spc_build_kmap(keys, desc, 3, 1, s_l, 0, B.LAYOUT_BOTH)
        assert km.n_out == 0 and km.export_triples(B.LAYOUT_OS).shape == (0, 3) and km.nnz().sum() == 0
        km.destroy()


def test_kmap_bad_arguments():
    desc = B.spc_pack_desc_fit([0, 0, 0], [10, 10, 10], 1, 2, 1)
    keys = torch.zeros(4, dtype=torch.int32, device="cuda")
    for args, code in (((4, 1, 1, 0, 3), B.ERR_UNSUPPORTED), ((3, 3, 1, 0, 3), B.ERR_ARG), ((3, 1, 1, 1, 3), B.ERR_ARG),
                       ((3, 1, 1, 0, 0), B.ERR_ARG)):
        with pytest.raises(B.SpcError) as e:
            B.spc_build_kmap(keys, desc, *args)
        assert e.value.code == code
    # descriptors that do not suit the layer (Section 5.3): guard band below the reach; field bias
    # that is not a multiple of the output stride
    for args in ((7, 1, 1, 0, 3), (2, 4, 2, 0, 3), (3, 1, 4, 0, 3)):
        with pytest.raises(B.SpcError) as e:
            B.spc_build_kmap(keys, desc, *args)
        assert e.value.code == B.ERR_ARG
    with pytest.raises(B.SpcError) as e:
        B.spc_build_kmaps_network(keys, desc, [(3, 1, 1, 0, 1), (3, 4, 1, 0, 1)])
    assert e.value.code == B.ERR_ARG


# ----------------------------------------------------------------------------- features
def _run_conv(c, K, s_l, transposed, cin, cout, dtype, seed=0, relu=False):
    desc = fit_desc(c, [(K, 1, s_l)])
    keys, perm = gpu_pack(c, desc)
    cs, operm = oracle.sort_coords(c)
    km = B.spc_build_kmap(keys, desc, K, 1, s_l, transposed, B.LAYOUT_BOTH)
    ci, co, M = oracle_layer(cs, K, 1, s_l, transposed)
    np_dt = np.float32 if dtype == torch.float32 else np.float16
    F = synth.features(len(ci), cin, np_dt, seed=seed + 1)
    W = synth.weights(K ** 3, cin, cout, np_dt, seed=seed + 2)
    Ft, F64 = to_torch(F, dtype)
    Wt, W64 = to_torch(W, dtype)
    ref = oracle.conv(M, F64, W64)
    if relu:
        ref = np.maximum(ref, 0)
    outs = {}
    # both OS kernels are forced in turn (the flags are ignored where no MFMA kernel runs)
    for df, variant in ((B.DATAFLOW_OS, B.CONV_OS_PHASE), (B.DATAFLOW_OS, B.CONV_OS_SPLITK), (B.DATAFLOW_OS, 0),
                        (B.DATAFLOW_WS, 0)):
        y = B.spc_conv_forward(km, Ft, Wt, df, (B.CONV_RELU if relu else 0) | variant)
        torch.cuda.synchronize()
        o = y.cpu().to(torch.float64).numpy()
        assert_close(o, ref, TOL[dtype], (df, variant))
        outs[df] = o
        outs[(df, variant)] = o
    # weights re-laid once (input channels padded to a multiple of 16 where needed): same kernels, same bits for OS
    if dtype != torch.float32 and cout % 32 == 0:
        packed = B.spc_conv_prepare_weights(Wt)
        assert packed.shape == (K ** 3, (cin + 15) // 16 * 16, cout)
        fl = (B.CONV_RELU if relu else 0) | B.CONV_PACKED_WEIGHTS
        for variant in (B.CONV_OS_PHASE, B.CONV_OS_SPLITK, 0):
            y = B.spc_conv_forward(km, Ft, packed, B.DATAFLOW_OS, fl | variant)
            assert np.array_equal(y.cpu().to(torch.float64).numpy(), outs[(B.DATAFLOW_OS, variant)]), ("packed", variant)
        if cout in (32, 64, 128, 256):
            y = B.spc_conv_forward(km, Ft, packed, B.DATAFLOW_WS, fl)
            assert_close(y.cpu().to(torch.float64).numpy(), ref, TOL[dtype], "packed ws")
    km.destroy()
    return outs, ref


@pytest.mark.parametrize("dtype,cin,cout", [
    (torch.float16, 64, 64), (torch.float16, 32, 32), (torch.float16, 64, 128), (torch.float16, 128, 256),
    (torch.float16, 16, 32), (torch.float16, 80, 64), (torch.bfloat16, 64, 64), (torch.bfloat16, 32, 128),
    (torch.float32, 16, 16), (torch.float32, 5, 7), (torch.float16, 4, 32), (torch.float16, 16, 16), (torch.float16, 24, 40),
    # output-channel slabs (several 64- or 32-wide slabs per layer) and zero-padded input channels
    (torch.float16, 32, 96), (torch.float16, 64, 192), (torch.bfloat16, 16, 320), (torch.float16, 4, 64),
    (torch.float16, 20, 128), (torch.bfloat16, 3, 96), (torch.float16, 1, 32),
])
def test_conv_submanifold_k3(dtype, cin, cout):
    _run_conv(_cloud("tiny"), 3, 1, 0, cin, cout, dtype)


@pytest.mark.parametrize("K,s_l,transposed", [(5, 1, 0), (3, 2, 0), (2, 2, 0), (2, 2, 1), (1, 1, 0), (7, 1, 0)])
def test_conv_other_layers(K, s_l, transposed):
    _run_conv(_cloud("tiny_neg"), K, s_l, transposed, 32, 64, torch.float16, relu=(K == 5))
    _run_conv(_cloud("ragged"), K, s_l, transposed, 6, 10, torch.float32)


def test_conv_selector_weight_checks_map_through_features():
    """W_k = I for one offset: the output must be the gathered input rows exactly."""
    c = _cloud("tiny")
    desc = fit_desc(c, [(3, 1, 1)])
    keys, _ = gpu_pack(c, desc)
    cs, _ = oracle.sort_coords(c)
    km = B.spc_build_kmap(keys, desc, 3)
    M = oracle.kernel_map(cs, cs, 3, 1)
    F = synth.features(len(cs), 32, np.float16, seed=5)
    Ft = torch.from_numpy(F).cuda()
    for k in (0, 13, 22):
        W = np.zeros((27, 32, 32), np.float16)
        W[k] = np.eye(32, dtype=np.float16)
        for df in (B.DATAFLOW_OS, B.DATAFLOW_WS):
            y = B.spc_conv_forward(km, Ft, torch.from_numpy(W).cuda(), df).cpu().numpy()
            ref = np.where(M[:, k:k + 1] >= 0, F[np.maximum(M[:, k], 0)], np.float16(0))
            assert np.array_equal(y, ref)
    km.destroy()


def test_conv_os_is_bit_reproducible_and_ws_stable():
    c = _cloud("rand_b3")
    outs1, _ = _run_conv(c, 3, 1, 0, 64, 64, torch.float16, seed=7)
    outs2, _ = _run_conv(c, 3, 1, 0, 64, 64, torch.float16, seed=7)
    assert np.array_equal(outs1[B.DATAFLOW_OS], outs2[B.DATAFLOW_OS])
    for v in (B.CONV_OS_PHASE, B.CONV_OS_SPLITK):
        assert np.array_equal(outs1[(B.DATAFLOW_OS, v)], outs2[(B.DATAFLOW_OS, v)])
    assert rel_err(outs1[B.DATAFLOW_WS], outs2[B.DATAFLOW_WS]) <= 1e-2


def test_conv_strided_rows_concat_buffer():
    """ld_in / ld_out: read from and write into column slices of wider buffers."""
    c = _cloud("tiny")
    desc = fit_desc(c, [(3, 1, 1)])
    keys, _ = gpu_pack(c, desc)
    cs, _ = oracle.sort_coords(c)
    km = B.spc_build_kmap(keys, desc, 3)
    M = oracle.kernel_map(cs, cs, 3, 1)
    n = len(cs)
    wide_in = torch.from_numpy(synth.features(n, 96, np.float16, seed=8)).cuda()
    W = torch.from_numpy(synth.weights(27, 32, 64, np.float16, seed=9)).cuda()
    wide_out = torch.full((n, 160), 7.0, dtype=torch.float16, device="cuda")
    fin = wide_in[:, 32:64]
    for df in (B.DATAFLOW_OS, B.DATAFLOW_WS):
        B.spc_conv_forward(km, fin, W, df, out=wide_out[:, 64:128])
        ref = oracle.conv(M, fin.cpu().double().numpy(), W.cpu().double().numpy())
        assert_close(wide_out[:, 64:128].cpu().double().numpy(), ref, 1e-2, df)
        assert bool((wide_out[:, :64] == 7).all()) and bool((wide_out[:, 128:] == 7).all())
    km.destroy()


@pytest.mark.parametrize("K,s_l", [(3, 1), (2, 2), (3, 2), (5, 1)])
def test_kmap_with_sort_permutation_folded_in(K, s_l):
    """spc_build_kmap_perm: the stored input indices are the caller's row numbers, so the layer runs on
    the unsorted feature matrix and gives the result of the sorted pipeline."""
    c = _cloud("rand_b3")
    desc = fit_desc(c, [(K, 1, s_l)])
    keys, perm = gpu_pack(c, desc)
    cs, operm = oracle.sort_coords(c)
    km = B.spc_build_kmap(keys, desc, K, 1, s_l, 0, B.LAYOUT_BOTH, in_perm=perm)
    ci, co, M = oracle_layer(cs, K, 1, s_l, 0)
    ref_t = oracle.triples(M)
    ref_t[:, 1] = operm[ref_t[:, 1]]  # sorted position -> original row
    ref_t = ref_t[np.lexsort((ref_t[:, 2], ref_t[:, 0]))]
    for which in (B.LAYOUT_OS, B.LAYOUT_WS):
        got = km.export_triples(which)
        assert np.array_equal(got[np.lexsort((got[:, 2], got[:, 0]))], ref_t), which
    F = synth.features(len(c), 32, np.float16, seed=31)  # rows in the cloud's original order
    W = synth.weights(K ** 3, 32, 64, np.float16, seed=32)
    ref = oracle.conv(M, F[operm].astype(np.float64), W.astype(np.float64))
    for df in (B.DATAFLOW_OS, B.DATAFLOW_WS):
        y = B.spc_conv_forward(km, torch.from_numpy(F).cuda(), torch.from_numpy(W).cuda(), df)
        assert_close(y.cpu().double().numpy(), ref, 1e-2, df)
    km.destroy()
    with pytest.raises(B.SpcError):
        B.spc_build_kmap(keys, desc, 2, 1, 2, 1, B.LAYOUT_OS, in_perm=perm)


@pytest.mark.parametrize("K,dtype,cin,cout", [(3, torch.float16, 32, 64), (5, torch.float16, 32, 32), (3, torch.float32, 6, 10),
                                               (2, torch.bfloat16, 16, 128), (3, torch.float16, 20, 96)])
def test_conv_hybrid_dataflow_every_threshold(K, dtype, cin, cout):
    """Hybrid dual dataflow: offsets with L1 norm < t output-stationary, the rest weight-stationary, for every
    t from 0 (all WS) to one above the largest norm (all OS); every split gives Eq. (2)."""
    c = _cloud("rand_b3")
    s_l = 2 if K == 2 else 1
    desc = fit_desc(c, [(K, 1, s_l)])
    keys, perm = gpu_pack(c, desc)
    cs, operm = oracle.sort_coords(c)
    km = B.spc_build_kmap(keys, desc, K, 1, s_l, 0, B.LAYOUT_BOTH)
    ci, co, M = oracle_layer(cs, K, 1, s_l, 0)
    np_dt = np.float32 if dtype == torch.float32 else np.float16
    F = synth.features(len(ci), cin, np_dt, seed=61)
    W = synth.weights(K ** 3, cin, cout, np_dt, seed=62)
    Ft, F64 = to_torch(F, dtype)
    Wt, W64 = to_torch(W, dtype)
    ref = np.maximum(oracle.conv(M, F64, W64), 0)
    l1_max = 3 if K == 2 else 3 * (K - 1) // 2
    for t in range(0, l1_max + 2):
        for variant in (0, B.CONV_OS_PHASE, B.CONV_OS_SPLITK):
            y = B.spc_conv_forward(km, Ft, Wt, flags=B.CONV_RELU | variant, hybrid_t=t)
            assert_close(y.cpu().to(torch.float64).numpy(), ref, TOL[dtype], (t, variant))
    # the ends of the range are the single dataflows: same kernels, same bits for OS
    y_os = B.spc_conv_forward(km, Ft, Wt, B.DATAFLOW_OS, B.CONV_RELU)
    y_t = B.spc_conv_forward(km, Ft, Wt, flags=B.CONV_RELU, hybrid_t=l1_max + 1)
    assert torch.equal(y_os, y_t)
    # a map without the WS layout serves only the all-OS end
    km_os = B.spc_build_kmap(keys, desc, K, 1, s_l, 0, B.LAYOUT_OS)
    B.spc_conv_forward(km_os, Ft, Wt, hybrid_t=l1_max + 1)
    with pytest.raises(B.SpcError):
        B.spc_conv_forward(km_os, Ft, Wt, hybrid_t=1)
    km_os.destroy()
    km.destroy()


@pytest.mark.parametrize("name,K,s_l,dtype,cin,cout", [("rand_b3", 3, 1, torch.float16, 32, 64), ("tiny_neg", 2, 2, torch.bfloat16, 16, 32),
                                                        ("tiny", 5, 1, torch.float32, 5, 7)])
def test_threshold_tuning_entry_point(name, K, s_l, dtype, cin, cout):
    """spc_conv_tune_threshold (Section 5.4, one-time tuning): one time per threshold, the fastest is reported
    and the output left behind is Eq. (2) computed with it."""
    import ctypes
    c = _cloud(name)
    desc = fit_desc(c, [(K, 1, s_l)])
    keys, _ = gpu_pack(c, desc)
    cs, _ = oracle.sort_coords(c)
    ci, co, M = oracle_layer(cs, K, 1, s_l, 0)
    np_dt = np.float32 if dtype == torch.float32 else np.float16
    Ft, F64 = to_torch(synth.features(len(ci), cin, np_dt, seed=91), dtype)
    Wt, W64 = to_torch(synth.weights(K ** 3, cin, cout, np_dt, seed=92), dtype)
    ref = oracle.conv(M, F64, W64)
    km = B.spc_build_kmap(keys, desc, K, 1, s_l, 0, B.LAYOUT_BOTH)
    l1_max = 3 if K == 2 else 3 * (K - 1) // 2
    packed = B.spc_conv_prepare_weights(Wt) if dtype != torch.float32 else None
    for pk in (None, packed):
        best, us, y = B.spc_conv_tune_threshold(km, Ft, Wt, pk, reps=2, ws_build_us=0.5)
        assert len(us) == l1_max + 2 and all(u > 0 for u in us)
        assert 0 <= best <= l1_max + 1 and us[best] == min(us)
        assert_close(y.cpu().to(torch.float64).numpy(), ref, TOL[dtype], (name, best))
    # the array is too short: the count still comes back
    n_t, b = ctypes.c_int32(0), ctypes.c_int32(0)
    us1 = (ctypes.c_float * 1)()
    out = torch.empty((km.n_out, cout), dtype=dtype, device="cuda")
    rc = B.lib().spc_conv_tune_threshold(km.handle, Ft.data_ptr(), Ft.stride(0), Wt.data_ptr(), None, out.data_ptr(), out.stride(0),
                                         cin, cout, B._TORCH_DTYPE[dtype], 0, 2, 0.0, us1, 1, ctypes.byref(n_t), ctypes.byref(b), None)
    assert rc == B.ERR_ARG and n_t.value == l1_max + 2
    with pytest.raises(B.SpcError):
        B.spc_conv_tune_threshold(km, Ft, Wt, reps=0)
    with pytest.raises(B.SpcError):  # prepacked weights go in their own argument
        B.spc_conv_tune_threshold(km, Ft, Wt, flags=B.CONV_PACKED_WEIGHTS)
    km.destroy()
    for layout in (B.LAYOUT_OS, B.LAYOUT_WS) + ((B.LAYOUT_BOTH | B.LAYOUT_HYBRID_T(1),) if s_l == 1 else ()):
        km = B.spc_build_kmap(keys, desc, K, 1, s_l, 0, layout)
        with pytest.raises(B.SpcError) as e:
            B.spc_conv_tune_threshold(km, Ft, Wt)
        assert e.value.code == B.ERR_ARG
        km.destroy()


@pytest.mark.parametrize("name,K,key_bits,with_os", [("tiny", 3, 0, False), ("tiny_neg", 5, 0, False), ("rand_b3", 3, 64, True),
                                                     ("ragged", 7, 0, False), ("grid", 3, 0, True)])
def test_symmetric_half_map(name, K, key_bits, with_os):
    """WS lists for the first half of the offsets only (submanifold layer): the exported triples, the
    per-offset counts and the features equal those of the full map."""
    c = _cloud(name)
    desc = fit_desc(c, [(K, 1, 1)], key_bits)
    keys, perm = gpu_pack(c, desc)
    cs, _ = oracle.sort_coords(c)
    layout = B.LAYOUT_WS | B.LAYOUT_WS_SYM | (B.LAYOUT_OS if with_os else 0)
    km = B.spc_build_kmap(keys, desc, K, 1, 1, 0, layout)
    M = oracle.kernel_map(cs, cs, K, 1)
    ref_t = oracle.triples(M)
    assert np.array_equal(km.export_triples(B.LAYOUT_WS), ref_t)
    if with_os:
        assert np.array_equal(km.export_triples(B.LAYOUT_OS), ref_t)
    assert np.array_equal(km.nnz(), np.bincount(ref_t[:, 0], minlength=K ** 3))
    for dtype, cin, cout in ((torch.float16, 32, 64), (torch.float32, 5, 7), (torch.bfloat16, 16, 32)):
        np_dt = np.float32 if dtype == torch.float32 else np.float16
        Ft, F64 = to_torch(synth.features(len(cs), cin, np_dt, seed=71), dtype)
        Wt, W64 = to_torch(synth.weights(K ** 3, cin, cout, np_dt, seed=72), dtype)
        ref = oracle.conv(M, F64, W64)
        y = B.spc_conv_forward(km, Ft, Wt, B.DATAFLOW_WS)
        assert_close(y.cpu().to(torch.float64).numpy(), ref, TOL[dtype], (dtype, "ws"))
        if with_os:  # hybrid dual dataflow on top of the half lists
            for t in (1, 2):
                y = B.spc_conv_forward(km, Ft, Wt, hybrid_t=t)
                assert_close(y.cpu().to(torch.float64).numpy(), ref, TOL[dtype], (dtype, t))
    km.destroy()


def test_symmetric_half_map_bad_arguments():
    c = _cloud("tiny")
    desc = fit_desc(c, [(3, 1, 2)])
    keys, _ = gpu_pack(c, desc)
    for K, s_l, tr, layout in ((3, 2, 0, B.LAYOUT_WS | B.LAYOUT_WS_SYM), (2, 2, 1, B.LAYOUT_WS | B.LAYOUT_WS_SYM),
                               (3, 1, 0, B.LAYOUT_OS | B.LAYOUT_WS_SYM), (1, 1, 0, B.LAYOUT_WS | B.LAYOUT_WS_SYM)):
        with pytest.raises(B.SpcError) as e:
            B.spc_build_kmap(keys, desc, K, 1, s_l, tr, layout)
        assert e.value.code == B.ERR_ARG
    keys1, perm1 = gpu_pack(c, fit_desc(c, [(3, 1, 1)]))
    with pytest.raises(B.SpcError) as e:  # swapped roles need one numbering of the rows
        B.spc_build_kmap(keys1, fit_desc(c, [(3, 1, 1)]), 3, 1, 1, 0, B.LAYOUT_WS | B.LAYOUT_WS_SYM, in_perm=perm1)
    assert e.value.code == B.ERR_ARG


def test_conv_unaligned_feature_rows():
    """Rows that do not start on 16-byte boundaries (odd column offset) still give the right result."""
    c = _cloud("tiny")
    desc = fit_desc(c, [(3, 1, 1)])
    keys, _ = gpu_pack(c, desc)
    cs, _ = oracle.sort_coords(c)
    km = B.spc_build_kmap(keys, desc, 3)
    M = oracle.kernel_map(cs, cs, 3, 1)
    wide_in = torch.from_numpy(synth.features(len(cs), 53, np.float16, seed=18)).cuda()
    W = torch.from_numpy(synth.weights(27, 32, 64, np.float16, seed=19)).cuda()
    fin = wide_in[:, 3:35]
    ref = oracle.conv(M, fin.cpu().double().numpy(), W.cpu().double().numpy())
    packed = B.spc_conv_prepare_weights(W)
    for df in (B.DATAFLOW_OS, B.DATAFLOW_WS):
        y = B.spc_conv_forward(km, fin, W, df)
        assert_close(y.cpu().double().numpy(), ref, 1e-2, df)
        y = B.spc_conv_forward(km, fin, packed, df, B.CONV_PACKED_WEIGHTS)
        assert_close(y.cpu().double().numpy(), ref, 1e-2, (df, "packed"))
    km.destroy()


def test_conv_bad_arguments():
    c = _cloud("one")
    desc = fit_desc(c, [(3, 1, 1)])
    keys, _ = gpu_pack(c, desc)
    km = B.spc_build_kmap(keys, desc, 3, layout=B.LAYOUT_OS)
    F = torch.zeros((1, 16), dtype=torch.float16, device="cuda")
    W = torch.zeros((27, 16, 16), dtype=torch.float16, device="cuda")
    with pytest.raises(B.SpcError) as e:
        B.spc_conv_forward(km, F, W, B.DATAFLOW_WS)
    assert e.value.code == B.ERR_ARG
    km.destroy()


# ----------------------------------------------------------------------------- large and random scenes
def _search_geometry(km):
    tile, cap = B.spc_kmap_search_info(km)
    assert tile in (64, 128) and cap >= 1024
    return tile, cap


def _exact_window_sizes(in_keys, out_keys, desc, K, s_p, tile):
    """Per tile of `tile` consecutive outputs and per (dx, dy) group: the number of input keys between the
    first output's smallest-z query and the last output's largest-z query (what the search kernel has to
    look through for that tile and group; its own windows are at least this wide)."""
    ax = [(i - (K - 1) // 2) * s_p for i in range(K)] if K % 2 else [i * s_p for i in range(K)]
    sh_y, sh_x = desc.bits_z, desc.bits_z + desc.bits_y
    ik = in_keys.astype(np.int64)
    ok = out_keys.astype(np.int64)
    first, last = ok[0::tile], ok[np.minimum(np.arange(tile - 1, len(ok) + tile - 1, tile), len(ok) - 1)]
    sizes = []
    for dx in ax:
        for dy in ax:
            d = dx * (1 << sh_x) + dy * (1 << sh_y)
            lo = np.searchsorted(ik, first + d + ax[0], "left")
            hi = np.searchsorted(ik, last + d + ax[-1], "right")
            sizes.append(np.maximum(hi - lo, 0))
    return np.stack(sizes, 1)  # [tiles, K^2]


@pytest.mark.parametrize("K,s_l,key_bits", [(3, 2, 0), (7, 1, 64), (5, 2, 64)])
def test_kmap_windows_beyond_the_lds_budget(K, s_l, key_bits):
    """Dense grids whose per-tile search windows do not fit the kernel's LDS budget: the groups past the
    budget are searched in global memory.  That the case is reached is shown on the host from the window
    sizes (exact ones, which the kernel's can only exceed) and the kernel's reported tile and budget."""
    c = synth.full_grid(22, batch=2)
    desc = fit_desc(c, [(K, 1, s_l)], key_bits)
    keys, _ = gpu_pack(c, desc)
    cs, _ = oracle.sort_coords(c)
    km = B.spc_build_kmap(keys, desc, K, 1, s_l, 0, B.LAYOUT_BOTH)
    ci, co, M = _check_map(cs, keys, desc, K, 1, s_l, 0, km)
    tile, cap = _search_geometry(km)
    w = _exact_window_sizes(oracle_keys(ci, desc), oracle_keys(co, desc), desc, K, 1, tile)
    over = (np.cumsum(w, axis=1) > cap).any(axis=1)
    assert over.mean() > 0.5, "most tiles must overflow the LDS window budget for this test to mean anything"
    km.destroy()


@pytest.mark.parametrize("n,key_bits", [(1_000_000, 0), (2_200_000, 0), (2_200_000, 64)])
def test_large_random_scene(n, key_bits):
    """Uniform random voxels at 1.25 % density (the ablation set-up of Section 6.6; no neighbouring
    structure): pack + sort, kernel map and features against the oracle at 10^6 voxels and above 2^21
    keys, both key widths."""
    c = synth.scaled_random_cloud(n)
    desc = fit_desc(c, [(3, 1, 1)], key_bits)
    assert desc.key_bits == (64 if key_bits == 64 else 32)
    keys, perm = gpu_pack(c, desc)
    cs, operm = oracle.sort_coords(c)
    assert np.array_equal(perm.cpu().numpy(), operm)
    assert np.array_equal(keys_to_u64(keys), oracle_keys(cs, desc))
    km = B.spc_build_kmap(keys, desc, 3, 1, 1, 0, B.LAYOUT_BOTH)
    M = oracle.kernel_map(cs, cs, 3, 1)
    ref_t = oracle.triples(M)
    assert np.array_equal(km.export_triples(B.LAYOUT_OS), ref_t)
    assert np.array_equal(km.export_triples(B.LAYOUT_WS), ref_t)
    F = synth.features(n, 32, np.float16, seed=91)
    W = synth.weights(27, 32, 32, np.float16, seed=92)
    Fs = B.spc_permute_rows(torch.from_numpy(F).cuda(), perm)
    ref = oracle.conv(M, F[operm].astype(np.float64), W.astype(np.float64))
    Wt = torch.from_numpy(W).cuda()
    for df, variant in ((B.DATAFLOW_OS, 0), (B.DATAFLOW_OS, B.CONV_OS_PHASE), (B.DATAFLOW_WS, 0)):
        y = B.spc_conv_forward(km, Fs, Wt, df, variant)
        assert_close(y.cpu().double().numpy(), ref, 1e-2, (n, df, variant))
    km.destroy()
    # 1x1x1: every voxel maps to itself
    km1 = B.spc_build_kmap(keys, desc, 1, 1, 1, 0, B.LAYOUT_BOTH)
    ident = np.stack([np.zeros(n, np.int32), np.arange(n, dtype=np.int32), np.arange(n, dtype=np.int32)], 1)
    assert np.array_equal(km1.export_triples(B.LAYOUT_OS), ident)
    assert np.array_equal(km1.export_triples(B.LAYOUT_WS), ident)
    km1.destroy()
    B.spc_release_cache()


def test_large_random_scene_levels():
    """Levels 2 and 4 straight from V_0 above 2^21 keys."""
    n = 2_200_000
    c = synth.scaled_random_cloud(n)
    desc = fit_desc(c, [(2, 2, 2)])
    keys, _ = gpu_pack(c, desc)
    cs, _ = oracle.sort_coords(c)
    maps = B.spc_build_kmaps_network(keys, desc, [(2, s, 2, 0, B.LAYOUT_OS) for s in (1, 2)])
    levels = {1: cs}
    for m, stride in zip(maps, (2, 4)):
        levels[stride] = oracle.downsample(cs, stride)
        ref = oracle_keys(levels[stride], desc)
        assert m.n_out == len(ref)
        assert np.array_equal(m.out_keys(), ref), stride
    # the strided 2x2x2 map onto the first level (long search tiles at this size)
    ref_t = oracle.triples(oracle.kernel_map(levels[1], levels[2], 2, 1))
    assert np.array_equal(maps[0].export_triples(B.LAYOUT_OS), ref_t)
    for m in maps:
        m.destroy()
    B.spc_release_cache()


def test_beyond_the_own_sort():
    """Above 8 Mi keys pack + sort and the downsampling fall back on the library sort (eager calls only): keys,
    permutation and the stride-2 level against the oracle at 8.5 million voxels."""
    n = 8_500_000
    c = synth.scaled_random_cloud(n)
    desc = fit_desc(c, [(2, 2, 2)])
    keys, perm = gpu_pack(c, desc)
    cs, operm = oracle.sort_coords(c)
    assert np.array_equal(perm.cpu().numpy(), operm)
    assert np.array_equal(keys_to_u64(keys), oracle_keys(cs, desc))
    m = B.spc_build_kmaps_network(keys, desc, [(2, 1, 2, 0, B.LAYOUT_OS)])[0]
    ref = oracle_keys(oracle.downsample(cs, 2), desc)
    assert m.n_out == len(ref)
    assert np.array_equal(m.out_keys(), ref)
    m.destroy()
    B.spc_release_cache()


def test_destroy_and_rebuild_while_another_stream_still_reads_the_map():
    """spc_kmap_destroy hands the map's arrays back to the build stream's block cache without waiting.  A
    feature layer enqueued on another stream must still see its map when the next build on the build
    stream takes those blocks again at once."""
    c1, c2 = synth.cloud("lidar"), synth.random_cloud(120_000, (1024, 1024, 80), seed=77)
    lo = np.minimum(c1[:, 1:].min(0), c2[:, 1:].min(0))
    hi = np.maximum(c1[:, 1:].max(0), c2[:, 1:].max(0))
    desc = B.spc_pack_desc_fit(lo, hi, 1, 1, 1)
    k1, p1 = gpu_pack(c1, desc)
    k2, _ = gpu_pack(c2, desc)
    F = torch.from_numpy(synth.features(len(c1), 64, np.float16, seed=3)).cuda()
    Fs = B.spc_permute_rows(F, p1)
    W = B.spc_conv_prepare_weights(torch.from_numpy(synth.weights(27, 64, 64, np.float16, seed=4)).cuda())
    km = B.spc_build_kmap(k1, desc, 3, 1, 1, 0, B.LAYOUT_OS)
    ref = B.spc_conv_forward(km, Fs, W, B.DATAFLOW_OS, B.CONV_PACKED_WEIGHTS).clone()
    torch.cuda.synchronize()
    km.destroy()
    build_stream, other = torch.cuda.current_stream(), torch.cuda.Stream()
    for rep in range(5):
        km = B.spc_build_kmap(k1, desc, 3, 1, 1, 0, B.LAYOUT_OS, stream=build_stream)
        other.wait_stream(build_stream)
        out = torch.empty_like(ref)
        with torch.cuda.stream(other):
            for _ in range(4):  # keeps `other` busy well past the destroy below
                B.spc_conv_forward(km, Fs, W, B.DATAFLOW_OS, B.CONV_PACKED_WEIGHTS, out=out, stream=other)
        km.destroy()  # no wait
        km2 = B.spc_build_kmap(k2, desc, 3, 1, 1, 0, B.LAYOUT_OS, stream=build_stream)  # same sizes: same blocks
        torch.cuda.synchronize()
        assert torch.equal(out, ref), rep
        km2.destroy()


@pytest.mark.parametrize("name,K,s_l,transposed,key_bits,with_perm", [
    ("tiny", 3, 1, 0, 0, False), ("tiny_neg", 5, 1, 0, 0, True), ("tiny", 7, 1, 0, 64, False), ("tiny", 1, 1, 0, 0, False),
    ("tiny_neg", 3, 2, 0, 0, True), ("tiny_neg", 2, 2, 0, 0, False), ("tiny_neg", 2, 2, 1, 0, False), ("tiny", 3, 2, 1, 64, False),
    ("rand_b3", 3, 1, 0, 0, True), ("rand_b3", 5, 1, 0, 64, False), ("grid", 3, 1, 0, 0, False), ("ragged", 5, 1, 0, 0, False),
    ("one", 3, 1, 0, 0, False), ("rand_n70001", 3, 1, 0, 0, True), ("skew_60k", 5, 1, 0, 0, False),
])
def test_kmap_ws_layout_alone(name, K, s_l, transposed, key_bits, with_perm):
    """The weight-stationary layout built on its own (no |V_q| x K^3 matrix is ever written): lists, counts
    and features equal the oracle's, with and without the sort permutation folded in."""
    c = _cloud(name)
    desc = fit_desc(c, [(K, 1, s_l)], key_bits)
    keys, perm = gpu_pack(c, desc)
    cs, operm = oracle.sort_coords(c)
    km = B.spc_build_kmap(keys, desc, K, 1, s_l, transposed, B.LAYOUT_WS, in_perm=perm if with_perm else None)
    ci, co, M = oracle_layer(cs, K, 1, s_l, transposed)
    ref_t = oracle.triples(M)
    assert km.n_out == len(co)
    got = km.export_triples(B.LAYOUT_WS)
    if with_perm:
        ref_t[:, 1] = operm[ref_t[:, 1]]  # sorted position -> original row
    assert np.array_equal(got, ref_t[np.lexsort((ref_t[:, 2], ref_t[:, 0]))])
    assert np.array_equal(km.nnz(), np.bincount(ref_t[:, 0], minlength=K ** 3))
    with pytest.raises(B.SpcError):
        km.export_triples(B.LAYOUT_OS)
    F = synth.features(len(c) if with_perm else len(ci), 32, np.float16, seed=41)
    W = synth.weights(K ** 3, 32, 64, np.float16, seed=42)
    ref = oracle.conv(M, (F[operm] if with_perm else F).astype(np.float64), W.astype(np.float64))
    y = B.spc_conv_forward(km, torch.from_numpy(F).cuda(), torch.from_numpy(W).cuda(), B.DATAFLOW_WS)
    assert_close(y.cpu().double().numpy(), ref, 1e-2, name)
    with pytest.raises(B.SpcError):
        B.spc_conv_forward(km, torch.from_numpy(F).cuda(), torch.from_numpy(W).cuda(), B.DATAFLOW_OS)
    km.destroy()


def _l1(K, k):
    iz, iy, ix = k % K, (k // K) % K, k // (K * K)
    if K % 2 == 0:
        return ix + iy + iz
    c = (K - 1) // 2
    return abs(ix - c) + abs(iy - c) + abs(iz - c)


@pytest.mark.parametrize("name,K,s_l,sym", [("rand_b3", 3, 1, False), ("tiny_neg", 5, 1, False), ("tiny", 3, 1, True),
                                            ("tiny_neg", 2, 2, False), ("rand_n70001", 3, 1, False), ("tiny", 5, 1, True)])
def test_hybrid_layout_holds_each_offset_once(name, K, s_l, sym):
    """Map built for one threshold t of the hybrid dual dataflow (Section 5.4): the OS matrix holds the offsets
    with L1 norm < t only, the WS lists the others only; together they are the oracle's map, and the hybrid
    feature computation with that t gives Eq. (2)."""
    c = _cloud(name)
    desc = fit_desc(c, [(K, 1, s_l)])
    keys, _ = gpu_pack(c, desc)
    cs, _ = oracle.sort_coords(c)
    ci, co, M = oracle_layer(cs, K, 1, s_l, 0)
    ref_t = oracle.triples(M)
    l1 = np.array([_l1(K, k) for k in range(K ** 3)])
    F, W = synth.features(len(ci), 32, np.float16, seed=81), synth.weights(K ** 3, 32, 64, np.float16, seed=82)
    Ft, Wt = torch.from_numpy(F).cuda(), torch.from_numpy(W).cuda()
    ref = oracle.conv(M, F.astype(np.float64), W.astype(np.float64))
    l1_max = int(l1.max())
    for t in range(1, l1_max + 1):
        layout = B.LAYOUT_BOTH | B.LAYOUT_HYBRID_T(t) | (B.LAYOUT_WS_SYM if sym else 0)
        km = B.spc_build_kmap(keys, desc, K, 1, s_l, 0, layout)
        dense = l1[ref_t[:, 0]] < t
        assert np.array_equal(km.export_triples(B.LAYOUT_OS), ref_t[dense]), t
        assert np.array_equal(km.export_triples(B.LAYOUT_WS), ref_t[~dense]), t
        assert np.array_equal(km.nnz(), np.bincount(ref_t[:, 0], minlength=K ** 3)), t
        y = B.spc_conv_forward(km, Ft, Wt, hybrid_t=t)
        assert_close(y.cpu().double().numpy(), ref, 1e-2, (name, t))
        for bad_t in (t + 1, t - 1):  # another split needs offsets this map does not hold in that layout
            if sym and bad_t == 0:
                continue  # (a symmetric map serves the centre offset in either dataflow: it pairs every voxel with itself)
            with pytest.raises(B.SpcError) as e:
                B.spc_conv_forward(km, Ft, Wt, hybrid_t=bad_t)
            assert e.value.code == B.ERR_ARG
        with pytest.raises(B.SpcError):
            B.spc_conv_forward(km, Ft, Wt, B.DATAFLOW_OS)
        km.destroy()
    with pytest.raises(B.SpcError):  # a threshold needs both layouts
        B.spc_build_kmap(keys, desc, K, 1, s_l, 0, B.LAYOUT_OS | B.LAYOUT_HYBRID_T(1))
