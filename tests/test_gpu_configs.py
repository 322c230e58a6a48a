"""Parity at the full sizes of the benchmark configurations (single layers 0-3),
through the same calls and launch configuration bench.py times."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_20834_amd import binding as B
from paper_2511_20834_amd import synth

from gpu_common import assert_close, oracle_keys

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg", [0, 1, 2, 3])
def test_config_full_size(cfg):
    c = synth.CONFIGS[cfg]
    K, s_l, cin, cout = c["K"], c["layer_stride"], c["cin"], c["cout"]
    coords = synth.cloud(c["cloud"])
    n = len(coords)
    F, W = synth.layer_tensors(cfg, n)
    reach = (K - 1) // 2
    desc = B.spc_pack_desc_fit(coords[:, 1:].min(0), coords[:, 1:].max(0), int(coords[:, 0].max()) + 1, s_l, reach)
    assert desc.key_bits == 32
    keys, perm = B.spc_pack_coords(torch.from_numpy(coords).cuda(), desc, True, B.PACK_VALIDATE)
    cs, operm = oracle.sort_coords(coords)
    assert np.array_equal(perm.cpu().numpy(), operm)
    km = B.spc_build_kmap(keys, desc, K, 1, s_l, 0, B.LAYOUT_BOTH)
    oc, M = oracle.layer(cs, K, 1, s_l)
    assert km.n_out == len(oc)
    assert np.array_equal(km.out_keys(), oracle_keys(oc, desc))
    ref_t = oracle.triples(M)
    assert np.array_equal(km.export_triples(B.LAYOUT_OS), ref_t)
    assert np.array_equal(km.export_triples(B.LAYOUT_WS), ref_t)
    Fs = B.spc_permute_rows(torch.from_numpy(F).cuda(), perm)
    assert np.array_equal(Fs.cpu().numpy(), F[operm])
    Wt = torch.from_numpy(W).cuda()
    ref = oracle.conv(M, F[operm].astype(np.float64), W.astype(np.float64))
    tol = 1e-5 if c["dtype"] == "f32" else 1e-2
    packed = B.spc_conv_prepare_weights(Wt) if c["dtype"] != "f32" else None
    for df in (B.DATAFLOW_OS, B.DATAFLOW_WS):
        y = B.spc_conv_forward(km, Fs, Wt, df).cpu().double().numpy()
        assert_close(y, ref, tol, (cfg, df))  # global and element-wise form of the tolerance
        if packed is not None:
            y2 = B.spc_conv_forward(km, Fs, packed, df, B.CONV_PACKED_WEIGHTS).cpu().double().numpy()
            if df == B.DATAFLOW_OS:
                assert np.array_equal(y2, y)
                # both OS kernels at full size, whichever one the size-based choice picked above
                for variant in (B.CONV_OS_PHASE, B.CONV_OS_SPLITK):
                    y3 = B.spc_conv_forward(km, Fs, packed, df, B.CONV_PACKED_WEIGHTS | variant).cpu().double().numpy()
                    assert_close(y3, ref, tol, (cfg, variant))
            else:
                assert_close(y2, ref, tol, (cfg, df, "packed"))
    km.destroy()
    # the step bench.py times: OS layout alone, the sort's permutation folded into the map, the caller's unsorted rows
    kmp = B.spc_build_kmap(keys, desc, K, 1, s_l, 0, B.LAYOUT_OS, in_perm=perm)
    ref_p = ref_t.copy()
    ref_p[:, 1] = operm[ref_p[:, 1]]
    got = kmp.export_triples(B.LAYOUT_OS)
    assert np.array_equal(got[np.lexsort((got[:, 2], got[:, 1], got[:, 0]))], ref_p[np.lexsort((ref_p[:, 2], ref_p[:, 1], ref_p[:, 0]))])
    Fu = torch.from_numpy(F).cuda()
    flags = B.CONV_PACKED_WEIGHTS if packed is not None else 0
    y = B.spc_conv_forward(kmp, Fu, packed if packed is not None else Wt, B.DATAFLOW_OS, flags).cpu().double().numpy()
    assert_close(y, ref, tol, (cfg, "permutation folded"))
    kmp.destroy()
