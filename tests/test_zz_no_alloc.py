"""The allocation-free entry point spc_pack_coords_noalloc against spc_pack_coords (bit-exact: keys and
permutation are integers), two calls in a row on the shared static scratch, the second one smaller."""
import numpy as np
import pytest
import torch

from paper_2511_20834_amd import binding as B
from paper_2511_20834_amd import synth

pytestmark = pytest.mark.gpu


def _both(c, desc, flags=0):
    coords = torch.from_numpy(np.ascontiguousarray(c)).cuda()
    keys_ref, perm_ref = B.spc_pack_coords(coords, desc, True, flags)
    kdt = torch.int32 if desc.key_bits == 32 else torch.int64
    keys = torch.full((len(c),), -1, dtype=kdt, device="cuda")
    perm = torch.full((len(c),), -1, dtype=torch.int32, device="cuda")
    B.spc_pack_coords_noalloc(coords, desc, keys, perm, flags)
    torch.cuda.synchronize()
    assert torch.equal(keys, keys_ref) and torch.equal(perm, perm_ref)
    return keys


@pytest.mark.parametrize("key_bits", [0, 64])
def test_noalloc_pack_matches_pack_coords_twice_in_a_row(key_bits):
    big = synth.cloud("lidar")                                                  # 120 000 voxels
    small = synth.random_cloud(9000, (300, 280, 40), seed=5, batch=2)           # second call: smaller input
    for c in (big, small, big[:70001]):
        lo, hi = c[:, 1:].min(0), c[:, 1:].max(0)
        desc = B.spc_pack_desc_fit(lo, hi, int(c[:, 0].max()) + 1, 16, 16, key_bits)
        k = _both(c, desc)
        a = k.cpu().numpy()
        a = a.view(np.uint32) if a.dtype == np.int32 else a.view(np.uint64)
        assert np.all(a[1:] > a[:-1])
    # validation mode reports through the same status word
    c = np.concatenate([small, small[:1]])
    desc = B.spc_pack_desc_fit(c[:, 1:].min(0), c[:, 1:].max(0), 2, 1, 1, key_bits)
    keys = torch.empty(len(c), dtype=torch.int32 if desc.key_bits == 32 else torch.int64, device="cuda")
    with pytest.raises(B.SpcError) as e:
        B.spc_pack_coords_noalloc(torch.from_numpy(c).cuda(), desc, keys, None, B.PACK_VALIDATE)
    assert e.value.code == B.ERR_DUP


def test_noalloc_pack_size_limits():
    desc = B.spc_pack_desc_fit([0, 0, 0], [2000, 2000, 200], 1, 1, 1)
    for n in (0, B.NOALLOC_MAX_N + 1):
        coords = torch.zeros((n, 4), dtype=torch.int32, device="cuda")
        keys = torch.empty(n, dtype=torch.int32, device="cuda")
        with pytest.raises(B.SpcError) as e:
            B.spc_pack_coords_noalloc(coords, desc, keys, None)
        assert e.value.code == B.ERR_UNSUPPORTED
    # small clouds go through the one-workgroup sort, on no scratch at all
    c = synth.random_cloud(777, (50, 40, 30), seed=10)
    _both(c, B.spc_pack_desc_fit(c[:, 1:].min(0), c[:, 1:].max(0), 1, 1, 1))
    # the largest size it takes
    c = synth.random_cloud(B.NOALLOC_MAX_N, (2000, 2000, 200), seed=9)
    d64 = B.spc_pack_desc_fit(c[:, 1:].min(0), c[:, 1:].max(0), 1, 16, 16, 64)
    _both(c, d64)
