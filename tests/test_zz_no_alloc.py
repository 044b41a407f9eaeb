"""The entry point that allocates nothing (basa_norm_sort_static, for callers that cannot call
hipMalloc): called through the C ABI and compared bit for bit with basa_norm_sort, which itself is
compared with the oracle in test_gpu_parity.py.  Two calls in a row share the library's static
scratch; the second is the smaller one, so stale words of the first lie beyond (and inside) what
it uses."""
import numpy as np
import pytest
import torch

from oracle import basa_oracle as o
from paper_2605_19726_amd import binding as bd
from paper_2605_19726_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(name, heads, L, d=128, block=128):
    w = synth.CONFIGS[4].scaled(name, heads_q=heads, heads_kv=heads, L=L, d=d, block=block)
    Q, _, _ = synth.make_qkv(w, device=DEV)
    return w, Q


def test_static_norm_sort_equals_workspace_norm_sort_on_two_calls_in_a_row():
    bd.load()
    bd.basa_static_init()
    assert bd.basa_static_scratch_size() == 32 << 20
    # several 4096-token tiles and merge passes, ragged tail; then a smaller input (one merge pass
    # less, fewer heads), then one that fits a single tile (no merge pass at all)
    for name, heads, L, window in (("big", 4, 40000 + 77, 0), ("small", 2, 9000 + 5, 0), ("windowed", 3, 20000, 4096),
                                   ("one_tile", 2, 3000, 0)):
        w, Q = _case(name, heads, L)
        Q[0, 0, 100:140] = Q[0, 0, 700:740]                      # exact ties
        want, want_keys = bd.basa_norm_sort(Q, w.block, window=window, return_keys=True)
        perm = torch.full((1, heads, L), -1, dtype=torch.int32, device=DEV)
        keys = torch.empty((1, heads, L), dtype=torch.float32, device=DEV)
        # (the number of allocations made so far, not the bytes in use: a tensor of an earlier test that
        #  the garbage collector happens to free during the call would change the latter)
        before = torch.cuda.memory_stats()["allocation.all.allocated"]
        bd.basa_norm_sort_static(Q, w.block, perm, window=window, keys=keys)
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
        torch.cuda.synchronize()
        assert torch.equal(perm, want), name
        assert torch.equal(keys, want_keys), name
        # and against the oracle directly on one head
        got = perm[0, heads - 1].cpu().numpy().astype(np.int64)
        assert np.array_equal(got, o.norm_sort(Q[0, heads - 1].cpu().double().numpy(), window)), name


def test_static_norm_sort_rejects_what_does_not_fit():
    bd.load()
    limit = bd.basa_static_scratch_size() // 16
    L = 1 << 16
    heads = limit // L + 1
    x = torch.empty((1, heads, L, 64), dtype=torch.bfloat16, device=DEV)
    perm = torch.empty((1, heads, L), dtype=torch.int32, device=DEV)
    with pytest.raises(bd.BasaError) as e:
        bd.basa_norm_sort_static(x, 64, perm)
    assert e.value.status_name == "BASA_ERR_WORKSPACE" and "static" in str(e.value)
