"""GPU parity of the causal variant (this library's reading of the future work named in Sec. 6:
visibility by ORIGINAL position, block pairs without a visible token pair dropped before the
ranking) against the oracle's select_causal / sparse_attention_causal / dense_causal_attention."""
import numpy as np
import pytest
import torch

from oracle import basa_oracle as o
from paper_2605_19726_amd import binding as bd
from paper_2605_19726_amd import synth
from parity_util import MASK_REL_BAND, check_output, np64, unpack_mask

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
C = synth.CONFIGS

CASES = [
    C[0],                                                                                  # fp32, d = 64, B = 64
    C[4].scaled("causal_b128", heads_q=2, heads_kv=2, L=2048 + 128 * 2 + 50, salient_frac=0.1),   # bf16 d = 128, ragged
    C[1].scaled("causal_b64_gqa", heads_q=4, heads_kv=2, L=1024 + 64 * 3 + 7, salient_frac=0.1),
    C[0].scaled("causal_bf16_d64", dtype="bf16", L=900),
]


def _select_parity(w, Q, K, s, sort):
    sel = bd.basa_select(Q, K, w.block, s, sort=sort, causal=True)
    torch.cuda.synchronize()
    gpu_mask = unpack_mask(sel.mask_bits, sel.n_k)
    group = Q.shape[1] // K.shape[1]
    refs = []
    for h in range(Q.shape[1]):
        ref = o.select_causal(np64(Q[0, h]), np64(K[0, h // group]), w.block, s, sort=sort)
        refs.append(ref)
        assert np.array_equal(sel.perm_q[0, h].cpu().numpy(), ref["perm_q"])
        assert np.array_equal(sel.perm_k[0, h // group].cpu().numpy(), ref["perm_k"])
        cnt = sel.row_count[0, h].cpu().numpy()
        assert np.array_equal(cnt, ref["count"]), f"{w.name} head {h}: kept counts differ"
        # kept sets: equal except for blocks whose oracle m' lies in the band around the row threshold
        th = ref["theta"][:, None]
        band = ref["live"] & (np.abs(ref["m"] - th) <= MASK_REL_BAND * th)
        diff = gpu_mask[0, h] != ref["mask"]
        assert not (diff & ~band).any(), f"{w.name} head {h}: mask differs outside the band"
        assert not (gpu_mask[0, h] & ~ref["live"]).any(), "a dead block was kept"
        cols = sel.row_cols[0, h].cpu().numpy()
        for r in range(cols.shape[0]):
            got = cols[r, :cnt[r]]
            assert np.array_equal(got, np.nonzero(gpu_mask[0, h, r])[0]), "list and bitmap disagree"
        mass = sel.row_mass[0, h].cpu().numpy()
        same = ~diff.any(axis=1)
        np.testing.assert_allclose(mass[same], ref["mass"][same], rtol=2e-5, atol=1e-6)
    return sel, refs


@pytest.mark.parametrize("sort", [bd.SORT_NONE, bd.SORT_QK])
@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_causal_selection_and_attention_match_oracle(w, sort):
    Q, K, V = synth.make_qkv(w, device=DEV)
    sel, refs = _select_parity(w, Q, K, 0.5, sort)
    group = Q.shape[1] // K.shape[1]
    # attention over the ORACLE's lists, so that both sides attend to the same blocks
    kappa = sel.row_cols.shape[-1]
    rc = torch.zeros_like(sel.row_cols)
    cnt = torch.zeros_like(sel.row_count)
    for h, ref in enumerate(refs):
        for r, c in enumerate(ref["cols"]):
            rc[0, h, r, :len(c)] = torch.from_numpy(c.astype(np.int32))
            cnt[0, h, r] = len(c)
    assert kappa >= int(cnt.max())
    out, lse = bd.basa_sparse_attn(Q, K, V, cnt, rc, w.block, sel.perm_q, sel.perm_k, want_lse=True, causal=True)
    torch.cuda.synchronize()
    bf16 = w.dtype == "bf16"
    for h, ref in enumerate(refs):
        O_ref, lse_ref = o.sparse_attention_causal(np64(Q[0, h]), np64(K[0, h // group]), np64(V[0, h // group]),
                                                   ref["perm_q"], ref["perm_k"], ref["cols"], w.block, return_lse=True)
        check_output(np64(out[0, h]), O_ref, bf16, f"causal {w.name} head {h}")
        got = lse[0, h].cpu().numpy()
        blind = np.isinf(lse_ref)
        assert np.array_equal(np.isinf(got) & (got < 0), blind), "queries that see nothing: lse must be -inf"
        np.testing.assert_allclose(got[~blind], lse_ref[~blind], rtol=0, atol=3e-2 if bf16 else 1e-4)
        assert np.abs(np64(out[0, h])[blind]).max(initial=0.0) == 0.0


@pytest.mark.parametrize("dtype,d,block,Lq,Lk", [(torch.bfloat16, 128, 128, 700, 700), (torch.bfloat16, 128, 64, 300, 777),
                                                  (torch.bfloat16, 64, 128, 777, 300), (torch.float32, 64, 64, 333, 333)])
def test_dense_causal_attention_matches_oracle(dtype, d, block, Lq, Lk):
    g = torch.Generator().manual_seed(31 + Lq + Lk)
    mk = lambda L: (torch.randn((1, 2, L, d), generator=g) * 1.2).to(dtype).to(DEV)
    Q, K, V = mk(Lq), mk(Lk), mk(Lk)
    out, lse = bd.basa_dense_attn(Q, K, V, block, want_lse=True, causal=True)
    torch.cuda.synchronize()
    bf16 = dtype == torch.bfloat16
    for h in range(2):
        O_ref, lse_ref = o.dense_causal_attention(np64(Q[0, h]), np64(K[0, h]), np64(V[0, h]), return_lse=True)
        check_output(np64(out[0, h]), O_ref, bf16, f"dense causal head {h}")
        got = lse[0, h].cpu().numpy()
        blind = np.isinf(lse_ref)
        assert np.array_equal(np.isinf(got), blind)
        np.testing.assert_allclose(got[~blind], lse_ref[~blind], rtol=0, atol=3e-2 if bf16 else 1e-4)
        if Lq > Lk:
            assert blind[:Lq - Lk].all() and np.abs(np64(out[0, h])[:Lq - Lk]).max() == 0.0


def test_causal_end_to_end_at_zero_sparsity_equals_dense_causal_for_sorted_and_unsorted():
    # sparsity 0 keeps every live block: whatever the sort, the result is dense causal attention
    w = C[4].scaled("causal_s0", heads_q=2, heads_kv=1, L=1500, salient_frac=0.1)
    Q, K, V = synth.make_qkv(w, device=DEV)
    dense = bd.basa_dense_attn(Q, K, V, w.block, causal=True)
    for sort in (bd.SORT_NONE, bd.SORT_Q, bd.SORT_K, bd.SORT_QK):
        sel = bd.basa_select(Q, K, w.block, 0.0, sort=sort, causal=True)
        out = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, w.block, sel.perm_q, sel.perm_k, causal=True)
        torch.cuda.synchronize()
        for h in range(2):
            O_ref = o.dense_causal_attention(np64(Q[0, h]), np64(K[0, 0]), np64(V[0, 0]))
            check_output(np64(out[0, h]), O_ref, True, f"sort {sort} head {h}")
            check_output(np64(dense[0, h]), O_ref, True, f"dense head {h}")
    # unsorted: the first rows have fewer live blocks than kappa
    sel = bd.basa_select(Q, K, w.block, 0.5, sort=bd.SORT_NONE, causal=True)
    cnt = sel.row_count[0, 0].cpu().numpy()
    n = sel.n_k
    assert list(cnt[:4]) == [1, 2, 3, 4] and (cnt == np.minimum(np.arange(1, n + 1), sel.kappa)).all()


@pytest.mark.parametrize("Lq,Lk", [(300, 1000), (1000, 300)])
@pytest.mark.parametrize("dtype,d,block", [(torch.bfloat16, 128, 64), (torch.float32, 64, 64)])
def test_causal_cross_lengths_through_selection(Lq, Lk, dtype, d, block):
    """Ends aligned: with L_q < L_k every query sees a long prefix; with L_q > L_k the first query blocks
    precede every key (no live block: count 0, zero rows)."""
    g = torch.Generator().manual_seed(5 + Lq)
    mk = lambda L: (torch.randn((1, 2, L, d), generator=g) * 1.1).to(dtype).to(DEV)
    Q, K, V = mk(Lq), mk(Lk), mk(Lk)
    for sort, mass in ((bd.SORT_NONE, 0.0), (bd.SORT_QK, 0.0), (bd.SORT_QK, 0.6)):
        sel = bd.basa_select(Q, K, block, 0.5, sort=sort, causal=True, mass_target=mass, min_keep=2)
        out, lse = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, block, sel.perm_q, sel.perm_k,
                                       want_lse=True, causal=True)
        torch.cuda.synchronize()
        bf16 = dtype == torch.bfloat16
        for h in range(2):
            q, k, v = np64(Q[0, h]), np64(K[0, h]), np64(V[0, h])
            ref = o.select_causal(q, k, block, 0.5, sort=sort)
            cnt = sel.row_count[0, h].cpu().numpy()
            cols = sel.row_cols[0, h].cpu().numpy().astype(np.int64)
            lists = [cols[r, :cnt[r]] for r in range(cols.shape[0])]
            n_live = ref["live"].sum(axis=1)
            if mass == 0.0:
                assert np.array_equal(cnt, ref["count"])
            else:                                # a mass budget keeps at most the fixed budget's count, at least min_keep
                assert (cnt <= ref["count"]).all() and (cnt >= np.minimum(2, n_live)).all()
            for r, c in enumerate(lists):
                assert ref["live"][r, c].all(), "a dead block was kept"
            if sort == bd.SORT_NONE and Lq > Lk:
                assert (cnt[:(Lq - Lk) // block] == 0).all()
            # attention over the GPU's own lists against the oracle on the same lists
            O_ref, lse_ref = o.sparse_attention_causal(q, k, v, ref["perm_q"], ref["perm_k"], lists, block, return_lse=True)
            check_output(np64(out[0, h]), O_ref, bf16, f"cross {Lq}x{Lk} sort {sort} mass {mass} head {h}")
            blind = np.isinf(lse_ref)
            assert np.array_equal(np.isinf(lse[0, h].cpu().numpy()), blind)
            assert np.abs(np64(out[0, h])[blind]).max(initial=0.0) == 0.0
