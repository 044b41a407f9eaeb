"""GPU parity: every stage of the HIP path, called through the C ABI, against the numpy
oracle on the same seeded inputs.  Sizes span several tiles and ragged tails; the
full-size configurations are checked on sampled (head, query block) units."""
import numpy as np
import pytest
import torch

from oracle import basa_oracle as o
from paper_2605_19726_amd import binding as bd
from paper_2605_19726_amd import synth
from parity_util import (check_output, mask_report, np64, oracle_select, unpack_mask)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
C = synth.CONFIGS

# scaled versions of the five workloads: same generators, sizes the oracle finishes in seconds
SMALL = [
    C[0],
    C[1].scaled("lowrank_b64", heads_q=2, heads_kv=2, L=4096 + 64 * 5, salient_frac=0.05),
    C[4].scaled("lowrank_b128", heads_q=2, heads_kv=2, L=8192 + 128 * 3, salient_frac=0.05),
    C[2].scaled("multimodal_gqa", heads_q=4, heads_kv=2, L=4096, image_side=32),
    C[3].scaled("video_ragged", heads_q=2, heads_kv=2, L=5 * 20 * 21, video_thw=(5, 20, 21)),
    C[0].scaled("tiny_f32_d128_ragged", L=1000, d=128, block=128, heads_q=2, heads_kv=1),
    C[0].scaled("tiny_bf16_d64", dtype="bf16", L=900),
]


def gen(w):
    return synth.make_qkv(w, device=DEV)


@pytest.fixture(scope="module", autouse=True)
def _lib():
    bd.load()


# ------------------------------------------------------------------ norm sort
@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
def test_norm_sort_matches_oracle(w):
    Q, K, V = gen(w)
    for x in (Q, K):
        perm, keys = bd.basa_norm_sort(x, w.block, return_keys=True)
        torch.cuda.synchronize()
        for h in range(x.shape[1]):
            xn = np64(x[0, h])
            assert np.array_equal(keys[0, h].cpu().numpy(), o.token_sort_keys(xn)), "fp32 sort keys differ"
            assert np.array_equal(perm[0, h].cpu().numpy().astype(np.int64), o.norm_sort(xn))


def test_norm_sort_windowed_and_ties():
    w = C[1].scaled("win", heads_q=2, heads_kv=2, L=10000 + 64)
    Q, _, _ = gen(w)
    Q[0, 0, 5000:5064] = Q[0, 0, 100:164]            # exact ties across distant positions
    for window in (0, 64, 1024, 4096, 8192):
        perm = bd.basa_norm_sort(Q, w.block, window=window)
        for h in range(2):
            want = o.norm_sort(np64(Q[0, h]), window)
            assert np.array_equal(perm[0, h].cpu().numpy().astype(np.int64), want), f"window={window}"


def test_norm_sort_with_runs_of_three_to_eighteen_tiles():
    """Segments longer than two sort tiles go through the kernel that merges four tiles in LDS: a ragged
    quad that is also the last pass (window of 3.03 tiles), whole quads followed by ordinary passes
    (10 tiles per window, the last window cut short), one run of 17.1 tiles, and a segment list."""
    w = C[1].scaled("quads", heads_q=2, heads_kv=2, L=70000 + 64)
    Q, _, _ = gen(w)
    for window in (12416, 40960, 16384, 0):
        perm = bd.basa_norm_sort(Q, w.block, window=window)
        for h in range(2):
            want = o.norm_sort(np64(Q[0, h]), window)
            assert np.array_equal(perm[0, h].cpu().numpy().astype(np.int64), want), f"window={window}"
    segs = [0, 9000, 30001, 50000]
    perm = bd.basa_norm_sort(Q, w.block, segments=segs)
    for h in range(2):
        assert np.array_equal(perm[0, h].cpu().numpy().astype(np.int64), o.norm_sort(np64(Q[0, h]), 0, segs))


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 64)])
def test_norm_sort_segments(dtype, d):
    L = 20000 + 37
    g = torch.Generator().manual_seed(77)
    X = torch.randn((1, 2, L, d), generator=g).to(dtype).to(DEV)
    X[0, 0, 9000:9064] = X[0, 0, 100:164]            # exact ties across segments and tiles
    X[0, 1, 4090:4100] = X[0, 1, 4080:4090]          # and around a tile edge
    cases = [[0], [0, 1], [0, L - 1], [0, 4096], [0, 4095, 4097], [0, 100, 101, 9000, 9032, 16384],
             list(range(0, 63 * 300, 300)),           # the maximum of 63 segments, several per tile
             [0] + list(range(5000, 5000 + 62))]      # one-token segments
    for starts in cases:
        perm = bd.basa_norm_sort(X, 128, segments=starts)
        for h in range(2):
            want = o.norm_sort(np64(X[0, h]), segments=starts)
            assert np.array_equal(perm[0, h].cpu().numpy().astype(np.int64), want), f"segments={starts[:8]}"


def test_select_and_attention_with_segments():
    # image + text segments as in the multimodal workload, scaled down; the segment edge is no
    # multiple of the block, so one block of the sorted order holds tokens of both
    w = C[2].scaled("seg", heads_q=4, heads_kv=2, L=6000 + 11, image_side=40)
    Q, K, V = gen(w)
    starts = [0, 1600, 3000]
    sel = bd.basa_select(Q, K, w.block, 0.5, want_scores=True, segments=starts)
    out = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, w.block, sel.perm_q, sel.perm_k)
    torch.cuda.synchronize()
    gpu_mask = unpack_mask(sel.mask_bits, sel.n_k)
    for h in range(4):
        q, k, v = np64(Q[0, h]), np64(K[0, h // 2]), np64(V[0, h // 2])
        ref = o.select(q, k, w.block, 0.5, segments=starts)
        assert np.array_equal(sel.perm_q[0, h].cpu().numpy(), ref["perm_q"])
        assert np.array_equal(sel.perm_k[0, h // 2].cpu().numpy(), ref["perm_k"])
        assert mask_report(gpu_mask[0, h], ref)[0] == 0
        cols = sel.row_cols[0, h].cpu().numpy().astype(np.int64)
        O_ref = o.sparse_attention(q, k, v, ref["perm_q"], ref["perm_k"], cols, w.block)
        check_output(np64(out[0, h]), O_ref, True, f"segments head {h}")


@pytest.mark.parametrize("dtype,d", [(torch.float32, 128), (torch.bfloat16, 128), (torch.float32, 64)])
def test_score_map_keeps_fp32_accuracy_over_a_wide_dynamic_range(dtype, d):
    """The score map multiplies three-part bf16 splits of fp32 features on the bf16 matrix cores;
    per-dimension scales over four decades and large offsets exercise every part of the split."""
    L, block = 3000 + 17, 64
    g = torch.Generator().manual_seed(2718)
    scale = 10.0 ** (torch.rand((1, 1, 1, d), generator=g) * 4 - 2)           # 0.01 .. 100 per dimension
    offset = torch.randn((1, 1, 1, d), generator=g) * 3
    Q = ((torch.randn((1, 2, L, d), generator=g) + offset) * scale).to(dtype).to(DEV)
    K = ((torch.randn((1, 2, L, d), generator=g) - offset) * scale.flip(-1)).to(dtype).to(DEV)
    for beta in (1.0, 0.0):
        sel = bd.basa_select(Q, K, block, 0.5, beta, want_scores=True)
        for h in range(2):
            ref = o.select(np64(Q[0, h]), np64(K[0, h]), block, 0.5, beta)
            got = sel.scores[0, h].cpu().numpy().astype(np.float64)
            err = np.abs(got - ref["logits"])
            big = np.abs(ref["logits"]).max()
            assert err.max() <= 1e-5 * max(1.0, big), (beta, h, err.max(), big)
            # the typical error is that of fp32 arithmetic, far inside the bound
            assert np.median(err) <= 2e-6 * max(1.0, big), (beta, h, np.median(err), big)


def test_norm_sort_keys_zeros_subnormals_and_scales():
    """Sort keys stay bit-identical to the oracle's when rows hold exact zeros, bf16 subnormals,
    all-zero rows, and values spread over many binades (within what an fp64 sum adds exactly)."""
    g = torch.Generator().manual_seed(77)
    L, d = 4096 + 37, 128
    x = torch.randn(L, d, generator=g)
    x *= torch.exp2(torch.randint(-12, 13, (L, 1), generator=g).float())      # row scales 2^-12 .. 2^12
    x *= torch.exp2(torch.randint(-4, 5, (L, d), generator=g).float())        # element scales on top
    x[torch.rand(L, d, generator=g) < 0.3] = 0.0                               # many exact zeros
    x[5] = 0.0
    x[6] = 0.0
    x[7, 3] = 1e-39                                                            # bf16 subnormal beside normals
    x[8] = 1e-39                                                               # a row of subnormals only
    x[9] = 3e-20                                                               # squares far below fp32 range
    x[10] = 2.0 ** -70
    x = x.to(torch.bfloat16).reshape(1, 1, L, d).to(DEV)
    perm, keys = bd.basa_norm_sort(x, 128, return_keys=True)
    torch.cuda.synchronize()
    xn = np64(x[0, 0])
    assert np.array_equal(keys[0, 0].cpu().numpy(), o.token_sort_keys(xn))
    assert np.array_equal(perm[0, 0].cpu().numpy().astype(np.int64), o.norm_sort(xn))


def test_norm_sort_strided_input():
    # heads interleaved in memory: [1, L, H, d] viewed as [1, H, L, d]
    w = C[1].scaled("strided", heads_q=3, heads_kv=3, L=5000)
    Q, _, _ = gen(w)
    Qs = Q.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert not Qs.is_contiguous()
    perm = bd.basa_norm_sort(Qs, w.block)
    ref = bd.basa_norm_sort(Q, w.block)
    assert torch.equal(perm, ref)


# ------------------------------------------------------------------ block statistics
@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
def test_downsample_matches_oracle(w):
    Q, K, V = gen(w)
    for x in (Q, K):
        perm = bd.basa_norm_sort(x, w.block)
        for pm in (None, perm):
            mean, var, xs = bd.basa_downsample(x, w.block, pm, want_sorted=True)
            for h in range(x.shape[1]):
                xn = np64(x[0, h])
                if pm is not None:
                    xn = xn[o.norm_sort(xn)]              # the oracle's own permutation
                # the materialised ordered sequence is a copy: bit-exact
                assert np.array_equal(np64(xs[0, h]), xn), "x_sorted differs from x[oracle perm]"
                m_ref, v_ref = o.block_stats(xn, w.block)
                np.testing.assert_allclose(mean[0, h].cpu().numpy(), m_ref, rtol=1e-5, atol=1e-6)
                np.testing.assert_allclose(var[0, h].cpu().numpy(), v_ref, rtol=1e-5, atol=1e-6)


# ------------------------------------------------------------------ selection
def _check_selection(w, Q, K, s, beta, sort, window=0, select_path=1):
    # select_path 2: the kernel that keeps the score map on chip (it has no `scores` output)
    sel = bd.basa_select(Q, K, w.block, s, beta, sort, window, want_scores=select_path != 2, select_path=select_path)
    torch.cuda.synchronize()
    n_k = sel.n_k
    gpu_mask = unpack_mask(sel.mask_bits, n_k)
    total_dc = 0
    for h in range(Q.shape[1]):
        ref = oracle_select(Q, K, h, w.block, s, beta, sort, window)
        hk = h // (Q.shape[1] // K.shape[1])
        assert sel.kappa == ref["kappa"]
        assert np.array_equal(sel.perm_q[0, h].cpu().numpy(), ref["perm_q"]), "perm_q"
        assert np.array_equal(sel.perm_k[0, hk].cpu().numpy(), ref["perm_k"]), "perm_k"
        if sel.scores is not None:
            sc = sel.scores[0, h].cpu().numpy().astype(np.float64)
            scale = max(1.0, np.abs(ref["logits"]).max())
            assert np.abs(sc - ref["logits"]).max() <= 1e-5 * scale, \
                f"logits off by {np.abs(sc - ref['logits']).max():.3e}"
        bad, dc = mask_report(gpu_mask[0, h], ref)
        total_dc += dc - ref["mask"].shape[0]          # every row's threshold block is in the band
        assert bad == 0, f"{bad} mask mismatches outside the don't-care band (head {h})"
        assert (sel.row_count[0, h].cpu().numpy() == ref["kappa"]).all()
        cols = sel.row_cols[0, h].cpu().numpy()
        assert (np.diff(cols, axis=1) > 0).all(), "columns not ascending"
        rebuilt = np.zeros_like(gpu_mask[0, h])
        np.put_along_axis(rebuilt, cols.astype(np.int64), True, axis=1)
        assert np.array_equal(rebuilt, gpu_mask[0, h]), "bitmap and column list disagree"
        if np.array_equal(gpu_mask[0, h], ref["mask"]):
            np.testing.assert_allclose(sel.row_mass[0, h].cpu().numpy(), ref["mass"], rtol=1e-4, atol=1e-6)
    return total_dc


@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
def test_select_matches_oracle(w):
    Q, K, _ = gen(w)
    for s in w.sparsities:
        _check_selection(w, Q, K, s, 1.0, o.SORT_QK)


@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
def test_select_with_the_map_on_chip_matches_oracle_and_the_two_kernel_path(w):
    """Eq. 2 / Eq. 14 and Alg. 1 steps 9-11 in one kernel: same parity bar against the oracle, and the
    same bits (bitmap, counts, lists) as the path through the score map in memory."""
    Q, K, _ = gen(w)
    for s in w.sparsities:
        for beta in (1.0, 0.0):
            _check_selection(w, Q, K, s, beta, o.SORT_QK, select_path=2)
            a = bd.basa_select(Q, K, w.block, s, beta, select_path=1)
            b = bd.basa_select(Q, K, w.block, s, beta, select_path=2)
            for name in ("mask_bits", "row_count", "row_cols", "perm_q", "perm_k"):
                assert torch.equal(getattr(a, name), getattr(b, name)), name
            assert (a.row_mass - b.row_mass).abs().max().item() <= 2e-6


def test_select_path_that_cannot_keep_the_map_on_chip_is_refused():
    w = SMALL[0]
    Q, K, _ = gen(w)
    for kw in (dict(want_scores=True), dict(mass_target=0.9), dict(budget_total=8), dict(causal=True)):
        with pytest.raises(bd.BasaError) as e:
            bd.basa_select(Q, K, w.block, 0.5, select_path=2, **kw)
        assert e.value.status_name == "BASA_ERR_UNSUPPORTED"
        # ... and the default takes the other path for them
        bd.basa_select(Q, K, w.block, 0.5, **kw)
    torch.cuda.synchronize()


@pytest.mark.parametrize("sort", [o.SORT_NONE, o.SORT_Q, o.SORT_K, o.SORT_QK])
@pytest.mark.parametrize("beta", [0.0, 1.0, 0.5])
def test_select_every_sort_mode_and_beta(sort, beta):
    w = C[0]
    Q, K, _ = gen(w)
    _check_selection(w, Q, K, 0.5, beta, sort)
    w2 = SMALL[1]
    Q, K, _ = gen(w2)
    _check_selection(w2, Q, K, 0.75, beta, sort)


def test_select_sparsity_extremes_and_window():
    w = SMALL[2]
    Q, K, _ = gen(w)
    for s in (0.0, 0.9, 0.999):
        _check_selection(w, Q, K, s, 1.0, o.SORT_QK)
    _check_selection(w, Q, K, 0.5, 1.0, o.SORT_QK, window=2048)


def test_select_cross_lengths():
    w = SMALL[1]
    Q, K, _ = gen(w)
    Qs = Q[:, :, :1000].contiguous()
    _check_selection(w, Qs, K, 0.5, 1.0, o.SORT_QK)


# ------------------------------------------------------------------ cumulative-mass selection
MASS_BAND = 1e-5     # a row whose cumulative mass comes this close to the target may keep one block more or fewer


def _check_mass_selection(w, Q, K, s_cap, p, min_keep):
    sel = bd.basa_select(Q, K, w.block, s_cap, mass_target=p, min_keep=min_keep)
    torch.cuda.synchronize()
    gpu_mask = unpack_mask(sel.mask_bits, sel.n_k)
    lo = max(1, min_keep)
    n_band = 0
    for h in range(Q.shape[1]):
        ref = o.select(np64(Q[0, h]), np64(K[0, h // (Q.shape[1] // K.shape[1])]), w.block, s_cap,
                       mass_target=p, min_keep=min_keep)
        cap, cum, m = ref["kappa"], ref["cum"], ref["m"]
        cnt = sel.row_count[0, h].cpu().numpy()
        cols = sel.row_cols[0, h].cpu().numpy()
        assert sel.row_cols.shape[-1] == cap
        for r in range(m.shape[0]):
            kg = int(cnt[r])
            assert min(lo, cap) <= kg <= cap, f"row {r}: count {kg} outside [{lo}, {cap}]"
            enough = kg == cap or cum[r, kg - 1] >= p - MASS_BAND
            minimal = kg == min(lo, cap) or cum[r, kg - 2] < p + MASS_BAND
            assert enough and minimal, f"head {h} row {r}: count {kg}, oracle {int(ref['count'][r])}"
            n_band += kg != int(ref["count"][r])
            # the kept set is the row's top-kg set (same tie band as the fixed-budget selection)
            top = o.select_top_kappa(m[r:r + 1], kg)
            top["m"] = m[r:r + 1]
            bad, _ = mask_report(gpu_mask[0, h, r:r + 1], top)
            assert bad == 0, f"head {h} row {r}: kept set is not the top-{kg} set"
            assert np.array_equal(np.flatnonzero(gpu_mask[0, h, r]), cols[r, :kg]), "bitmap and list disagree"
            if np.array_equal(gpu_mask[0, h, r], ref["mask"][r]):
                assert abs(float(sel.row_mass[0, h, r]) - ref["mass"][r]) <= 1e-4
    return sel, n_band


@pytest.mark.parametrize("w", [SMALL[0], SMALL[1], SMALL[3]], ids=lambda w: w.name)
def test_mass_selection_matches_oracle(w):
    Q, K, _ = gen(w)
    for p, min_keep, s_cap in ((0.5, 0, 0.0), (0.9, 4, 0.0), (0.95, 1, 0.5), (1.0, 0, 0.0), (1e-6, 3, 0.0)):
        _check_mass_selection(w, Q, K, s_cap, p, min_keep)


def test_mass_selection_then_attention_with_ragged_row_counts():
    """Rows keep different numbers of blocks; the attention kernel walks each row's own count."""
    w = SMALL[1]
    Q, K, V = gen(w)
    sel, _ = _check_mass_selection(w, Q, K, 0.0, 0.8, 2)
    cnt = sel.row_count.cpu().numpy()
    assert cnt.min() < cnt.max(), "the target mass should give rows of different lengths on this input"
    out = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, w.block, sel.perm_q, sel.perm_k)
    torch.cuda.synchronize()
    group = Q.shape[1] // K.shape[1]
    for h in range(Q.shape[1]):
        q, k, v = np64(Q[0, h]), np64(K[0, h // group]), np64(V[0, h // group])
        pq, pk = sel.perm_q[0, h].cpu().numpy().astype(np.int64), sel.perm_k[0, h // group].cpu().numpy().astype(np.int64)
        cols = sel.row_cols[0, h].cpu().numpy().astype(np.int64)
        out_h = np64(out[0, h])
        for g in range(sel.n_q):
            rows, O_ref, _ = o.sparse_attention_block(q, k, v, pq, pk, g, cols[g, :cnt[0, h, g]], w.block)
            check_output(out_h[rows], O_ref, w.dtype == "bf16", f"head {h} block {g}")


@pytest.mark.parametrize("mode", ["mass", "fixed"])
def test_total_budget_trims_rows_to_a_common_cap(mode):
    """budget_total: the integer rule is checked exactly on the counts the GPU itself asked for
    (they may differ from the fp64 oracle's by one near the mass target), the kept sets against
    the oracle's ranking of every row."""
    w = SMALL[1]
    Q, K, V = gen(w)
    kw = dict(mass_target=0.8, min_keep=2) if mode == "mass" else {}
    s_cap = 0.0 if mode == "mass" else 0.25
    free = bd.basa_select(Q, K, w.block, s_cap, **kw)
    asked = free.row_count.cpu().numpy().astype(np.int64)              # [1, H, Nq]
    H, n_q = asked.shape[1], asked.shape[2]
    floor = 2 if mode == "mass" else 1
    for G in (int(asked[0, 0].sum()) - 7, n_q * floor + 3, 1, int(asked.max()) * n_q + 5):
        sel = bd.basa_select(Q, K, w.block, s_cap, want_scores=True, budget_total=G, **kw)
        out = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, w.block, sel.perm_q, sel.perm_k)
        torch.cuda.synchronize()
        cnt = sel.row_count.cpu().numpy().astype(np.int64)
        gpu_mask = unpack_mask(sel.mask_bits, sel.n_k)
        group = H // K.shape[1]
        for h in range(H):
            cap = o.budget_cap(asked[0, h], G, floor, free.kappa)
            assert np.array_equal(cnt[0, h], np.minimum(asked[0, h], cap)), (mode, G, h)
            if cnt[0, h].sum() > G:
                assert cap == floor                                     # only the per-row minimum may break the budget
            ref = oracle_select(Q, K, h, w.block, s_cap, 1.0, o.SORT_QK)
            cols = sel.row_cols[0, h].cpu().numpy().astype(np.int64)
            for r in range(n_q):
                top = o.select_top_kappa(ref["m"][r:r + 1], int(cnt[0, h, r]))
                top["m"] = ref["m"][r:r + 1]
                assert mask_report(gpu_mask[0, h, r:r + 1], top)[0] == 0, (mode, G, h, r)
                assert np.array_equal(np.flatnonzero(gpu_mask[0, h, r]), cols[r, :cnt[0, h, r]])
            lists = [cols[r, :cnt[0, h, r]] for r in range(n_q)]
            O_ref = o.sparse_attention(np64(Q[0, h]), np64(K[0, h // group]), np64(V[0, h // group]),
                                       sel.perm_q[0, h].cpu().numpy(), sel.perm_k[0, h // group].cpu().numpy(),
                                       lists, w.block)
            check_output(np64(out[0, h]), O_ref, w.dtype == "bf16", f"budget {G} head {h}")
    if mode == "mass":
        assert asked.min() < asked.max(), "rows should ask for different numbers of blocks on this input"


# ------------------------------------------------------------------ attention
def _oracle_attention(Q, K, V, h, sel, block):
    hk = h // (Q.shape[1] // K.shape[1])
    return o.sparse_attention(np64(Q[0, h]), np64(K[0, hk]), np64(V[0, hk]), sel["perm_q"],
                              sel["perm_k"], sel["cols"], block, return_lse=True)


def _attn_with_oracle_selection(w, Q, K, V, s, beta=1.0, sort=o.SORT_QK):
    """GPU attention fed with the ORACLE's permutation and block lists."""
    H = Q.shape[1]
    refs = [oracle_select(Q, K, h, w.block, s, beta, sort) for h in range(H)]
    group = H // K.shape[1]
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a).astype(np.int32)).to(DEV)
    perm_q = i32(np.stack([r["perm_q"] for r in refs]))[None]
    perm_k = i32(np.stack([refs[hk * group]["perm_k"] for hk in range(K.shape[1])]))[None]
    cols = i32(np.stack([r["cols"] for r in refs]))[None]
    count = torch.full(cols.shape[:3], refs[0]["kappa"], dtype=torch.int32, device=DEV)
    out, lse = bd.basa_sparse_attn(Q, K, V, count, cols, w.block, perm_q, perm_k, want_lse=True)
    torch.cuda.synchronize()
    for h in range(H):
        O_ref, lse_ref = _oracle_attention(Q, K, V, h, refs[h], w.block)
        check_output(np64(out[0, h]), O_ref, w.dtype == "bf16", f"{w.name} head {h} s={s}")
        np.testing.assert_allclose(lse[0, h].cpu().numpy(), lse_ref, rtol=0, atol=2e-2 if w.dtype == "bf16" else 1e-4)


@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
def test_sparse_attention_matches_oracle(w):
    Q, K, V = gen(w)
    for s in w.sparsities:
        _attn_with_oracle_selection(w, Q, K, V, s)


@pytest.mark.parametrize("sort", [o.SORT_NONE, o.SORT_Q, o.SORT_K, o.SORT_QK])
def test_sparse_attention_every_sort_mode(sort):
    for w in (C[0], SMALL[4]):
        Q, K, V = gen(w)
        _attn_with_oracle_selection(w, Q, K, V, 0.5, 1.0, sort)


@pytest.mark.parametrize("w", [SMALL[0], SMALL[2], SMALL[3], SMALL[4], SMALL[6]], ids=lambda w: w.name)
def test_zero_sparsity_and_dense_entry_equal_dense_attention(w):
    Q, K, V = gen(w)
    sel = bd.basa_select(Q, K, w.block, 0.0)
    out = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, w.block, sel.perm_q, sel.perm_k)
    dense, lse = bd.basa_dense_attn(Q, K, V, w.block, want_lse=True)
    torch.cuda.synchronize()
    group = Q.shape[1] // K.shape[1]
    for h in range(Q.shape[1]):
        ref, lse_ref = o.dense_attention(np64(Q[0, h]), np64(K[0, h // group]), np64(V[0, h // group]), True)
        check_output(np64(out[0, h]), ref, w.dtype == "bf16", "s=0")
        check_output(np64(dense[0, h]), ref, w.dtype == "bf16", "dense entry")
        np.testing.assert_allclose(lse[0, h].cpu().numpy(), lse_ref, atol=2e-2 if w.dtype == "bf16" else 1e-4)


def test_end_to_end_gpu_selection_then_attention():
    for w in (SMALL[1], SMALL[4]):
        Q, K, V = gen(w)
        s = 0.5
        sel = bd.basa_select(Q, K, w.block, s)
        out = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, w.block, sel.perm_q, sel.perm_k)
        torch.cuda.synchronize()
        gpu_mask = unpack_mask(sel.mask_bits, sel.n_k)
        for h in range(Q.shape[1]):
            ref = oracle_select(Q, K, h, w.block, s, 1.0, o.SORT_QK)
            assert np.array_equal(sel.perm_q[0, h].cpu().numpy(), ref["perm_q"])
            assert np.array_equal(sel.perm_k[0, h // (Q.shape[1] // K.shape[1])].cpu().numpy(), ref["perm_k"])
            if not np.array_equal(gpu_mask[0, h], ref["mask"]):
                # differs only inside the don't-care band: the output is then checked against the
                # oracle's attention over the lists the GPU chose
                assert mask_report(gpu_mask[0, h], ref)[0] == 0
                ref = dict(ref, cols=sel.row_cols[0, h].cpu().numpy().astype(np.int64))
            O_ref, _ = _oracle_attention(Q, K, V, h, ref, w.block)
            check_output(np64(out[0, h]), O_ref, True, f"e2e {w.name} head {h}")


def test_cross_attention_lengths():
    w = SMALL[2]
    Q, K, V = gen(w)
    Qs = Q[:, :, :1000].contiguous()              # L_q != L_k, ragged query tail
    _attn_with_oracle_selection(w, Qs, K, V, 0.5)


def test_results_are_deterministic():
    w = SMALL[2]
    Q, K, V = gen(w)
    a = bd.basa_select(Q, K, w.block, 0.5)
    b = bd.basa_select(Q, K, w.block, 0.5)
    assert torch.equal(a.mask_bits, b.mask_bits) and torch.equal(a.row_cols, b.row_cols)
    o1 = bd.basa_sparse_attn(Q, K, V, a.row_count, a.row_cols, w.block, a.perm_q, a.perm_k)
    o2 = bd.basa_sparse_attn(Q, K, V, a.row_count, a.row_cols, w.block, a.perm_q, a.perm_k)
    assert torch.equal(o1, o2)
