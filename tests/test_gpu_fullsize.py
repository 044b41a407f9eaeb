"""GPU parity at the benchmark's full sizes (configurations 1-4), in the launch configuration
bench.py times.  Selection (permutations, logits, block mask) is compared with the oracle on
every head; attention output is compared on sampled (head, query block) units, which the
oracle computes one by one."""
import numpy as np
import pytest
import torch

from oracle import basa_oracle as o
from paper_2605_19726_amd import binding as bd
from paper_2605_19726_amd import synth
from parity_util import check_output, mask_report, np64, unpack_mask

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
UNITS_PER_CONFIG = 64


def _sample_units(w, rng):
    """(head, query block) units: block 0 and the last (possibly ragged) block of some heads,
    one unit per KV group, the rest random."""
    n_q = w.n_blocks
    group = w.heads_q // w.heads_kv
    units = {(0, 0), (0, n_q - 1), (w.heads_q - 1, n_q - 1)}
    for hk in range(w.heads_kv):
        units.add((hk * group + int(rng.integers(group)), int(rng.integers(n_q))))
    heads = rng.choice(w.heads_q, size=min(8, w.heads_q), replace=False)
    while len(units) < UNITS_PER_CONFIG:
        units.add((int(rng.choice(heads)), int(rng.integers(n_q))))
    return sorted(units)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_full_size_selection_and_attention(cfg):
    w = synth.CONFIGS[cfg]
    Q, K, V = synth.make_qkv(w, device=DEV)
    group = w.heads_q // w.heads_kv
    rng = np.random.default_rng(1000 + cfg)
    units = _sample_units(w, rng)
    unit_heads = sorted({h for h, _ in units})

    sels = {s: bd.basa_select(Q, K, w.block, s, want_scores=(s == w.sparsities[0])) for s in w.sparsities}
    outs = {}
    for s, sel in sels.items():
        outs[s] = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, w.block, sel.perm_q, sel.perm_k)
    torch.cuda.synchronize()
    s0 = w.sparsities[0]
    scores = sels[s0].scores
    masks = {s: unpack_mask(sel.mask_bits, sel.n_k) for s, sel in sels.items()}

    stats = dict(dontcare=0, max_logit_err=0.0, max_abs=0.0, max_rel=0.0)
    k_cache = {}
    for h in range(w.heads_q):
        hk = h // group
        q = np64(Q[0, h])
        if hk not in k_cache:
            k_cache.clear()
            k_cache[hk] = np64(K[0, hk])
        k = k_cache[hk]
        base = o.select(q, k, w.block, s0)          # permutations, statistics, logits: sparsity-free
        assert np.array_equal(sels[s0].perm_q[0, h].cpu().numpy(), base["perm_q"]), f"perm_q head {h}"
        assert np.array_equal(sels[s0].perm_k[0, hk].cpu().numpy(), base["perm_k"]), f"perm_k head {hk}"
        err = np.abs(scores[0, h].cpu().numpy().astype(np.float64) - base["logits"]).max()
        scale = max(1.0, np.abs(base["logits"]).max())
        stats["max_logit_err"] = max(stats["max_logit_err"], err / scale)
        assert err <= 1e-5 * scale, f"head {h}: logits off by {err:.3e} (scale {scale:.2f})"
        refs = {}
        for s in w.sparsities:
            ref = dict(base)
            ref["kappa"] = o.kappa_from_sparsity(base["m"].shape[1], s)
            ref.update(o.select_top_kappa(base["m"], ref["kappa"]))
            bad, dc = mask_report(masks[s][0, h], ref)
            stats["dontcare"] += dc - ref["mask"].shape[0]
            assert bad == 0, f"cfg{cfg} s={s} head {h}: {bad} mask mismatches outside the don't-care band"
            assert (sels[s].row_count[0, h].cpu().numpy() == ref["kappa"]).all()
            refs[s] = ref
        if h in unit_heads:
            v = np64(V[0, hk])
            for s in w.sparsities:
                cols_gpu = sels[s].row_cols[0, h].cpu().numpy().astype(np.int64)
                out_h = np64(outs[s][0, h])
                for (hh, g) in units:
                    if hh != h:
                        continue
                    # the attention kernel is checked on the block list it was given (equal to the
                    # oracle's except inside the don't-care band, which the mask check above covers)
                    rows, O_ref, _ = o.sparse_attention_block(q, k, v, base["perm_q"], base["perm_k"], g,
                                                              cols_gpu[g], w.block)
                    ma, rl = check_output(out_h[rows], O_ref, True, f"cfg{cfg} s={s} unit ({h},{g})")
                    stats["max_abs"] = max(stats["max_abs"], ma)
                    stats["max_rel"] = max(stats["max_rel"], rl)
    print(f"\n[cfg{cfg}] units={len(units)} dontcare_blocks={stats['dontcare']} "
          f"max_rel_logit_err={stats['max_logit_err']:.2e} out_max_abs={stats['max_abs']:.2e} "
          f"out_max_relL2={stats['max_rel']:.2e}")


def test_full_size_dense_entry_sampled():
    """Dense baseline at the largest configuration, checked on sampled query blocks of one head."""
    w = synth.CONFIGS[4]
    Q, K, V = synth.make_qkv(w, device=DEV)
    out = bd.basa_dense_attn(Q, K, V, w.block)
    torch.cuda.synchronize()
    h = 5
    q, k, v = np64(Q[0, h]), np64(K[0, h]), np64(V[0, h])
    for g in (0, 511, w.n_blocks - 1):
        rows = np.arange(g * w.block, (g + 1) * w.block)
        ref = o.dense_attention(q[rows], k, v)
        check_output(np64(out[0, h, rows]), ref, True, f"dense block {g}")


def test_full_size_cumulative_mass_selection():
    """Cumulative-mass selection at the largest configuration: per-row counts on four heads against
    the oracle (inside the mass band), the kept sets being the rows' top-count sets."""
    w = synth.CONFIGS[4]
    Q, K, _ = synth.make_qkv(w, device=DEV)
    p_mass, band = 0.6, 1e-5
    sel = bd.basa_select(Q, K, w.block, 0.0, mass_target=p_mass, min_keep=8)
    torch.cuda.synchronize()
    mask = unpack_mask(sel.mask_bits, sel.n_k)
    for h in (0, 7, 19, 31):
        ref = o.select(np64(Q[0, h]), np64(K[0, h]), w.block, 0.0, mass_target=p_mass, min_keep=8)
        cnt = sel.row_count[0, h].cpu().numpy()
        cum, m = ref["cum"], ref["m"]
        rows = np.arange(m.shape[0])
        enough = (cnt == ref["kappa"]) | (cum[rows, cnt - 1] >= p_mass - band)
        minimal = (cnt == 8) | (cum[rows, np.maximum(cnt - 2, 0)] < p_mass + band)
        assert enough.all() and minimal.all(), f"head {h}: counts outside the band"
        order = np.argsort(-m, axis=1, kind="stable")
        for r in range(m.shape[0]):
            want = np.zeros(m.shape[1], dtype=bool)
            want[order[r, :cnt[r]]] = True
            diff = want != mask[0, h, r]
            if diff.any():
                theta = m[r, order[r, cnt[r] - 1]]
                assert (np.abs(m[r, diff] - theta) <= 1e-5 * theta).all(), f"head {h} row {r}"
        print(f"\n[cfg4 mass {p_mass}] head {h}: kept per row min {cnt.min()} mean {cnt.mean():.1f} max {cnt.max()}, "
              f"rows off the fp64 count: {(cnt != ref['count']).sum()}")


def test_full_size_block_mass_sampled():
    """Oracle block distribution (Eq. 3) at 128K on the GPU, checked on sampled query blocks of two
    heads against the oracle's dense attention rows of those queries."""
    w = synth.CONFIGS[4]
    Q, K, _ = synth.make_qkv(w, device=DEV)
    sel = bd.basa_select(Q, K, w.block, 0.5, beta=0.0, want_scores=True)
    m_hat, dev, _ = bd.basa_block_mass(Q, K, w.block, sel.perm_q, sel.perm_k, base_logits=sel.scores, want_dev=True)
    torch.cuda.synchronize()
    np.testing.assert_allclose(m_hat.sum(-1).cpu().numpy(), 1.0, atol=5e-5)
    B, n = w.block, w.n_blocks
    for h in (3, 30):
        q = np64(Q[0, h])[sel.perm_q[0, h].cpu().numpy()]
        k = np64(K[0, h])[sel.perm_k[0, h].cpu().numpy()]
        k_mean, _ = o.block_stats(k, B)
        for g in (0, 500, n - 1):
            qb = q[g * B:(g + 1) * B]
            A = o.attention_matrix(qb, k)                               # [128, L]
            want = A.reshape(B, n, B).sum(axis=(0, 2)) / B
            np.testing.assert_allclose(m_hat[0, h, g].cpu().numpy(), want, rtol=3e-4, atol=1e-9)
            l_tok = (qb @ k.T) / np.sqrt(w.d)
            l_blk = (qb.mean(0) @ k_mean.T) / np.sqrt(w.d)
            want_dev = np.abs(l_tok.reshape(B, n, B) - l_blk[None, :, None]).max(axis=(0, 2))
            np.testing.assert_allclose(dev[0, h, g].cpu().numpy(), want_dev, rtol=1e-4, atol=1e-4)


@pytest.mark.parametrize("sort", [o.SORT_QK, o.SORT_NONE])
def test_full_size_causal_attention_sampled(sort):
    """The causal variant at the largest configuration: the permutations are the oracle's, every sampled
    query block attends to its listed key blocks under the original-position mask (oracle, block by
    block, on the lists the GPU selection produced), the dense causal entry on sampled blocks too."""
    w = synth.CONFIGS[4]
    Q, K, V = synth.make_qkv(w, device=DEV)
    sel = bd.basa_select(Q, K, w.block, 0.5, sort=sort, causal=True)
    out, lse = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, w.block, sel.perm_q, sel.perm_k,
                                   causal=True, want_lse=True)
    torch.cuda.synchronize()
    n = w.n_blocks
    rng = np.random.default_rng(77)
    worst = 0.0
    for h in (0, 13, w.heads_q - 1):
        q, k, v = np64(Q[0, h]), np64(K[0, h]), np64(V[0, h])
        perm_q, perm_k = sel.perm_q[0, h].cpu().numpy(), sel.perm_k[0, h].cpu().numpy()
        if sort == o.SORT_QK:
            assert np.array_equal(perm_q, o.norm_sort(q)) and np.array_equal(perm_k, o.norm_sort(k))
        cnt = sel.row_count[0, h].cpu().numpy()
        cols = sel.row_cols[0, h].cpu().numpy().astype(np.int64)
        out_h, lse_h = np64(out[0, h]), lse[0, h].cpu().numpy().astype(np.float64)
        for g in [0, 1, n - 1] + rng.integers(n, size=4).tolist():
            rows, O_ref, lse_ref = o.sparse_attention_causal_block(q, k, v, perm_q, perm_k, g, cols[g, :cnt[g]], w.block)
            ma, _ = check_output(out_h[rows], O_ref, True, f"causal sort={sort} unit ({h},{g})")
            worst = max(worst, ma)
            seen = np.isfinite(lse_ref)
            assert np.array_equal(np.isfinite(lse_h[rows]), seen)
            # the row sum is taken over the bf16-rounded probabilities (relative error of each at most
            # 2^-9, so of the sum too: 1.95e-3 in the logarithm, reached by a row that sees one key whose
            # probability is not an exact power of two), plus the hardware exp2 / log2
            np.testing.assert_allclose(lse_h[rows][seen], lse_ref[seen], rtol=0, atol=2.5e-3)
    print(f"\n[cfg4 causal sort={sort}] kept per row mean {float(sel.row_count.float().mean()):.1f}, out_max_abs={worst:.2e}")
    if sort == o.SORT_NONE:
        dense = bd.basa_dense_attn(Q, K, V, w.block, causal=True)
        torch.cuda.synchronize()
        h = 5
        q, k, v = np64(Q[0, h]), np64(K[0, h]), np64(V[0, h])
        # rows a .. b-1 of the causal map are the oracle's suffix-aligned case with the keys cut at b
        for a, b in ((0, 128), (65536 - 64, 65536 + 64), (w.L - 128, w.L)):
            ref = o.dense_causal_attention(q[a:b], k[:b], v[:b])
            check_output(np64(dense[0, h, a:b]), ref, True, f"dense causal rows {a}..{b}")


def test_full_size_results_are_the_same_bits_on_every_run():
    """Selection and attention at the largest configuration, three runs into separate buffers: every
    output identical (both attention shapes the library chooses between, and the causal variant)."""
    w = synth.CONFIGS[4]
    Q, K, V = synth.make_qkv(w, device=DEV)
    first = None
    for _ in range(3):
        sel = bd.basa_select(Q, K, w.block, 0.5)
        outs = [bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, w.block, sel.perm_q, sel.perm_k,
                                    attn_shape=shape, want_lse=True) for shape in (3, 2)]
        selc = bd.basa_select(Q, K, w.block, 0.75, causal=True)
        outs.append(bd.basa_sparse_attn(Q, K, V, selc.row_count, selc.row_cols, w.block, selc.perm_q, selc.perm_k,
                                        causal=True, want_lse=True))
        torch.cuda.synchronize()
        got = [sel.mask_bits, sel.row_cols, sel.row_mass, sel.perm_q, sel.perm_k, selc.row_count, selc.row_cols]
        for o_, l_ in outs:
            got += [o_, l_]
        if first is None:
            first = got
        else:
            for i, (a, b) in enumerate(zip(first, got)):
                # (-inf == -inf in the log-sum-exp of blind causal rows; NaN nowhere)
                assert torch.equal(a, b), f"output {i} differs between runs"
