"""Pins for the CPU oracle: each test ties one oracle function to something the
paper or the mathematics fixes independently of the oracle's own code
(definitions written out by brute force in pure Python loops, closed forms,
invariants, special cases).  No GPU, no HIP library."""
import itertools
import math

import numpy as np
import pytest

from oracle import basa_oracle as o

RNG = np.random.default_rng(20260519)


def rand(L, d, scale=1.0):
    return RNG.standard_normal((L, d)) * scale


# ---------------------------------------------------------------- brute force helpers
def loop_dense_attention(Q, K, V):
    """Eq. 1 with explicit Python loops (no matmul, no broadcasting)."""
    L_q, d = Q.shape
    L_k = K.shape[0]
    O = np.zeros((L_q, V.shape[1]))
    A = np.zeros((L_q, L_k))
    for i in range(L_q):
        s = [sum(Q[i, t] * K[j, t] for t in range(d)) / math.sqrt(d) for j in range(L_k)]
        mx = max(s)
        e = [math.exp(x - mx) for x in s]
        den = sum(e)
        for j in range(L_k):
            A[i, j] = e[j] / den
            for t in range(V.shape[1]):
                O[i, t] += A[i, j] * V[j, t]
    return O, A


# ---------------------------------------------------------------- kappa
@pytest.mark.parametrize("n,s,expect", [
    (16, 0.5, 8), (512, 0.5, 256), (591, 0.5, 296), (591, 0.75, 148),
    (1024, 0.0, 1024), (1024, 0.5, 512), (1024, 0.75, 256), (1024, 0.9, 103),
    (590, 0.6, 236), (3, 0.99, 1), (1, 0.5, 1)])
def test_kappa_spot_values(n, s, expect):
    # kept = N - floor(s N), never below one block; every row keeps >= (1-s) N blocks
    k = o.kappa_from_sparsity(n, s)
    assert k == expect
    assert k >= (1 - s) * n - 1e-9 and k >= 1


def test_kappa_rejects_bad_sparsity():
    for s in (-0.1, 1.0, 1.5):
        with pytest.raises(ValueError):
            o.kappa_from_sparsity(10, s)


# ---------------------------------------------------------------- dense attention (Eq. 1)
def test_dense_attention_matches_python_loops():
    Q, K, V = rand(7, 5), rand(9, 5), rand(9, 3)
    O_loop, A_loop = loop_dense_attention(Q, K, V)
    np.testing.assert_allclose(o.dense_attention(Q, K, V), O_loop, rtol=0, atol=1e-13)
    np.testing.assert_allclose(o.attention_matrix(Q, K), A_loop, rtol=0, atol=1e-14)


def test_dense_attention_closed_forms():
    # all keys equal -> uniform weights -> output is the mean of V
    K = np.tile(rand(1, 4), (6, 1))
    V = rand(6, 4)
    np.testing.assert_allclose(o.dense_attention(rand(3, 4), K, V),
                               np.tile(V.mean(0), (3, 1)), atol=1e-14)
    # two keys, d=1: weight of key 0 is the logistic function of q (k0-k1)
    Q = np.array([[0.7]]); K = np.array([[1.5], [-0.5]]); V = np.array([[1.0], [0.0]])
    expect = 1.0 / (1.0 + math.exp(-0.7 * 2.0))
    assert abs(o.dense_attention(Q, K, V)[0, 0] - expect) < 1e-15
    # lse closed form for zero queries: log(L_k)
    _, lse = o.dense_attention(np.zeros((2, 3)), rand(5, 3), rand(5, 3), return_lse=True)
    np.testing.assert_allclose(lse, math.log(5), atol=1e-15)


# ---------------------------------------------------------------- P1: sparsity 0 == dense
@pytest.mark.parametrize("sort", [o.SORT_NONE, o.SORT_Q, o.SORT_K, o.SORT_QK])
@pytest.mark.parametrize("L,B", [(48, 8), (45, 8)])
def test_zero_sparsity_equals_dense_for_every_sort_mode(sort, L, B):
    Q, K, V = rand(L, 6), rand(L, 6), rand(L, 6)
    O, sel = o.ba_att(Q, K, V, B, 0.0, 1.0, sort)
    assert sel["mask"].all()
    O_loop, _ = loop_dense_attention(Q, K, V)
    np.testing.assert_allclose(O, O_loop, rtol=0, atol=1e-12)


def test_zero_sparsity_equals_dense_cross_lengths():
    Q, K, V = rand(20, 4), rand(37, 4), rand(37, 4)     # L_q != L_k, ragged key tail
    O, _ = o.ba_att(Q, K, V, 8, 0.0)
    np.testing.assert_allclose(O, o.dense_attention(Q, K, V), atol=1e-12)


# ---------------------------------------------------------------- P7: norm sort
def test_norm_sort_is_sorted_stable_permutation():
    x = rand(200, 8)
    x[50] = x[10]; x[120] = x[10]; x[11] = -x[10]        # constructed ties (same norm)
    perm = o.norm_sort(x)
    assert sorted(perm.tolist()) == list(range(200))
    norms = [math.sqrt(sum(float(v) ** 2 for v in x[i])) for i in perm]
    assert all(norms[i] <= norms[i + 1] * (1 + 1e-7) for i in range(199))
    pos = {int(t): i for i, t in enumerate(perm)}
    assert pos[10] < pos[11] < pos[50] < pos[120]        # ties keep original order
    assert pos[11] == pos[10] + 1 and pos[50] == pos[10] + 2 and pos[120] == pos[10] + 3


def test_norm_sort_matches_python_sorted():
    x = rand(97, 3)
    keys = [np.float32(sum(float(v) * float(v) for v in row)) for row in x]
    expect = sorted(range(97), key=lambda i: (keys[i], i))
    assert o.norm_sort(x).tolist() == expect


def test_windowed_sort_stays_in_window():
    x = rand(100, 4)
    perm = o.norm_sort(x, window=32)
    for w0 in range(0, 100, 32):
        seg = perm[w0:w0 + 32]
        assert sorted(seg.tolist()) == list(range(w0, min(w0 + 32, 100)))
        k = o.token_sort_keys(x)[seg]
        assert (np.diff(k) >= 0).all()
    assert o.norm_sort(x, window=0).tolist() == o.norm_sort(x, window=100).tolist()


def test_segment_sort_against_python_sorted_per_segment():
    x = rand(97, 3)
    x[40] = x[12]                                  # a tie across segments and one inside
    x[13] = x[12]
    keys = [np.float32(sum(float(v) * float(v) for v in row)) for row in x]
    starts = [0, 5, 6, 50]
    perm = o.norm_sort(x, segments=starts)
    expect = []
    for a, b in zip(starts, starts[1:] + [97]):
        expect += sorted(range(a, b), key=lambda i: (keys[i], i))
    assert perm.tolist() == expect
    assert perm[5] == 5                            # a one-token segment stays where it is
    # one segment is the global sort; equal segments are the windowed sort
    assert o.norm_sort(x, segments=[0]).tolist() == o.norm_sort(x).tolist()
    assert o.norm_sort(x, segments=[0, 32, 64, 96]).tolist() == o.norm_sort(x, window=32).tolist()
    for bad in ([], [1, 5], [0, 5, 5], [0, 97], [0, 9, 3]):
        with pytest.raises(ValueError):
            o.norm_sort(x, segments=bad)
    with pytest.raises(ValueError):
        o.norm_sort(x, window=32, segments=[0, 32])


def test_select_with_segments_only_changes_the_permutations():
    Q, K = rand(70, 4), rand(70, 4)
    starts = [0, 16, 48]
    ref = o.select(Q, K, 8, 0.5, segments=starts)
    assert ref["perm_q"].tolist() == o.norm_sort(Q, segments=starts).tolist()
    assert ref["perm_k"].tolist() == o.norm_sort(K, segments=starts).tolist()
    qm, qv = o.block_stats(Q[ref["perm_q"]], 8)
    assert np.array_equal(qm, ref["q_mean"]) and np.array_equal(qv, ref["q_var"])


def test_budget_cap_against_brute_force_and_its_properties():
    rng = np.random.default_rng(8)
    for _ in range(200):
        n, kappa = int(rng.integers(1, 9)), int(rng.integers(1, 7))
        floor = int(rng.integers(1, kappa + 1))
        count = rng.integers(floor, kappa + 1, size=n)
        G = int(rng.integers(0, n * kappa + 3))
        t = o.budget_cap(count, G, floor, kappa)
        total = lambda c: int(np.minimum(count, c).sum())
        fits = [c for c in range(floor, kappa + 1) if total(c) <= G]
        assert t == (max(fits) if fits else floor)
        assert floor <= t <= kappa
        if fits:
            assert total(t) <= G and (t == kappa or total(t + 1) > G)
        # rows that asked for no more than the cap keep what they asked for
        assert (np.minimum(count, t)[count <= t] == count[count <= t]).all()
        # a larger budget never lowers the cap
        assert o.budget_cap(count, G + 1, floor, kappa) >= t
    # closed forms: equal requests share the budget evenly; a budget that covers everything changes nothing
    assert o.budget_cap([5, 5, 5, 5], 12, 1, 5) == 3
    assert o.budget_cap([5, 2, 1], 8, 1, 5) == 5
    assert o.budget_cap([5, 2, 1], 7, 1, 5) == 4
    assert o.budget_cap([4, 4], 1, 2, 4) == 2                      # the per-row minimum wins


def test_select_with_a_total_budget_trims_the_greediest_rows():
    Q, K = rand(128, 4), rand(128, 4)
    free = o.select(Q, K, 8, 0.0, mass_target=0.7, min_keep=2)
    asked = free["count"]
    assert asked.min() < asked.max() and asked.sum() - 5 >= 2 * len(asked)     # the case is not degenerate
    G = int(asked.sum()) - 5
    ref = o.select(Q, K, 8, 0.0, mass_target=0.7, min_keep=2, budget_total=G)
    assert ref["count"].sum() <= G and (ref["count"] == np.minimum(asked, ref["cap"])).all()
    for r in range(len(asked)):
        # the kept set of a trimmed row is the head of its own ranking
        top = o.select_top_kappa(ref["m"][r:r + 1], int(ref["count"][r]))
        assert np.array_equal(top["mask"][0], ref["mask"][r])
        assert set(ref["cols"][r]) <= set(free["cols"][r])
    # fixed-count mode: the budget lowers the common count
    fixed = o.select(Q, K, 8, 0.0, budget_total=16 * 3 + 2)
    assert (fixed["count"] == 3).all()
    # a budget nobody exceeds changes nothing
    same = o.select(Q, K, 8, 0.0, mass_target=0.7, min_keep=2, budget_total=int(asked.sum()))
    assert np.array_equal(same["mask"], free["mask"])


def test_sort_key_is_fp32_rounded_squared_norm():
    x = np.array([[3.0, 4.0], [1e-3, 0.0]])
    k = o.token_sort_keys(x)
    assert k.dtype == np.float32 and k[0] == np.float32(25.0) and k[1] == np.float32(1e-6)


# ---------------------------------------------------------------- block stats (mean pooling, Sec. 3.1; variances Sec. 3.4)
def test_block_stats_against_loops_and_ragged_tail():
    x = rand(21, 3)
    mean, var = o.block_stats(x, 8)
    assert mean.shape == (3, 3)
    for g, (a, b) in enumerate([(0, 8), (8, 16), (16, 21)]):
        n = b - a
        for t in range(3):
            mu = sum(x[i, t] for i in range(a, b)) / n
            vv = sum((x[i, t] - mu) ** 2 for i in range(a, b)) / n
            assert abs(mean[g, t] - mu) < 1e-14 and abs(var[g, t] - vv) < 1e-14
    # deviations from the block mean average to zero (Sec. 3.4, below Eq. 11)
    assert np.abs((x[:8] - mean[0]).mean(0)).max() < 1e-15
    # single-token block: zero variance
    m1, v1 = o.block_stats(rand(9, 2), 8)
    assert (v1[1] == 0).all()


# ---------------------------------------------------------------- P2: Eq. 3 oracle distribution
def test_oracle_block_mass_is_pooled_dense_attention():
    L, B, d = 6, 2, 3            # the shape of the paper's Fig. 1 illustration
    Q, K = rand(L, d), rand(L, d)
    _, A = loop_dense_attention(Q, K, np.zeros((L, 1)))
    m_hat = o.oracle_block_mass(Q, K, B)
    for gq, gk in itertools.product(range(3), range(3)):
        acc = 0.0
        for i in range(gq * B, (gq + 1) * B):
            for j in range(gk * B, (gk + 1) * B):
                acc += A[i, j]
        assert abs(m_hat[gq, gk] - acc / B) < 1e-14
    np.testing.assert_allclose(m_hat.sum(1), 1.0, atol=1e-14)
    assert (m_hat >= 0).all()


# ---------------------------------------------------------------- P3: homogeneous blocks (Sec. 3.2 interpretation)
def test_homogeneous_blocks_make_pre_and_post_downsample_agree():
    B, nb, d = 4, 5, 6
    Q = np.repeat(rand(nb, d), B, axis=0)
    K = np.repeat(rand(nb, d), B, axis=0)
    sel = o.select(Q, K, B, 0.4, 1.0, o.SORT_NONE)
    assert np.abs(sel["q_var"]).max() == 0 and np.abs(sel["k_var"]).max() == 0
    assert np.abs(o.diag_compensation(sel["q_mean"], sel["q_var"], sel["k_mean"], sel["k_var"])).max() == 0
    assert np.abs(o.deviation_bound(Q, K, B)).max() < 1e-14
    np.testing.assert_allclose(sel["m"], o.oracle_block_mass(Q, K, B), atol=1e-14)


# ---------------------------------------------------------------- P4: Eq. 5 decomposition and Eq. 8 bound
def test_logit_decomposition_and_deviation_bound():
    L, B, d = 24, 6, 5
    Q, K = rand(L, d, 1.3), rand(L, d, 0.8)
    qm, _ = o.block_stats(Q, B)
    km, _ = o.block_stats(K, B)
    l = o.baseline_logits(qm, km)
    U = o.deviation_bound(Q, K, B)
    for i in range(L):
        for j in range(L):
            gq, gk = i // B, j // B
            lhat = float(Q[i] @ K[j]) / math.sqrt(d)
            dq, dk = Q[i] - qm[gq], K[j] - km[gk]
            rhs = (dq @ km[gk] + qm[gq] @ dk + dq @ dk) / math.sqrt(d)
            assert abs((lhat - l[gq, gk]) - rhs) < 1e-13          # Eq. 5 / Eq. 11
            assert abs(lhat - l[gq, gk]) <= U[gq, gk] + 1e-13       # Eq. 8


def test_baseline_logits_loop():
    qm, km = rand(3, 4), rand(5, 4)
    l = o.baseline_logits(qm, km)
    for a in range(3):
        for b in range(5):
            assert abs(l[a, b] - sum(qm[a, t] * km[b, t] for t in range(4)) / 2.0) < 1e-14


# ---------------------------------------------------------------- P5: Eq. 14 == variance of token logits under diagonal covariance
def test_compensation_is_token_logit_variance_for_d1():
    # d = 1: covariances are scalars, so the diagonal form of Eq. 14 is exact and must
    # equal the population variance of the n_q*n_k token logits of the block pair.
    L, B = 12, 4
    Q, K = rand(L, 1), rand(L, 1)
    qm, qv = o.block_stats(Q, B)
    km, kv = o.block_stats(K, B)
    delta = o.diag_compensation(qm, qv, km, kv)
    for gq in range(3):
        for gk in range(3):
            logits = [Q[i, 0] * K[j, 0] for i in range(gq * B, gq * B + B)
                      for j in range(gk * B, gk * B + B)]
            mu = sum(logits) / len(logits)
            var = sum((x - mu) ** 2 for x in logits) / len(logits)
            assert abs(delta[gq, gk] - var) < 1e-13


def test_compensation_with_axis_aligned_blocks():
    # tokens of a block vary along one coordinate axis at a time (different axis per
    # token pair, symmetric +-), so the block covariance is exactly diagonal for any d.
    d, B = 4, 8
    def axis_block(center, amps):
        rows = []
        for t in range(d):
            e = np.zeros(d); e[t] = amps[t]
            rows += [center + e, center - e]
        return np.array(rows)
    Qb = axis_block(rand(1, d)[0], [0.5, 1.0, 0.2, 0.7])
    Kb = axis_block(rand(1, d)[0], [0.3, 0.1, 0.9, 0.4])
    qm, qv = o.block_stats(Qb, B)
    km, kv = o.block_stats(Kb, B)
    cov_q = (Qb - qm[0]).T @ (Qb - qm[0]) / B
    assert np.abs(cov_q - np.diag(np.diag(cov_q))).max() < 1e-15
    logits = np.array([[Qb[i] @ Kb[j] / math.sqrt(d) for j in range(B)] for i in range(B)])
    var = ((logits - logits.mean()) ** 2).mean()
    assert abs(o.diag_compensation(qm, qv, km, kv)[0, 0] - var) < 1e-13


def test_compensation_terms_by_loops_and_beta():
    qm, qv, km, kv = rand(2, 3), np.abs(rand(2, 3)), rand(4, 3), np.abs(rand(4, 3))
    delta = o.diag_compensation(qm, qv, km, kv)
    for a in range(2):
        for b in range(4):
            acc = 0.0
            for t in range(3):
                acc += qv[a, t] * km[b, t] ** 2 + kv[b, t] * qm[a, t] ** 2 + qv[a, t] * kv[b, t]
            assert abs(delta[a, b] - acc / 3) < 1e-14
    base = o.baseline_logits(qm, km)
    np.testing.assert_allclose(o.block_logits(qm, qv, km, kv, 0.0), base, atol=0)
    np.testing.assert_allclose(o.block_logits(qm, qv, km, kv, 0.5), base + 0.5 * delta, atol=1e-15)
    np.testing.assert_allclose(o.block_logits(qm, qv, km, kv, 1.0), base + delta, atol=1e-15)


def test_single_contraction_form_of_compensated_logits():
    # l' is one dot product of length 3d between per-block feature vectors
    d = 6
    qm, qv, km, kv = rand(3, d), np.abs(rand(3, d)), rand(5, d), np.abs(rand(5, d))
    beta = 0.7
    fq = np.concatenate([qm / math.sqrt(d), beta * qv / d, beta * qm ** 2 / d], axis=1)
    fk = np.concatenate([km, km ** 2 + kv, kv], axis=1)
    np.testing.assert_allclose(fq @ fk.T, o.block_logits(qm, qv, km, kv, beta), atol=1e-12)


# ---------------------------------------------------------------- softmax (Eq. 2)
def test_row_softmax():
    l = rand(4, 7, 3.0)
    m = o.row_softmax(l)
    for r in range(4):
        den = sum(math.exp(v) for v in l[r])
        for c in range(7):
            assert abs(m[r, c] - math.exp(l[r, c]) / den) < 1e-14
    np.testing.assert_allclose(o.row_softmax(l + 1000.0), m, atol=1e-12)   # shift invariant, no overflow


# ---------------------------------------------------------------- P6: selection
def test_selection_properties_and_bruteforce():
    m = o.row_softmax(rand(9, 13, 2.0))
    for kappa in (1, 4, 13):
        sel = o.select_top_kappa(m, kappa)
        assert (sel["mask"].sum(1) == kappa).all()
        for r in range(9):
            ranked = sorted(range(13), key=lambda c: (-m[r, c], c))[:kappa]
            assert sorted(ranked) == sel["cols"][r].tolist()
            assert set(np.flatnonzero(sel["mask"][r]).tolist()) == set(ranked)
            kept = m[r, sel["mask"][r]]
            assert abs(sel["mass"][r] - kept.sum()) < 1e-15
            assert sel["mass"][r] >= kappa / 13 - 1e-15          # top-kappa mass >= uniform share
            assert sel["theta"][r] == kept.min()
            if kappa < 13:
                assert kept.min() >= m[r, ~sel["mask"][r]].max() == sel["next"][r]


def test_selection_ties_prefer_lower_block_index():
    m = np.array([[0.2, 0.2, 0.2, 0.2, 0.2], [0.1, 0.3, 0.3, 0.2, 0.1]])
    sel = o.select_top_kappa(m, 2)
    assert sel["cols"].tolist() == [[0, 1], [1, 2]]
    sel = o.select_top_kappa(m, 3)
    assert sel["cols"].tolist() == [[0, 1, 2], [1, 2, 3]]


def test_selection_is_nested_in_sparsity():
    Q, K = rand(96, 8), rand(96, 8)
    prev = None
    for s in (0.0, 0.25, 0.5, 0.75, 0.9):
        mask = o.select(Q, K, 8, s)["mask"]
        if prev is not None:
            assert (prev | mask == prev).all()
        prev = mask


# ---------------------------------------------------------------- cumulative-mass selection
def test_top_mass_is_the_smallest_sufficient_subset_bruteforce():
    """Over ALL subsets of a small row: no smaller subset reaches the target, and no subset of
    the same size carries more mass."""
    import itertools
    m = o.row_softmax(rand(5, 9, 2.0))
    for p in (0.05, 0.4, 0.7, 0.95, 0.999999):
        sel = o.select_top_mass(m, p)
        for r in range(5):
            k = int(sel["count"][r])
            best = {size: max(sum(m[r, c] for c in sub) for sub in itertools.combinations(range(9), size))
                    for size in range(1, 10)}
            smallest = min(size for size in range(1, 10) if best[size] >= p) if best[9] >= p else 9
            assert k == smallest
            assert abs(sel["mass"][r] - best[k]) < 1e-15
            assert sel["mask"][r].sum() == k and sel["cols"][r].tolist() == np.flatnonzero(sel["mask"][r]).tolist()
            assert abs(m[r, sel["mask"][r]].sum() - sel["mass"][r]) < 1e-15


def test_top_mass_closed_forms_and_limits():
    n = 16
    uniform = np.full((1, n), 1.0 / n)
    for p, want in ((0.01, 1), (0.25, 4), (0.26, 5), (0.5, 8), (1.0, 16)):
        sel = o.select_top_mass(uniform, p)
        assert sel["count"][0] == want and sel["cols"][0].tolist() == list(range(want))   # ties: lower index
    geo = np.array([[0.5, 0.25, 0.125, 0.0625, 0.0625]])
    assert [int(o.select_top_mass(geo, p)["count"][0]) for p in (0.5, 0.51, 0.75, 0.9, 1.0)] == [1, 2, 2, 4, 5]
    assert o.select_top_mass(geo[:, ::-1].copy(), 0.75)["cols"][0].tolist() == [3, 4]
    # floor and ceiling on the count
    assert o.select_top_mass(geo, 0.1, min_keep=3)["count"][0] == 3
    assert o.select_top_mass(geo, 0.99, cap=2)["count"][0] == 2
    assert o.select_top_mass(geo, 0.99, min_keep=4, cap=2)["count"][0] == 2
    # a target no prefix reaches (rounding): everything is kept
    assert o.select_top_mass(geo, 1.0 + 1e-9)["count"][0] == 5


def test_top_mass_agrees_with_top_kappa_and_is_nested_in_target():
    Q, K = rand(96, 8), rand(96, 8)
    prev = None
    for p in (0.2, 0.5, 0.8, 0.95):
        sel = o.select(Q, K, 8, 0.0, mass_target=p)
        m = sel["m"]
        for r in range(m.shape[0]):
            k = int(sel["count"][r])
            top = o.select_top_kappa(m[r:r + 1], k)
            assert (top["mask"][0] == sel["mask"][r]).all()
            assert sel["mass"][r] >= p and (k == 1 or sel["mass"][r] - top["theta"][0] < p)
        if prev is not None:
            assert (prev | sel["mask"] == sel["mask"]).all()
        prev = sel["mask"]
    capped = o.select(Q, K, 8, 0.75, mass_target=0.95)
    assert capped["count"].max() <= capped["kappa"] == 3


# ---------------------------------------------------------------- P8: sparse attention
def _tiny_case(L=40, d=4, B=8, s=0.5, sort=o.SORT_QK):
    Q, K, V = rand(L, d), rand(L, d), rand(L, d)
    sel = o.select(Q, K, B, s, 1.0, sort)
    return Q, K, V, sel


def test_sparse_attention_against_python_loops():
    # literal masked softmax over the tokens of the kept blocks, rows put back by pi_q
    L, d, B = 22, 3, 4                                   # ragged tails on both sides
    Q, K, V, sel = _tiny_case(L, d, B, 0.5)
    O = o.sparse_attention(Q, K, V, sel["perm_q"], sel["perm_k"], sel["cols"], B)
    Qs, Ks, Vs = Q[sel["perm_q"]], K[sel["perm_k"]], V[sel["perm_k"]]
    for i in range(L):
        gq = i // B
        js = [j for j in range(L) if sel["mask"][gq, j // B]]
        s = [sum(Qs[i, t] * Ks[j, t] for t in range(d)) / math.sqrt(d) for j in js]
        mx = max(s); e = [math.exp(x - mx) for x in s]; den = sum(e)
        for t in range(d):
            acc = sum(e[n] / den * Vs[j, t] for n, j in enumerate(js))
            assert abs(O[sel["perm_q"][i], t] - acc) < 1e-13


def test_sparse_attention_constant_values_and_linearity():
    Q, K, V, sel = _tiny_case()
    args = (sel["perm_q"], sel["perm_k"], sel["cols"], 8)
    c = np.tile(rand(1, 4), (40, 1))
    np.testing.assert_allclose(o.sparse_attention(Q, K, c, *args), c, atol=1e-14)
    V2 = rand(40, 4)
    lhs = o.sparse_attention(Q, K, 2.0 * V - 3.0 * V2, *args)
    rhs = 2.0 * o.sparse_attention(Q, K, V, *args) - 3.0 * o.sparse_attention(Q, K, V2, *args)
    np.testing.assert_allclose(lhs, rhs, atol=1e-13)


def test_kappa_one_is_dense_attention_inside_one_block():
    L, B = 32, 8
    Q, K, V = rand(L, 4), rand(L, 4), rand(L, 4)
    sel = o.select(Q, K, B, 0.99)
    assert sel["kappa"] == 1
    O = o.sparse_attention(Q, K, V, sel["perm_q"], sel["perm_k"], sel["cols"], B)
    for g in range(L // B):
        rows = sel["perm_q"][g * B:(g + 1) * B]
        c = int(sel["cols"][g, 0])
        kr = sel["perm_k"][c * B:(c + 1) * B]
        np.testing.assert_allclose(O[rows], o.dense_attention(Q[rows], K[kr], V[kr]), atol=1e-13)


def test_sparse_lse_ties_selection_to_oracle_block_mass():
    # exp(lse_sparse - lse_dense) is the dense attention mass that falls on the kept
    # tokens; its mean over a query block is the sum of m_hat (Eq. 3) over kept blocks.
    L, B = 48, 8
    Q, K, V, sel = _tiny_case(L, 4, B, 0.5)
    _, lse_s = o.sparse_attention(Q, K, V, sel["perm_q"], sel["perm_k"], sel["cols"], B, True)
    _, lse_d = o.dense_attention(Q, K, V, return_lse=True)
    ratio = np.exp(lse_s - lse_d)
    assert ((ratio > 0) & (ratio <= 1 + 1e-14)).all()
    m_hat_sorted = o.oracle_block_mass(Q[sel["perm_q"]], K[sel["perm_k"]], B)
    for g in range(L // B):
        rows = sel["perm_q"][g * B:(g + 1) * B]
        assert abs(ratio[rows].mean() - m_hat_sorted[g, sel["mask"][g]].sum()) < 1e-13


def test_key_permutation_invariance_and_query_equivariance():
    # permuting keys together with values leaves bidirectional attention unchanged;
    # permuting queries permutes output rows.
    Q, K, V = rand(16, 4), rand(16, 4), rand(16, 4)
    pk, pq = RNG.permutation(16), RNG.permutation(16)
    base = o.dense_attention(Q, K, V)
    np.testing.assert_allclose(o.dense_attention(Q, K[pk], V[pk]), base, atol=1e-14)
    np.testing.assert_allclose(o.dense_attention(Q[pq], K, V), base[pq], atol=1e-14)


# ---------------------------------------------------------------- P10: generator sanity on the tiny workload
def test_tiny_workload_selection_is_not_flat():
    from paper_2605_19726_amd import synth
    w = synth.CONFIGS[0]
    Q, K, V = synth.make_qkv(w)
    q, k = Q[0, 0].double().numpy(), K[0, 0].double().numpy()
    sel = o.select(q, k, w.block, 0.5)
    assert sel["kappa"] == 8
    # the shifted ("salient") key tokens carry the largest norms: they fill the last
    # sorted key blocks, which every query block keeps
    norms = np.sqrt((k ** 2).sum(1))
    salient_tokens = np.argsort(norms)[-3 * w.block:]
    last_blocks = sel["perm_k"][-3 * w.block:]
    assert len(set(salient_tokens.tolist()) & set(last_blocks.tolist())) == 3 * w.block
    assert sel["mask"][:, -3:].all()
    assert sel["mass"].min() > 0.5
    # without sorting, different query blocks keep different key blocks
    sel_ns = o.select(q, k, w.block, 0.5, 1.0, o.SORT_NONE)
    assert len({tuple(r) for r in sel_ns["cols"].tolist()}) > 4


# ---------------------------------------------------------------- fidelity diagnostics
def test_max_logit_deviation_by_loops_and_under_the_bound():
    Q, K = rand(22, 5), rand(19, 5)            # ragged last blocks on both sides
    B = 4
    dev = o.max_logit_deviation(Q, K, B)
    qm, _ = o.block_stats(Q, B)
    km, _ = o.block_stats(K, B)
    for gq in range(dev.shape[0]):
        for gk in range(dev.shape[1]):
            lb = float(qm[gq] @ km[gk]) / math.sqrt(5)
            want = max(abs(float(Q[i] @ K[j]) / math.sqrt(5) - lb)
                       for i in range(gq * B, min((gq + 1) * B, 22)) for j in range(gk * B, min((gk + 1) * B, 19)))
            assert abs(dev[gq, gk] - want) < 1e-13
    assert (dev <= o.deviation_bound(Q, K, B) + 1e-12).all()                      # Eq. 8
    same = np.repeat(rand(3, 5), 4, axis=0)                                        # homogeneous blocks
    assert np.abs(o.max_logit_deviation(same, same, 4)).max() < 1e-13


def test_pearson_r_closed_forms_and_library():
    x = rand(50, 1)[:, 0]
    assert abs(o.pearson_r(x, 2.0 * x + 1.0) - 1.0) < 1e-12
    assert abs(o.pearson_r(x, -0.5 * x) + 1.0) < 1e-12
    y = rand(50, 1)[:, 0]
    assert abs(o.pearson_r(x, y) - np.corrcoef(x, y)[0, 1]) < 1e-12
    assert abs(o.pearson_r(x, y) - o.pearson_r(y, x)) < 1e-15
    assert abs(o.pearson_r([0, 0, 1, 1], [0, 1, 0, 1])) < 1e-15


def test_selection_fidelity_limits():
    Q, K = rand(48, 6), rand(48, 6)
    sel = o.select(Q, K, 8, 0.5, sort=o.SORT_NONE)
    m_hat = o.oracle_block_mass(Q, K, 8)
    recall, l1 = o.selection_fidelity(sel["m"], sel["mask"], m_hat)
    full, _ = o.selection_fidelity(sel["m"], np.ones_like(sel["mask"]), m_hat)
    np.testing.assert_allclose(full, 1.0, atol=1e-12)                 # keeping everything keeps all mass
    assert ((recall > 0) & (recall < 1)).all() and ((l1 >= 0) & (l1 <= 2)).all()
    for r in range(6):
        assert abs(recall[r] - sum(m_hat[r, c] for c in sel["cols"][r])) < 1e-15
    _, zero = o.selection_fidelity(m_hat, sel["mask"], m_hat)
    assert np.abs(zero).max() == 0.0


# ---------------------------------------------------------------- value pins of the diagnostics (Eq. 3, Eq. 7-8, l1)
def test_block_radius_and_max_norm_closed_form():
    # Eq. 7 on blocks built from known points.  Block 0: {c, c + 2e1, c - 2e1} (mean c, every
    # deviation 0 or 2, so R = 2; norms |c|, |c + 2e1|, |c - 2e1|).  Block 1: a 3-4-0 triangle
    # {(0,0,0), (3,0,0), (0,4,0)}: mean (1, 4/3, 0), the farthest token from it is (0,4,0).
    c = np.array([1.0, -2.0, 0.5])
    e1 = np.array([1.0, 0.0, 0.0])
    x = np.stack([c, c + 2 * e1, c - 2 * e1, np.zeros(3), np.array([3.0, 0, 0]), np.array([0, 4.0, 0])])
    R, M = o.block_norm_metrics(x, 3)
    assert abs(R[0] - 2.0) < 1e-15
    assert abs(M[0] - math.sqrt(9.0 + 4.0 + 0.25)) < 1e-15               # |c + 2e1| = |(3, -2, 0.5)|
    assert abs(R[1] - math.sqrt(1.0 + (8.0 / 3.0) ** 2)) < 1e-15
    assert abs(M[1] - 4.0) < 1e-15
    # the values that plausible wrong definitions would give on block 1, all different from R, M
    rms = math.sqrt((1 + 16 / 9.0 + 4 + 16 / 9.0 + 1 + 64 / 9.0) / 3.0)
    for wrong in (rms, 2 * R[1], 1.0 + 8.0 / 3.0):                         # RMS radius, diameter-like, l1 radius
        assert abs(R[1] - wrong) > 0.1
    for wrong in (7.0 / 3.0, math.sqrt(1.0 + 16.0 / 9.0)):                 # mean norm, norm of the mean
        assert abs(M[1] - wrong) > 0.1


def test_block_norm_metrics_and_bound_by_python_loops():
    L_q, L_k, B, d = 23, 18, 5, 4                                          # ragged last blocks: 3 and 3 tokens
    Q, K = rand(L_q, d, 1.4) + 0.3, rand(L_k, d, 0.7) - 0.2

    def loops(x):
        L = x.shape[0]
        R, M = [], []
        for g in range((L + B - 1) // B):
            idx = range(g * B, min((g + 1) * B, L))
            mean = [sum(x[i, t] for i in idx) / len(idx) for t in range(d)]
            R.append(max(math.sqrt(sum((x[i, t] - mean[t]) ** 2 for t in range(d))) for i in idx))
            M.append(max(math.sqrt(sum(x[i, t] ** 2 for t in range(d))) for i in idx))
        return R, M

    Rq, Mq = o.block_norm_metrics(Q, B)
    Rk, Mk = o.block_norm_metrics(K, B)
    wRq, wMq = loops(Q)
    wRk, wMk = loops(K)
    for got, want in ((Rq, wRq), (Mq, wMq), (Rk, wRk), (Mk, wMk)):
        assert len(got) == len(want)
        for a, b in zip(got, want):
            assert abs(a - b) < 1e-14
    U = o.deviation_bound(Q, K, B)
    assert U.shape == (5, 4)
    for a in range(5):
        for b in range(4):
            want = (wRq[a] * wMk[b] + wMq[a] * wRk[b] + wRq[a] * wRk[b]) / math.sqrt(d)      # Eq. 8
            assert abs(U[a, b] - want) < 1e-13
    # closed form: blocks {+a, -a} along one axis have mean 0 and R = M = |a|, so U = 3 |a|^2 / sqrt(d)
    a = np.array([[2.0, 0.0], [-2.0, 0.0]])
    assert abs(o.deviation_bound(a, a, 2)[0, 0] - 3 * 4.0 / math.sqrt(2)) < 1e-14


def test_selection_fidelity_l1_and_recall_by_hand():
    m = np.array([[0.7, 0.3], [0.25, 0.75]])
    m_hat = np.array([[0.4, 0.6], [0.5, 0.5]])
    mask = np.array([[True, False], [False, True]])
    recall, l1 = o.selection_fidelity(m, mask, m_hat)
    assert abs(l1[0] - 0.6) < 1e-15 and abs(l1[1] - 0.5) < 1e-15           # |.3| + |.3| ; |.25| + |.25|
    assert abs(recall[0] - 0.4) < 1e-15 and abs(recall[1] - 0.5) < 1e-15
    # against explicit loops on a ragged random case (the sum of abs differs from their max)
    Q, K = rand(29, 3), rand(26, 3)
    sel = o.select(Q, K, 4, 0.5, sort=o.SORT_NONE)
    mh = o.oracle_block_mass(Q, K, 4)
    recall, l1 = o.selection_fidelity(sel["m"], sel["mask"], mh)
    for r in range(mh.shape[0]):
        want = 0.0
        for c in range(mh.shape[1]):
            want += abs(sel["m"][r, c] - mh[r, c])
        assert abs(l1[r] - want) < 1e-14
        assert l1[r] > np.abs(sel["m"][r] - mh[r]).max() + 1e-6
        assert abs(recall[r] - sum(mh[r, c] for c in range(mh.shape[1]) if sel["mask"][r, c])) < 1e-15


def test_oracle_block_mass_ragged_blocks_by_python_loops():
    # Eq. 3 with ragged last query AND key blocks: the mean is over the rows the block HAS
    L_q, L_k, B, d = 11, 14, 4, 3                                          # last blocks: 3 queries, 2 keys
    Q, K = rand(L_q, d, 1.2), rand(L_k, d, 0.9)
    A = [[0.0] * L_k for _ in range(L_q)]
    for i in range(L_q):
        logit = [sum(Q[i, t] * K[j, t] for t in range(d)) / math.sqrt(d) for j in range(L_k)]
        mx = max(logit)
        e = [math.exp(v - mx) for v in logit]
        z = sum(e)
        A[i] = [v / z for v in e]
    m_hat = o.oracle_block_mass(Q, K, B)
    assert m_hat.shape == (3, 4)
    for gq in range(3):
        rows = range(gq * B, min((gq + 1) * B, L_q))
        for gk in range(4):
            cols = range(gk * B, min((gk + 1) * B, L_k))
            want = sum(A[i][j] for i in rows for j in cols) / len(rows)
            assert abs(m_hat[gq, gk] - want) < 1e-14
        assert abs(sum(m_hat[gq]) - 1.0) < 1e-13                           # every row is a distribution
    # dividing the ragged row by B instead of its 3 rows would give 3/4
    assert abs(m_hat[2].sum() - 0.75) > 0.2


# ---------------------------------------------------------------- causal variant (our reading; Sec. 6 future work)
def loop_causal_attention(Q, K, V):
    L_q, L_k, d = Q.shape[0], K.shape[0], Q.shape[1]
    off = L_k - L_q
    O = [[0.0] * V.shape[1] for _ in range(L_q)]
    lse = [-math.inf] * L_q
    for i in range(L_q):
        js = [j for j in range(L_k) if j <= i + off]
        if not js:
            continue
        logit = [sum(Q[i, t] * K[j, t] for t in range(d)) / math.sqrt(d) for j in js]
        mx = max(logit)
        e = [math.exp(v - mx) for v in logit]
        z = sum(e)
        for c in range(V.shape[1]):
            O[i][c] = sum(e[a] * V[j, c] for a, j in enumerate(js)) / z
        lse[i] = mx + math.log(z)
    return np.array(O), np.array(lse)


@pytest.mark.parametrize("L_q,L_k", [(13, 13), (5, 12), (12, 5), (1, 9)])
def test_dense_causal_attention_matches_python_loops(L_q, L_k):
    Q, K, V = rand(L_q, 3, 1.5), rand(L_k, 3, 1.5), rand(L_k, 4)
    O, lse = o.dense_causal_attention(Q, K, V, return_lse=True)
    O_ref, lse_ref = loop_causal_attention(Q, K, V)
    np.testing.assert_allclose(O, O_ref, atol=1e-13)
    np.testing.assert_array_equal(np.isinf(lse), np.isinf(lse_ref))
    fin = np.isfinite(lse_ref)
    np.testing.assert_allclose(lse[fin], lse_ref[fin], atol=1e-13)
    if L_q > L_k:                                  # the first L_q - L_k queries precede every key
        assert np.abs(O[:L_q - L_k]).max() == 0 and np.isinf(lse[:L_q - L_k]).all()


def test_dense_causal_closed_forms():
    L, d = 9, 4
    Q, K, V = rand(L, d), rand(L, d), rand(L, 3)
    O, lse = o.dense_causal_attention(Q, K, V, return_lse=True)
    np.testing.assert_allclose(O[0], V[0], atol=1e-15)                       # the first token sees itself only
    assert abs(lse[0] - float(Q[0] @ K[0]) / math.sqrt(d)) < 1e-14
    O0, lse0 = o.dense_causal_attention(Q, np.zeros_like(K), V, return_lse=True)   # equal logits: prefix means
    for i in range(L):
        np.testing.assert_allclose(O0[i], V[:i + 1].mean(axis=0), atol=1e-14)
        assert abs(lse0[i] - math.log(i + 1)) < 1e-14
    # one query that follows every key: plain attention of that query
    q1 = rand(1, d)
    np.testing.assert_allclose(o.dense_causal_attention(q1, K, V), o.dense_attention(q1, K, V), atol=1e-14)
    # the last query of a square problem sees everything too
    np.testing.assert_allclose(O[-1], o.dense_attention(Q[-1:], K, V)[0], atol=1e-14)


def test_causal_live_blocks_bruteforce():
    rng = np.random.default_rng(3)
    for L_q, L_k, B in ((22, 22, 4), (10, 19, 4), (19, 10, 4)):
        pq, pk = rng.permutation(L_q), rng.permutation(L_k)
        live = o.causal_live_blocks(pq, pk, B)
        off = L_k - L_q
        for gq in range(live.shape[0]):
            for gk in range(live.shape[1]):
                want = any(pk[j] <= pq[i] + off for i in range(gq * B, min((gq + 1) * B, L_q))
                           for j in range(gk * B, min((gk + 1) * B, L_k)))
                assert live[gq, gk] == want
    # original order, equal lengths, B divides L: the block-lower-triangular pattern
    ident = np.arange(24)
    assert np.array_equal(o.causal_live_blocks(ident, ident, 4), np.tril(np.ones((6, 6), dtype=bool)))


@pytest.mark.parametrize("sort", [o.SORT_NONE, o.SORT_Q, o.SORT_K, o.SORT_QK])
@pytest.mark.parametrize("L_q,L_k,B", [(48, 48, 8), (45, 45, 8), (20, 37, 8)])
def test_causal_zero_sparsity_equals_dense_causal_for_every_sort_mode(sort, L_q, L_k, B):
    # sorting permutes keys (with their values) and output rows; visibility follows original positions
    Q, K, V = rand(L_q, 5, 1.3), rand(L_k, 5, 1.3), rand(L_k, 3)
    sel = o.select_causal(Q, K, B, 0.0, sort=sort)
    O, lse = o.sparse_attention_causal(Q, K, V, sel["perm_q"], sel["perm_k"], sel["cols"], B, return_lse=True)
    O_ref, lse_ref = o.dense_causal_attention(Q, K, V, return_lse=True)
    np.testing.assert_allclose(O, O_ref, atol=1e-12)
    np.testing.assert_allclose(lse, lse_ref, atol=1e-12)
    assert all(np.array_equal(c, np.nonzero(l)[0]) for c, l in zip(sel["cols"], sel["live"]))   # all live blocks, no dead one


def test_causal_selection_ranks_live_blocks_only():
    L, B, d = 64, 8, 4
    Q, K = rand(L, d, 1.5), rand(L, d, 1.5)
    for sort in (o.SORT_NONE, o.SORT_QK):
        plain = o.select(Q, K, B, 0.5, sort=sort)
        sel = o.select_causal(Q, K, B, 0.5, sort=sort)
        assert sel["kappa"] == 4
        for r in range(8):
            live = [c for c in range(8) if sel["live"][r, c]]
            assert sel["count"][r] == min(4, len(live)) == len(sel["cols"][r])
            # brute force: the live blocks by decreasing plain logit (ties: lower index)
            want = sorted(sorted(live, key=lambda c: (-plain["logits"][r, c], c))[:sel["count"][r]])
            assert list(sel["cols"][r]) == want
            assert np.isinf(sel["logits"][r][~sel["live"][r]]).all() and (sel["m"][r][~sel["live"][r]] == 0).all()
            assert abs(sel["m"][r].sum() - 1.0) < 1e-13
            # the distribution over the live blocks is the softmax of their plain logits
            z = np.array([plain["logits"][r, c] for c in live])
            ref = np.exp(z - z.max()) / np.exp(z - z.max()).sum()
            np.testing.assert_allclose(sel["m"][r][live], ref, atol=1e-14)
    # without sorting, row g sees blocks 0..g: the first rows keep fewer than kappa
    sel = o.select_causal(Q, K, B, 0.5, sort=o.SORT_NONE)
    assert list(sel["count"]) == [1, 2, 3, 4, 4, 4, 4, 4]


def test_sparse_causal_attention_against_python_loops_and_empty_rows():
    L, B, d = 40, 8, 4
    Q, K, V = rand(L, d, 1.4), rand(L, d, 1.4), rand(L, 3)
    sel = o.select_causal(Q, K, B, 0.5)
    pq, pk = sel["perm_q"], sel["perm_k"]
    O, lse = o.sparse_attention_causal(Q, K, V, pq, pk, sel["cols"], B, return_lse=True)
    for g in range(5):
        for i in range(g * B, (g + 1) * B):
            qi = pq[i]
            js = [pk[j] for c in sel["cols"][g] for j in range(c * B, (c + 1) * B) if pk[j] <= qi]
            if not js:
                assert np.abs(O[qi]).max() == 0 and np.isinf(lse[qi])
                continue
            logit = [float(Q[qi] @ K[j]) / math.sqrt(d) for j in js]
            mx = max(logit)
            e = [math.exp(v - mx) for v in logit]
            want = sum(w * V[j] for w, j in zip(e, js)) / sum(e)
            np.testing.assert_allclose(O[qi], want, atol=1e-13)
            assert abs(lse[qi] - (mx + math.log(sum(e)))) < 1e-13
    # a list that holds no visible key for the earliest queries: zero rows, lse -inf
    ident = np.arange(L)
    rows, Ob, lb = o.sparse_attention_causal_block(Q, K, V, ident, ident, 0, [0], B)
    assert np.isfinite(lb).all()                                         # the diagonal block: every query sees itself
    rows, Ob, lb = o.sparse_attention_causal_block(Q, K, V, ident, ident, 1, [2], B)
    assert np.abs(Ob).max() == 0 and np.isinf(lb).all()                  # a block that lies wholly in the future
    # constant values: every row with a visible key returns the constant
    Vc = np.full((L, 2), 0.75)
    Oc, lc = o.sparse_attention_causal(Q, K, Vc, pq, pk, sel["cols"], B, return_lse=True)
    np.testing.assert_allclose(Oc[np.isfinite(lc)], 0.75, atol=1e-14)


# ---------------------------------------------------------------- drift guard (no paper values: see the script's header)
def test_oracle_reproduces_its_stored_tiny_results():
    import importlib.util
    import json
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_oracle_fixtures", os.path.join(here, "make_oracle_fixtures.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.compute()
    with open(os.path.join(here, "oracle_tiny.json")) as f:
        stored = json.load(f)

    def same(a, b, path):
        if isinstance(a, dict):
            assert a.keys() == b.keys(), path
            for k in a:
                same(a[k], b[k], f"{path}/{k}")
        elif isinstance(a, list):
            assert len(a) == len(b), path
            for i, (x, y) in enumerate(zip(a, b)):
                same(x, y, f"{path}[{i}]")
        elif isinstance(a, float):
            assert abs(a - b) <= 1e-12 * max(1.0, abs(a)), f"{path}: {a} vs {b}"
        else:
            assert a == b, f"{path}: {a} vs {b}"
    same(now, stored, "")
