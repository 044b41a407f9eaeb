"""CPU oracle for Block Approximate Sparse Attention (BA-Att).

TEST INFRASTRUCTURE ONLY.  This module is a plain, slow, fp64 numpy statement of
what the method computes.  It is imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg, never by the product path, and it shares no code,
tables or helpers with the HIP library.

Every function names the passage of the paper it follows (section, equation or
algorithm).  Where the paper leaves a choice open the choice is stated in the
docstring ("Reading:").

Conventions: one (batch, head) at a time; Q is [L_q, d], K and V are [L_k, d];
all arithmetic is float64 on the exact input values; block g of a (sorted)
sequence is positions [g*B, min((g+1)*B, L)).
"""
from __future__ import annotations

import math

import numpy as np

SORT_NONE, SORT_Q, SORT_K, SORT_QK = 0, 1, 2, 3


# --------------------------------------------------------------------------- #
# Budget
# --------------------------------------------------------------------------- #
def kappa_from_sparsity(n_k: int, sparsity: float) -> int:
    """Per-query-block budget kappa (Alg. 1, inputs) from a target sparsity.

    Reading: the paper links kappa and sparsity by no formula.  A sparsity s drops
    floor(s * N_k) key blocks from every row and keeps the rest, at least one:
    kappa = max(1, N_k - floor(s*N_k + 1e-9)).  The 1e-9 guards products such as
    0.6*590 that land a hair below an integer in binary.
    """
    if not (0.0 <= sparsity < 1.0):
        raise ValueError("sparsity must lie in [0, 1)")
    dropped = int(math.floor(float(sparsity) * n_k + 1e-9))
    return max(1, n_k - dropped)


def num_blocks(L: int, B: int) -> int:
    """N = ceil(L / B) (Sec. 2 defines N = L/B for L divisible by B).

    Reading: a ragged tail forms one short last block."""
    return (L + B - 1) // B


# --------------------------------------------------------------------------- #
# Norm-based ranking (Sec. 3.3, Eq. 9-10; Alg. 1 steps 1-2)
# --------------------------------------------------------------------------- #
def token_sort_keys(x: np.ndarray) -> np.ndarray:
    """Sort key of every token: its squared L2 norm (Eq. 9 up to a monotone map).

    Reading: the paper does not fix the precision of the norm.  The key is the
    fp64 sum of squares rounded once to fp32; equal fp32 keys are ties.  Squaring
    keeps the order of the norms and avoids a square root.
    """
    x64 = np.asarray(x, dtype=np.float64)
    return (x64 * x64).sum(axis=-1).astype(np.float32)


def norm_sort(x: np.ndarray, window: int = 0, segments=None) -> np.ndarray:
    """Permutation pi with keys non-decreasing along pi (Eq. 10).

    Reading: ties keep the original order (stable sort).  "(windowed) sort" of
    Alg. 1 step 1 is not defined in the paper; window = 0 is one sort over the
    whole sequence, window = W sorts each run of W consecutive tokens by itself.
    segments = [0, s_1, s_2, ...] (ascending token indices) is the same with runs
    of unequal length: tokens s_j .. s_{j+1}-1 (the last run ends at L) are sorted
    among themselves, so a modality or a frame keeps its range of positions.
    """
    keys = token_sort_keys(x)
    L = keys.shape[0]
    if segments is not None:
        if window:
            raise ValueError("window and segments exclude each other")
        starts = [int(v) for v in segments]
        if not starts or starts[0] != 0 or any(b <= a for a, b in zip(starts, starts[1:])) or starts[-1] >= max(L, 1):
            raise ValueError("segments must start at 0, ascend strictly and stay below L")
        bounds = starts + [L]
    else:
        W = L if not window else int(window)
        bounds = list(range(0, L, W)) + [L]
    perm = np.empty(L, dtype=np.int64)
    for w0, w1 in zip(bounds, bounds[1:]):
        perm[w0:w1] = w0 + np.argsort(keys[w0:w1], kind="stable")
    return perm


def identity_perm(L: int) -> np.ndarray:
    return np.arange(L, dtype=np.int64)


# --------------------------------------------------------------------------- #
# Block statistics (Sec. 3.1 mean pooling; Sec. 3.4 variances; Alg. 1 steps 3-4)
# --------------------------------------------------------------------------- #
def block_stats(x_sorted: np.ndarray, B: int):
    """Per-block mean and per-dimension variance of an already ordered sequence.

    Reading: Sigma = E[delta delta^T] over the block's tokens, so the variance is
    the population one (divide by the number of tokens in the block); a ragged
    last block uses its true token count.
    Returns (mean [N, d], var [N, d]).
    """
    x = np.asarray(x_sorted, dtype=np.float64)
    L, d = x.shape
    N = num_blocks(L, B)
    mean = np.zeros((N, d), dtype=np.float64)
    var = np.zeros((N, d), dtype=np.float64)
    for g in range(N):
        blk = x[g * B:min((g + 1) * B, L)]
        mean[g] = blk.sum(axis=0) / blk.shape[0]
        dev = blk - mean[g]
        var[g] = (dev * dev).sum(axis=0) / blk.shape[0]
    return mean, var


# --------------------------------------------------------------------------- #
# Block logits (Eq. 2), diagonal-variance compensation (Eq. 14), Alg. 1 steps 5-7
# --------------------------------------------------------------------------- #
def baseline_logits(q_mean: np.ndarray, k_mean: np.ndarray) -> np.ndarray:
    """l[g_q, g_k] = (Qbar . Kbar) / sqrt(d)   (Eq. 2, first line)."""
    d = q_mean.shape[1]
    return (q_mean @ k_mean.T) / math.sqrt(d)


def diag_compensation(q_mean, q_var, k_mean, k_var) -> np.ndarray:
    """Delta^[g_q, g_k] of Eq. 14: the three additive variance terms over d.

    Reading: Alg. 1 step 6 names Eq. 14, so all three printed terms are used,
    with the 1/d prefactor."""
    d = q_mean.shape[1]
    t1 = q_var @ (k_mean * k_mean).T       # Var[Q_t] * Kbar_t^2
    t2 = (q_mean * q_mean) @ k_var.T       # Var[K_t] * Qbar_t^2
    t3 = q_var @ k_var.T                   # Var[Q_t] * Var[K_t]
    return (t1 + t2 + t3) / d


def block_logits(q_mean, q_var, k_mean, k_var, beta: float = 1.0) -> np.ndarray:
    """l' = l + beta * Delta^   (Eq. 13 with Eq. 14; Alg. 1 step 7)."""
    l = baseline_logits(q_mean, k_mean)
    if beta == 0.0:
        return l
    return l + beta * diag_compensation(q_mean, q_var, k_mean, k_var)


def row_softmax(logits: np.ndarray) -> np.ndarray:
    """m' = softmax over key blocks of every query-block row (Eq. 2, second line)."""
    z = logits - logits.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


# --------------------------------------------------------------------------- #
# Selection (Alg. 1 steps 8-11)
# --------------------------------------------------------------------------- #
def select_top_kappa(m: np.ndarray, kappa: int):
    """Keep the kappa key blocks of largest m' in every row.

    Reading: equal values are ranked by lower key-block index first.
    Returns dict(mask [N_q, N_k] bool, cols [N_q, kappa] ascending int64,
    mass [N_q], theta [N_q] (smallest kept m'), next [N_q] (largest dropped m',
    -inf when nothing is dropped)).
    """
    n_q, n_k = m.shape
    kappa = min(int(kappa), n_k)
    mask = np.zeros((n_q, n_k), dtype=bool)
    cols = np.zeros((n_q, kappa), dtype=np.int64)
    mass = np.zeros(n_q)
    theta = np.zeros(n_q)
    nxt = np.full(n_q, -np.inf)
    for r in range(n_q):
        order = np.argsort(-m[r], kind="stable")      # descending, ties -> lower index
        keep = order[:kappa]
        mask[r, keep] = True
        cols[r] = np.sort(keep)
        mass[r] = m[r, keep].sum()
        theta[r] = m[r, order[kappa - 1]]
        if kappa < n_k:
            nxt[r] = m[r, order[kappa]]
    return dict(mask=mask, cols=cols, mass=mass, theta=theta, next=nxt)


def select_top_mass(m: np.ndarray, mass_target: float, min_keep: int = 1, cap: int | None = None):
    """Cumulative-mass reading of "the mask is built from m under a computational budget"
    (Sec. 3.1, sentence after Eq. 2): in every row keep the FEWEST key blocks, taken in order
    of decreasing m' (equal values: lower index first), whose m' sum to at least mass_target;
    never fewer than min_keep nor more than cap blocks (cap None: no cap).

    Returns dict(mask [N_q, N_k] bool, count [N_q] int64, cols: list of ascending int64 arrays,
    mass [N_q], cum [N_q, N_k]: cum[r, k-1] = sum of the k largest m' of row r).
    """
    n_q, n_k = m.shape
    cap = n_k if cap is None else min(int(cap), n_k)
    min_keep = max(1, min(int(min_keep), cap))
    mask = np.zeros((n_q, n_k), dtype=bool)
    count = np.zeros(n_q, dtype=np.int64)
    mass = np.zeros(n_q)
    cum = np.zeros((n_q, n_k))
    cols = []
    for r in range(n_q):
        order = np.argsort(-m[r], kind="stable")      # descending, ties -> lower index
        c = np.cumsum(m[r, order])
        cum[r] = c
        reached = np.nonzero(c >= mass_target)[0]
        k = int(reached[0]) + 1 if reached.size else n_k
        k = max(min_keep, min(k, cap))
        keep = order[:k]
        mask[r, keep] = True
        count[r] = k
        cols.append(np.sort(keep))
        mass[r] = c[k - 1]
    return dict(mask=mask, count=count, cols=cols, mass=mass, cum=cum)


def budget_cap(count, budget_total: int, floor: int, kappa: int) -> int:
    """Common per-row cap that fits a head's rows into a total budget of kept blocks.

    Reading (the paper speaks of "computational budgets", Sec. 3.1 after Eq. 2, without a rule
    for sharing one between rows): the rows that ask for the most are trimmed first, to a common
    cap t, the largest t in [floor, kappa] with sum_r min(count_r, t) <= budget_total; rows that
    ask for no more than t keep what they asked for.  If even t = floor does not fit, t = floor
    (the per-row minimum wins over the budget).
    """
    count = [int(c) for c in count]
    floor = max(1, min(int(floor), int(kappa)))
    best = floor
    for t in range(floor, int(kappa) + 1):
        if sum(min(c, t) for c in count) <= budget_total:
            best = t
    return best


def select_top_counts(m: np.ndarray, counts):
    """Row r keeps its counts[r] key blocks of largest m' (equal values: lower index first).
    Returns dict(mask, count, cols: list of ascending arrays, mass)."""
    n_q, n_k = m.shape
    mask = np.zeros((n_q, n_k), dtype=bool)
    cols, mass = [], np.zeros(n_q)
    for r in range(n_q):
        order = np.argsort(-m[r], kind="stable")
        keep = order[:int(counts[r])]
        mask[r, keep] = True
        cols.append(np.sort(keep))
        mass[r] = m[r, keep].sum()
    return dict(mask=mask, count=np.asarray(counts, dtype=np.int64), cols=cols, mass=mass)


# --------------------------------------------------------------------------- #
# Attention (Eq. 1; Sec. 2 block-sparse attention; Alg. 1 step 12)
# --------------------------------------------------------------------------- #
def dense_attention(Q, K, V, return_lse: bool = False):
    """softmax(Q K^T / sqrt(d)) V, every query against every key (Eq. 1)."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    d = Q.shape[1]
    S = (Q @ K.T) / math.sqrt(d)
    mx = S.max(axis=1, keepdims=True)
    P = np.exp(S - mx)
    den = P.sum(axis=1, keepdims=True)
    O = (P / den) @ V
    if return_lse:
        return O, (mx[:, 0] + np.log(den[:, 0]))
    return O


def attention_matrix(Q, K) -> np.ndarray:
    """A of Eq. 1 as an explicit L_q x L_k matrix (tiny inputs only)."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    S = (Q @ K.T) / math.sqrt(Q.shape[1])
    P = np.exp(S - S.max(axis=1, keepdims=True))
    return P / P.sum(axis=1, keepdims=True)


def sparse_attention_block(Q, K, V, perm_q, perm_k, g_q: int, cols_row, B: int):
    """Output rows of ONE query block g_q of the sorted order (Alg. 1 step 12).

    The block's queries Q'[i] = Q[perm_q[i]] attend to the tokens of the listed key
    blocks of K' = K[perm_k], V' = V[perm_k] only.
    Reading: the softmax is normalised over the kept tokens (Sec. 2: only the
    selected blocks' logits are computed).
    Returns (rows_original [n], O_rows [n, d], lse [n]).
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    L_q, d = Q.shape
    L_k = K.shape[0]
    qpos = np.arange(g_q * B, min((g_q + 1) * B, L_q))
    rows = np.asarray(perm_q)[qpos]
    kpos = np.concatenate([np.arange(c * B, min((c + 1) * B, L_k)) for c in cols_row])
    krows = np.asarray(perm_k)[kpos]
    S = (Q[rows] @ K[krows].T) / math.sqrt(d)
    mx = S.max(axis=1, keepdims=True)
    P = np.exp(S - mx)
    den = P.sum(axis=1, keepdims=True)
    O = (P / den) @ V[krows]
    return rows, O, mx[:, 0] + np.log(den[:, 0])


def sparse_attention(Q, K, V, perm_q, perm_k, cols, B: int, return_lse: bool = False):
    """Block-sparse attention over all query blocks, rows back in original order
    (Alg. 1 step 12: the inverse of pi_q is applied by writing row pi_q[i])."""
    L_q, d = np.asarray(Q).shape
    O = np.zeros((L_q, d), dtype=np.float64)
    lse = np.zeros(L_q, dtype=np.float64)
    for g in range(num_blocks(L_q, B)):
        rows, o, l = sparse_attention_block(Q, K, V, perm_q, perm_k, g, cols[g], B)
        O[rows] = o
        lse[rows] = l
    return (O, lse) if return_lse else O


# --------------------------------------------------------------------------- #
# The whole operator (Alg. 1)
# --------------------------------------------------------------------------- #
def select(Q, K, B: int, sparsity: float, beta: float = 1.0, sort: int = SORT_QK,
           window: int = 0, mass_target: float | None = None, min_keep: int = 1, segments=None,
           budget_total: int = 0):
    """Alg. 1 steps 1-11 for one head: permutations, block statistics, compensated
    logits, row distribution, top-kappa mask.  Returns a dict with every
    intermediate.  With mass_target the mask is the cumulative-mass one instead
    (select_top_mass), capped at the kappa that `sparsity` gives."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    perm_q = norm_sort(Q, window, segments) if sort in (SORT_Q, SORT_QK) else identity_perm(Q.shape[0])
    perm_k = norm_sort(K, window, segments) if sort in (SORT_K, SORT_QK) else identity_perm(K.shape[0])
    q_mean, q_var = block_stats(Q[perm_q], B)
    k_mean, k_var = block_stats(K[perm_k], B)
    logits = block_logits(q_mean, q_var, k_mean, k_var, beta)
    m = row_softmax(logits)
    kappa = kappa_from_sparsity(k_mean.shape[0], sparsity)
    if mass_target is None:
        sel = select_top_kappa(m, kappa)
    else:
        sel = select_top_mass(m, mass_target, min_keep, cap=kappa)
    out = dict(perm_q=perm_q, perm_k=perm_k, q_mean=q_mean, q_var=q_var, k_mean=k_mean,
               k_var=k_var, logits=logits, m=m, kappa=kappa)
    out.update(sel)
    if budget_total:
        # the head's rows share a total budget: a common cap on top of the per-row rule
        asked = sel["count"] if mass_target is not None else np.full(m.shape[0], min(kappa, m.shape[1]))
        cap = budget_cap(asked, budget_total, min_keep if mass_target is not None else 1, kappa)
        out.update(select_top_counts(m, np.minimum(asked, cap)))
        out["asked"], out["cap"] = asked, cap
    return out


def ba_att(Q, K, V, B: int, sparsity: float, beta: float = 1.0, sort: int = SORT_QK,
           window: int = 0):
    """Alg. 1 end to end for one head.  Returns (O [L_q, d], selection dict)."""
    sel = select(Q, K, B, sparsity, beta, sort, window)
    O = sparse_attention(Q, K, V, sel["perm_q"], sel["perm_k"], sel["cols"], B)
    return O, sel


# --------------------------------------------------------------------------- #
# Causal variant (Sec. 6 names autoregressive attention as future work; the paper's method is
# bidirectional).  Reading, all of it ours: causality is a property of ORIGINAL positions, so
# after any sorting the query at original index i may attend to the key at original index j
# iff j <= i + (L_k - L_q) (ends aligned when the lengths differ).  Block selection keeps its
# form (same statistics, same compensated logits of Eq. 2 / Eq. 14 over ALL tokens of a block);
# a block pair in which no token pair is visible is removed before the row softmax and the
# ranking, and a row keeps min(kappa, number of its live blocks) blocks.  No block is forced in:
# a query none of whose visible keys lie in its block's kept blocks attends to nothing and gets
# a zero output row and lse = -inf.
# --------------------------------------------------------------------------- #
def causal_offset(L_q: int, L_k: int) -> int:
    return int(L_k) - int(L_q)


def dense_causal_attention(Q, K, V, return_lse: bool = False):
    """Eq. 1 restricted to keys j <= i + (L_k - L_q); rows without a visible key are zero."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    L_q, d = Q.shape
    L_k = K.shape[0]
    off = causal_offset(L_q, L_k)
    S = (Q @ K.T) / math.sqrt(d)
    vis = np.arange(L_k)[None, :] <= (np.arange(L_q)[:, None] + off)
    S = np.where(vis, S, -np.inf)
    O = np.zeros((L_q, V.shape[1]))
    lse = np.full(L_q, -np.inf)
    for i in range(L_q):
        if not vis[i].any():
            continue
        mx = S[i].max()
        p = np.exp(S[i] - mx)
        den = p.sum()
        O[i] = (p / den) @ V
        lse[i] = mx + math.log(den)
    return (O, lse) if return_lse else O


def causal_live_blocks(perm_q, perm_k, B: int) -> np.ndarray:
    """live[g_q, g_k]: some query of block g_q (sorted order) may see some key of block g_k, i.e.
    the smallest original key index of g_k is <= the largest original query index of g_q + offset."""
    perm_q = np.asarray(perm_q)
    perm_k = np.asarray(perm_k)
    L_q, L_k = perm_q.shape[0], perm_k.shape[0]
    off = causal_offset(L_q, L_k)
    n_q, n_k = num_blocks(L_q, B), num_blocks(L_k, B)
    q_max = np.array([perm_q[g * B:min((g + 1) * B, L_q)].max() for g in range(n_q)])
    k_min = np.array([perm_k[g * B:min((g + 1) * B, L_k)].min() for g in range(n_k)])
    return k_min[None, :] <= (q_max[:, None] + off)


def select_causal(Q, K, B: int, sparsity: float, beta: float = 1.0, sort: int = SORT_QK, window: int = 0):
    """Alg. 1 steps 1-11 under the causal reading above.  Returns the dict of `select` with the
    logits of dead block pairs at -inf, `live`, per-row `count` and `cols` as a list of arrays."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    perm_q = norm_sort(Q, window) if sort in (SORT_Q, SORT_QK) else identity_perm(Q.shape[0])
    perm_k = norm_sort(K, window) if sort in (SORT_K, SORT_QK) else identity_perm(K.shape[0])
    q_mean, q_var = block_stats(Q[perm_q], B)
    k_mean, k_var = block_stats(K[perm_k], B)
    live = causal_live_blocks(perm_q, perm_k, B)
    logits = np.where(live, block_logits(q_mean, q_var, k_mean, k_var, beta), -np.inf)
    n_q, n_k = logits.shape
    kappa = kappa_from_sparsity(n_k, sparsity)
    m = np.zeros_like(logits)
    count = np.zeros(n_q, dtype=np.int64)
    mask = np.zeros((n_q, n_k), dtype=bool)
    cols, mass = [], np.zeros(n_q)
    theta = np.zeros(n_q)
    for r in range(n_q):
        n_live = int(live[r].sum())
        if n_live == 0:                       # every key lies after every query of the block
            cols.append(np.zeros(0, dtype=np.int64))
            continue
        z = logits[r] - logits[r][live[r]].max()
        e = np.where(live[r], np.exp(z), 0.0)
        m[r] = e / e.sum()
        count[r] = min(kappa, n_live)
        # ranking among the live blocks only; equal values: lower index first
        order = [c for c in np.argsort(-m[r], kind="stable") if live[r, c]]
        keep = np.array(order[:count[r]], dtype=np.int64)
        mask[r, keep] = True
        cols.append(np.sort(keep))
        mass[r] = m[r, keep].sum()
        theta[r] = m[r, order[count[r] - 1]]
    return dict(perm_q=perm_q, perm_k=perm_k, q_mean=q_mean, q_var=q_var, k_mean=k_mean, k_var=k_var,
                logits=logits, m=m, kappa=kappa, live=live, count=count, mask=mask, cols=cols, mass=mass,
                theta=theta)


def sparse_attention_causal_block(Q, K, V, perm_q, perm_k, g_q: int, cols_row, B: int):
    """Alg. 1 step 12 for one query block under the causal reading: the block's queries attend to
    the tokens of the listed key blocks whose original index does not exceed their own (+ offset);
    the softmax is over those tokens.  Returns (rows_original, O_rows, lse)."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    L_q, d = Q.shape
    L_k = K.shape[0]
    off = causal_offset(L_q, L_k)
    qpos = np.arange(g_q * B, min((g_q + 1) * B, L_q))
    rows = np.asarray(perm_q)[qpos]
    O = np.zeros((rows.shape[0], V.shape[1]))
    lse = np.full(rows.shape[0], -np.inf)
    if len(cols_row) == 0:
        return rows, O, lse
    kpos = np.concatenate([np.arange(c * B, min((c + 1) * B, L_k)) for c in cols_row])
    krows = np.asarray(perm_k)[kpos]
    S = (Q[rows] @ K[krows].T) / math.sqrt(d)
    vis = krows[None, :] <= (rows[:, None] + off)
    S = np.where(vis, S, -np.inf)
    for a in range(rows.shape[0]):
        if not vis[a].any():
            continue
        mx = S[a].max()
        p = np.exp(S[a] - mx)
        den = p.sum()
        O[a] = (p / den) @ V[krows]
        lse[a] = mx + math.log(den)
    return rows, O, lse


def sparse_attention_causal(Q, K, V, perm_q, perm_k, cols, B: int, return_lse: bool = False):
    L_q = np.asarray(Q).shape[0]
    O = np.zeros((L_q, np.asarray(V).shape[1]))
    lse = np.full(L_q, -np.inf)
    for g in range(num_blocks(L_q, B)):
        rows, o, l = sparse_attention_causal_block(Q, K, V, perm_q, perm_k, g, cols[g], B)
        O[rows] = o
        lse[rows] = l
    return (O, lse) if return_lse else O


# --------------------------------------------------------------------------- #
# Analysis quantities (Sec. 3.1 Eq. 3; Sec. 3.2 Eq. 5-8).  Tiny inputs only.
# --------------------------------------------------------------------------- #
def oracle_block_mass(Q, K, B: int) -> np.ndarray:
    """m_hat[g_q, g_k] (Eq. 3): mean over the block's query rows of the summed
    dense attention weight falling into key block g_k."""
    A = attention_matrix(Q, K)
    L_q, L_k = A.shape
    n_q, n_k = num_blocks(L_q, B), num_blocks(L_k, B)
    m_hat = np.zeros((n_q, n_k))
    for gq in range(n_q):
        rows = A[gq * B:min((gq + 1) * B, L_q)]
        for gk in range(n_k):
            m_hat[gq, gk] = rows[:, gk * B:min((gk + 1) * B, L_k)].sum() / rows.shape[0]
    return m_hat


def block_norm_metrics(x, B: int):
    """Radius R and max norm M of every block (Eq. 7)."""
    x = np.asarray(x, dtype=np.float64)
    mean, _ = block_stats(x, B)
    N = mean.shape[0]
    R = np.zeros(N)
    M = np.zeros(N)
    for g in range(N):
        blk = x[g * B:min((g + 1) * B, x.shape[0])]
        R[g] = np.sqrt(((blk - mean[g]) ** 2).sum(axis=1)).max()
        M[g] = np.sqrt((blk ** 2).sum(axis=1)).max()
    return R, M


def deviation_bound(Q, K, B: int) -> np.ndarray:
    """U[g_q, g_k] = (R^Q M^K + M^Q R^K + R^Q R^K) / sqrt(d)   (Eq. 8)."""
    d = np.asarray(Q).shape[1]
    Rq, Mq = block_norm_metrics(Q, B)
    Rk, Mk = block_norm_metrics(K, B)
    return (np.outer(Rq, Mk) + np.outer(Mq, Rk) + np.outer(Rq, Rk)) / math.sqrt(d)


def max_logit_deviation(Q, K, B: int) -> np.ndarray:
    """max over the token pairs (i, j) of a block pair of |l^_ij - l_{g_q,g_k}| with
    l^_ij = Q_i.K_j / sqrt(d) and l of Eq. 2: the observed deviation that Eq. 8 bounds and
    Fig. 2 plots against the bound.  Q and K are taken in the order given."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    d = Q.shape[1]
    q_mean, _ = block_stats(Q, B)
    k_mean, _ = block_stats(K, B)
    l_blk = baseline_logits(q_mean, k_mean)
    l_tok = (Q @ K.T) / math.sqrt(d)
    n_q, n_k = l_blk.shape
    dev = np.zeros((n_q, n_k))
    for gq in range(n_q):
        for gk in range(n_k):
            blk = l_tok[gq * B:(gq + 1) * B, gk * B:(gk + 1) * B]
            dev[gq, gk] = np.abs(blk - l_blk[gq, gk]).max()
    return dev


def pearson_r(x, y) -> float:
    """Pearson correlation coefficient (the R of Fig. 2)."""
    x = np.asarray(x, dtype=np.float64).ravel()
    y = np.asarray(y, dtype=np.float64).ravel()
    xc, yc = x - x.mean(), y - y.mean()
    return float((xc * yc).sum() / math.sqrt((xc * xc).sum() * (yc * yc).sum()))


def selection_fidelity(m: np.ndarray, mask: np.ndarray, m_hat: np.ndarray):
    """Per query block: the oracle mass (Eq. 3) that the kept blocks hold, and the l1
    distance between the block distribution m' and the oracle distribution m_hat
    (the quantity the deviation analysis of Sec. 3.2 sets out to control)."""
    recall = np.where(mask, m_hat, 0.0).sum(axis=1)
    l1 = np.abs(m - m_hat).sum(axis=1)
    return recall, l1
