"""GPU parity of the selection-fidelity diagnostics (oracle block distribution of Eq. 3, block
norm metrics of Eq. 7, deviation bound of Eq. 8, recall / l1 / Pearson sums) against the numpy
oracle, through the C ABI.  Sizes keep the oracle's dense L x L map in memory."""
import numpy as np
import pytest
import torch

from oracle import basa_oracle as o
from paper_2605_19726_amd import binding as bd
from paper_2605_19726_amd import synth
from parity_util import np64, unpack_mask

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
C = synth.CONFIGS

# bf16 workloads on the matrix-core kernel (d = 128 and d = 64), ragged and GQA cases included, and the
# f32 configuration on the exact-arithmetic kernel
CASES = [
    C[1].scaled("lowrank_b64", heads_q=2, heads_kv=2, L=1536 + 64 * 3 + 17, salient_frac=0.05),
    C[4].scaled("lowrank_b128", heads_q=2, heads_kv=2, L=2048 + 128 + 5, salient_frac=0.05),
    C[2].scaled("multimodal_gqa", heads_q=4, heads_kv=2, L=2048, image_side=16),
    C[3].scaled("video_ragged", heads_q=2, heads_kv=2, L=4 * 20 * 21, video_thw=(4, 20, 21)),
    C[0].scaled("tiny_bf16_d64", dtype="bf16", L=900),
    C[1].scaled("lowrank_d64_b128", heads_q=2, heads_kv=1, d=64, block=128, L=1024 + 128 + 77, salient_frac=0.05),
    C[0],
    C[0].scaled("tiny_f32_d128_ragged", L=700, d=128, block=128, heads_q=2, heads_kv=1),
]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
@pytest.mark.parametrize("sorted_", [False, True])
def test_block_mass_deviation_and_lse(w, sorted_):
    Q, K, _ = synth.make_qkv(w, device=DEV)
    group = w.heads_q // w.heads_kv
    sort = bd.SORT_QK if sorted_ else bd.SORT_NONE
    sel = bd.basa_select(Q, K, w.block, 0.5, beta=0.0, sort=sort, want_scores=True)   # beta = 0: l of Eq. 2
    pq, pk = (sel.perm_q, sel.perm_k) if sorted_ else (None, None)
    m_hat, dev, lse = bd.basa_block_mass(Q, K, w.block, pq, pk, base_logits=sel.scores, want_dev=True, want_lse=True)
    torch.cuda.synchronize()
    for h in range(w.heads_q):
        q, k = np64(Q[0, h]), np64(K[0, h // group])
        if sorted_:
            q_ord, k_ord = q[sel.perm_q[0, h].cpu().numpy()], k[sel.perm_k[0, h // group].cpu().numpy()]
        else:
            q_ord, k_ord = q, k
        want = o.oracle_block_mass(q_ord, k_ord, w.block)
        got = m_hat[0, h].cpu().numpy().astype(np.float64)
        np.testing.assert_allclose(got.sum(1), 1.0, atol=2e-5)
        np.testing.assert_allclose(got, want, rtol=2e-4, atol=1e-7)
        want_dev = o.max_logit_deviation(q_ord, k_ord, w.block)
        np.testing.assert_allclose(dev[0, h].cpu().numpy(), want_dev, rtol=1e-4, atol=1e-4)
        _, lse_ref = o.dense_attention(q, k, k, return_lse=True)
        np.testing.assert_allclose(lse[0, h].cpu().numpy(), lse_ref, rtol=0, atol=1e-4)


@pytest.mark.parametrize("w", [C[0], CASES[0], CASES[3],
                               C[0].scaled("tiny_f32_d128_ragged", L=1000, d=128, block=128, heads_q=2, heads_kv=1)],
                         ids=lambda w: w.name)
def test_block_radius_and_deviation_bound(w):
    Q, K, _ = synth.make_qkv(w, device=DEV)
    group = w.heads_q // w.heads_kv
    perm_q = bd.basa_norm_sort(Q, w.block)
    rq, mq = bd.basa_block_radius(Q, w.block, perm_q)
    rk, mk = bd.basa_block_radius(K, w.block, None)
    U = bd.basa_deviation_bound(rq, mq, rk, mk, w.d)
    torch.cuda.synchronize()
    for h in range(w.heads_q):
        q = np64(Q[0, h])[perm_q[0, h].cpu().numpy()]
        k = np64(K[0, h // group])
        R, M = o.block_norm_metrics(q, w.block)
        np.testing.assert_allclose(rq[0, h].cpu().numpy(), R, rtol=2e-5)
        np.testing.assert_allclose(mq[0, h].cpu().numpy(), M, rtol=2e-5)
        Rk, Mk = o.block_norm_metrics(k, w.block)
        np.testing.assert_allclose(rk[0, h // group].cpu().numpy(), Rk, rtol=2e-5)
        np.testing.assert_allclose(mk[0, h // group].cpu().numpy(), Mk, rtol=2e-5)
        np.testing.assert_allclose(U[0, h].cpu().numpy(), o.deviation_bound(q, k, w.block), rtol=1e-4)


def test_selection_fidelity_and_pearson():
    w = CASES[1]
    Q, K, _ = synth.make_qkv(w, device=DEV)
    sel = bd.basa_select(Q, K, w.block, 0.5, want_scores=True)
    m_hat, _, _ = bd.basa_block_mass(Q, K, w.block, sel.perm_q, sel.perm_k)
    recall, l1 = bd.basa_selection_fidelity(sel.scores, sel.mask_bits, m_hat)
    sums = bd.basa_pearson_sums(sel.scores, m_hat)
    torch.cuda.synchronize()
    mask = unpack_mask(sel.mask_bits, sel.n_k)
    for h in range(w.heads_q):
        # fed with the GPU's own logits, mask and m_hat: this checks the row kernel alone
        m = o.row_softmax(sel.scores[0, h].cpu().numpy().astype(np.float64))
        rec_ref, l1_ref = o.selection_fidelity(m, mask[0, h], m_hat[0, h].cpu().numpy().astype(np.float64))
        np.testing.assert_allclose(recall[0, h].cpu().numpy(), rec_ref, rtol=1e-5, atol=1e-6)
        np.testing.assert_allclose(l1[0, h].cpu().numpy(), l1_ref, rtol=1e-4, atol=1e-6)
    x = sel.scores.cpu().numpy().astype(np.float64).ravel()
    y = m_hat.cpu().numpy().astype(np.float64).ravel()
    n, sx, sy, sxx, syy, sxy = sums.cpu().numpy()
    assert n == x.size
    r = (n * sxy - sx * sy) / np.sqrt((n * sxx - sx * sx) * (n * syy - sy * sy))
    assert abs(r - o.pearson_r(x, y)) < 1e-9
    np.testing.assert_allclose([sx, sy, sxx, syy, sxy], [x.sum(), y.sum(), (x * x).sum(), (y * y).sum(), (x * y).sum()],
                               rtol=1e-12)


def test_block_mass_without_deviation_output_and_its_limit():
    w = CASES[4]
    Q, K, _ = synth.make_qkv(w, device=DEV)
    m_hat, dev, lse = bd.basa_block_mass(Q, K, w.block)
    torch.cuda.synchronize()
    assert dev is None and lse is None
    want = o.oracle_block_mass(np64(Q[0, 0]), np64(K[0, 0]), w.block)
    np.testing.assert_allclose(m_hat[0, 0].cpu().numpy(), want, rtol=2e-4, atol=1e-7)
    # the deviation output keeps a row of block logits per query block in LDS: B = 64 allows 4096 key blocks
    L = 64 * 4097
    q = torch.zeros((1, 1, 64, 128), dtype=torch.bfloat16, device=DEV)
    k = torch.zeros((1, 1, L, 128), dtype=torch.bfloat16, device=DEV)
    base = torch.zeros((1, 1, 1, 4097), dtype=torch.float32, device=DEV)
    with pytest.raises(bd.BasaError) as e:
        bd.basa_block_mass(q, k, 64, base_logits=base, want_dev=True)
    assert e.value.status_name == "BASA_ERR_UNSUPPORTED"


@pytest.mark.parametrize("block", [128, 64])
def test_block_mass_is_the_same_bits_on_every_run_at_a_size_with_many_key_tiles(block):
    """Eq. 3 at 64K tokens, two heads, three runs: identical bits, and rows that sum to one.  (The block
    totals travel through LDS between the waves of a workgroup once per key block; a wait missing
    there showed as a few stale totals per ten thousand entries, different from run to run, and only
    at sizes like this one.)"""
    w = synth.CONFIGS[4].scaled("det", heads_q=2, heads_kv=2, L=65536, block=block)
    Q, K, _ = synth.make_qkv(w, device=DEV)
    perm_q, perm_k = bd.basa_norm_sort(Q, block), bd.basa_norm_sort(K, block)
    runs = []
    for _ in range(3):
        m_hat, _, lse = bd.basa_block_mass(Q, K, block, perm_q, perm_k, want_lse=True)
        torch.cuda.synchronize()
        runs.append((m_hat, lse))
    for m_hat, lse in runs[1:]:
        assert torch.equal(m_hat, runs[0][0]) and torch.equal(lse, runs[0][1])
    np.testing.assert_allclose(runs[0][0].sum(-1).cpu().numpy(), 1.0, atol=5e-5)
