"""Randomised differential test: many small random shapes and parameter combinations through
basa_select + basa_sparse_attn against the oracle (every head, every row).  Seeds are fixed, so
a failure names a reproducible case."""
import numpy as np
import pytest
import torch

from oracle import basa_oracle as o
from paper_2605_19726_amd import binding as bd
from parity_util import check_output, mask_report, np64, unpack_mask

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
N_CASES = 160
MASS_BAND = 1e-5


def _case(i):
    rng = np.random.default_rng(31000 + i)
    bf16 = bool(rng.integers(4))                    # three in four cases on the matrix-core path
    d = int(rng.choice([64, 128]))
    block = int(rng.choice([64, 128]))
    hk = int(rng.choice([1, 2, 3]))
    hq = hk * int(rng.choice([1, 2]))
    Lk = int(rng.integers(1, 900))
    Lq = Lk if rng.integers(3) else int(rng.integers(1, 900))
    s = float(rng.choice([0.0, 0.3, 0.5, 0.75, 0.9, 0.99]))
    sort = int(rng.integers(4))
    beta = float(rng.choice([0.0, 1.0, 0.5]))
    window = int(rng.choice([0, 0, block, 2 * block, 4 * block]))
    mass = float(rng.choice([0.0, 0.0, 0.6, 0.95]))
    min_keep = int(rng.choice([0, 1, 3]))
    scale = float(rng.choice([0.25, 1.0, 3.0]))
    segments = None
    if Lq == Lk and Lk > 4 and rng.integers(4) == 0:       # drawn last: earlier cases keep their inputs
        window = 0
        cuts = np.sort(rng.choice(np.arange(1, Lk), size=int(rng.integers(1, 4)), replace=False))
        segments = [0] + [int(v) for v in cuts]
    return dict(segments=segments, bf16=bf16, d=d, block=block, hq=hq, hk=hk, Lq=Lq, Lk=Lk, s=s, sort=sort, beta=beta, window=window,
                mass=mass, min_keep=min_keep, scale=scale, seed=int(rng.integers(1 << 30)))


@pytest.mark.parametrize("i", range(N_CASES))
def test_random_case(i):
    c = _case(i)
    g = torch.Generator().manual_seed(c["seed"])
    dt = torch.bfloat16 if c["bf16"] else torch.float32
    mk = lambda h, L, scale: (torch.randn((1, h, L, c["d"]), generator=g) * scale).to(dt).to(DEV)
    Q, K, V = mk(c["hq"], c["Lq"], c["scale"]), mk(c["hk"], c["Lk"], c["scale"]), mk(c["hk"], c["Lk"], 1.0)
    B = c["block"]
    sel = bd.basa_select(Q, K, B, c["s"], c["beta"], c["sort"], c["window"], want_scores=True,
                         mass_target=c["mass"], min_keep=c["min_keep"], segments=c["segments"])
    out, lse = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, B, sel.perm_q, sel.perm_k, want_lse=True,
                                    attn_shape=i % 4)
    torch.cuda.synchronize()
    if c["mass"] == 0:
        # the kernel that keeps the score map on chip: same bitmap, counts and lists
        chip = bd.basa_select(Q, K, B, c["s"], c["beta"], c["sort"], c["window"], segments=c["segments"], select_path=2)
        for name in ("mask_bits", "row_count", "row_cols", "perm_q", "perm_k"):
            assert torch.equal(getattr(chip, name), getattr(sel, name)), f"select_path 2, {name}: {c}"
        assert (chip.row_mass - sel.row_mass).abs().max().item() <= 2e-6, str(c)
    gpu_mask = unpack_mask(sel.mask_bits, sel.n_k)
    group = c["hq"] // c["hk"]
    what = str(c)
    for h in range(c["hq"]):
        q, k, v = np64(Q[0, h]), np64(K[0, h // group]), np64(V[0, h // group])
        ref = o.select(q, k, B, c["s"], c["beta"], c["sort"], c["window"],
                       mass_target=c["mass"] if c["mass"] > 0 else None, min_keep=c["min_keep"],
                       segments=c["segments"])
        assert np.array_equal(sel.perm_q[0, h].cpu().numpy(), ref["perm_q"]), what
        assert np.array_equal(sel.perm_k[0, h // group].cpu().numpy(), ref["perm_k"]), what
        sc = sel.scores[0, h].cpu().numpy().astype(np.float64)
        assert np.abs(sc - ref["logits"]).max() <= 1e-5 * max(1.0, np.abs(ref["logits"]).max()), what
        cnt = sel.row_count[0, h].cpu().numpy()
        cols = sel.row_cols[0, h].cpu().numpy().astype(np.int64)
        m = ref["m"]
        if c["mass"] > 0:
            cap, lo, cum = ref["kappa"], min(max(1, c["min_keep"]), ref["kappa"]), ref["cum"]
            for r in range(m.shape[0]):
                kg = int(cnt[r])
                assert lo <= kg <= cap, what
                assert kg == cap or cum[r, kg - 1] >= c["mass"] - MASS_BAND, what
                assert kg == lo or cum[r, kg - 2] < c["mass"] + MASS_BAND, what
                top = o.select_top_kappa(m[r:r + 1], kg)
                top["m"] = m[r:r + 1]
                assert mask_report(gpu_mask[0, h, r:r + 1], top)[0] == 0, what
        else:
            assert (cnt == ref["kappa"]).all(), what
            assert mask_report(gpu_mask[0, h], ref)[0] == 0, what
        lists = [cols[r, :cnt[r]] for r in range(m.shape[0])]
        for r, lst in enumerate(lists):
            assert np.array_equal(np.flatnonzero(gpu_mask[0, h, r]), lst), what
        O_ref, lse_ref = o.sparse_attention(q, k, v, ref["perm_q"], ref["perm_k"], lists, B, return_lse=True)
        check_output(np64(out[0, h]), O_ref, c["bf16"], what)
        np.testing.assert_allclose(lse[0, h].cpu().numpy(), lse_ref, rtol=0,
                                   atol=(3e-2 if c["bf16"] else 2e-4) * max(1.0, c["scale"] ** 2), err_msg=what)
