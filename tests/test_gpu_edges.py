"""GPU parity on the edges of the path: degenerate lengths (a single short block, one token),
batch > 1 with strided batches, inputs that tie everywhere, and the largest block map the
library accepts (4096 key blocks per row)."""
import numpy as np
import pytest
import torch

from oracle import basa_oracle as o
from paper_2605_19726_amd import binding as bd
from paper_2605_19726_amd import synth
from parity_util import check_output, mask_report, np64, unpack_mask

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
C = synth.CONFIGS


def _randn(shape, seed, dtype):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(shape, generator=g).to(dtype).to(DEV)


def _full_check(Q, K, V, block, s, bf16, what):
    """select + attention of [1, H, L, d] tensors against the oracle, every head, every row."""
    sel = bd.basa_select(Q, K, block, s, want_scores=True)
    out = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, block, sel.perm_q, sel.perm_k)
    torch.cuda.synchronize()
    gpu_mask = unpack_mask(sel.mask_bits, sel.n_k)
    group = Q.shape[1] // K.shape[1]
    for h in range(Q.shape[1]):
        q, k, v = np64(Q[0, h]), np64(K[0, h // group]), np64(V[0, h // group])
        ref = o.select(q, k, block, s)
        assert np.array_equal(sel.perm_q[0, h].cpu().numpy(), ref["perm_q"]), what
        assert np.array_equal(sel.perm_k[0, h // group].cpu().numpy(), ref["perm_k"]), what
        assert mask_report(gpu_mask[0, h], ref)[0] == 0, what
        assert (sel.row_count[0, h].cpu().numpy() == ref["kappa"]).all(), what
        cols = sel.row_cols[0, h].cpu().numpy().astype(np.int64)
        O_ref = o.sparse_attention(q, k, v, ref["perm_q"], ref["perm_k"], cols, block)
        check_output(np64(out[0, h]), O_ref, bf16, what)


@pytest.mark.parametrize("L", [1, 2, 63, 64, 65, 127, 128, 129, 257])
@pytest.mark.parametrize("block", [64, 128])
def test_degenerate_lengths_bf16(L, block):
    Q, K, V = (_randn((1, 2, L, 128), 100 + i + L, torch.bfloat16) for i in range(3))
    _full_check(Q, K, V, block, 0.5, True, f"bf16 L={L} B={block}")


@pytest.mark.parametrize("L", [1, 3, 64, 65, 130])
def test_degenerate_lengths_f32(L):
    Q, K, V = (_randn((1, 1, L, 64), 200 + i + L, torch.float32) for i in range(3))
    _full_check(Q, K, V, 64, 0.5, False, f"f32 L={L}")


def test_short_queries_long_keys_and_the_reverse():
    K, V = _randn((1, 2, 1000, 128), 301, torch.bfloat16), _randn((1, 2, 1000, 128), 302, torch.bfloat16)
    Q = _randn((1, 2, 5, 128), 303, torch.bfloat16)
    _full_check(Q, K, V, 128, 0.75, True, "5 queries, 1000 keys")
    _full_check(K, Q, Q, 128, 0.0, True, "1000 queries, 5 keys")


def test_inputs_that_tie_everywhere():
    """All tokens identical (every norm, every block logit ties), and all-zero queries: the order
    of equal keys is the original order, equal logits keep the lower block indices, attention
    over equal scores is the mean of the kept values."""
    L, block = 1024, 128           # full blocks only: every block mean is exact, so the logits tie bit for bit
    row = _randn((1, 1, 1, 128), 401, torch.bfloat16)
    same = row.expand(1, 1, L, 128).contiguous()
    V = _randn((1, 1, L, 128), 402, torch.bfloat16)
    _full_check(same, same, V, block, 0.5, True, "identical tokens")
    sel = bd.basa_select(same, same, block, 0.5)
    assert torch.equal(sel.perm_q[0, 0].cpu(), torch.arange(L, dtype=torch.int32))
    assert sel.row_cols[0, 0, 0].cpu().tolist() == list(range(sel.kappa))
    zeros = torch.zeros_like(same)
    _full_check(zeros, V, V, block, 0.5, True, "zero queries")


def test_batch_two_with_strided_batches():
    """Two batches living in one buffer with a gap between them: each batch must come out exactly
    as it does when passed alone, and batch 1 must match the oracle."""
    w = C[4].scaled("batch2", heads_q=2, heads_kv=2, L=1024 + 128 + 9)
    parts = [synth.make_qkv(w.scaled(f"b{i}", index=40 + i), device=DEV) for i in range(2)]
    def pack(i):
        buf = torch.zeros((2, w.heads_q + 1, w.L, w.d), dtype=parts[0][i].dtype, device=DEV)   # padded head axis
        buf[0, :w.heads_q], buf[1, :w.heads_q] = parts[0][i][0], parts[1][i][0]
        return buf[:, :w.heads_q]
    Q, K, V = pack(0), pack(1), pack(2)
    assert not Q.is_contiguous()
    sel = bd.basa_select(Q, K, w.block, 0.5)
    out = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, w.block, sel.perm_q, sel.perm_k)
    for b in range(2):
        q1, k1, v1 = parts[b]
        s1 = bd.basa_select(q1, k1, w.block, 0.5)
        o1 = bd.basa_sparse_attn(q1, k1, v1, s1.row_count, s1.row_cols, w.block, s1.perm_q, s1.perm_k)
        assert torch.equal(sel.perm_q[b], s1.perm_q[0]) and torch.equal(sel.perm_k[b], s1.perm_k[0])
        assert torch.equal(sel.mask_bits[b], s1.mask_bits[0]) and torch.equal(sel.row_cols[b], s1.row_cols[0])
        assert torch.equal(out[b], o1[0])
    _full_check(Q[1:2], K[1:2], V[1:2], w.block, 0.5, True, "batch 1 of 2")


def test_largest_block_map():
    """4096 key blocks per row (the limit of the row-selection kernel and of the attention
    kernel's block-list storage in LDS): selection on every row, attention on sampled query blocks."""
    block, n = 64, 4096
    L = n * block - 13                         # ragged last block
    w = C[1].scaled("max_blocks", heads_q=1, heads_kv=1, L=L, salient_frac=0.01)
    Q, K, V = synth.make_qkv(w, device=DEV)
    s = 0.9
    sel = bd.basa_select(Q, K, block, s, want_scores=True)
    out = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, block, sel.perm_q, sel.perm_k)
    torch.cuda.synchronize()
    assert sel.n_k == n
    q, k, v = np64(Q[0, 0]), np64(K[0, 0]), np64(V[0, 0])
    ref = o.select(q, k, block, s)
    assert np.array_equal(sel.perm_q[0, 0].cpu().numpy(), ref["perm_q"])
    assert np.array_equal(sel.perm_k[0, 0].cpu().numpy(), ref["perm_k"])
    sc = sel.scores[0, 0].cpu().numpy().astype(np.float64)
    assert np.abs(sc - ref["logits"]).max() <= 1e-5 * max(1.0, np.abs(ref["logits"]).max())
    assert mask_report(unpack_mask(sel.mask_bits, n)[0, 0], ref)[0] == 0
    cols = sel.row_cols[0, 0].cpu().numpy().astype(np.int64)
    out_h = np64(out[0, 0])
    rng = np.random.default_rng(5)
    for g in [0, n - 1] + rng.integers(n, size=6).tolist():
        rows, O_ref, _ = o.sparse_attention_block(q, k, v, ref["perm_q"], ref["perm_k"], g, cols[g], block)
        check_output(out_h[rows], O_ref, True, f"query block {g}")
    with pytest.raises(bd.BasaError) as e:     # one block more is refused, not mishandled
        Kbig = torch.zeros((1, 1, (n + 1) * block, 128), dtype=torch.bfloat16, device=DEV)
        bd.basa_select(Q, Kbig, block, s)
    assert e.value.status_name == "BASA_ERR_UNSUPPORTED"


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 64)])
def test_malformed_block_lists_are_ignored_not_followed(dtype, d):
    """Block lists are device data the host cannot validate: entries outside [0, N_k) are skipped,
    counts above the list stride are cut, and a query block with no valid entry yields zeros."""
    L, block = 5 * 128 + 40, 128
    n = (L + block - 1) // block
    Q, K, V = (_randn((1, 1, L, d), 600 + i, dtype) for i in range(3))
    stride = 4
    cols = torch.tensor([[0, 2, 5, 4],            # fine (ragged last block 5 included)
                         [1, -7, 3, 99999],       # two entries that are no key blocks
                         [n, -1, 2 ** 30, -2 ** 31],   # nothing valid
                         [3, 4, 5, 0],            # count says 9, the stride is 4
                         [2, 0, 0, 0],            # count 1
                         [5, 1, 0, 0]], dtype=torch.int32, device=DEV).reshape(1, 1, n, stride)
    count = torch.tensor([4, 4, 4, 9, 1, 2], dtype=torch.int32, device=DEV).reshape(1, 1, n)
    out, lse = bd.basa_sparse_attn(Q, K, V, count, cols, block, None, None, want_lse=True)
    torch.cuda.synchronize()
    valid = [[0, 2, 4, 5], [1, 3], [], [0, 3, 4, 5], [2], [1, 5]]
    q, k, v = np64(Q[0, 0]), np64(K[0, 0]), np64(V[0, 0])
    ident = np.arange(L)
    for g, lst in enumerate(valid):
        rows = np.arange(g * block, min((g + 1) * block, L))
        got = np64(out[0, 0, rows])
        if not lst:
            assert (got == 0).all() and np.isneginf(lse[0, 0, rows].cpu().numpy()).all()
            continue
        _, O_ref, _ = o.sparse_attention_block(q, k, v, ident, ident, g, lst, block)
        check_output(got, O_ref, dtype == torch.bfloat16, f"query block {g}")
    # two neighbouring query blocks (one workgroup of the matrix-core kernel) without any valid entry
    count[0, 0, 3] = 0
    out = bd.basa_sparse_attn(Q, K, V, count, cols, block, None, None)
    torch.cuda.synchronize()
    assert (np64(out[0, 0, 2 * block:4 * block]) == 0).all()
    _, O_ref, _ = o.sparse_attention_block(q, k, v, ident, ident, 4, [2], block)
    check_output(np64(out[0, 0, 4 * block:5 * block]), O_ref, dtype == torch.bfloat16, "query block 4")


def test_malformed_key_permutation_stays_inside_the_tensor():
    """A permutation entry that is no index falls back to its own position: wrong rows for the
    caller, but never an access outside K or V.  Checked against the oracle fed with the same
    (sanitised) index array, through pooling and through both attention kernels."""
    L, block = 3 * 128 + 17, 128
    rng = np.random.default_rng(9)
    for dtype, d in ((torch.bfloat16, 128), (torch.float32, 64)):
        Q, K, V = (_randn((1, 1, L, d), 700 + i, dtype) for i in range(3))
        perm = rng.permutation(L).astype(np.int32)
        bad = perm.copy()
        bad[[3, 100, 250, L - 1]] = [L, -1, 2 ** 31 - 1, -2 ** 31]
        clean = np.where((bad >= 0) & (bad < L), bad, np.arange(L)).astype(np.int64)
        pk = torch.from_numpy(bad).to(DEV).reshape(1, 1, L)
        mean, var = bd.basa_downsample(K, block, pk)
        m_ref, v_ref = o.block_stats(np64(K[0, 0])[clean], block)
        np.testing.assert_allclose(mean[0, 0].cpu().numpy(), m_ref, rtol=1e-5, atol=1e-6)
        np.testing.assert_allclose(var[0, 0].cpu().numpy(), v_ref, rtol=1e-5, atol=1e-6)
        n = (L + block - 1) // block
        cols = torch.arange(n, dtype=torch.int32, device=DEV).repeat(n, 1).reshape(1, 1, n, n)
        count = torch.full((1, 1, n), n, dtype=torch.int32, device=DEV)
        out = bd.basa_sparse_attn(Q, K, V, count, cols, block, None, pk)
        torch.cuda.synchronize()
        ref = o.dense_attention(np64(Q[0, 0]), np64(K[0, 0])[clean], np64(V[0, 0])[clean])
        check_output(np64(out[0, 0]), ref, dtype == torch.bfloat16, f"{dtype}")


@pytest.mark.parametrize("block", [64, 128])
@pytest.mark.parametrize("L", [1, 64, 130, 1000, 2048 + 77])
def test_bf16_head_dim_64(L, block):
    """bf16 with head dimension 64 runs on the matrix-core kernel too (half-size rows and tiles)."""
    Hq, Hk = 4, 2
    Q = _randn((1, Hq, L, 64), 800 + L, torch.bfloat16)
    K, V = _randn((1, Hk, L, 64), 801 + L, torch.bfloat16), _randn((1, Hk, L, 64), 802 + L, torch.bfloat16)
    _full_check(Q, K, V, block, 0.5, True, f"d=64 L={L} B={block}")
    if L >= 1000:
        dense, lse = bd.basa_dense_attn(Q, K, V, block, want_lse=True)
        torch.cuda.synchronize()
        for h in range(Hq):
            ref, lse_ref = o.dense_attention(np64(Q[0, h]), np64(K[0, h // 2]), np64(V[0, h // 2]), True)
            check_output(np64(dense[0, h]), ref, True, "dense d=64")
            np.testing.assert_allclose(lse[0, h].cpu().numpy(), lse_ref, atol=2e-2)


def test_hip_graph_capture_and_replay():
    """With caller-owned buffers the library allocates nothing and never synchronises, so a
    select + attention pass can be captured into a HIP graph; every replay, with eager work
    and synchronisation in between, must reproduce the eager result bit for bit."""
    w = C[4].scaled("graph", heads_q=4, heads_kv=4, L=4096 + 128 + 31)
    Q, K, V = synth.make_qkv(w, device=DEV)
    p = bd.params(w.block, 0.5)
    ws_sel = torch.empty(bd.select_workspace_size(Q, K, p), dtype=torch.uint8, device=DEV)
    ws_att = torch.empty(bd.attn_workspace_size(Q, K, p), dtype=torch.uint8, device=DEV)
    sel = bd.basa_select(Q, K, w.block, 0.5, ws=ws_sel)
    out = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, w.block, sel.perm_q, sel.perm_k, ws=ws_att)
    torch.cuda.synchronize()
    want_out, want_cols, want_perm = out.clone(), sel.row_cols.clone(), sel.perm_k.clone()

    def step():
        bd.basa_select(Q, K, w.block, 0.5, ws=ws_sel, out=sel)
        bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, w.block, sel.perm_q, sel.perm_k, ws=ws_att, out=out)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for rep in range(4):
        out.zero_(); sel.row_cols.zero_(); sel.perm_k.zero_()      # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want_out), f"replay {rep}: output differs"
        assert torch.equal(sel.row_cols, want_cols) and torch.equal(sel.perm_k, want_perm), f"replay {rep}"
        # a different eager call in between must not disturb the next replay
        bd.basa_select(Q, K, w.block, 0.75)


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.bfloat16, 64), (torch.float32, 64)])
def test_packed_qkv_views(dtype, d):
    """Q, K and V as strided views of one packed [1, L, 3, H, d] buffer (token-major, heads
    interleaved): every kernel follows the strides; results equal those on contiguous copies."""
    H, L, block = 3, 777, 128
    packed = _randn((1, L, 3, H, d), 900 + d, dtype)
    Q, K, V = (packed[:, :, i].permute(0, 2, 1, 3) for i in range(3))          # [1, H, L, d] views
    assert not Q.is_contiguous() and Q.stride(2) == 3 * H * d
    Qc, Kc, Vc = Q.contiguous(), K.contiguous(), V.contiguous()
    sel = bd.basa_select(Q, K, block, 0.5)
    ref = bd.basa_select(Qc, Kc, block, 0.5)
    for name in ("perm_q", "perm_k", "mask_bits", "row_cols", "row_count", "row_mass"):
        assert torch.equal(getattr(sel, name), getattr(ref, name)), name
    out = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, block, sel.perm_q, sel.perm_k)
    want = bd.basa_sparse_attn(Qc, Kc, Vc, ref.row_count, ref.row_cols, block, ref.perm_q, ref.perm_k)
    assert out.is_contiguous() and torch.equal(out, want)
    mean, var = bd.basa_downsample(K, block, sel.perm_k)
    mean_c, var_c = bd.basa_downsample(Kc, block, ref.perm_k)
    assert torch.equal(mean, mean_c) and torch.equal(var, var_c)
    _full_check(Q, K, V, block, 0.5, dtype == torch.bfloat16, f"packed qkv {dtype} d={d}")


def test_optional_outputs_may_be_null():
    w = C[4].scaled("nulls", heads_q=2, heads_kv=2, L=1500)
    Q, K, V = synth.make_qkv(w, device=DEV)
    full = bd.basa_select(Q, K, w.block, 0.5)
    lean = bd.basa_select(Q, K, w.block, 0.5, want_mask=False, want_mass=False)
    assert lean.mask_bits is None and lean.row_mass is None
    assert torch.equal(lean.row_cols, full.row_cols) and torch.equal(lean.perm_k, full.perm_k)
    mean, var = bd.basa_downsample(K, w.block, full.perm_k, want_var=False)
    assert var is None
    mean2, _ = bd.basa_downsample(K, w.block, full.perm_k)
    assert torch.equal(mean, mean2)


def test_two_streams_with_their_own_buffers_do_not_interfere():
    """The library keeps no device-side state of its own: calls on two streams, each with its own
    workspaces and outputs, may overlap and give what they give when run alone."""
    wa = C[4].scaled("sa", heads_q=4, heads_kv=4, L=8192 + 50)
    wb = C[1].scaled("sb", heads_q=4, heads_kv=4, L=6000)
    A = synth.make_qkv(wa, device=DEV)
    Bt = synth.make_qkv(wb, device=DEV)

    def run(w, qkv):
        Q, K, V = qkv
        sel = bd.basa_select(Q, K, w.block, 0.5)
        return bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, w.block, sel.perm_q, sel.perm_k)

    alone_a, alone_b = run(wa, A), run(wb, Bt)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    for _ in range(3):
        with torch.cuda.stream(s1):
            oa = run(wa, A)
        with torch.cuda.stream(s2):
            ob = run(wb, Bt)
        outs.append((oa, ob))
    torch.cuda.synchronize()
    for oa, ob in outs:
        assert torch.equal(oa, alone_a) and torch.equal(ob, alone_b)


@pytest.mark.parametrize("block,d", [(128, 128), (64, 128), (128, 64), (64, 64)])
@pytest.mark.parametrize("L", [1, 100, 640 + 33, 2048 + 77])
def test_every_workgroup_shape_against_the_oracle(L, block, d):
    # the 256-query and the 128-query workgroup are two schedules of the same arithmetic; the
    # 512-query one (64 queries per wave) exponentiates against a reference that is not the running
    # maximum (shape 3) or against a maximum refreshed every 32 keys instead of every 64 (shape 4),
    # so its bits differ while it meets the same tolerance
    Q, K, V = (_randn((1, 2, L, d), 600 + i, torch.bfloat16) for i in range(3))
    sel = bd.basa_select(Q, K, block, 0.5, 0.0, bd.SORT_NONE)           # lists with little in common
    outs = [bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, block, sel.perm_q, sel.perm_k,
                                want_lse=True, attn_shape=shape) for shape in (1, 2, 3, 0, 4)]
    torch.cuda.synchronize()
    for h in range(2):
        q, k, v = np64(Q[0, h]), np64(K[0, h]), np64(V[0, h])
        cnt = sel.row_count[0, h].cpu().numpy()
        cols = sel.row_cols[0, h].cpu().numpy().astype(np.int64)
        lists = [cols[r, :cnt[r]] for r in range(cols.shape[0])]
        O_ref, lse_ref = o.sparse_attention(q, k, v, sel.perm_q[0, h].cpu().numpy(), sel.perm_k[0, h].cpu().numpy(),
                                            lists, block, return_lse=True)
        for (out, lse), name in zip(outs, ("shared", "solo", "wide", "auto", "wide with running maxima")):
            check_output(np64(out[0, h]), O_ref, True, f"{name} L={L} B={block} d={d} head {h}")
            np.testing.assert_allclose(lse[0, h].cpu().numpy(), lse_ref, rtol=0, atol=3e-2)
    # 32 queries per wave: every wave walks its own tiles in the same order in both shapes: identical bits
    assert torch.equal(outs[0][0], outs[1][0])
    # too small for the overlap probe: the library takes the 512-query shape
    assert torch.equal(outs[3][0], outs[2][0]) and torch.equal(outs[3][1], outs[2][1])


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [128, 64])
def test_scores_outside_the_range_of_the_pass_without_running_maxima(d, causal):
    """The 512-query shape first exponentiates against a reference that starts at 0 and only moves up
    in steps of 2^40; a workgroup with a row sum outside [2^-60, 2^100] is computed again with running
    maxima.  Heads whose scaled scores sit near +300, near -300, climb by hundreds from tile to tile,
    or are ordinary, next to each other: every one must come out as the oracle's (a row that the
    first pass overflowed or flushed to zero and that was not repeated would be NaN, inf or zero)."""
    H, L, B = 5, 1024 + 40, 128
    g = torch.Generator().manual_seed(910 + d)
    u = torch.randn(d, generator=g, dtype=torch.float64)
    u /= u.norm()
    noise = lambda sc: sc * torch.randn(L, d, generator=g, dtype=torch.float64)
    amp = (300.0 * (d ** 0.5) / 1.4426950408889634) ** 0.5        # (amp u) . (amp u) / sqrt(d) * log2(e) = 300
    Q = torch.empty(1, H, L, d, dtype=torch.float64)
    K = torch.empty(1, H, L, d, dtype=torch.float64)
    Q[0, 0], K[0, 0] = amp * u + noise(0.5), amp * u + noise(0.5)          # every score near +300 (in log2 units)
    Q[0, 1], K[0, 1] = amp * u + noise(0.5), -amp * u + noise(0.5)         # every score near -300
    ramp = torch.linspace(0.0, 1.0, L, dtype=torch.float64)[:, None]
    Q[0, 2], K[0, 2] = amp * u + noise(0.5), 2.0 * amp * ramp * u + noise(0.5)    # climbing from 0 to +600 along the keys
    Q[0, 3], K[0, 3] = noise(1.0), noise(1.0)                               # ordinary
    Q[0, 4], K[0, 4] = amp * u + noise(0.5), 2.0 * amp * (1.0 - ramp) * u + noise(0.5)   # falling from +600 to 0
    V = torch.randn(1, H, L, d, generator=g, dtype=torch.float64)
    Q, K, V = (t.to(torch.bfloat16).to(DEV) for t in (Q, K, V))
    n = (L + B - 1) // B
    rng = np.random.default_rng(12)
    keep = n - 2
    cols = np.stack([np.sort(rng.choice(n, keep, replace=False)) for _ in range(H * n)]).reshape(H, n, keep)
    if causal:                        # every query block lists its own key block, so that no row is empty
        for h in range(H):
            for r in range(n):
                if r not in cols[h, r]:
                    cols[h, r, 0] = r
                    cols[h, r].sort()
    row_cols = torch.from_numpy(cols.astype(np.int32)).reshape(1, H, n, keep).contiguous().to(DEV)
    row_count = torch.full((1, H, n), keep, dtype=torch.int32, device=DEV)
    out3, lse3 = bd.basa_sparse_attn(Q, K, V, row_count, row_cols, B, want_lse=True, attn_shape=3, causal=causal)
    out4, lse4 = bd.basa_sparse_attn(Q, K, V, row_count, row_cols, B, want_lse=True, attn_shape=4, causal=causal)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out3.float()).all()) and bool(torch.isfinite(lse3).all())
    ident = np.arange(L)
    for h in range(H):
        q, k, v = np64(Q[0, h]), np64(K[0, h]), np64(V[0, h])
        lists = [cols[h, r] for r in range(n)]
        O_ref, lse_ref = (o.sparse_attention_causal if causal else o.sparse_attention)(q, k, v, ident, ident, lists, B,
                                                                                      return_lse=True)
        for out, lse, name in ((out3, lse3, "two passes"), (out4, lse4, "running maxima")):
            check_output(np64(out[0, h]), O_ref, True, f"{name} head {h} d={d} causal={causal}")
            np.testing.assert_allclose(lse[0, h].cpu().numpy(), lse_ref, rtol=1e-4, atol=3e-2)
    # the heads that cannot but be repeated carry the bits of the pass with running maxima (the climbing
    # head is followed by the moving reference, the ordinary one never leaves the range)
    for h in (0, 1, 4):
        assert torch.equal(out3[0, h], out4[0, h]), h


@pytest.mark.parametrize("kind", ["overlapping", "disjoint", "ragged"])
def test_workgroup_shape_chosen_on_the_device(kind):
    # large enough for the library to measure the overlap of neighbouring lists and choose;
    # whichever shape it takes, the output is the forced shapes' output
    H, L, B, d = 8, 32768 + 50, 128, 128
    Q, K, V = (_randn((1, H, L, d), 700 + i, torch.bfloat16) for i in range(3))
    n = (L + B - 1) // B
    rng = np.random.default_rng(5)
    keep = n // 4
    if kind == "overlapping":        # the four neighbours (4g .. 4g+3) that share a 512-query workgroup share their list
        base = np.stack([np.sort(rng.choice(n, keep, replace=False)) for _ in range(H * ((n + 3) // 4))])
        cols = np.repeat(base.reshape(H, (n + 3) // 4, keep), 4, axis=1)[:, :n]
        cnt = np.full((H, n), keep)
    elif kind == "disjoint":         # even rows list even blocks, odd rows odd blocks
        cols = np.stack([np.sort(rng.choice(n // 2, keep, replace=False)) * 2 + (r & 1) for _ in range(H)
                         for r in range(n)]).reshape(H, n, keep)
        cnt = np.full((H, n), keep)
    else:
        cols = np.stack([np.sort(rng.choice(n, keep, replace=False)) for _ in range(H * n)]).reshape(H, n, keep)
        cnt = rng.integers(1, keep + 1, size=(H, n))
    row_cols = torch.from_numpy(cols.astype(np.int32)).reshape(1, H, n, keep).contiguous().to(DEV)
    row_count = torch.from_numpy(cnt.astype(np.int32)).reshape(1, H, n).contiguous().to(DEV)
    outs = [bd.basa_sparse_attn(Q, K, V, row_count, row_cols, B, want_lse=True, attn_shape=shape) for shape in (1, 2, 3, 0)]
    torch.cuda.synchronize()
    assert torch.equal(outs[0][0], outs[1][0])
    # lists that overlap go to the 512-query shape, the others to the 128-query one
    chosen = 2 if kind == "overlapping" else 1
    assert torch.equal(outs[3][0], outs[chosen][0]) and torch.equal(outs[3][1], outs[chosen][1]), kind
    # sampled query blocks against the oracle
    h = 3
    q, k, v = np64(Q[0, h]), np64(K[0, h]), np64(V[0, h])
    ident = np.arange(L)
    for g in (0, 1, n // 2, n - 1):
        rows, O_ref, _ = o.sparse_attention_block(q, k, v, ident, ident, g, cols[h, g, :cnt[h, g]], B)
        for i in (0, 2):
            check_output(np64(outs[i][0][0, h])[rows], O_ref, True, f"{kind} block {g} shape {i + 1}")


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.bfloat16, 64), (torch.float32, 64)])
def test_token_major_output_through_out_strides(dtype, d):
    """out as a strided view: a token-major [2, L, H, d] buffer (what the next projection reads)
    with two extra slots per token that must stay untouched."""
    Bt, H, L, block = 2, 4, 500, 64
    Q, K, V = (_randn((Bt, H, L, d), 950 + i, dtype) for i in range(3))
    sel = bd.basa_select(Q, K, block, 0.5)
    want, lse_want = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, block, sel.perm_q, sel.perm_k, want_lse=True)
    buf = torch.full((Bt, L, H + 2, d), 7.0, dtype=dtype, device=DEV)
    view = buf[:, :, 1:H + 1].permute(0, 2, 1, 3)                              # [Bt, H, L, d]
    got, lse = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, block, sel.perm_q, sel.perm_k, want_lse=True,
                                   out=view)
    torch.cuda.synchronize()
    assert got.data_ptr() == view.data_ptr()
    assert torch.equal(view, want) and torch.equal(lse, lse_want)
    assert (buf[:, :, 0] == 7).all() and (buf[:, :, H + 1] == 7).all()
    dense_want = bd.basa_dense_attn(Q, K, V, block)
    buf.fill_(7.0)
    bd.basa_dense_attn(Q, K, V, block, out=view)
    assert torch.equal(view, dense_want) and (buf[:, :, 0] == 7).all() and (buf[:, :, H + 1] == 7).all()
    with pytest.raises(ValueError):
        bd.basa_dense_attn(Q, K, V, block, out=buf[:, :, 1:H + 1].permute(0, 2, 3, 1))   # d not innermost


def test_variable_length_batch_packed_token_major():
    """Three sequences of different lengths packed token-major, each its own problem."""
    Hq, Hk, d, block = 4, 2, 128, 64
    lens = [700, 1, 1333]
    cu = [0, 700, 701, 2034]
    T = cu[-1]
    g = torch.Generator().manual_seed(4242)
    q = torch.randn((T, Hq, d), generator=g).to(torch.bfloat16).to(DEV)
    k = torch.randn((T, Hk, d), generator=g).to(torch.bfloat16).to(DEV)
    v = torch.randn((T, Hk, d), generator=g).to(torch.bfloat16).to(DEV)
    out = bd.ba_att_varlen(q, k, v, cu, block, 0.5)
    torch.cuda.synchronize()
    assert out.shape == q.shape
    for a, b in zip(cu[:-1], cu[1:]):
        for h in range(Hq):
            O_ref, _ = o.ba_att(np64(q[a:b, h]), np64(k[a:b, h // 2]), np64(v[a:b, h // 2]), block, 0.5)
            check_output(np64(out[a:b, h]), O_ref, True, f"sequence [{a},{b}) head {h}")
    # an empty sequence in the list is skipped
    out2 = bd.ba_att_varlen(q, k, v, [0, 700, 700, 701, 2034], block, 0.5)
    assert torch.equal(out, out2)


def test_two_runs_give_identical_bits():
    """Nothing on the path depends on the order in which workgroups finish: two runs of selection
    (fixed count, cumulative mass with a total budget, segments) and attention agree bit for bit."""
    H, L, B, d = 8, 32768 + 50, 128, 128
    Q, K, V = (_randn((1, H, L, d), 990 + i, torch.bfloat16) for i in range(3))
    for kw in (dict(), dict(mass_target=0.9, min_keep=2, budget_total=40000), dict(segments=[0, 5000, 20001])):
        runs = []
        for _ in range(2):
            sel = bd.basa_select(Q, K, B, 0.5, want_scores=True, **kw)
            out, lse = bd.basa_sparse_attn(Q, K, V, sel.row_count, sel.row_cols, B, sel.perm_q, sel.perm_k, want_lse=True)
            torch.cuda.synchronize()
            runs.append((sel, out, lse))
        (s0, o0, l0), (s1, o1, l1) = runs
        for name in ("perm_q", "perm_k", "mask_bits", "row_count", "row_mass", "scores"):
            assert torch.equal(getattr(s0, name), getattr(s1, name)), (kw, name)
        # list entries past a row's count are not written: compare the counted part
        cnt = s0.row_count[..., None]
        live = torch.arange(s0.row_cols.shape[-1], device=DEV) < cnt
        assert torch.equal(s0.row_cols * live, s1.row_cols * live), kw
        assert torch.equal(o0, o1) and torch.equal(l0, l1), kw


def test_downsample_x_sorted_from_strided_fp32_and_ragged_input():
    """x_sorted of a non-contiguous fp32 tensor with a ragged last block and a batch of two: a plain
    gather, compared with torch indexing bit for bit; the statistics do not change with it."""
    Bt, H, L, d, block = 2, 3, 64 * 5 + 17, 64, 64
    big = _randn((Bt, H + 1, L + 3, d), 1234, torch.float32)
    x = big[:, :H, 2:L + 2]
    assert not x.is_contiguous()
    perm = bd.basa_norm_sort(x, block)
    mean, var, xs = bd.basa_downsample(x, block, perm, want_sorted=True)
    mean0, var0 = bd.basa_downsample(x, block, perm)
    want = torch.gather(x, 2, perm.long()[..., None].expand(-1, -1, -1, d))
    assert xs.is_contiguous() and torch.equal(xs, want)
    assert torch.equal(mean, mean0) and torch.equal(var, var0)
