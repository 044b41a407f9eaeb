#!/usr/bin/env python3
"""Benchmark of the BA-Att hot path on one MI355X.

A step is one pass of the whole path on one batch of synthetic input already resident
in HBM: basa_select (norm sort, block pooling, compensated score map, top-kappa) followed
by basa_sparse_attn (gather + bf16-MFMA block-sparse attention).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--sparsity 0.5]
                    [--sweep] [--no-cpu-baseline] [--fidelity] [--sweep-len]

--sweep additionally times every configuration / sparsity of the benchmark and writes the
table to <out-dir>/bench_sweep.json (the printed line stays the headline workload).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2605_19726_amd import binding as bd   # noqa: E402
from paper_2605_19726_amd import synth           # noqa: E402

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
# HBM traffic cannot be counted from inside this process: the figures come from the committed
# rocprofv3 summary of this same command (FETCH_SIZE / WRITE_SIZE per dispatch, scaled by a plain-copy
# calibration), which carries them in a machine-readable comment line together with their spread
# over the profiled launches.  The bench line names that file; a workload it does not cover gets null.
TRAFFIC_PROFILE = os.path.join("profiles", "attn_and_select_cfg4_s50.md")


def profiled_traffic(workload, sparsity):
    """{'attn': {...}, 'select': {...}} from the profile summary, or {} if it does not cover this workload."""
    try:
        with open(os.path.join(ROOT, TRAFFIC_PROFILE)) as f:
            for line in f:
                if line.startswith("<!-- traffic-json:"):
                    rec = json.loads(line[len("<!-- traffic-json:"):].rsplit("-->", 1)[0])
                    if rec.get("workload") == workload and abs(rec.get("sparsity", -1) - sparsity) < 1e-9:
                        return rec
    except (OSError, ValueError):
        pass
    return {}


def executed_flops(w, kappa):
    """4 * n_q * n_k * d per executed block pair, ragged tails counted at their true size."""
    B, L, d = w.block, w.L, w.d
    n = w.n_blocks
    # every row keeps kappa key blocks; the ragged last key block (if kept) is shorter, which
    # at most changes the total by one block per row: count whole blocks except for the tail
    # of the query side, which is exact.
    return 4.0 * w.heads_q * L * (kappa * B if kappa < n else L) * d


def selection_bytes(w):
    """Algorithmic HBM bytes of the selection stage: Q and K are read twice (norm pass, then the
    gather + pooling pass, which depends on the finished sort), plus the sort's key/index words
    (one 8-byte word per token written by the key + tile-sort pass, then read and written by
    every merge pass), the block features, the score map and the block lists."""
    e = 2 if w.dtype == "bf16" else 4
    rows = (w.heads_q + w.heads_kv) * w.L
    n = w.n_blocks
    qk = rows * w.d * e
    merges = max(0, int(np.ceil(np.log2(max(w.L, 1) / 4096.0))))
    sort = rows * 8 * (1 + 2 * merges)      # the tile sort writes each word once, every merge pass reads and writes it
    feats = (w.heads_q + w.heads_kv) * n * 3 * w.d * 4 * 2
    scores = w.heads_q * n * n * 4 * 2
    return dict(two_pass=2 * qk, compulsory=qk, sort=sort, small=feats + scores,
                total=2 * qk + sort + feats + scores)


class Pipeline:
    """Preallocated buffers for repeated select + attention calls on one workload."""

    def __init__(self, w, sparsity, Q, K, V, beta=1.0, sort=bd.SORT_QK, mass_target=0.0, causal=False):
        self.w, self.s, self.beta, self.sort, self.mass_target = w, sparsity, beta, sort, mass_target
        self.causal = causal
        self.Q, self.K, self.V = Q, K, V
        # Inputs that fit the 256 MB Infinity Cache would be served from it on every step after the
        # first: rotate over enough copies (same values, other addresses) that each step finds its
        # inputs in HBM only.
        nbytes = sum(t.numel() * t.element_size() for t in (Q, K, V))
        self.copies = [(Q, K, V)]
        if nbytes < 512e6:
            for _ in range(min(7, int(1.0e9 // nbytes))):
                self.copies.append((Q.clone(), K.clone(), V.clone()))
        self.turn = 0
        dev = Q.device
        p = bd.params(w.block, sparsity, beta, sort, causal=causal)
        self.ws_sel = torch.empty(bd.select_workspace_size(Q, K, p), dtype=torch.uint8, device=dev)
        self.ws_att = torch.empty(bd.attn_workspace_size(Q, K, p), dtype=torch.uint8, device=dev)
        self.sel = bd.basa_select(Q, K, w.block, sparsity, beta, sort, ws=self.ws_sel, mass_target=mass_target,
                                  causal=causal)
        self.out = torch.empty_like(Q)

    def _next(self):
        self.turn = (self.turn + 1) % len(self.copies)
        self.Q, self.K, self.V = self.copies[self.turn]

    def select(self, rotate=True):
        if rotate:
            self._next()
        bd.basa_select(self.Q, self.K, self.w.block, self.s, self.beta, self.sort, ws=self.ws_sel,
                       out=self.sel, mass_target=self.mass_target, causal=self.causal)

    def attn(self, rotate=True):
        if rotate:
            self._next()
        s = self.sel
        bd.basa_sparse_attn(self.Q, self.K, self.V, s.row_count, s.row_cols, self.w.block, s.perm_q,
                            s.perm_k, ws=self.ws_att, out=self.out, causal=self.causal)

    def dense(self):
        self._next()
        bd.basa_dense_attn(self.Q, self.K, self.V, self.w.block, ws=self.ws_att, out=self.out, causal=self.causal)

    def step(self):
        self._next()
        self.select(rotate=False)
        self.attn(rotate=False)


def timed(fn, reps):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / reps


def attainable_mfma(dev, iters=60000):
    """The bf16 matrix-core rate a bare loop of independent MFMAs sustains on this chip, with
    constant and with pseudo-random operand values (TFLOP/s each).  Context for the roofline
    fraction: the nominal peak is only reached while the operand bits do not toggle."""
    out = torch.empty(1 << 17, dtype=torch.float32, device=dev)
    rates = {}
    for name, rnd in (("constant_operands", False), ("random_operands", True)):
        bd.basa_calibrate_mfma(rnd, 2000, out)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flops = bd.basa_calibrate_mfma(rnd, iters, out)
        e1.record()
        e1.synchronize()
        rates[name] = flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    return rates


def attainable_read(dev, gib=2):
    """GB/s of a read-only 16-byte-per-lane stream over `gib` GiB (the access pattern of the key pass)."""
    buf = torch.zeros(gib << 28, dtype=torch.int32, device=dev)
    out = torch.zeros(4, dtype=torch.int32, device=dev)
    bd.basa_calibrate_read(buf, out)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    nbytes = 0
    for _ in range(3):
        nbytes += bd.basa_calibrate_read(buf, out)
    e1.record()
    e1.synchronize()
    return nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9


def fidelity_report(w, Q, K, sparsities):
    """How much of the dense attention mass the selected blocks hold (recall of the oracle block
    distribution, Eq. 3), how far m' is from it (l1), and how well the norm bound U (Eq. 8)
    tracks the observed logit deviation (Pearson R, as in Fig. 2) - for the four combinations
    of norm sorting and covariance compensation, on this workload's synthetic tensors."""
    dev = Q.device
    rows = []
    # the four sort modes of the paper's ablation (Tab. 7), plus a per-segment sort where the
    # workload has segments
    variants = [(bd.SORT_NONE, "none", None), (bd.SORT_Q, "Q", None), (bd.SORT_K, "K", None), (bd.SORT_QK, "QK", None)]
    if synth.segments_of(w) is not None:
        variants.append((bd.SORT_QK, "QK per segment", synth.segments_of(w)))
    for sort, sort_name, segments in variants:
        base = bd.basa_select(Q, K, w.block, 0.5, beta=0.0, sort=sort, want_scores=True, segments=segments)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        m_hat, max_dev, _ = bd.basa_block_mass(Q, K, w.block, base.perm_q, base.perm_k,
                                               base_logits=base.scores, want_dev=True)
        e1.record()
        rq, mq = bd.basa_block_radius(Q, w.block, base.perm_q)
        rk, mk = bd.basa_block_radius(K, w.block, base.perm_k)
        U = bd.basa_deviation_bound(rq, mq, rk, mk, w.d)
        n, sx, sy, sxx, syy, sxy = bd.basa_pearson_sums(U, max_dev).cpu().tolist()
        pearson = (n * sxy - sx * sy) / max(1e-300, ((n * sxx - sx * sx) * (n * syy - sy * sy)) ** 0.5)
        mass_ms = e0.elapsed_time(e1)
        mass_flops = 2 * 2.0 * w.heads_q * w.L * w.L * w.d          # two QK^T passes
        for beta in (0.0, 1.0):
            for s in sparsities:
                sel = base if (beta == 0.0 and s == 0.5) else bd.basa_select(Q, K, w.block, s, beta=beta, sort=sort,
                                                                             want_scores=True, segments=segments)
                recall, l1 = bd.basa_selection_fidelity(sel.scores, sel.mask_bits, m_hat)
                rows.append({"workload": w.name, "sort": sort_name, "beta": beta, "sparsity": s,
                             "kept_fraction": sel.kappa / sel.n_k, "recall_mean": float(recall.mean()),
                             "recall_min": float(recall.min()), "l1_mean": float(l1.mean()),
                             "bound_mean": float(U.mean()), "observed_dev_mean": float(max_dev.mean()),
                             "pearson_bound_vs_observed": pearson, "block_mass_ms": mass_ms,
                             "block_mass_tflops": mass_flops / (mass_ms * 1e-3) / 1e12})
        del m_hat, max_dev, U, base
        torch.cuda.empty_cache()
    return rows


def graph_step_ms(pipe, reps=20):
    """Milliseconds per step when the whole step (about 14 launches) is replayed from a HIP graph:
    what a caller sees who captures the path once, as serving loops on short sequences do."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pipe.step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    n = len(pipe.copies)          # one step per input copy in the graph, so that replays stay HBM-fed too
    with torch.cuda.graph(graph, stream=side):
        for _ in range(n):
            pipe.step()
    graph.replay()
    return timed(graph.replay, max(2, reps // n)) * 1e3 / n


def measure(w, sparsity, Q, K, V, steps, warmup, dense_reps=1, beta=1.0, sort=bd.SORT_QK, mass_target=0.0,
            causal=False):
    pipe = Pipeline(w, sparsity, Q, K, V, beta, sort, mass_target, causal)
    for _ in range(warmup):
        pipe.step()
    torch.cuda.synchronize()
    bd.basa_profile_enable(True)
    bd.basa_profile_read()
    t_step = timed(pipe.step, steps)
    prof = bd.basa_profile_read()
    bd.basa_profile_enable(False)
    # the same step again, one pair of events per step on the stream the library launches on
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for e0, e1 in evs:
        e0.record()
        pipe.step()
        e1.record()
    torch.cuda.synchronize()
    per_step = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    t_sel = timed(pipe.select, max(2, steps))
    t_att = timed(pipe.attn, max(2, steps))
    t_dense = None
    if dense_reps > 0:
        pipe.dense()
        t_dense = timed(pipe.dense, dense_reps)
    kern_ms = {k: (ms / cnt if cnt else 0.0) for k, (ms, cnt) in prof.items()}
    kern_per_step = {k: ms / steps for k, (ms, cnt) in prof.items() if cnt}
    kappa = pipe.sel.kappa
    fl_exec = executed_flops(w, kappa)
    kept_mean = float(kappa)
    if mass_target > 0.0 or causal:       # rows keep different numbers of blocks: count the listed pairs
        kept_mean = float(pipe.sel.row_count.double().mean())
        fl_exec = 4.0 * w.block * float(pipe.sel.row_count.sum()) * min(w.block, w.L) * w.d
    fl_dense = 4.0 * w.heads_q * float(w.L) ** 2 * w.d
    if causal:                  # the token pairs a causal mask leaves: L (L + 1) / 2 per head
        fl_dense = 4.0 * w.heads_q * (float(w.L) * (w.L + 1) / 2) * w.d
    attn_kernel_s = kern_ms.get("attn_mfma_kernel", 0.0) * 1e-3
    sb = selection_bytes(w)
    res = dict(
        workload=w.name, sparsity=sparsity, kappa=kappa, n_blocks=w.n_blocks, mass_target=mass_target,
        input_copies=len(pipe.copies),
        step_ms_median=per_step[len(per_step) // 2], step_ms_min=per_step[0],
        kept_blocks_per_row_mean=kept_mean,
        t_e2e_ms=t_step * 1e3, t_select_ms=t_sel * 1e3, t_attn_ms=t_att * 1e3,
        t_dense_ms=None if t_dense is None else t_dense * 1e3,
        speedup_vs_dense=None if t_dense is None else t_dense / t_step,
        effective_tflops=fl_dense / t_step / 1e12,
        executed_tflops_attn_call=fl_exec / t_att / 1e12,
        executed_tflops_attn_kernel=(fl_exec / attn_kernel_s / 1e12) if attn_kernel_s else None,
        dense_tflops=None if t_dense is None else fl_dense / t_dense / 1e12,
        selection_gbs_two_pass=sb["two_pass"] / t_sel / 1e9,
        selection_gbs_total=sb["total"] / t_sel / 1e9,
        kernel_avg_ms=kern_ms, kernel_ms_per_step=kern_per_step,
        executed_flops=fl_exec, selection_bytes=sb,
    )
    return res, pipe


def cpu_baseline(w, sparsity, Q, K, V, pipe, n_units=64):
    """Time the numpy oracle on a bounded sample and extrapolate to the whole workload: the
    selection oracle runs in full on every head, the attention oracle on n_units (head, query
    block) units spread over all heads (so every KV group is hit), always including the first
    block of the first head and the last block of the last.  The GPU output rows of the sampled
    units are compared with the oracle's on the way."""
    from oracle import basa_oracle as o
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    group = w.heads_q // w.heads_kv
    pipe.step()                 # the dense baseline shares the output buffer: recompute the sparse result
    torch.cuda.synchronize()
    n_q = w.n_blocks
    rng = np.random.default_rng(7)
    per_head = [[] for _ in range(w.heads_q)]
    for i in range(max(n_units, w.heads_q)):
        per_head[i % w.heads_q].append(int(rng.integers(n_q)))
    per_head[0][0] = 0
    per_head[-1][-1] = n_q - 1
    t_sel = t_att = 0.0
    n_att = 0
    max_err, n_checked = 0.0, 0
    f64 = lambda t: t.to("cpu").to(torch.float64).numpy()
    for h in range(w.heads_q):
        q, k, v = f64(Q[0, h]), f64(K[0, h // group]), f64(V[0, h // group])
        t0 = time.perf_counter()
        sel = o.select(q, k, w.block, sparsity, pipe.beta, pipe.sort)
        t_sel += time.perf_counter() - t0
        cols_gpu = pipe.sel.row_cols[0, h].cpu().numpy()
        for g in sorted(set(per_head[h])):
            t0 = time.perf_counter()
            rows, O, _ = o.sparse_attention_block(q, k, v, sel["perm_q"], sel["perm_k"], g, sel["cols"][g], w.block)
            t_att += time.perf_counter() - t0
            n_att += 1
            if np.array_equal(cols_gpu[g], sel["cols"][g]):       # same kept blocks: the rows must agree
                got = pipe.out[0, h, torch.as_tensor(rows)].to("cpu").to(torch.float64).numpy()
                max_err = max(max_err, float(np.abs(got - O).max()))
                n_checked += 1
    t_unit = t_att / n_att
    t_total = t_sel + t_unit * w.heads_q * n_q
    fl_dense = 4.0 * w.heads_q * float(w.L) ** 2 * w.d
    return dict(value=fl_dense / t_total / 1e12, unit="TFLOP/s", cores=int(threads), kind="oracle",
                sample=f"numpy fp64 oracle: selection of all {w.heads_q} heads in full ({t_sel:.1f} s) + "
                       f"attention of {n_att} of {w.heads_q * n_q} (head, query-block) units over all heads "
                       f"and KV groups, first and last block included ({t_unit:.3f} s each), the attention "
                       f"part extrapolated linearly to the whole workload ({t_total:.0f} s)",
                est_total_s=t_total, cpu_seconds_spent=t_sel + t_att,
                gpu_vs_oracle_sample_maxabs=max_err if n_checked else None, units_compared_with_gpu=n_checked)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--sparsity", type=float, default=0.5)
    ap.add_argument("--sweep", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--out-dir", default=os.path.join(ROOT, "bench_out"),
                    help="where --sweep, --sweep-len and --fidelity write their tables")
    ap.add_argument("--sweep-len", action="store_true",
                    help="instead of the headline line: the sequence-length sweep of the paper's operator "
                         "benchmark (Sec. 4.3, Fig. 4 axes), L = 16K .. 256K on the 128K workload's generator, "
                         "sparse vs our dense at several sparsities; table written to <out-dir>/bench_len_sweep.json")
    ap.add_argument("--fidelity", action="store_true",
                    help="instead of timing the path: selection-fidelity diagnostics (recall of the dense "
                         "attention mass, l1 distance, bound-vs-deviation correlation) for every bf16 "
                         "configuration; table written to <out-dir>/fidelity.json")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run plain 4 GiB device copies: the known-size kernel against which "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    bd.load()
    dev = "cuda:0"
    if args.calibrate_copy:
        src = torch.ones(1 << 30, dtype=torch.float32, device=dev)      # 4 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4, "calibrate_copy_bytes_written": src.numel() * 4}))
        return
    if args.sweep_len:
        table = []
        for L in (16384, 32768, 65536, 131072, 262144):
            c = synth.CONFIGS[4].scaled(f"dlm_len_{L // 1024}k", L=L)
            q2, k2, v2 = synth.make_qkv(c, device=dev)
            first = True
            for s_ in (0.5, 0.75, 0.9):
                r, pipe_ = measure(c, s_, q2, k2, v2, 2, 1, dense_reps=1 if first else 0)
                r["t_e2e_graph_ms"] = graph_step_ms(pipe_)
                del pipe_
                if first:
                    t_dense = r["t_dense_ms"]
                first = False
                r["t_dense_ms"], r["speedup_vs_dense"] = t_dense, t_dense / r["t_e2e_ms"]
                table.append({k: r[k] for k in ("workload", "sparsity", "kappa", "n_blocks", "t_e2e_ms", "t_select_ms",
                                                "t_attn_ms", "t_dense_ms", "t_e2e_graph_ms", "speedup_vs_dense", "effective_tflops",
                                                "executed_tflops_attn_call", "dense_tflops")})
            del q2, k2, v2
            torch.cuda.empty_cache()
        os.makedirs(args.out_dir, exist_ok=True)
        with open(os.path.join(args.out_dir, "bench_len_sweep.json"), "w") as f:
            json.dump(table, f, indent=1)
        print(json.dumps({"len_sweep_rows": len(table), "table": table}))
        return
    if args.fidelity:
        table = []
        for c in synth.CONFIGS:
            q2, k2, _ = synth.make_qkv(c, device=dev)
            table += fidelity_report(c, q2, k2, c.sparsities if 0.5 in c.sparsities else (0.5,) + tuple(c.sparsities))
            del q2, k2
            torch.cuda.empty_cache()
        os.makedirs(args.out_dir, exist_ok=True)
        with open(os.path.join(args.out_dir, "fidelity.json"), "w") as f:
            json.dump(table, f, indent=1)
        print(json.dumps({"fidelity_rows": len(table), "table": table}))
        return
    w = synth.CONFIGS[args.config]
    Q, K, V = synth.make_qkv(w, device=dev)
    res, pipe = measure(w, args.sparsity, Q, K, V, args.steps, args.warmup,
                        dense_reps=0 if args.no_dense else 1)
    attn_ms = res["kernel_avg_ms"].get("attn_mfma_kernel", 0.0) or res["kernel_avg_ms"].get("attn_simple_kernel", 0.0)
    achieved = res["executed_flops"] / (attn_ms * 1e-3) / 1e12 if attn_ms else None
    traffic = profiled_traffic(w.name, args.sparsity)

    def traffic_note(key):
        t = traffic.get(key)
        if not t:
            return None
        return (f"not counted in this run: rocprofv3 FETCH_SIZE + WRITE_SIZE of the same command, {TRAFFIC_PROFILE}, "
                f"{t['launches']} profiled launches, min {t['min_bytes']:.3g} max {t['max_bytes']:.3g} bytes")

    line = {
        "metric": "BA-Att effective (dense-equivalent) TFLOP/s at 50% sparsity, L=128K; latency in ms_per_step; vs dense in speedup_vs_dense",
        "value": res["effective_tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": res["t_e2e_ms"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "heads_q": w.heads_q, "heads_kv": w.heads_kv, "L": w.L,
                   "head_dim": w.d, "block": w.block, "sparsity": args.sparsity, "kappa": res["kappa"],
                   "sort": "QK", "beta": 1.0},
        "latency_ms": {"select": res["t_select_ms"], "attn": res["t_attn_ms"], "e2e": res["t_e2e_ms"],
                       "dense": res["t_dense_ms"]},
        "step_ms_median": res["step_ms_median"], "step_ms_min": res["step_ms_min"],
        "speedup_vs_dense": res["speedup_vs_dense"],
        "executed_tflops": res["executed_tflops_attn_call"],
        "dense_tflops": res["dense_tflops"],
        "roofline": {"kernel": "attn_mfma_kernel", "bound": "mfma", "achieved": achieved,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": (achieved / PEAK_BF16_TFLOPS) if achieved else None,
                     "traffic": traffic.get("attn", {}).get("mean_bytes"),
                     "traffic_source": traffic_note("attn"),
                     "avg_launch_ms": attn_ms},
        "roofline_select": {"stage": "basa_select (all kernels)", "bound": "hbm",
                            "achieved": res["selection_gbs_total"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                            "frac": res["selection_gbs_total"] / PEAK_HBM_GBS,
                            "traffic": traffic.get("select", {}).get("mean_bytes"),
                            "traffic_source": traffic_note("select"),
                            "achieved_two_pass_qk_only": res["selection_gbs_two_pass"],
                            "bytes": res["selection_bytes"]},
        "kernel_ms_per_step": res["kernel_ms_per_step"],
    }
    if achieved:
        rates = attainable_mfma(dev)
        line["roofline"]["mfma_loop_tflops"] = rates
        line["roofline"]["frac_of_random_operand_loop"] = achieved / rates["random_operands"]
    read_gbs = attainable_read(dev)
    line["roofline_select"]["read_stream_gbs"] = read_gbs
    line["roofline_select"]["frac_of_read_stream"] = res["selection_gbs_total"] / read_gbs
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, args.sparsity, Q, K, V, pipe)
    if args.sweep:
        rows = [res]
        del pipe
        for s in w.sparsities:
            if s != args.sparsity:
                rows.append(measure(w, s, Q, K, V, 2, 1, dense_reps=0)[0])
        rows.append(measure(w, args.sparsity, Q, K, V, 2, 1, dense_reps=0, beta=0.0)[0] | {"variant": "beta=0"})
        rows.append(measure(w, args.sparsity, Q, K, V, 2, 1, dense_reps=0, sort=bd.SORT_NONE)[0] | {"variant": "sort=none"})
        for p_mass in (0.5, 0.9):
            rows.append(measure(w, 0.0, Q, K, V, 2, 1, dense_reps=0, mass_target=p_mass)[0]
                        | {"variant": f"cumulative mass {p_mass}"})
        # the causal variant (visibility on original positions): listed block pairs are all computed and
        # masked score by score, so `executed` counts listed pairs and `effective` the visible token pairs
        rows.append(measure(w, args.sparsity, Q, K, V, 2, 1, dense_reps=1, causal=True)[0] | {"variant": "causal"})
        rows.append(measure(w, args.sparsity, Q, K, V, 2, 1, dense_reps=0, sort=bd.SORT_NONE, causal=True)[0]
                    | {"variant": "causal, sort=none"})
        del Q, K, V
        torch.cuda.empty_cache()
        # the headline workload with head dimension 64 (same generator), then the other configurations
        for c in [w.scaled(w.name + "_d64", d=64)] + list(synth.CONFIGS):
            if c.index == w.index and c.d == w.d:
                continue
            q2, k2, v2 = synth.make_qkv(c, device=dev)
            for s in c.sparsities:
                rows.append(measure(c, s, q2, k2, v2, 2, 1, dense_reps=1 if s == c.sparsities[0] else 0)[0])
            del q2, k2, v2
            torch.cuda.empty_cache()
        os.makedirs(args.out_dir, exist_ok=True)
        with open(os.path.join(args.out_dir, "bench_sweep.json"), "w") as f:
            json.dump(rows, f, indent=1)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
