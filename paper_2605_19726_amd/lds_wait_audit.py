"""Check of the compiled kernels: no workgroup barrier may be reachable from an LDS instruction of the
same wave (store, atomic, and load or permute as well) without an `s_waitcnt` that brings lgkmcnt to 0
in between.

Why it exists: a wave that stores to LDS and then meets its workgroup at `s_barrier` has to wait for
that store first, or another wave can pass the barrier and read the old value.  The fence inside
`__syncthreads()` asks for this wait, but the compiler's wait-count pass was found to drop the LDS
part in one loop of the block-mass diagnostic kernel (a store in a conditional tail of the loop body,
the barrier at the top of the next iteration): rare stale partial sums, different from run to run.
The same gap came back once more, in the key pass, when a barrier was added after its loop, and was
caught here before any test saw it.  The source spells the wait out in both places; this audit reads the assembly the build keeps
(`_build/*-gfx950.s`, written with -save-temps) and reports every place where the pattern comes
back, in any kernel.

    python -m paper_2605_19726_amd.lds_wait_audit [files...]      # exit status 1 if anything is found
"""
from __future__ import annotations

import glob
import os
import re
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
_LDS_OP = re.compile(r"^ds_(?!nop)")          # loads too: an LDS load still in flight at the barrier can be overtaken by another wave's store
_LABEL = re.compile(r"^(\.LBB\d+_\d+):")


def default_files():
    return sorted(glob.glob(os.path.join(PKG, "_build", "*-hip-amdgcn-amd-amdhsa-gfx950.s")))


def _functions(lines):
    cur = None
    for i, l in enumerate(lines):
        m = re.match(r"^(_Z\w+):", l)
        if m:
            cur = (m.group(1), i)
        elif l.startswith(".Lfunc_end") and cur:
            yield cur[0], lines[cur[1]:i]
            cur = None


def audit_function(body):
    """[(barrier block, store instruction, store block)] for one function's assembly lines."""
    blocks, order, label = {"entry": []}, ["entry"], "entry"
    for l in body:
        t = l.strip()
        m = _LABEL.match(t)
        if m:
            label = m.group(1)
            blocks[label] = []
            order.append(label)
            continue
        if t and not t.startswith((";", ".")):
            blocks[label].append(t)
    pred = {k: [] for k in order}
    for i, k in enumerate(order):
        falls = True
        for t in blocks[k]:
            m = re.match(r"^s_cbranch_\w+\s+(\.LBB\d+_\d+)", t)
            if m and m.group(1) in pred:
                pred[m.group(1)].append(k)
            m = re.match(r"^s_branch\s+(\.LBB\d+_\d+)", t)
            if m:
                if m.group(1) in pred:
                    pred[m.group(1)].append(k)
                falls = False
            if t.startswith("s_endpgm"):
                falls = False
        if falls and i + 1 < len(order):
            pred[order[i + 1]].append(k)
    found = []
    for k in order:
        for idx, t in enumerate(blocks[k]):
            if t != "s_barrier":
                continue
            seen, stack, hit = set(), [(k, idx)], None
            while stack and hit is None:
                blk, upto = stack.pop()
                settled = False
                for j in range(upto - 1, -1, -1):
                    u = blocks[blk][j]
                    if u.startswith("s_waitcnt") and "lgkmcnt(0)" in u:
                        settled = True
                        break
                    if _LDS_OP.match(u):
                        hit = (k, u, blk)
                        break
                if settled or hit:
                    continue
                for p in pred[blk]:
                    if p not in seen:
                        seen.add(p)
                        stack.append((p, len(blocks[p])))
            if hit:
                found.append(hit)
    return found


def audit_files(files):
    """[(file, kernel, barrier block, store, store block)] over the assembly files."""
    out = []
    for path in files:
        with open(path) as f:
            lines = f.read().split("\n")
        for name, body in _functions(lines):
            for b, store, sb in audit_function(body):
                out.append((os.path.basename(path), name, b, store, sb))
    return out


def main(argv):
    files = argv or default_files()
    if not files:
        print("no assembly files: build first (python -m paper_2605_19726_amd.build)", file=sys.stderr)
        return 2
    bad = audit_files(files)
    for f, name, b, store, sb in bad:
        print(f"{f}: {name}: s_barrier in {b} reachable from `{store}` ({sb}) without s_waitcnt lgkmcnt(0)")
    print(f"{len(files)} files, {len(bad)} findings")
    return 1 if bad else 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
