"""Writes tests/golden/oracle_tiny.json: the oracle's own results on a tiny seeded input.

The paper prints no numeric worked example for this path, so this file holds no paper values.
It is a drift guard: the stored numbers were produced by oracle/basa_oracle.py alone (this
script imports nothing else of the repository), and tests/test_oracle_pins.py checks that
the oracle still reproduces them, so that a change to the oracle's arithmetic cannot pass
unnoticed.  Regenerate only together with a commit that says which passage of the paper
justifies the change:

    python tests/golden/make_oracle_fixtures.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import basa_oracle as o  # noqa: E402

L, D, B, SEED = 26, 4, 4, 20260519          # ragged: 6 full blocks and one of 2 tokens


def inputs():
    rng = np.random.default_rng(SEED)
    # multiples of 1/8: exactly representable, so the JSON round trip is exact
    return tuple(np.round(rng.standard_normal((L, D)) * 8) / 8 for _ in range(3))


def compute():
    Q, K, V = inputs()
    out = {"L": L, "d": D, "B": B, "seed": SEED}
    for name, kw in (("topk_s50", dict(sparsity=0.5)), ("topk_s50_beta0_sortK", dict(sparsity=0.5, beta=0.0, sort=o.SORT_K)),
                     ("mass_p60", dict(sparsity=0.0, mass_target=0.6, min_keep=2))):
        sel = o.select(Q, K, B, **kw)
        cols = [c.tolist() for c in sel["cols"]]
        O = o.sparse_attention(Q, K, V, sel["perm_q"], sel["perm_k"], sel["cols"], B)
        out[name] = {"perm_q": sel["perm_q"].tolist(), "perm_k": sel["perm_k"].tolist(),
                     "logits": sel["logits"].tolist(), "m": sel["m"].tolist(), "cols": cols,
                     "mass": np.asarray(sel["mass"]).tolist(), "O": O.tolist()}
    out["m_hat"] = o.oracle_block_mass(Q, K, B).tolist()
    out["bound"] = o.deviation_bound(Q, K, B).tolist()
    out["max_dev"] = o.max_logit_deviation(Q, K, B).tolist()
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_tiny.json")
    with open(path, "w") as f:
        json.dump(compute(), f, indent=1)
    print("wrote", path)
