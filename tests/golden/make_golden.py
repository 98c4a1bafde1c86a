#!/usr/bin/env python3
"""Writes the stored expected values under tests/golden/ by calling only oracle/.

The paper prints no worked numerical example, so these fixtures are the
oracle's own results on small fixed inputs: they pin the oracle against silent
changes (a later edit that moves any of them must be justified by the paper),
they do not pin it against the paper.  Every value is written with 17
significant digits.  Run from the repository root:

    python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
from oracle import dash_oracle as orc  # noqa: E402
from oracle import dash_oracle_bwd as bwd  # noqa: E402


def entmax_cases():
    """alpha-entmax (Eq. 2; App. A) of three fixed score vectors at four alphas."""
    vecs = {
        "ramp8": [0.1 * i for i in range(8)],
        "two_close_one_far": [1.0, 0.9, -2.0],
        "mixed12": [0.3, -1.2, 2.5, 2.4, 0.0, 1.1, -0.7, 2.45, 0.9, -3.0, 1.6, 2.0],
    }
    out = []
    for name, v in vecs.items():
        for alpha in (1.25, 1.5, 2.0, 3.0):
            s = np.asarray(v, dtype=np.float64)
            x = (alpha - 1.0) * s
            tau = orc.entmax_threshold(x, alpha)
            p = orc.entmax(s, alpha)
            out.append({"name": name, "alpha": alpha, "scores": v, "tau": repr(float(tau)),
                        "p": [repr(float(t)) for t in p]})
    return out


def path_case():
    """The whole forward path (Alg. 1-3, Prop. 1) on a tiny causal GQA problem:
    N = 16, chunk 4, d = 4, 4 query heads on 2 kv-heads, alpha = 1.5, sigma = 2."""
    rng = np.random.default_rng(20240607)
    n, d = 16, 4
    q = rng.standard_normal((1, 4, n, d)).round(3)
    k = rng.standard_normal((1, 2, n, d)).round(3)
    v = rng.standard_normal((1, 2, n, d)).round(3)
    k[0, :, 8:12] += 1.5          # one chunk with a shifted mean so that routing is sparse
    prm = orc.DashParams(block=4, alpha=1.5, gamma=2.0, sigma=2.0, causal=True)
    o, kbar, rows = orc.dash_forward_full(q, k, v, prm)
    return {
        "q": q.tolist(), "k": k.tolist(), "v": v.tolist(),
        "params": {"block": 4, "alpha": 1.5, "gamma": 2.0, "sigma": 2.0, "causal": True},
        "o": [[[[repr(float(t)) for t in row] for row in head] for head in b] for b in o],
        "routed": [[int(c) for c in rr.routed] for rr in rows],
        "bias": [[repr(float(t)) for t in rr.bias] for rr in rows],
        "tau": [[repr(float(t)) for t in rr.tau] for rr in rows],
    }


def backward_case():
    """The backward pass (end of Sec. 3.3; sparse entmax Jacobian) on the tiny problem of
    path_case with a fixed upstream gradient: dq, dk, dv and the summaries' gradient of
    each kv-head."""
    rng = np.random.default_rng(20240607)
    n, d = 16, 4
    q = rng.standard_normal((1, 4, n, d)).round(3)
    k = rng.standard_normal((1, 2, n, d)).round(3)
    v = rng.standard_normal((1, 2, n, d)).round(3)
    k[0, :, 8:12] += 1.5
    d_o = np.random.default_rng(77).standard_normal((1, 4, n, d)).round(3)
    prm = orc.DashParams(block=4, alpha=1.5, gamma=2.0, sigma=2.0, causal=True)
    heads = []
    for r in range(2):
        dq, dk, dv, dkbar = bwd.dash_backward_group(q[0, 2 * r:2 * r + 2], k[0, r], v[0, r], d_o[0, 2 * r:2 * r + 2], prm)
        heads.append({n_: [[repr(float(t)) for t in row] for row in a.reshape(-1, d)]
                      for n_, a in (("dq", dq), ("dk", dk), ("dv", dv), ("dkbar", dkbar))})
    return {"d_o": d_o.tolist(), "kv_heads": heads}


def main():
    with open(os.path.join(HERE, "entmax_cases.json"), "w") as f:
        json.dump({"what": "alpha-entmax threshold and probabilities (Eq. 2; App. A), oracle-generated",
                   "cases": entmax_cases()}, f, indent=1)
    with open(os.path.join(HERE, "tiny_path.json"), "w") as f:
        json.dump({"what": "DashAttention forward on a tiny causal GQA input (Alg. 1-3, Prop. 1), oracle-generated",
                   **path_case()}, f, indent=1)
    with open(os.path.join(HERE, "tiny_backward.json"), "w") as f:
        json.dump({"what": "DashAttention backward on the input of tiny_path.json (end of Sec. 3.3), oracle-generated",
                   **backward_case()}, f, indent=1)
    print("wrote entmax_cases.json, tiny_path.json, tiny_backward.json")


if __name__ == "__main__":
    main()
