"""The oracle against its stored results (tests/golden/, written by
tests/golden/make_golden.py from oracle/ alone).  The paper prints no worked
example; these fixtures guard the oracle against silent changes."""
import json
import os

import numpy as np

from oracle import dash_oracle as orc
from oracle import dash_oracle_bwd as bwd

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _load(name):
    with open(os.path.join(GOLD, name)) as f:
        return json.load(f)


def test_entmax_golden():
    for c in _load("entmax_cases.json")["cases"]:
        s = np.asarray(c["scores"], dtype=np.float64)
        p = orc.entmax(s, c["alpha"])
        tau = orc.entmax_threshold((c["alpha"] - 1.0) * s, c["alpha"])
        assert abs(tau - float(c["tau"])) < 1e-13, (c["name"], c["alpha"])
        assert np.allclose(p, np.asarray([float(t) for t in c["p"]]), rtol=0, atol=1e-13)
        assert abs(p.sum() - 1.0) < 1e-12


def test_tiny_path_golden():
    g = _load("tiny_path.json")
    q, k, v = (np.asarray(g[n], dtype=np.float64) for n in ("q", "k", "v"))
    prm = orc.DashParams(**g["params"])
    o, _, rows = orc.dash_forward_full(q, k, v, prm)
    want = np.asarray([[[[float(t) for t in row] for row in head] for head in b] for b in g["o"]])
    assert np.allclose(o, want, rtol=0, atol=1e-12)
    assert [[int(c) for c in rr.routed] for rr in rows] == g["routed"]
    for rr in rows:
        assert list(rr.routed) == sorted(rr.routed) and all(0 <= c < rr.n_cand for c in rr.routed)


def test_tiny_backward_golden():
    g, gb = _load("tiny_path.json"), _load("tiny_backward.json")
    q, k, v = (np.asarray(g[n], dtype=np.float64) for n in ("q", "k", "v"))
    d_o = np.asarray(gb["d_o"], dtype=np.float64)
    prm = orc.DashParams(**g["params"])
    for r, want in enumerate(gb["kv_heads"]):
        got = bwd.dash_backward_group(q[0, 2 * r:2 * r + 2], k[0, r], v[0, r], d_o[0, 2 * r:2 * r + 2], prm)
        for name, arr in zip(("dq", "dk", "dv", "dkbar"), got):
            ref = np.asarray([[float(t) for t in row] for row in want[name]])
            assert np.allclose(arr.reshape(ref.shape), ref, rtol=0, atol=1e-12 * max(1.0, np.abs(ref).max())), name
        assert np.abs(np.asarray([[float(t) for t in row] for row in want["dkbar"]])).max() > 0
