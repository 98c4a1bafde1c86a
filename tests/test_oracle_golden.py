"""The oracle against its stored results (tests/golden/, written by
tests/golden/make_golden.py from oracle/ alone).  The paper prints no worked
example; these fixtures guard the oracle against silent changes."""
import json
import os

import numpy as np

from oracle import dash_oracle as orc

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
