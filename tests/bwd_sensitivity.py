"""Test-side conditioning estimate for the backward comparison.

The backward oracle is the plain chain rule and stays untouched; this module
only calls it again on inputs perturbed by the size of an fp32 rounding error and
reports how far each gradient element moves.  The GPU evaluates the routing
scores x = gamma (alpha-1) <q, kbar> scale and the sums of dz in fp32, so its
scores and bias gradients differ from the fp64 ones by about 1e-6 of their
magnitude; ln w and 1/w are singular at the edge of the support, so a few
elements of the exact gradient move by far more than that under such a change.

Perturbation: every element of the summaries is multiplied by 1 + eps * xi and
every element of dO by 1 + eps * eta, with xi, eta independent uniform signs
(seeded); the oracle is evaluated at +/- the same signs.  The summaries are
passed to the oracle as an input of their own, so for block-mean summaries this
module folds their gradient into dk itself (each key of a complete chunk receives
1/B of its summary's gradient), exactly as the oracle does.
"""
from __future__ import annotations

import numpy as np

from oracle import dash_oracle as orc
from oracle import dash_oracle_bwd as bwd


def _group(q, k, v, d_o, prm, kbar, fold):
    dq, dk, dv, dkb = bwd.dash_backward_group(q, k, v, d_o, prm, kbar=kbar)
    if fold:
        blk = prm.block
        dk = dk.copy()
        for c in range(dkb.shape[0]):
            dk[c * blk:(c + 1) * blk] += dkb[c] / float(blk)
    return dq, dk, dv, dkb


def perturbed_pair(q, k, v, d_o, prm, kbar=None, eps=1e-6, seed=0):
    """The oracle's gradients (dq, dk, dv, dkbar) at the two perturbed inputs.
    kbar None: block-mean summaries (their gradient folded into dk)."""
    fold = kbar is None
    kb = orc.block_mean_summaries(np.asarray(k, dtype=np.float64), prm.block) if fold else np.asarray(kbar, np.float64)
    rng = np.random.default_rng(seed)
    xi = rng.integers(0, 2, kb.shape) * 2.0 - 1.0
    eta = rng.integers(0, 2, np.shape(d_o)) * 2.0 - 1.0
    out = []
    for s in (+1.0, -1.0):
        out.append(_group(q, k, v, np.asarray(d_o, np.float64) * (1.0 + s * eps * eta), prm,
                          kb * (1.0 + s * eps * xi), fold))
    return out


def perturbed_row_pair(qh, k, v, kbar, doh, prm, pos, eps=1e-6, seed=0):
    """dq of one query row (backward_row) at the two perturbed inputs; the sums into
    dk, dv and dkbar go to arrays nobody reads."""
    kb = np.asarray(kbar, np.float64)
    rng = np.random.default_rng(seed)
    xi = rng.integers(0, 2, kb.shape) * 2.0 - 1.0
    eta = rng.integers(0, 2, np.shape(doh)) * 2.0 - 1.0
    scr = (np.zeros(np.shape(k)), np.zeros(np.shape(v)), np.zeros(kb.shape))
    return [bwd.backward_row(qh, k, v, kb * (1.0 + s * eps * xi), np.asarray(doh, np.float64) * (1.0 + s * eps * eta),
                             prm, pos, *scr)[0] for s in (+1.0, -1.0)]


def allowance(ref, pair, factor=3.0):
    """Element-wise allowance for each of the gradients in `ref`: factor times the
    sum of the two perturbed evaluations' distances from it."""
    return [factor * (np.abs(pair[0][j] - ref[j]) + np.abs(pair[1][j] - ref[j])) for j in range(len(ref))]


def rowwise_report(got, ref, allow, tol, cap=10.0):
    """Row by row (last axis = head_dim), scale_row = the row's largest reference
    magnitude floored at a tenth of the median over rows.  Returns a dict:
      plain_worst   largest |got - ref| / scale_row with no allowance at all
      median, p99   of the per-row largest |got - ref| / scale_row
      need_allow    fraction of elements with |got - ref| > tol * scale_row
      ill           fraction of elements whose allowance exceeds cap * tol * scale_row
                    (the exact gradient itself moves by more than cap * tol there)
      excess        largest (|got - ref| - tol * scale_row - allow) / scale_row (<= 0 passes)
      capped_excess the same with the allowance cut at cap * tol * scale_row, over the
                    elements that are not ill
    """
    rowmax = np.abs(ref).max(axis=-1, keepdims=True)
    floor = 0.1 * np.median(rowmax)
    scale = np.maximum(np.maximum(rowmax, floor), 1e-300)
    err = np.abs(got - ref)
    rel = err / scale
    per_row = rel.max(axis=-1)
    ill = allow > cap * tol * scale
    capped = np.minimum(allow, cap * tol * scale)
    ex_c = np.where(ill, -np.inf, (err - tol * scale - capped) / scale)
    return {
        "plain_worst": float(rel.max()),
        "median": float(np.median(per_row)),
        "p99": float(np.quantile(per_row, 0.99)),
        "need_allow": float((err > tol * scale).mean()),
        "ill": float(ill.mean()),
        "excess": float(((err - tol * scale - allow) / scale).max()),
        "capped_excess": float(ex_c.max()),
    }
