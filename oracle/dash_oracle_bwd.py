"""CPU oracle for the DashAttention backward pass -- TEST INFRASTRUCTURE ONLY.

Plain numpy, fp64, one query row at a time, the chain rule applied step by
step to the forward path of dash_oracle.dash_row_at; nothing in the product
path may import it.  It shares no code with the HIP path.

The paper states that the Stage-2 output (Sec. 3.3) is differentiable with respect to q, k, v and the
prior, that the gradient reaches the Stage-1 entmax weights and, through them,
the Stage-0 summaries (end of Sec. 3.3), and that the backward pass reuses the
forward's chunk mask because the entmax Jacobian is sparse (Sec. 3.5 / App. on
differentiability): inside a region of fixed support the Jacobian of
p = entmax_alpha(s) is  diag(g) - g g^T / sum(g)  with  g_c = p_c^(2-alpha) on
the support and 0 elsewhere (Peters et al., 2019).  At a support change the
map is only piecewise differentiable; the oracle, like automatic
differentiation, takes the Jacobian of the current support.

Chain, for the g_q query heads of one kv-head at one position (notation of
dash_oracle: x = gamma (alpha-1) <q, kbar> scale, u = x - tau, w_hat = u^p with
p = 1/(alpha-1), w = mean over heads of w_hat, bias d_c = (ln w_c - mu)/sigma
with mu the mean of ln w over the routed set R, logits z + d over the routed
chunks and z over the always-attended local tokens):

  attention      P = softmax(z + d),  o = P V
                 dP = V do,  dz = P * (dP - <P, dP>)
                 dq += scale K^T dz,  dK += scale dz q^T,  dV += P do^T
  bias           dd_c = sum over heads and over the tokens of chunk c of dz
  prior          dlnw_c = (dd_c - mean_R dd) / sigma        (mu depends on every ln w)
                 dw_c = dlnw_c / w_c,  dw_hat_{h,c} = dw_c / g_q
  entmax         g_{h,c} = p u_{h,c}^(p-1) on head h's support,
                 dx_{h,c} = g_{h,c} (dw_hat_{h,c} - sum_j g_{h,j} dw_hat_{h,j} / sum_j g_{h,j})
  scores         dq_h += c sum_c dx_{h,c} kbar_c,  dkbar_c += c sum_h dx_{h,c} q_h,
                 c = gamma (alpha-1) scale
  summaries      block mean: dK_j += dkbar_c / B for every key j of chunk c
                 (the rounding of the summary cache to fp32 is treated as the identity)

  learned summary  kbar_c = a^T K_c with a = softmax(K_c qbar scale) (Eq. 3): for a given
                 dkbar_c,  da = K_c dkbar_c,  ds = a * (da - <a, da>),
                 dK_c += a dkbar_c^T + scale ds qbar^T,  dqbar_c = scale K_c^T ds
                 (local_attention_summaries_backward; the gradient of the trainable
                 Stage 0 the paper refers to at the end of Sec. 3.3)

Pins (tests/test_oracle_backward.py, CPU): central finite differences of the
forward oracle's own outputs on tiny inputs with sparse supports (q, k, v, all
alpha modes, GQA, window, non-causal); the entmax Jacobian against finite
differences of entmax; the gamma -> 0 limit against a library's automatic
differentiation of causal softmax attention; sum_c dx_{h,c} = 0 (shift
invariance of entmax); zero gradient for keys and values no query attends;
the learned-summary backward against finite differences of
local_attention_summaries and, at a zero query, against the block-mean rule.
"""
from __future__ import annotations

import math
from typing import Optional, Tuple

import numpy as np

from . import dash_oracle as orc


def entmax_jacobian_vjp(x: np.ndarray, tau: float, alpha: float, dw: np.ndarray) -> np.ndarray:
    """Vector-Jacobian product of w = [x - tau(x)]_+^p, p = 1/(alpha-1), where
    tau(x) keeps sum w = 1: returns dL/dx for a given dL/dw.  Entries of dw
    outside the support are ignored."""
    p = 1.0 / (alpha - 1.0)
    u = x - tau
    sup = u > 0.0
    g = np.zeros_like(x)
    g[sup] = p * u[sup] ** (p - 1.0)
    gs = g.sum()
    dws = np.where(sup, dw, 0.0)
    return g * (dws - (g * dws).sum() / gs)


def backward_row(qh: np.ndarray, k: np.ndarray, v: np.ndarray, kbar: np.ndarray, d_o: np.ndarray,
                 prm: orc.DashParams, pos: int, dk: np.ndarray, dv: np.ndarray, dkbar: np.ndarray):
    """Backward of dash_oracle.dash_row_at for the g_q heads qh [g_q, d] at
    position pos with upstream gradient d_o [g_q, d].  Adds this row's
    contributions into dk, dv [n_kv, d] and dkbar [T_c, d]; returns
    (dq [g_q, d], dx [g_q, n_cand], dd [len(routed)])."""
    qh = np.asarray(qh, dtype=np.float64)
    d_o = np.asarray(d_o, dtype=np.float64)
    g_q, d = qh.shape
    rr = orc.dash_row_at(qh, k, v, kbar, prm, pos)
    scale = prm.scale if prm.scale is not None else 1.0 / math.sqrt(d)
    blk = prm.block
    # the attended tokens and their bias, in the forward's order
    tok = [np.arange(c * blk, (c + 1) * blk) for c in rr.routed]
    dtok = [np.full(blk, b) for b in rr.bias]
    chunk_of = [np.full(blk, j) for j in range(len(rr.routed))]
    if rr.diag[1] > rr.diag[0]:
        tok.append(np.arange(rr.diag[0], rr.diag[1]))
        dtok.append(np.zeros(rr.diag[1] - rr.diag[0]))
        chunk_of.append(np.full(rr.diag[1] - rr.diag[0], -1))
    tok = np.concatenate(tok)
    dtok = np.concatenate(dtok)
    chunk_of = np.concatenate(chunk_of)
    kk = np.asarray(k[tok], dtype=np.float64)
    vv = np.asarray(v[tok], dtype=np.float64)

    dq = np.zeros((g_q, d))
    dd = np.zeros(len(rr.routed))
    for h in range(g_q):
        z = kk @ qh[h] * scale + dtok
        e = np.exp(z - z.max())
        P = e / e.sum()
        dP = vv @ d_o[h]
        dz = P * (dP - P @ dP)
        dq[h] += scale * (kk.T @ dz)
        np.add.at(dk, tok, scale * np.outer(dz, qh[h]))
        np.add.at(dv, tok, np.outer(P, d_o[h]))
        for j in range(len(rr.routed)):
            dd[j] += dz[chunk_of == j].sum()

    dx = np.zeros((g_q, rr.n_cand))
    if len(rr.routed):
        dlnw = (dd - dd.mean()) / prm.sigma
        dw = np.zeros(rr.n_cand)
        dw[rr.routed] = dlnw / rr.w[rr.routed]
        c_x = prm.gamma * (prm.alpha - 1.0) * scale
        for h in range(g_q):
            dx[h] = entmax_jacobian_vjp(rr.x[h], rr.tau[h], prm.alpha, dw / float(g_q))
            dq[h] += c_x * (dx[h] @ np.asarray(kbar[:rr.n_cand], dtype=np.float64))
            dkbar[:rr.n_cand] += c_x * np.outer(dx[h], qh[h])
    return dq, dx, dd


def dash_backward_group(q: np.ndarray, k: np.ndarray, v: np.ndarray, d_o: np.ndarray,
                        prm: orc.DashParams, kbar: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """Backward for one (batch, kv-head) pair: q, d_o [g_q, n_q, d]; k, v
    [n_kv, d]; query t sits at position n_kv - n_q + t.  kbar None: block-mean
    summaries, whose gradient is folded into dk; otherwise the given summaries
    are an independent input and only dkbar carries their gradient.
    Returns (dq [g_q, n_q, d], dk, dv [n_kv, d], dkbar [T_c, d])."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    g_q, n_q, d = q.shape
    n_kv = k.shape[0]
    fold = kbar is None
    if fold:
        kbar = orc.block_mean_summaries(k, prm.block)
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    dkbar = np.zeros_like(np.asarray(kbar, dtype=np.float64))
    for t in range(n_q):
        dq[:, t], _, _ = backward_row(q[:, t], k, v, kbar, d_o[:, t], prm, n_kv - n_q + t, dk, dv, dkbar)
    if fold:
        blk = prm.block
        for c in range(dkbar.shape[0]):
            dk[c * blk:(c + 1) * blk] += dkbar[c] / float(blk)
    return dq, dk, dv, dkbar


def local_attention_summaries_backward(k: np.ndarray, qbar: np.ndarray, block: int, dkbar: np.ndarray,
                                       scale: Optional[float] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Backward of dash_oracle.local_attention_summaries for one kv-head:
    k [n, d], qbar [d] (one query for all chunks) or [T_c, d] (one per chunk),
    dkbar [T_c, d].  Returns (dk [n, d], dqbar_c [T_c, d]): the gradient of the
    keys through their chunk's summary and the gradient of the summary query
    per chunk (a shared query's gradient is their sum).  The fp32 rounding of
    the summaries is treated as the identity."""
    k = np.asarray(k, dtype=np.float64)
    n, d = k.shape
    t_c = n // block
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    qb = np.broadcast_to(np.asarray(qbar, dtype=np.float64), (t_c, d))
    dk = np.zeros_like(k)
    dq = np.zeros((t_c, d))
    for c in range(t_c):
        keys = k[c * block:(c + 1) * block]
        s = keys @ qb[c] * scale
        e = np.exp(s - s.max())
        a = e / e.sum()
        g = np.asarray(dkbar[c], dtype=np.float64)
        da = keys @ g
        ds = a * (da - a @ da)
        dk[c * block:(c + 1) * block] = np.outer(a, g) + scale * np.outer(ds, qb[c])
        dq[c] = scale * (keys.T @ ds)
    return dk, dq
