"""CPU oracle for the DashAttention forward path -- TEST INFRASTRUCTURE ONLY.

Plain numpy, fp64, one query row at a time, no blocking, no fusion, no
reordering beyond what the paper's definitions state.  It exists so that the
HIP library can be checked element by element; nothing in the product path may
import it (only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline
leg do).  It shares no code, table or constant with the HIP path.

What each function follows (paper sections / equations / algorithms):

  block_mean_summaries   Stage 0, Eq. 3 with the summary query at its zero
                         initial value (uniform mean pooling), Alg. 1
  local_attention_summaries
                         Stage 0 with a learned summary query, Eq. 3 / Alg. 1
  entmax_threshold_*     Eq. 2 / App. A Eq. 11: tau with sum_i [x_i-tau]_+^(1/(a-1)) = 1
  entmax                 Eq. 2
  route_token            Stage 1, Eq. 4 and the GQA averaging paragraph; Alg. 2
  prior_bias             Proposition 1 (mu_i, d_ij)
  attend_bias_form       Proposition 1 / Alg. 3: softmax(z + d) V over R_i u D_i
  prior_literal,
  attend_literal         Eq. 5-8 taken literally (w', lambda via KL + sigmoid, g)
  dense_attention        Eq. 1
  dash_row_at, dash_row,
  dash_rows              the whole path for one (batch, kv-head, query) triple

Pins (tests/test_oracle_*.py, all CPU): entmax closed forms, simplex
invariants, alpha=2 == Euclidean projection, alpha->1 == softmax, brute force
over supports on tiny inputs, exact-vs-bisection agreement, Proposition 1
(literal form == bias form), sigma->inf == masked softmax, gamma->0 == dense
causal attention, block-permutation invariance; learned summaries: zero query
== block mean (bit for bit), a library softmax + matmul per chunk, the
argmax-key limit, convex-hull bounds, shift equivariance.

Parity unpinned: the paper prints no worked numerical example, so absolute
output values at finite sigma are pinned only through Proposition 1 and the
limits above.  The readings of silent/ambiguous points (candidate set c < c_i,
non-causal case, fp32 summaries, decode position, empty candidate set) are
conventions of this build, listed in the design notes.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Iterable, List, Optional, Sequence, Tuple

import numpy as np

__all__ = [
    "block_mean_summaries", "local_attention_summaries", "entmax_threshold_exact", "entmax_threshold_bisect",
    "entmax_threshold", "entmax", "route_token", "prior_bias",
    "attend_bias_form", "prior_literal", "attend_literal", "dense_attention",
    "DashParams", "RowResult", "dash_row_at", "dash_row", "dash_rows", "dash_forward_full",
]


# --------------------------------------------------------------------------
# Stage 0
# --------------------------------------------------------------------------
def block_mean_summaries(k: np.ndarray, block: int) -> np.ndarray:
    """Uniform mean of every complete chunk of `block` keys (Stage 0 with the
    zero summary query).  k: [..., n, d].  Returns [..., floor(n/block), d] as
    fp64 values that are exactly representable in fp32: the summary cache is
    defined as the fp64 mean rounded once to fp32.
    """
    k = np.asarray(k, dtype=np.float64)
    n, d = k.shape[-2], k.shape[-1]
    t_c = n // block
    body = k[..., : t_c * block, :].reshape(k.shape[:-2] + (t_c, block, d))
    mean = body.sum(axis=-2) / float(block)
    return mean.astype(np.float32).astype(np.float64)


def local_attention_summaries(k: np.ndarray, qbar: np.ndarray, block: int,
                              scale: Optional[float] = None) -> np.ndarray:
    """Stage 0 with a learned summary query (Eq. 3; Alg. 1): every complete
    chunk is summarised by one softmax attention of the summary query over the
    chunk's own keys, the keys serving as values as well.

    k: [..., h_kv, n, d]; qbar: broadcastable to [..., h_kv, T_c, d] (one vector
    per kv-head as in Sec. 3.1, or one per chunk as in Alg. 1, where the
    rotary embedding has been applied to it); scale defaults to 1/sqrt(d).
    Returns [..., h_kv, T_c, d] as fp64 values exactly representable in fp32
    (the summary cache is fp32).
    """
    k = np.asarray(k, dtype=np.float64)
    n, d = k.shape[-2], k.shape[-1]
    t_c = n // block
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    body = k[..., : t_c * block, :].reshape(k.shape[:-2] + (t_c, block, d))
    qb = np.broadcast_to(np.asarray(qbar, dtype=np.float64), body.shape[:-2] + (d,))
    out = np.empty(body.shape[:-2] + (d,), dtype=np.float64)
    for idx in np.ndindex(*body.shape[:-2]):
        keys = body[idx]                      # [block, d]
        s = keys @ qb[idx] * scale            # s_t = <qbar, k_t> / sqrt(d)
        e = np.exp(s - s.max())
        out[idx] = (e / e.sum()) @ keys       # softmax(s)^T K_c
    return out.astype(np.float32).astype(np.float64)


# --------------------------------------------------------------------------
# alpha-entmax
# --------------------------------------------------------------------------
def _entmax_residual(x: np.ndarray, tau: float, p: float) -> float:
    u = np.maximum(x - tau, 0.0)
    return float(np.sum(u ** p) - 1.0)


def entmax_threshold_bisect(x: np.ndarray, alpha: float, width: float = 1e-15) -> float:
    """tau solving sum_i [x_i - tau]_+^(1/(alpha-1)) = 1 by bisection.

    x already carries the (alpha-1) factor of Eq. 2.  Bracket: at max(x)-1 the
    largest entry alone contributes 1 (residual >= 0); at max(x)-n^-(alpha-1)
    every entry contributes at most 1/n (residual <= 0).
    """
    x = np.asarray(x, dtype=np.float64).ravel()
    n = x.size
    assert n >= 1 and alpha > 1.0
    p = 1.0 / (alpha - 1.0)
    mx = float(x.max())
    lo = mx - 1.0
    hi = mx - float(n) ** (-(alpha - 1.0))
    for _ in range(200):
        if hi - lo <= width:
            break
        mid = 0.5 * (lo + hi)
        if mid <= lo or mid >= hi:
            break
        if _entmax_residual(x, mid, p) >= 0.0:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def entmax_threshold_exact(x: np.ndarray, alpha: float) -> float:
    """Sort-based tau for alpha in {1.5, 2}.

    With the entries sorted decreasingly and k of them kept, the
    normalisation condition is, for alpha=2, sum_{j<=k}(x_j - tau) = 1, i.e.
    tau_k = (sum_{j<=k} x_j - 1)/k; for alpha=1.5, sum_{j<=k}(x_j - tau)^2 = 1,
    i.e. k (M_k - tau)^2 + SS_k = 1 with M_k the mean and SS_k the centred sum
    of squares of the k largest, so tau_k = M_k - sqrt((1 - SS_k)/k).  The
    support is the largest k whose tau_k still lies below its smallest kept
    entry.
    """
    xs = np.sort(np.asarray(x, dtype=np.float64).ravel())[::-1]
    n = xs.size
    best = None
    for k in range(1, n + 1):
        head = xs[:k]
        if alpha == 2.0:
            tau_k = (head.sum() - 1.0) / k
        elif alpha == 1.5:
            m_k = head.mean()
            ss_k = float(np.sum((head - m_k) ** 2))
            if ss_k > 1.0:
                continue
            tau_k = m_k - math.sqrt((1.0 - ss_k) / k)
        else:
            raise ValueError("exact threshold only for alpha in {1.5, 2}")
        if tau_k < xs[k - 1]:
            best = tau_k
    assert best is not None
    return float(best)


def entmax_threshold(x: np.ndarray, alpha: float) -> float:
    if alpha == 2.0 or alpha == 1.5:
        return entmax_threshold_exact(x, alpha)
    return entmax_threshold_bisect(x, alpha)


def entmax(s: np.ndarray, alpha: float) -> np.ndarray:
    """alpha-entmax of a score vector s (Eq. 2)."""
    x = (alpha - 1.0) * np.asarray(s, dtype=np.float64)
    tau = entmax_threshold(x, alpha)
    return np.maximum(x - tau, 0.0) ** (1.0 / (alpha - 1.0))


# --------------------------------------------------------------------------
# Stage 1
# --------------------------------------------------------------------------
def route_token(q_heads: np.ndarray, kbar_cand: np.ndarray, alpha: float,
                gamma: float, scale: float):
    """Stage-1 routing of one token for one kv-head.

    q_heads [g_q, d]: the query vectors of the g_q heads that share the
    kv-head; kbar_cand [n_cand, d]: summaries of the candidate chunks.
    Returns (x [g_q,n_cand], tau [g_q], w_hat [g_q,n_cand], w [n_cand]) where
    x = gamma (alpha-1) <q, kbar> scale is the entmax-domain score, w_hat the
    per-head entmax probabilities and w their average over the group.
    """
    q_heads = np.asarray(q_heads, dtype=np.float64)
    kbar_cand = np.asarray(kbar_cand, dtype=np.float64)
    g_q = q_heads.shape[0]
    n_cand = kbar_cand.shape[0]
    x = np.empty((g_q, n_cand))
    tau = np.empty(g_q)
    w_hat = np.empty((g_q, n_cand))
    p = 1.0 / (alpha - 1.0)
    for h in range(g_q):
        zbar = kbar_cand @ q_heads[h] * scale
        x[h] = gamma * (alpha - 1.0) * zbar
        tau[h] = entmax_threshold(x[h], alpha)
        w_hat[h] = np.maximum(x[h] - tau[h], 0.0) ** p
    w = w_hat.sum(axis=0) / float(g_q)
    return x, tau, w_hat, w


def prior_bias(w: np.ndarray, sigma: float):
    """Proposition 1: routed set R = {c : w_c > 0} (ascending), mu = mean over
    R of ln w, bias d_c = (ln w_c - mu) / sigma."""
    w = np.asarray(w, dtype=np.float64)
    routed = np.nonzero(w > 0.0)[0]
    if routed.size == 0:
        return routed, np.zeros(0)
    logw = np.log(w[routed])
    mu = logw.mean()
    return routed, (logw - mu) / sigma


# --------------------------------------------------------------------------
# Stage 2
# --------------------------------------------------------------------------
def _softmax_weighted_sum(logits: np.ndarray, values: np.ndarray) -> np.ndarray:
    m = logits.max()
    e = np.exp(logits - m)
    return (e @ values) / e.sum()


def attend_bias_form(q_heads, k, v, scale, block, routed_chunks, bias,
                     diag_lo: int, diag_hi: int) -> np.ndarray:
    """softmax(z + d) V over the tokens of the routed chunks (bias d_c each)
    and the diagonal tokens diag_lo..diag_hi-1 (bias 0).  k, v: [n, d]."""
    q_heads = np.asarray(q_heads, dtype=np.float64)
    idx: List[np.ndarray] = []
    dvec: List[np.ndarray] = []
    for c, d_c in zip(routed_chunks, bias):
        idx.append(np.arange(c * block, (c + 1) * block))
        dvec.append(np.full(block, d_c))
    if diag_hi > diag_lo:
        idx.append(np.arange(diag_lo, diag_hi))
        dvec.append(np.zeros(diag_hi - diag_lo))
    tok = np.concatenate(idx)
    dtok = np.concatenate(dvec)
    kk = np.asarray(k[tok], dtype=np.float64)
    vv = np.asarray(v[tok], dtype=np.float64)
    out = np.empty((q_heads.shape[0], vv.shape[1]))
    for h in range(q_heads.shape[0]):
        z = kk @ q_heads[h] * scale
        out[h] = _softmax_weighted_sum(z + dtok, vv)
    return out


def prior_literal(w: np.ndarray, sigma: float, block: int, n_diag: int):
    """The prior g of Eq. 7 with lambda of Eq. 8, token by token.

    Returns (routed_chunks, g_routed_token [one value per routed chunk: the
    prior of each of its `block` tokens], g_diag_token, lam).
    """
    w = np.asarray(w, dtype=np.float64)
    routed = np.nonzero(w > 0.0)[0]
    n_r_tok = routed.size * block
    if n_r_tok == 0:
        return routed, np.zeros(0), (1.0 / n_diag if n_diag else 0.0), 0.0
    ws = w[routed] ** (1.0 / sigma)
    w_prime = ws / (block * ws.sum())              # per token of each routed chunk
    if n_diag == 0:
        lam = 1.0
    else:
        # KL(u_R || w'_R) over the routed tokens, u_R uniform on them
        u = 1.0 / n_r_tok
        kl = float(np.sum(block * u * np.log(u / w_prime)))
        t = kl + math.log(n_r_tok / n_diag)
        lam = 1.0 / (1.0 + math.exp(-t))
    g_r = lam * w_prime
    g_d = (1.0 - lam) / n_diag if n_diag else 0.0
    return routed, g_r, g_d, lam


def attend_literal(q_heads, k, v, scale, block, w, sigma,
                   diag_lo: int, diag_hi: int) -> np.ndarray:
    """Eq. 6: o = sum_j g_j exp(z_j) v_j / sum_t g_t exp(z_t) with g of Eq. 7."""
    routed, g_r, g_d, _ = prior_literal(w, sigma, block, diag_hi - diag_lo)
    q_heads = np.asarray(q_heads, dtype=np.float64)
    idx, gvec = [], []
    for c, g_c in zip(routed, g_r):
        idx.append(np.arange(c * block, (c + 1) * block))
        gvec.append(np.full(block, g_c))
    if diag_hi > diag_lo:
        idx.append(np.arange(diag_lo, diag_hi))
        gvec.append(np.full(diag_hi - diag_lo, g_d))
    tok = np.concatenate(idx)
    g = np.concatenate(gvec)
    kk = np.asarray(k[tok], dtype=np.float64)
    vv = np.asarray(v[tok], dtype=np.float64)
    out = np.empty((q_heads.shape[0], vv.shape[1]))
    for h in range(q_heads.shape[0]):
        z = kk @ q_heads[h] * scale
        e = g * np.exp(z - z.max())
        out[h] = (e @ vv) / e.sum()
    return out


def dense_attention(q, k, v, scale: float, causal: bool, q_pos0: int = 0) -> np.ndarray:
    """Eq. 1 for one head: q [n_q, d], k, v [n_kv, d]; query row t sits at
    position q_pos0 + t and, if causal, sees keys 0..position."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    out = np.empty((q.shape[0], v.shape[1]))
    for t in range(q.shape[0]):
        hi = q_pos0 + t + 1 if causal else k.shape[0]
        z = k[:hi] @ q[t] * scale
        out[t] = _softmax_weighted_sum(z, v[:hi])
    return out


# --------------------------------------------------------------------------
# The whole path
# --------------------------------------------------------------------------
@dataclass
class DashParams:
    block: int
    alpha: float = 1.5
    gamma: float = 1.0
    sigma: float = 1.0
    causal: bool = True
    scale: Optional[float] = None      # None -> 1/sqrt(d)
    window: int = 0                    # complete chunks before the diagonal one that are always attended


@dataclass
class RowResult:
    b: int
    r: int
    iq: int
    pos: int
    n_cand: int
    x: np.ndarray          # [g_q, n_cand] entmax-domain scores
    tau: np.ndarray        # [g_q]
    w: np.ndarray          # [n_cand] group-averaged weights
    routed: np.ndarray     # ascending chunk ids with w > 0
    bias: np.ndarray       # d_c for the routed chunks
    diag: Tuple[int, int]  # [lo, hi) token range of the diagonal branch
    o: np.ndarray          # [g_q, d]


def dash_row_at(qh, k, v, kbar, prm: DashParams, pos: int, ident=(0, 0, 0)) -> RowResult:
    """The forward path for the g_q query heads qh [g_q, d] of one kv-head at
    sequence position pos, against that head's keys/values k, v [n_kv, d] and
    summaries kbar [T_c, d].

    Causal: candidates are the chunks strictly before the query's own chunk,
    and the diagonal branch is the causal part of that chunk (Alg. 2).  With
    prm.window = W > 0 the W complete chunks just before the query's own are
    part of the always-attended local set as well (the local window of the
    trained models, App. B.1: the diagonal block and the last block, W = 1):
    they leave the candidate set and their tokens join the diagonal branch
    D_i of Proposition 1 with bias 0.  Non-causal: all chunks are candidates
    and there is no diagonal branch.
    """
    qh = np.asarray(qh, dtype=np.float64)
    g_q, d = qh.shape
    n_kv = k.shape[0]
    scale = prm.scale if prm.scale is not None else 1.0 / math.sqrt(d)
    blk = prm.block
    if prm.causal:
        n_cand = max(pos // blk - prm.window, 0)
        diag = (n_cand * blk, pos + 1)
    else:
        assert n_kv % blk == 0
        n_cand = n_kv // blk
        diag = (0, 0)
    if n_cand > 0:
        x, tau, _, w = route_token(qh, kbar[:n_cand], prm.alpha, prm.gamma, scale)
        routed, bias = prior_bias(w, prm.sigma)
    else:
        x = np.zeros((g_q, 0)); tau = np.zeros(g_q); w = np.zeros(0)
        routed = np.zeros(0, dtype=np.int64); bias = np.zeros(0)
    o = attend_bias_form(qh, k, v, scale, blk, routed, bias, diag[0], diag[1])
    return RowResult(ident[0], ident[1], ident[2], pos, n_cand, x, tau, w, routed, bias, diag, o)


def dash_row(q, k, v, kbar, prm: DashParams, b: int, r: int, iq: int) -> RowResult:
    """One (batch b, kv-head r, query index iq) of the forward path.

    q [B,H_q,n_q,d], k, v [B,H_kv,n_kv,d] hold run-dtype values; kbar
    [B,H_kv,T_c,d] comes from block_mean_summaries.  Query iq sits at position
    n_kv - n_q + iq (prefill: iq; decode with n_q = 1: the last cached token).
    """
    n_q = q.shape[2]
    n_kv = k.shape[2]
    g_q = q.shape[1] // k.shape[1]
    pos = n_kv - n_q + iq
    return dash_row_at(q[b, r * g_q:(r + 1) * g_q, iq, :], k[b, r], v[b, r], kbar[b, r], prm, pos,
                       (b, r, iq))


def dash_rows(q, k, v, prm: DashParams, rows: Iterable[Tuple[int, int, int]],
              kbar: Optional[np.ndarray] = None) -> List[RowResult]:
    if kbar is None:
        kbar = block_mean_summaries(k, prm.block)
    return [dash_row(q, k, v, kbar, prm, b, r, iq) for (b, r, iq) in rows]


def dash_forward_full(q, k, v, prm: DashParams):
    """Every row.  Returns (O [B,H_q,n_q,d] fp64, kbar, list of RowResult)."""
    B, h_q, n_q, d = q.shape
    h_kv = k.shape[1]
    g_q = h_q // h_kv
    kbar = block_mean_summaries(k, prm.block)
    out = np.empty((B, h_q, n_q, d))
    res = []
    for b in range(B):
        for r in range(h_kv):
            for iq in range(n_q):
                rr = dash_row(q, k, v, kbar, prm, b, r, iq)
                out[b, r * g_q:(r + 1) * g_q, iq, :] = rr.o
                res.append(rr)
    return out, kbar, res
