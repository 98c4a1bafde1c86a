"""Pins of the backward oracle (CPU only): finite differences of the forward
oracle, the entmax Jacobian, a library's automatic differentiation in the
dense limit, and structural invariants."""
import math

import numpy as np
import pytest
import torch

from oracle import dash_oracle as orc
from oracle import dash_oracle_bwd as bwd


def tiny_inputs(seed, g_q, n, d, block, spread=2.0):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((g_q, n, d)) * 1.5
    k = rng.standard_normal((n, d))
    k += np.repeat(rng.standard_normal((-(-n // block), d)) * spread, block, axis=0)[:n]
    v = rng.standard_normal((n, d))
    d_o = rng.standard_normal((g_q, n, d))
    return q, k, v, d_o


def exact_mean(k, block):
    t_c = k.shape[0] // block
    return k[: t_c * block].reshape(t_c, block, -1).mean(axis=1)


def loss(q, k, v, d_o, prm, kbar=None):
    """sum over rows of <o, d_o> with the forward oracle; kbar None -> the
    unrounded block mean of k (so that the loss is smooth in k)."""
    if kbar is None:
        kbar = exact_mean(k, prm.block)
    n_q, n_kv = q.shape[1], k.shape[0]
    tot = 0.0
    for t in range(n_q):
        rr = orc.dash_row_at(q[:, t], k, v, kbar, prm, n_kv - n_q + t)
        tot += float((rr.o * d_o[:, t]).sum())
    return tot


def min_margin(q, k, prm):
    kbar = exact_mean(k, prm.block)
    m = np.inf
    kept = total = 0
    for t in range(q.shape[1]):
        rr = orc.dash_row_at(q[:, t], k, k, kbar, prm, k.shape[0] - q.shape[1] + t)
        if rr.n_cand:
            m = min(m, np.abs(rr.x - rr.tau[:, None]).min())
            kept += len(rr.routed)
            total += rr.n_cand
    return m, kept, total


CASES = [
    # name, g_q, n, d, block, params
    ("alpha15_gqa2", 2, 40, 8, 8, dict(alpha=1.5)),
    ("alpha2_gqa3", 3, 36, 8, 6, dict(alpha=2.0, gamma=1.5)),
    ("alpha125_mha", 1, 40, 8, 8, dict(alpha=1.25, sigma=0.5)),
    ("alpha3_gqa2", 2, 40, 8, 8, dict(alpha=3.0, sigma=2.0)),
    ("window1_ragged", 2, 43, 8, 8, dict(alpha=1.5, window=1)),
    ("noncausal", 2, 32, 8, 8, dict(alpha=1.5, causal=False)),
    ("scale_given", 2, 40, 8, 8, dict(alpha=1.5, scale=0.2, gamma=2.0)),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_backward_matches_finite_differences_of_the_forward(case):
    name, g_q, n, d, block, kw = case
    prm = orc.DashParams(block=block, **kw)
    q, k, v, d_o = tiny_inputs(13 if name == "alpha3_gqa2" else 11, g_q, n, d, block)
    margin, kept, total = min_margin(q, k, prm)
    # the pin needs a fixed support inside the difference stencil and a support
    # that is neither empty nor full
    assert margin > 1e-3, margin
    assert 0 < kept < total, (kept, total)
    kbar_used = orc.block_mean_summaries(k, block)
    dq, dk, dv, dkbar = bwd.dash_backward_group(q, k, v, d_o, prm)
    rng = np.random.default_rng(5)
    h = 1e-6
    for name_t, arr, grad in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        worst = 0.0
        for _ in range(24):
            idx = tuple(int(rng.integers(0, s)) for s in arr.shape)
            keep = arr[idx]
            arr[idx] = keep + h
            lp = loss(q, k, v, d_o, prm)
            arr[idx] = keep - h
            lm = loss(q, k, v, d_o, prm)
            arr[idx] = keep
            fd = (lp - lm) / (2 * h)
            worst = max(worst, abs(fd - grad[idx]))
        assert worst <= 2e-6 * max(1.0, np.abs(grad).max()), (name_t, worst, np.abs(grad).max())
    # summaries as an independent input: dkbar alone, dk without the folded term
    dq2, dk2, dv2, dkbar2 = bwd.dash_backward_group(q, k, v, d_o, prm, kbar=kbar_used)
    assert np.array_equal(dkbar, dkbar2) and np.array_equal(dq, dq2) and np.array_equal(dv, dv2)
    t_c = n // block
    fold = np.zeros_like(dk)
    fold[: t_c * block] = np.repeat(dkbar / block, block, axis=0)
    assert np.allclose(dk2 + fold, dk, rtol=0, atol=1e-12 * np.abs(dk).max())
    worst = 0.0
    kb = kbar_used.copy()
    for _ in range(24):
        idx = tuple(int(rng.integers(0, s)) for s in kb.shape)
        keep = kb[idx]
        kb[idx] = keep + h
        lp = loss(q, k, v, d_o, prm, kb)
        kb[idx] = keep - h
        lm = loss(q, k, v, d_o, prm, kb)
        kb[idx] = keep
        worst = max(worst, abs((lp - lm) / (2 * h) - dkbar[idx]))
    assert worst <= 2e-6 * max(1.0, np.abs(dkbar).max()), worst
    assert np.abs(dkbar).max() > 1e-3          # the routing path carries a real gradient


@pytest.mark.parametrize("alpha", [1.25, 1.5, 2.0, 3.0])
def test_entmax_jacobian_against_finite_differences(alpha):
    rng = np.random.default_rng(3)
    s = rng.standard_normal(12) * 0.8 / (alpha - 1.0) ** 0.5 * 0.5
    x = (alpha - 1.0) * s
    tau = orc.entmax_threshold(x, alpha)
    assert 1 < (x > tau).sum() < 12 and np.abs(x - tau).min() > 1e-3, (x - tau)
    dw = rng.standard_normal(12)
    got = bwd.entmax_jacobian_vjp(x, tau, alpha, dw)
    h = 1e-6
    for i in range(12):
        sp, sm = s.copy(), s.copy()
        sp[i] += h
        sm[i] -= h
        # entmax takes s and multiplies by (alpha-1) itself: d/dx = d/ds / (alpha-1)
        fd = (orc.entmax(sp, alpha) - orc.entmax(sm, alpha)) @ dw / (2 * h) / (alpha - 1.0)
        assert abs(fd - got[i]) <= 1e-7 * max(1.0, np.abs(got).max())
    assert abs(got.sum()) <= 1e-12 * max(1.0, np.abs(got).max())     # shift invariance
    assert np.all(got[x <= tau] == 0.0)                            # sparse Jacobian


def test_entmax_jacobian_is_the_published_closed_form():
    """diag(g) - g g^T / sum(g) with g = p^(2-alpha) on the support (Peters et
    al., 2019), applied to probabilities as a function of the scores s."""
    rng = np.random.default_rng(8)
    for alpha in (1.5, 2.0, 1.3):
        s = rng.standard_normal(9) * 1.5
        prob = orc.entmax(s, alpha)
        g = np.where(prob > 0, prob ** (2.0 - alpha), 0.0)
        jac = np.diag(g) - np.outer(g, g) / g.sum()
        dw = rng.standard_normal(9)
        x = (alpha - 1.0) * s
        tau = orc.entmax_threshold(x, alpha)
        # ours is d/dx with x = (alpha-1) s, so d/ds = (alpha-1) d/dx
        got = (alpha - 1.0) * bwd.entmax_jacobian_vjp(x, tau, alpha, dw)
        assert np.allclose(got, jac @ dw, rtol=1e-10, atol=1e-12)


def test_dense_limit_matches_autograd_of_causal_attention():
    g_q, n, d, block = 2, 48, 16, 8
    q, k, v, d_o = tiny_inputs(2, g_q, n, d, block, spread=0.5)
    prm = orc.DashParams(block=block, gamma=1e-10)
    dq, dk, dv, dkbar = bwd.dash_backward_group(q, k, v, d_o, prm)
    tq = torch.tensor(q, requires_grad=True)
    tk = torch.tensor(k, requires_grad=True)
    tv = torch.tensor(v, requires_grad=True)
    o = torch.nn.functional.scaled_dot_product_attention(tq[None], tk[None, None].expand(1, g_q, n, d),
                                                         tv[None, None].expand(1, g_q, n, d), is_causal=True)
    (o[0] * torch.tensor(d_o)).sum().backward()
    for got, ref in ((dq, tq.grad), (dk, tk.grad), (dv, tv.grad)):
        assert np.allclose(got, ref.numpy(), rtol=0, atol=1e-7 * np.abs(ref.numpy()).max())


def test_structure_of_the_gradients():
    g_q, n, d, block = 2, 64, 8, 8
    q, k, v, d_o = tiny_inputs(4, g_q, n, d, block, spread=3.0)
    prm = orc.DashParams(block=block, alpha=1.5, gamma=2.0)
    kbar = orc.block_mean_summaries(k, block)
    attended = np.zeros(n, bool)
    dk = np.zeros_like(k); dv = np.zeros_like(v); dkbar = np.zeros_like(kbar)
    for t in range(n):
        rr = orc.dash_row_at(q[:, t], k, v, kbar, prm, t)
        for c in rr.routed:
            attended[c * block:(c + 1) * block] = True
        attended[rr.diag[0]:rr.diag[1]] = True
        dq, dx, dd = bwd.backward_row(q[:, t], k, v, kbar, d_o[:, t], prm, t, dk, dv, dkbar)
        if rr.n_cand:
            assert np.abs(dx.sum(axis=1)).max() <= 1e-9 * max(1.0, np.abs(dx).max())
            off = np.setdiff1d(np.arange(rr.n_cand), rr.routed)
            assert np.all(dx[:, off] == 0.0)
    assert attended.all()                      # every key is on its own diagonal
    # a value row only receives gradient from queries that attend it: the last key from one query
    # the last key is attended by the last query only: dV = P do^T summed over its heads
    rr = orc.dash_row_at(q[:, n - 1], k, v, kbar, prm, n - 1)
    tok = np.concatenate([np.arange(c * block, (c + 1) * block) for c in rr.routed] + [np.arange(*rr.diag)])
    dtok = np.concatenate([np.full(block, b) for b in rr.bias] + [np.zeros(rr.diag[1] - rr.diag[0])])
    want = np.zeros(d)
    for h in range(g_q):
        z = k[tok] @ q[h, n - 1] / math.sqrt(d) + dtok
        p_last = np.exp(z[-1] - z.max()) / np.exp(z - z.max()).sum()
        want += p_last * d_o[h, n - 1]
    assert np.allclose(dv[n - 1], want, rtol=1e-12, atol=0)


def test_no_candidates_means_plain_causal_gradients():
    """First-chunk rows route nothing: their backward is that of causal softmax
    attention over the diagonal branch and the summaries get no gradient."""
    g_q, n, d, block = 2, 8, 8, 8
    q, k, v, d_o = tiny_inputs(6, g_q, n, d, block)
    dq, dk, dv, dkbar = bwd.dash_backward_group(q, k, v, d_o, orc.DashParams(block=block))
    assert np.all(dkbar == 0.0)
    tq = torch.tensor(q, requires_grad=True)
    tk = torch.tensor(k, requires_grad=True)
    tv = torch.tensor(v, requires_grad=True)
    o = torch.nn.functional.scaled_dot_product_attention(tq[None], tk[None, None].expand(1, g_q, n, d),
                                                         tv[None, None].expand(1, g_q, n, d), is_causal=True)
    (o[0] * torch.tensor(d_o)).sum().backward()
    for got, ref in ((dq, tq.grad), (dk, tk.grad), (dv, tv.grad)):
        assert np.allclose(got, ref.numpy(), rtol=0, atol=1e-12 * max(1.0, np.abs(ref.numpy()).max()))


@pytest.mark.parametrize("per_chunk", [False, True])
def test_learned_summary_backward_against_finite_differences(per_chunk):
    rng = np.random.default_rng(12)
    n, d, block = 45, 8, 8                    # 5 complete chunks and a tail
    t_c = n // block
    k = rng.standard_normal((n, d))
    qbar = rng.standard_normal((t_c, d) if per_chunk else d) * 2.0
    G = rng.standard_normal((t_c, d))

    def smooth(kk, qq):                        # the summaries without their fp32 rounding
        out = np.empty((t_c, d))
        qb = np.broadcast_to(qq, (t_c, d))
        for c in range(t_c):
            keys = kk[c * block:(c + 1) * block]
            out[c] = scipy_softmax(keys @ qb[c] / math.sqrt(d)) @ keys
        return out

    from scipy.special import softmax as scipy_softmax
    # the smooth form is the oracle's forward up to the rounding of its result
    assert np.allclose(smooth(k, qbar), orc.local_attention_summaries(k[None], qbar, block)[0], rtol=0, atol=1e-6)
    dk, dq = bwd.local_attention_summaries_backward(k, qbar, block, G)
    assert np.all(dk[t_c * block:] == 0.0)     # the incomplete chunk has no summary
    h = 1e-6
    for _ in range(40):
        i, j = int(rng.integers(0, t_c * block)), int(rng.integers(0, d))
        kp, km = k.copy(), k.copy()
        kp[i, j] += h
        km[i, j] -= h
        fd = ((smooth(kp, qbar) - smooth(km, qbar)) * G).sum() / (2 * h)
        assert abs(fd - dk[i, j]) <= 1e-7 * max(1.0, np.abs(dk).max())
    dq_total = dq if per_chunk else dq.sum(axis=0)
    for idx in np.ndindex(*np.shape(qbar)):
        qp, qm = np.array(qbar, dtype=np.float64), np.array(qbar, dtype=np.float64)
        qp[idx] += h
        qm[idx] -= h
        fd = ((smooth(k, qp) - smooth(k, qm)) * G).sum() / (2 * h)
        assert abs(fd - dq_total[idx]) <= 1e-7 * max(1.0, np.abs(dq_total).max())


def test_learned_summary_backward_at_a_zero_query_is_the_block_mean_rule():
    rng = np.random.default_rng(13)
    n, d, block = 32, 8, 8
    k = rng.standard_normal((n, d))
    G = rng.standard_normal((n // block, d))
    dk, dq = bwd.local_attention_summaries_backward(k, np.zeros(d), block, G)
    assert np.allclose(dk, np.repeat(G / block, block, axis=0), rtol=1e-14, atol=0)
    # and the query's gradient is the covariance-like term scale * K^T (a * (da - mean da))
    for c in range(n // block):
        keys = k[c * block:(c + 1) * block]
        da = keys @ G[c]
        assert np.allclose(dq[c], keys.T @ ((da - da.mean()) / block) / math.sqrt(d), rtol=1e-12, atol=1e-15)


def test_noncausal_bias_gradients_of_a_row_sum_to_zero():
    """Non-causal: every attended token lies in a routed chunk, so the bias
    gradients of a row are the sums of all dz of the row, and sum_j dz_j = 0."""
    g_q, n, d, block = 2, 48, 8, 8
    q, k, v, d_o = tiny_inputs(6, g_q, n, d, block, spread=3.0)
    prm = orc.DashParams(block=block, alpha=1.5, gamma=2.0, causal=False)
    kbar = orc.block_mean_summaries(k, block)
    scr = (np.zeros_like(k), np.zeros_like(v), np.zeros_like(kbar))
    for t in (0, 17, n - 1):
        _, _, dd = bwd.backward_row(q[:, t], k, v, kbar, d_o[:, t], prm, t, *scr)
        assert abs(dd.sum()) <= 1e-13 * np.abs(d_o[:, t]).sum() * np.abs(v).max()      # the scale of dP
