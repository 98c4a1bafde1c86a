"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI
binding, run the oracle on the same bits, compare by the build's parity rules.

Support rule: the GPU's attended-chunk set of a (batch, kv-head, query) row must
equal the oracle's, except for chunks within 1e-6 of the entmax threshold: a
chunk is exempt if, in the oracle, no head of the group has margin
x - tau > 1e-6 and at least one head has |x - tau| <= 1e-6.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Iterable, List, Optional, Sequence, Tuple

import numpy as np
import torch

from oracle import dash_oracle as orc
from paper_2605_18753_amd import binding as B
from paper_2605_18753_amd.inputs import Workload, make_inputs

BAND = 1e-6


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


@dataclass
class HipRun:
    o: torch.Tensor
    kbar: torch.Tensor
    lists: B.Lists
    params: B.dash_params


def run_prefill(w: Workload, q, k, v, *, want_idx=True) -> HipRun:
    dev = q.device
    o = torch.empty_like(q)
    p = B.make_params(q, k, v, o, w.block, w.alpha, w.gamma, w.sigma, w.causal, window=w.window)
    kbar = torch.empty(B.kbar_shape(p), dtype=torch.float32, device=dev)
    lists = B.Lists.allocate(p, dev, idx=want_idx)
    ws = B.alloc_workspace(p, dev)
    B.dash_attn_prefill(p, q, k, v, o, kbar, lists, ws)
    torch.cuda.synchronize()
    return HipRun(o, kbar, lists, p)


def run_prefill_learned(w: Workload, q, k, v, qbar: torch.Tensor) -> HipRun:
    """The path with the learned Stage 0: summaries from dash_kbar_summarize, then
    the Stage-1 and Stage-2 entry points."""
    dev = q.device
    o = torch.empty_like(q)
    p = B.make_params(q, k, v, o, w.block, w.alpha, w.gamma, w.sigma, w.causal, window=w.window)
    kbar = torch.empty(B.kbar_shape(p), dtype=torch.float32, device=dev)
    lists = B.Lists.allocate(p, dev)
    ws = B.alloc_workspace(p, dev)
    B.dash_kbar_summarize(p, k, qbar, kbar)
    B.dash_stage1_route(p, q, kbar, lists, ws)
    B.dash_stage2_attend(p, q, k, v, o, lists, ws)
    torch.cuda.synchronize()
    return HipRun(o, kbar, lists, p)


def ulp_diff(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Distance in units of the last place between two fp32 arrays (finite values)."""
    def key(x):
        i = np.ascontiguousarray(x, dtype=np.float32).view(np.int32).astype(np.int64)
        return np.where(i < 0, -(i & 0x7FFFFFFF), i)
    return np.abs(key(a) - key(b))


def run_decode(w: Workload, q, k, v, kbar: Optional[torch.Tensor] = None) -> HipRun:
    dev = q.device
    o = torch.empty_like(q)
    p = B.make_params(q, k, v, o, w.block, w.alpha, w.gamma, w.sigma, True, window=w.window)
    if kbar is None:
        kbar = torch.empty(B.kbar_shape(p), dtype=torch.float32, device=dev)
        B.dash_kbar_compress(p, k, kbar)
    lists = B.Lists.allocate(p, dev)
    ws = B.alloc_workspace(p, dev)
    B.dash_attn_decode(p, q, k, v, kbar, o, lists, ws)
    torch.cuda.synchronize()
    return HipRun(o, kbar, lists, p)


def oracle_params(w: Workload) -> orc.DashParams:
    return orc.DashParams(block=w.block, alpha=w.alpha, gamma=w.gamma, sigma=w.sigma, causal=w.causal,
                          window=w.window)


@dataclass
class SupportReport:
    rows: int = 0
    blocks: int = 0          # candidate chunks examined
    kept: int = 0            # chunks the oracle routes
    exempt: int = 0
    mismatched: int = 0
    exempt_rows: set = field(default_factory=set)
    worst_bias_err: float = 0.0
    worst_tau_err: float = 0.0
    # output error: tensor-relative (the metric of the stated tolerance) and per row relative to
    # the row's own largest magnitude (median / 99th percentile / max over the compared rows)
    err_plain: float = 0.0           # worst tensor-relative row error (no allowance exists)
    row_rel_median: float = 0.0
    row_rel_p99: float = 0.0
    row_rel_max: float = 0.0

    @property
    def sparsity(self) -> float:
        return 1.0 - self.kept / max(1, self.blocks)

    def errors(self) -> str:
        return (f"out_err {self.err_plain:.2e} "
                f"per-row rel median {self.row_rel_median:.2e} p99 {self.row_rel_p99:.2e} max {self.row_rel_max:.2e}")


def mask_bits(words: np.ndarray, n_bits: int) -> np.ndarray:
    w = words.astype(np.uint32)
    bits = ((w[:, None] >> np.arange(32, dtype=np.uint32)[None, :]) & 1).astype(bool).reshape(-1)
    return bits[:n_bits]


def lnw_error_bound(rr: orc.RowResult, alpha: float) -> np.ndarray:
    """Per candidate chunk, a bound on the fp32 error of ln w, where
    w = mean_h [x_h - tau_h]_+^p and p = 1/(alpha-1) (Eq. 4 with the group mean
    of Sec. 3.3).  An fp32 error eps ~ 1e-6 (generous) in each head's margin
    u_h = x_h - tau_h moves ln w by eps * sum_h p u_h^(p-1) / sum_h u_h^p.  For
    p >= 1 the largest margin dominates (about p eps / u_max); for p < 1 a head
    that keeps the chunk by a hair contributes the most."""
    p = 1.0 / (alpha - 1.0)
    u = np.maximum(rr.x - rr.tau[:, None], 0.0)               # [g_q, n_cand]
    pos = u > 0
    uf = np.where(pos, np.maximum(u, 1e-9), 1.0)
    num = np.where(pos, p * uf ** (p - 1.0), 0.0).sum(axis=0)
    den = np.where(pos, uf ** p, 0.0).sum(axis=0)
    return 1e-6 * num / np.maximum(den, 1e-300)


def mu_error_bound(rr: orc.RowResult, alpha: float) -> float:
    """Bound on the fp32 error of mu = mean_R ln w: the mean of the routed
    chunks' ln w bounds."""
    if rr.routed.size == 0:
        return 0.0
    return float(np.mean(lnw_error_bound(rr, alpha)[rr.routed]))


def compare_row(rr: orc.RowResult, w: Workload, mask_words: np.ndarray, cnt: int,
                idx: Optional[np.ndarray], bias: np.ndarray, tau: Optional[np.ndarray],
                rep: SupportReport, t_all: int) -> None:
    """Checks one row's support, list structure, bias and tau against the oracle."""
    rep.rows += 1
    bits = mask_bits(mask_words, t_all)
    gpu_set = set(np.nonzero(bits)[0].tolist())
    ref_set = set(rr.routed.tolist())
    diag_chunk = None
    local: List[int] = []            # always-attended chunks: the window, then the diagonal chunk
    if w.causal:
        diag_chunk = rr.pos // w.block
        local = list(range(rr.n_cand, diag_chunk + 1))
        assert len(local) == min(w.window, diag_chunk) + 1
        for c in local:
            assert c in gpu_set, f"row {rr.b,rr.r,rr.iq}: local chunk {c} missing"
            gpu_set.discard(c)
    assert all(c < rr.n_cand for c in gpu_set), f"row {rr.b,rr.r,rr.iq}: non-candidate chunk attended"
    rep.blocks += rr.n_cand
    rep.kept += len(ref_set)
    if rr.n_cand:
        margin = rr.x - rr.tau[:, None]                       # [g_q, n_cand]
        exempt = (~(margin > BAND).any(axis=0)) & (np.abs(margin) <= BAND).any(axis=0)
    else:
        exempt = np.zeros(0, bool)
    diff = gpu_set ^ ref_set
    for c in diff:
        if exempt[c]:
            rep.exempt += 1
            rep.exempt_rows.add((rr.b, rr.r, rr.iq))
        else:
            rep.mismatched += 1
    # list structure: count, ascending ids, diagonal last, agreement with the mask
    n_expected = len(gpu_set) + len(local)
    assert cnt == n_expected, f"row {rr.b,rr.r,rr.iq}: cnt {cnt} != popcount {n_expected}"
    if idx is not None:
        ids = idx[:cnt].tolist()
        want = sorted(gpu_set) + local
        assert ids == want, f"row {rr.b,rr.r,rr.iq}: idx list {ids[:8]}.. != mask order"
    for j in range(len(local)):
        assert bias[cnt - 1 - j] == 0.0
    # bias of the chunks both sides keep (skip rows whose support differs: mu shifts)
    if not diff and len(ref_set):
        order = sorted(gpu_set)
        ref_bias = dict(zip(rr.routed.tolist(), rr.bias.tolist()))
        lnw_slack = lnw_error_bound(rr, w.alpha)
        mu_slack = mu_error_bound(rr, w.alpha)
        for j, c in enumerate(order):
            tol = (2e-4 + lnw_slack[c] + mu_slack) / w.sigma + 1e-6 * abs(ref_bias[c])
            err = abs(bias[j] - ref_bias[c])
            rep.worst_bias_err = max(rep.worst_bias_err, err * w.sigma)
            assert err <= tol, f"row {rr.b,rr.r,rr.iq} chunk {c}: bias {bias[j]} vs {ref_bias[c]}"
    if tau is not None and rr.n_cand:
        err = float(np.abs(tau - rr.tau).max())
        rep.worst_tau_err = max(rep.worst_tau_err, err)
        # fp32 scores and thresholds: a few ulp of the largest magnitude in the row
        assert err <= 2e-6 * max(1.0, float(np.abs(rr.x).max())), f"row {rr.b,rr.r,rr.iq}: tau {tau} vs {rr.tau}"


def check_against_oracle(w: Workload, q, k, v, run: HipRun,
                         rows: Optional[Sequence[Tuple[int, int, int]]] = None,
                         out_tol: Optional[float] = None, max_exempt_frac: float = 1e-3,
                         summaries=None):
    """Element-wise comparison on `rows` (default: all).  Tensors may live on the
    GPU; only the (batch, kv-head) slices that `rows` touch are copied to the host.
    `summaries(b, r, keys)` gives the oracle's Stage-0 result for one (batch, kv-head)
    pair when it is not the block mean; the GPU's must then agree to 1 ulp of fp32
    everywhere and bit for bit on all but 1e-4 of the elements (both sides round an
    fp64 evaluation once).  Returns (report, worst relative output error)."""
    prm = oracle_params(w)
    if rows is None:
        rows = [(b, r, i) for b in range(w.batch) for r in range(w.h_kv) for i in range(w.n_q)]
    rows = sorted(rows)
    g = w.g_q
    t_all = B.list_stride(run.params)
    pos0 = w.n_kv - w.n_q
    rep = SupportReport()
    o_ref = np.zeros((len(rows), g, w.head_dim))
    o_got = np.zeros_like(o_ref)
    cur = None
    for n, (b, r, i) in enumerate(rows):
        if cur != (b, r):
            cur = (b, r)
            kn, vn = to_np(k[b, r]), to_np(v[b, r])
            kbar_ref = summaries(b, r, kn) if summaries else orc.block_mean_summaries(kn, w.block)
            if kbar_ref.shape[0]:
                kbar_gpu = run.kbar[b, r].cpu().numpy()
                assert kbar_gpu.dtype == np.float32
                if summaries:
                    ud = ulp_diff(kbar_gpu, kbar_ref.astype(np.float32))
                    assert ud.max() <= 1 and (ud > 0).mean() <= 1e-4, "learned kbar off"
                else:
                    assert np.array_equal(kbar_gpu, kbar_ref.astype(np.float32)), "kbar not bit-exact"
        qh = to_np(q[b, r * g:(r + 1) * g, i])
        rr = orc.dash_row_at(qh, kn, vn, kbar_ref, prm, pos0 + i, (b, r, i))
        L = run.lists
        compare_row(rr, w, L.mask[b, r, i].cpu().numpy(), int(L.cnt[b, r, i]),
                    L.idx[b, r, i].cpu().numpy() if L.idx is not None else None,
                    L.bias[b, r, i].cpu().numpy(),
                    L.tau[b, r * g:(r + 1) * g, i].cpu().numpy() if L.tau is not None else None, rep, t_all)
        o_ref[n] = rr.o
        o_got[n] = to_np(run.o[b, r * g:(r + 1) * g, i]).astype(np.float64)
    assert rep.mismatched == 0, f"{rep.mismatched} support mismatches outside the 1e-6 band"
    assert rep.exempt <= max(2, max_exempt_frac * rep.blocks), f"too many exempt chunks: {rep.exempt}"
    tol = out_tol if out_tol is not None else (2e-2 if w.dtype == "bf16" else 1e-5)
    # a flipped near-threshold chunk changes the output discontinuously only when
    # the prior is weak (large sigma); such rows are left out and counted
    keep = np.ones(len(rows), bool)
    if w.sigma > 1.0:
        for n, row in enumerate(rows):
            if row in rep.exempt_rows:
                keep[n] = False
    denom = np.abs(o_ref).max()
    row_abs = np.abs(o_got - o_ref).max(axis=(1, 2))
    row_err = row_abs / denom
    bad = keep & (row_err > tol)
    assert not bad.any(), (f"output error {row_err[bad].max():.3e} > {tol} on {int(bad.sum())} rows, "
                           f"first {rows[int(np.nonzero(bad)[0][0])]}")
    if keep.any():
        rep.err_plain = float(row_err[keep].max())
        rel = (row_abs / np.maximum(np.abs(o_ref).max(axis=(1, 2)), 1e-300))[keep]
        rep.row_rel_median, rep.row_rel_p99, rep.row_rel_max = (float(np.median(rel)), float(np.quantile(rel, 0.99)),
                                                                 float(rel.max()))
    return rep, rep.err_plain


def sample_rows(w: Workload, n_rows: int, seed: int = 0, heads: Optional[Sequence[Tuple[int, int]]] = None):
    """Uniform sample of query rows plus the first and last rows of the sequence
    and the rows around a chunk boundary, for a few (batch, kv-head) pairs."""
    rng = np.random.default_rng(seed)
    if heads is None:
        heads = [(0, 0), (w.batch - 1, w.h_kv - 1)]
    heads = sorted(set(heads))
    rows = set()
    per = max(1, n_rows // len(heads))
    for (b, r) in heads:
        fixed = [0, 1, w.block - 1, w.block, w.n_q - 1, w.n_q - 2, w.n_q // 2]
        for i in fixed:
            if 0 <= i < w.n_q:
                rows.add((b, r, int(i)))
        for i in rng.integers(0, w.n_q, size=per):
            rows.add((b, r, int(i)))
    return sorted(rows)
