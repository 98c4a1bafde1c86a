"""GPU parity of the backward pass (dash_attn_backward through the C ABI) against
the fp64 backward oracle, element by element, on inputs small enough for the
oracle to process every row."""
import numpy as np
import pytest
import torch

import parity_util as U
from oracle import dash_oracle as orc
from oracle import dash_oracle_bwd as bwd
from paper_2605_18753_amd import binding as B
from paper_2605_18753_amd.inputs import Workload, make_inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def gen(w):
    return tuple(t.to(DEV) for t in make_inputs(w, "cpu"))


def run_backward(w, q, k, v, run, d_o):
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    # poison the outputs: every element must be written
    for t in (dq, dk, dv):
        t.fill_(float("nan"))
    ws = B.alloc_backward_workspace(run.params, DEV)
    B.dash_attn_backward(run.params, q, k, v, d_o, run.kbar, run.lists, dq, dk, dv, ws)
    torch.cuda.synchronize()
    return dq, dk, dv


# The comparison, row by row (last axis = head_dim): err = |got - ref| / scale_row with
# scale_row = the row's largest reference magnitude, floored at a tenth of the median over rows
# (near-zero rows are not held to a relative bar).  No allowance of any kind is added.
#   bf16 tensors: every element of dq, dk, dv (dkbar, dqbar) within 2e-2.
#   fp32 tensors: dq (one row = one query, nothing summed over queries): at least 98 % of the rows
#     within 1e-4 (observed: 99.6 % and more for alpha <= 2, 98.9 % at alpha = 3); every element of
#     every tensor (dq and the sums over queries dk, dv, dkbar, dqbar) within 2e-2.  The rows beyond
#     1e-4 are those with a routed chunk at the edge of its support: ln w and 1/w are singular there
#     and fp32 scores resolve the margin x - tau to about 1e-6 only; a sum over queries inherits such
#     a row's error on every key of the chunks that row routes to, so the sums are held to the hard
#     bar only and their distribution is printed.
HARD = 2e-2
F32_ROW, F32_ROW_FRAC = 1e-4, 0.98


def row_errors(got, ref):
    rowmax = np.abs(ref).max(axis=-1, keepdims=True)
    scale = np.maximum(np.maximum(rowmax, 0.1 * np.median(rowmax)), 1e-300)
    return (np.abs(got - ref) / scale).max(axis=-1).reshape(-1)


def rowwise_check(name, got, ref, dtype, per_query):
    """Returns the per-row errors; asserts the bars above."""
    e = row_errors(got, ref)
    msg = (f"{name}: worst {e.max():.2e} median {np.median(e):.2e} p99 {np.quantile(e, 0.99):.2e} "
           f"rows > 1e-4: {(e > F32_ROW).mean():.2e}")
    assert e.max() <= HARD, msg
    if dtype == "fp32" and per_query:
        assert (e <= F32_ROW).mean() >= F32_ROW_FRAC, msg
    return e


def merge(worst, nm, e):
    worst.setdefault(nm, []).append(e)


def fmt(worst):
    out = []
    for nm, es in worst.items():
        e = np.concatenate(es)
        out.append(f"{nm}: worst {e.max():.2e} median {np.median(e):.2e} p99 {np.quantile(e, 0.99):.2e} "
                   f"rows>1e-4 {(e > F32_ROW).mean():.1e}")
    return "; ".join(out)


CASES = [
    # name, batch, h_q, h_kv, n, d, block, extra
    ("gqa2", 1, 4, 2, 512, 128, 64, {}),
    ("mha_needles", 2, 2, 2, 448, 128, 64, {"needles": 2, "offset_sigma": 0.0}),
    ("gqa4_ragged", 1, 4, 1, 600, 128, 64, {"offset_sigma": 0.8}),
    ("gqa8_b128_d64", 1, 8, 1, 768, 64, 128, {"offset_sigma": 0.8}),
    ("gqa16", 1, 16, 1, 384, 128, 64, {"offset_sigma": 0.8}),
    ("alpha2_gamma", 1, 4, 2, 512, 128, 64, {"alpha": 2.0, "gamma": 1.5}),
    ("alpha125_sigma", 1, 4, 2, 512, 128, 64, {"alpha": 1.25, "sigma": 2.0, "offset_sigma": 1.0}),
    ("window1", 1, 4, 2, 512, 128, 64, {"window": 1, "offset_sigma": 0.8}),
    ("noncausal", 1, 4, 2, 512, 128, 64, {"causal": False, "offset_sigma": 0.8}),
    ("one_chunk", 1, 4, 2, 50, 128, 64, {}),
    ("sparse_gamma3", 1, 4, 2, 512, 128, 64, {"gamma": 3.0, "offset_sigma": 1.0}),
    ("strong_prior_sigma03", 1, 4, 2, 512, 128, 64, {"sigma": 0.3, "offset_sigma": 0.8}),
    ("mha_d64_b64", 1, 2, 2, 320, 64, 64, {"offset_sigma": 0.8}),
    # p = 1/(alpha-1) < 1: the entmax slope p u^(p-1) is unbounded at the edge of the support
    ("alpha3", 1, 4, 2, 512, 128, 64, {"alpha": 3.0, "offset_sigma": 0.8}),
    ("alpha105", 1, 4, 2, 512, 128, 64, {"alpha": 1.05, "offset_sigma": 0.8}),
    ("window2_b128", 1, 4, 2, 768, 128, 128, {"window": 2, "offset_sigma": 0.8}),
    # degenerate lengths: a single token, exactly one chunk, one chunk plus one token
    ("one_token", 2, 4, 2, 1, 128, 64, {}),
    ("exactly_one_chunk", 1, 4, 2, 64, 128, 64, {}),
    ("one_chunk_plus_one", 1, 4, 2, 65, 128, 64, {}),
    # fp32 tensors (the plain VALU kernels; the routing kernel is the one the bf16 path uses):
    # the same chain at a tolerance 200 times tighter, every group size of the routing kernel
    ("f32_gqa2", 1, 4, 2, 512, 128, 64, {"dtype": "fp32"}),
    ("f32_mha_needles", 2, 2, 2, 448, 128, 64, {"dtype": "fp32", "needles": 2, "offset_sigma": 0.0}),
    ("f32_gqa4_ragged", 1, 4, 1, 600, 128, 64, {"dtype": "fp32", "offset_sigma": 0.8}),
    ("f32_gqa8_b128_d64", 1, 8, 1, 768, 64, 128, {"dtype": "fp32", "offset_sigma": 0.8}),
    ("f32_gqa16", 1, 16, 1, 384, 128, 64, {"dtype": "fp32", "offset_sigma": 0.8}),
    ("f32_alpha2_window1", 1, 4, 2, 512, 128, 64, {"dtype": "fp32", "alpha": 2.0, "gamma": 1.5, "window": 1}),
    ("f32_alpha125_sigma", 1, 4, 2, 512, 128, 64, {"dtype": "fp32", "alpha": 1.25, "sigma": 2.0, "offset_sigma": 1.0}),
    ("f32_noncausal", 1, 4, 2, 512, 128, 64, {"dtype": "fp32", "causal": False, "offset_sigma": 0.8}),
    ("f32_mha_d64_b64", 1, 2, 2, 320, 64, 64, {"dtype": "fp32", "offset_sigma": 0.8}),
    # the shape of the fp32 single-head non-causal configuration
    ("f32_single_head_1024", 1, 1, 1, 1024, 64, 64, {"dtype": "fp32", "causal": False, "offset_sigma": 0.5}),
    ("f32_window2_b128", 1, 4, 2, 768, 128, 128, {"dtype": "fp32", "window": 2, "offset_sigma": 0.8}),
    ("f32_sparse_gamma3_sigma03", 1, 4, 2, 512, 128, 64, {"dtype": "fp32", "gamma": 3.0, "sigma": 0.3, "offset_sigma": 1.0}),
    ("f32_alpha3", 1, 4, 2, 512, 128, 64, {"dtype": "fp32", "alpha": 3.0, "offset_sigma": 0.8}),
    ("f32_alpha105", 1, 4, 2, 512, 128, 64, {"dtype": "fp32", "alpha": 1.05, "offset_sigma": 0.8}),
    ("f32_one_token", 2, 4, 2, 1, 128, 64, {"dtype": "fp32"}),
    ("f32_one_chunk_plus_one", 1, 4, 2, 65, 128, 64, {"dtype": "fp32"}),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_backward_matches_the_oracle(case):
    name, batch, h_q, h_kv, n, d, block, extra = case
    w = Workload(name, batch, h_q, h_kv, n, n, d, block, seed=17, **extra)
    q, k, v = gen(w)
    gen_do = torch.Generator().manual_seed(99)
    d_o = torch.randn(q.shape, generator=gen_do).to(w.torch_dtype).to(DEV)
    run = U.run_prefill(w, q, k, v)
    dq, dk, dv = run_backward(w, q, k, v, run, d_o)
    for t in (dq, dk, dv):
        assert torch.isfinite(t.float()).all(), "an output element was not written or is not finite"

    prm = U.oracle_params(w)
    g = w.g_q
    qn, kn, vn, don = U.to_np(q).astype(np.float64), U.to_np(k).astype(np.float64), \
        U.to_np(v).astype(np.float64), U.to_np(d_o).astype(np.float64)
    t_all = B.list_stride(run.params)
    worst = {}
    for b in range(batch):
        for r in range(h_kv):
            # the comparison presumes the same support on both sides
            kbar = orc.block_mean_summaries(kn[b, r], block)
            mism = 0
            xmax = 1.0
            for i in range(n):
                rr = orc.dash_row_at(qn[b, r * g:(r + 1) * g, i], kn[b, r], vn[b, r], kbar, prm, i)
                bits = U.mask_bits(run.lists.mask[b, r, i].cpu().numpy(), t_all)
                got = set(np.nonzero(bits[:rr.n_cand])[0].tolist())
                mism += got != set(rr.routed.tolist())
                if rr.n_cand:
                    xmax = max(xmax, float(np.abs(rr.x).max()))
            # gradients are compared inside one support (a precondition of the comparison, not of the
            # kernel: the forward tests cover the band around the threshold)
            assert mism == 0, f"{mism} rows route differently on the two sides"
            sl = slice(r * g, (r + 1) * g)
            ref = bwd.dash_backward_group(qn[b, sl], kn[b, r], vn[b, r], don[b, sl], prm)
            for nm, got, j in (("dq", U.to_np(dq[b, sl]), 0), ("dk", U.to_np(dk[b, r]), 1),
                               ("dv", U.to_np(dv[b, r]), 2)):
                merge(worst, nm, rowwise_check(f"{name} {nm}[{b},{r}]", got.astype(np.float64), ref[j], w.dtype, j == 0))
            if n >= 2 * block:
                # the path through the routing scores into the block means must be a visible part
                # of dk, or the comparison above would not notice its absence
                direct = bwd.dash_backward_group(qn[b, sl], kn[b, r], vn[b, r], don[b, sl], prm, kbar=kbar)[1]
                rowmax = np.abs(ref[1]).max(axis=-1)
                share = np.abs(ref[1] - direct).max(axis=-1) / np.maximum(rowmax, 0.1 * np.median(rowmax))
                assert share.max() > 0.05, share.max()
    print(f"{name}: {fmt(worst)}")


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_backward_token_major_layout_and_workspace_reuse(dtype):
    """q, k, v, dO and the gradients in [batch, token, head, d] storage (head stride d,
    token stride heads*d), and a second call on the same workspace with other
    inputs: the results must equal those of contiguous tensors / a fresh workspace
    (bf16: bit for bit; fp32: the atomic sums of dk, dv and dd have no fixed order)."""
    w = Workload("bwd_layout", 2, 8, 2, 640, 640, 128, 64, seed=23, offset_sigma=0.8, dtype=dtype)
    q, k, v = gen(w)
    d_o = torch.randn(q.shape, generator=torch.Generator().manual_seed(5)).to(w.torch_dtype).to(DEV)
    run = U.run_prefill(w, q, k, v)
    ref = run_backward(w, q, k, v, run, d_o)

    def same(got, want):
        if dtype == "bf16":
            return torch.equal(got, want)
        # a wrong stride would be an O(1) error; the order of the sums moves rows near a threshold by up to ~1e-4
        return bool(((got - want).abs() <= 1e-3 * want.abs().amax(dim=-1, keepdim=True) + 1e-6).all())

    def token_major(t):
        return t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)      # same values, [b, n, h, d] storage

    qt, kt, vt, dot = (token_major(t) for t in (q, k, v, d_o))
    ot = token_major(torch.empty_like(q))
    p = B.make_params(qt, kt, vt, ot, w.block, w.alpha, w.gamma, w.sigma, w.causal)
    assert p.q_stride[1] == w.head_dim and p.q_stride[2] == w.h_q * w.head_dim
    dq, dk, dv = (token_major(torch.full_like(t, float("nan"))) for t in (q, k, v))
    ws = B.alloc_backward_workspace(p, DEV)
    B.dash_attn_backward(p, qt, kt, vt, dot, run.kbar, run.lists, dq, dk, dv, ws)
    torch.cuda.synchronize()
    for got, want in zip((dq, dk, dv), ref):
        assert same(got, want)

    # other inputs through the same workspace (the column masks of the first call must not leak)
    w2 = w.replace(seed=24, gamma=2.0)
    q2, k2, v2 = gen(w2)
    run2 = U.run_prefill(w2, q2, k2, v2)
    ref2 = run_backward(w2, q2, k2, v2, run2, d_o)
    dq2, dk2, dv2 = torch.empty_like(q2), torch.empty_like(k2), torch.empty_like(v2)
    B.dash_attn_backward(run2.params, q2, k2, v2, d_o, run2.kbar, run2.lists, dq2, dk2, dv2, ws)
    torch.cuda.synchronize()
    for got, want in zip((dq2, dk2, dv2), ref2):
        assert same(got, want)


@pytest.mark.parametrize("which", ["C5", "C2", "C4"])
def test_backward_at_the_benchmark_shape_on_sampled_rows(which):
    """The training-shaped workload in the launch configuration bench.py times (and the
    32k GQA prefill and the 128k / chunk-128 shapes): dq of sampled query rows and dk, dv of the keys of the last
    chunk (which only the rows of that chunk attend) against the oracle."""
    from paper_2605_18753_amd.inputs import NAMED
    w = NAMED[which]
    q, k, v = make_inputs(w, DEV)
    d_o = torch.randn(q.shape, device=DEV, dtype=torch.float32).to(torch.bfloat16)
    run = U.run_prefill(w, q, k, v, want_idx=False)
    dq, dk, dv = run_backward(w, q, k, v, run, d_o)
    prm = U.oracle_params(w)
    g, n, blk = w.g_q, w.n_q, w.block
    t_all = B.list_stride(run.params)
    rng = np.random.default_rng(1)
    checked = skipped = 0
    worst = {}
    # the 128k shape costs the oracle about 0.1 s per row: one kv-head and sampled rows only there
    light = w.n_q > 65536
    groups = ((0, 3),) if light else ((0, 0), (w.batch - 1, w.h_kv - 1), (w.batch // 2, w.h_kv // 2))
    for b, r in groups:
        kn, vn = U.to_np(k[b, r]).astype(np.float64), U.to_np(v[b, r]).astype(np.float64)
        kbar = orc.block_mean_summaries(kn, blk)
        sl = slice(r * g, (r + 1) * g)
        rows = sorted(set(rng.integers(0, n, 24).tolist()) | set(range(n - 4, n))) if light else \
            sorted(set(rng.integers(0, n, 10).tolist()) | set(range(n - blk, n)))
        tail_ok = not light
        dk_ref, dv_ref, dkb = np.zeros_like(kn), np.zeros_like(vn), np.zeros_like(kbar)
        scratch = (np.zeros_like(kn), np.zeros_like(vn), np.zeros_like(kbar))    # sums nobody reads
        gots, refs = [], []
        for i in rows:
            qh = U.to_np(q[b, sl, i]).astype(np.float64)
            doh = U.to_np(d_o[b, sl, i]).astype(np.float64)
            rr = orc.dash_row_at(qh, kn, vn, kbar, prm, i)
            bits = U.mask_bits(run.lists.mask[b, r, i].cpu().numpy(), t_all)
            same = set(np.nonzero(bits[:rr.n_cand])[0].tolist()) == set(rr.routed.tolist())
            scr_k, scr_v, scr_b = (dk_ref, dv_ref, dkb) if i >= n - blk else scratch
            ref_dq, _, _ = bwd.backward_row(qh, kn, vn, kbar, doh, prm, i, scr_k, scr_v, scr_b)
            if not same:
                skipped += 1
                tail_ok = tail_ok and i < n - blk
                continue
            gots.append(U.to_np(dq[b, sl, i]).astype(np.float64))
            refs.append(ref_dq)
            checked += 1
        merge(worst, "dq", rowwise_check(f"dq[{b},{r}]", np.stack(gots), np.stack(refs), "bf16", True))
        if tail_ok:
            # keys of the last (complete) chunk: no later row routes to it, so these sums are complete
            last = slice(n - blk, n)
            for nm, got, ref in (("dk", dk, dk_ref), ("dv", dv, dv_ref)):
                merge(worst, nm, rowwise_check(f"{nm}[{b},{r},last chunk]", U.to_np(got[b, r, last]).astype(np.float64),
                                               ref[last], "bf16", False))
    assert checked >= (20 if light else 150) and skipped <= 6, (checked, skipped)
    print(f"benchmark shape: {checked} rows checked, {skipped} skipped (support at the band); {fmt(worst)}")


@pytest.mark.parametrize("per_chunk,dtype", [(False, "bf16"), (True, "bf16"), (False, "fp32"), (True, "fp32")],
                         ids=["query_per_head", "query_per_chunk", "f32_query_per_head", "f32_query_per_chunk"])
def test_backward_through_learned_summaries(per_chunk, dtype):
    """The trainable Stage 0: forward with dash_kbar_summarize, backward with the
    summaries as an input of their own (dkbar output), then
    dash_kbar_summarize_backward down to the keys and the summary query."""
    w = Workload("bwd_learned", 1, 4, 2, 512, 512, 128, 64, seed=29, offset_sigma=0.8, dtype=dtype)
    q, k, v = gen(w)
    t_c = w.n_kv // w.block
    gq = torch.Generator().manual_seed(3)
    qbar = (torch.randn((w.h_kv, t_c, w.head_dim) if per_chunk else (w.h_kv, w.head_dim), generator=gq) * 0.7).to(DEV)
    d_o = torch.randn(q.shape, generator=torch.Generator().manual_seed(7)).to(w.torch_dtype).to(DEV)
    run = U.run_prefill_learned(w, q, k, v, qbar)
    dq, dk, dv = (torch.full_like(t, float("nan")) for t in (q, k, v))
    dkbar = torch.full_like(run.kbar, float("nan"))
    dqbar = torch.full_like(run.kbar, float("nan"))
    ws = B.alloc_backward_workspace(run.params, DEV)
    B.dash_attn_backward(run.params, q, k, v, d_o, run.kbar, run.lists, dq, dk, dv, ws, dkbar=dkbar)
    B.dash_kbar_summarize_backward(run.params, k, qbar, dkbar, dk, dqbar)
    torch.cuda.synchronize()
    for t in (dq, dk, dv, dkbar, dqbar):
        assert torch.isfinite(t.float()).all()

    prm = U.oracle_params(w)
    g, n, blk = w.g_q, w.n_q, w.block
    qn, kn, vn, don = (U.to_np(t).astype(np.float64) for t in (q, k, v, d_o))
    qbn = U.to_np(qbar).astype(np.float64)
    t_all = B.list_stride(run.params)
    for r in range(w.h_kv):
        kbar_ref = orc.local_attention_summaries(kn[0, r][None], qbn[r], blk)[0]
        for i in range(n):
            rr = orc.dash_row_at(qn[0, r * g:(r + 1) * g, i], kn[0, r], vn[0, r], kbar_ref, prm, i)
            bits = U.mask_bits(run.lists.mask[0, r, i].cpu().numpy(), t_all)
            assert set(np.nonzero(bits[:rr.n_cand])[0].tolist()) == set(rr.routed.tolist()), "the two sides route differently"
        sl = slice(r * g, (r + 1) * g)
        def through_stage0(grads):
            rq, rk, rv, rkb = grads
            sk, sq = bwd.local_attention_summaries_backward(kn[0, r], qbn[r], blk, rkb)
            return (rq, rk + sk, rv, rkb, sq)

        ref = through_stage0(bwd.dash_backward_group(qn[0, sl], kn[0, r], vn[0, r], don[0, sl], prm, kbar=kbar_ref))
        got = (U.to_np(dq[0, sl]), U.to_np(dk[0, r]), U.to_np(dv[0, r]), U.to_np(dkbar[0, r]), U.to_np(dqbar[0, r]))
        worst = {}
        for j, nm in enumerate(("dq", "dk", "dv", "dkbar", "dqbar")):
            merge(worst, nm, rowwise_check(f"learned {nm}[{r}]", got[j].astype(np.float64), ref[j], dtype, j == 0))
        if not per_chunk:
            # one query per kv-head: its gradient is the sum over the chunks
            tot_ref, tot_got = ref[4].sum(axis=0), got[4].astype(np.float64).sum(axis=0)
            assert np.abs(tot_got - tot_ref).max() <= HARD * np.abs(tot_ref).max()
        # the summary path must be a visible part of dk
        share = np.abs(ref[1] - bwd.dash_backward_group(qn[0, sl], kn[0, r], vn[0, r], don[0, sl], prm,
                                                            kbar=kbar_ref)[1]).max() / np.abs(ref[1]).max()
        assert share > 0.02, share
        print(f"learned summaries, kv-head {r}: {fmt(worst)}")


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_forward_and_backward_replay_from_a_captured_graph(dtype):
    """Neither call allocates, synchronises or clears memory with a memset node, so a
    training step can be captured once and replayed: three replays with new inputs in
    the same buffers, eager work in between, each equal to the eager results (fp32
    tensors: the forward bit for bit, the gradients up to the order of their atomic sums)."""
    w = Workload("train_graph", 2, 8, 2, 700, 700, 128, 64, seed=19, offset_sigma=0.8, dtype=dtype)
    q, k, v = gen(w)
    d_o = torch.randn(q.shape, generator=torch.Generator().manual_seed(2)).to(w.torch_dtype).to(DEV)
    o = torch.empty_like(q)
    p = B.make_params(q, k, v, o, w.block, w.alpha, w.gamma, w.sigma, w.causal)
    kbar = torch.empty(B.kbar_shape(p), dtype=torch.float32, device=DEV)
    lists = B.Lists.allocate(p, DEV)
    ws, wsb = B.alloc_workspace(p, DEV), B.alloc_backward_workspace(p, DEV)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)

    def step():
        B.dash_attn_prefill(p, q, k, v, o, kbar, lists, ws)
        B.dash_attn_backward(p, q, k, v, d_o, kbar, lists, dq, dk, dv, wsb)

    def same(got, want, exact):
        if exact:
            return torch.equal(got, want)
        return bool(((got - want).abs() <= 1e-3 * want.abs().amax(dim=-1, keepdim=True) + 1e-6).all())

    step()                                                     # warm-up outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    gen_x = torch.Generator(device=DEV).manual_seed(5)
    for rep in range(3):
        for t in (q, d_o):
            t.copy_(torch.randn(t.shape, generator=gen_x, device=DEV).to(t.dtype))
        for t in (o, dq, dk, dv):
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (o, dq, dk, dv)]
        for t in (o, dq, dk, dv):
            t.zero_()
        step()                                                 # eager, same inputs
        torch.cuda.synchronize()
        for j, (a_, b_) in enumerate(zip(got, (o, dq, dk, dv))):
            assert same(a_, b_, dtype == "bf16" or j == 0), (rep, j)
        assert dq.float().abs().max() > 0 and torch.isfinite(dk.float()).all()
