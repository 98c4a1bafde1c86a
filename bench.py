#!/usr/bin/env python3
"""Benchmark of the DashAttention forward hot path on one MI355X.

A step is one pass of the whole prefill path (Stage 0 block means -> Stage 1
entmax routing -> Stage 2 block-sparse attention) over the causal GQA prefill
workload (B=1, H_q=32, H_kv=8, N=32768, d=128, block 64, alpha=1.5, bf16),
inputs resident in HBM.  Prints ONE JSON line.

  value      dense-equivalent causal attention flops / step time (TFLOP/s)
  roofline   Stage-2 kernel: algorithmic flops (exact per-token sparsity) per
             launch / its average duration, against the bf16 MFMA peak
  extras     stage times, speed-up over the in-library dense kernel at the
             config's gamma and at the gamma that gives ~75 % chunk sparsity,
             MFMA flops actually issued, decode step time and HBM rate
  cpu_baseline  the fp64 oracle timed on a bounded row sample
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0
HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the Stage-2 kernel on the full C2 workload, from the two
# rocprofv3 --pmc runs summarised in profiles/bench_c2_c3_hbm_traffic.md
# (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0).  Not measurable from inside this script.
S2_TRAFFIC_BYTES_C2 = 2.539e9 + 0.388e9


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-backward", action="store_true")
    ap.add_argument("--backward-only", action="store_true",
                    help="time only the forward + backward of the training-shaped workload and print its JSON line "
                         "(the command of the backward kernels' rocprofv3 summaries)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--small", action="store_true", help="shrunken shapes (debugging)")
    ap.add_argument("--paper-protocol", action="store_true",
                    help="run the kernel-benchmark protocol of the paper instead (H_q=32, H_kv=2, d=128, chunk 64, "
                         "N in 16K..96K, Stage-2 mask randomised to 75 / 87.5 / 93.75 % sparsity, speed-up over the "
                         "in-library dense kernel; prefill batch 1, decode batch 24) and print its JSON line")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 1 GiB device copy three times (known traffic, to scale the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    return ap.parse_args()


def timed(fn, steps, warmup, torch):
    """Average ms per call over `steps` calls, HIP events on the current stream."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def popcount32(x, torch):
    x = x.to(torch.int64) & 0xFFFFFFFF
    x = x - ((x >> 1) & 0x55555555)
    x = (x & 0x33333333) + ((x >> 2) & 0x33333333)
    x = (x + (x >> 4)) & 0x0F0F0F0F
    return ((x * 0x01010101) & 0xFFFFFFFF) >> 24


def prefill_stats(w, lists, torch):
    """Flop counts from the Stage-1 outputs (reporting only).

    f_alg  : 4 d per attended key and query head (exact per-token sparsity)
    f_exec : flops of the MFMA tiles Stage 2 issues: a wave owns 32 rows (all
             heads of 32/g_q tokens) and computes every chunk one of them kept
    f_dense: causal dense attention
    """
    d, g, blk, n = w.head_dim, w.g_q, w.block, w.n_q
    cnt = lists.cnt.to(torch.int64)                               # [B,Hkv,N] incl. diagonal
    pos = torch.arange(n, device=cnt.device, dtype=torch.int64)
    diag_keys = (pos % blk) + 1
    keys = (cnt - 1) * blk + diag_keys                            # routed chunks are complete
    f_alg = 4.0 * d * g * float(keys.sum())
    tokw = 32 // g
    m = lists.mask                                                # [B,Hkv,N,W] int32
    B_, H_, N_, W_ = m.shape
    pad = (-N_) % tokw
    if pad:
        m = torch.cat([m, torch.zeros((B_, H_, pad, W_), dtype=m.dtype, device=m.device)], 2)
    mg = m.view(B_, H_, -1, tokw, W_)
    u = mg[:, :, :, 0]
    for t in range(1, tokw):
        u = u | mg[:, :, :, t]
    wave_chunks = float(popcount32(u, torch).sum())
    f_exec = wave_chunks * 4.0 * 32 * blk * d
    f_dense = 4.0 * d * w.h_q * w.batch * n * (n + 1) / 2.0
    cand = (pos // blk).to(torch.float64).sum() * w.batch * w.h_kv
    sparsity = 1.0 - float((cnt - 1).sum()) / float(cand)
    return dict(f_alg=f_alg, f_exec=f_exec, f_dense=f_dense, sparsity=sparsity)


def bench_prefill(w, steps, warmup, torch, B, make_inputs):
    dev = "cuda:0"
    q, k, v = make_inputs(w, dev)
    o = torch.empty_like(q)
    p = B.make_params(q, k, v, o, w.block, w.alpha, w.gamma, w.sigma, w.causal)
    kbar = torch.empty(B.kbar_shape(p), dtype=torch.float32, device=dev)
    lists = B.Lists.allocate(p, dev, idx=False, tau=False)
    ws = B.alloc_workspace(p, dev)
    B.dash_attn_prefill(p, q, k, v, o, kbar, lists, ws)
    torch.cuda.synchronize()
    st = prefill_stats(w, lists, torch)
    t_all = timed(lambda: B.dash_attn_prefill(p, q, k, v, o, kbar, lists, ws), steps, warmup, torch)
    t_s0 = timed(lambda: B.dash_kbar_compress(p, k, kbar), steps, 1, torch)
    # Stage 0 in its learned form (one summary query per kv-head), timed beside the block mean
    qbar = torch.randn((w.h_kv, w.head_dim), dtype=torch.float32, device=dev)
    kbar_l = torch.empty_like(kbar)
    t_s0l = timed(lambda: B.dash_kbar_summarize(p, k, qbar, kbar_l), steps, 1, torch)
    t_s1 = timed(lambda: B.dash_stage1_route(p, q, kbar, lists, ws), steps, 1, torch)
    t_s2 = timed(lambda: B.dash_stage2_attend(p, q, k, v, o, lists, ws), steps, 1, torch)
    od = torch.empty_like(q)
    t_dense = timed(lambda: B.dense_attn(p, q, k, v, od, ws), steps, warmup, torch)
    res = dict(ms_step=t_all, ms_stage0=t_s0, ms_stage0_learned=t_s0l, ms_stage1=t_s1, ms_stage2=t_s2, ms_dense=t_dense, **st)
    del q, k, v, o, od, ws, lists, kbar, kbar_l
    torch.cuda.empty_cache()
    return res


def bench_backward(w, steps, warmup, torch, B, make_inputs):
    """Forward and backward of the training-shaped workload (the backward reuses the
    forward's mask, bias and thresholds)."""
    dev = "cuda:0"
    q, k, v = make_inputs(w, dev)
    o = torch.empty_like(q)
    d_o = torch.randn(q.shape, device=dev, dtype=torch.float32).to(q.dtype)
    p = B.make_params(q, k, v, o, w.block, w.alpha, w.gamma, w.sigma, w.causal)
    kbar = torch.empty(B.kbar_shape(p), dtype=torch.float32, device=dev)
    lists = B.Lists.allocate(p, dev, idx=False)
    ws = B.alloc_workspace(p, dev)
    wsb = B.alloc_backward_workspace(p, dev)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    B.dash_attn_prefill(p, q, k, v, o, kbar, lists, ws)
    torch.cuda.synchronize()
    st = prefill_stats(w, lists, torch)
    t_f = timed(lambda: B.dash_attn_prefill(p, q, k, v, o, kbar, lists, ws), steps, warmup, torch)
    t_b = timed(lambda: B.dash_attn_backward(p, q, k, v, d_o, kbar, lists, dq, dk, dv, wsb), steps, warmup, torch)
    # the learned Stage 0's own backward (summary gradient -> keys and summary query), timed alone
    qbar = torch.randn((w.h_kv, w.head_dim), dtype=torch.float32, device=dev)
    dkbar = torch.randn(B.kbar_shape(p), dtype=torch.float32, device=dev)
    dqbar = torch.empty_like(dkbar)
    t_sb = timed(lambda: B.dash_kbar_summarize_backward(p, k, qbar, dkbar, dk, dqbar), steps, 1, torch)
    res = dict(ms_forward=t_f, ms_backward=t_b, ms_summarize_backward=t_sb, **st)
    del q, k, v, o, d_o, dq, dk, dv, ws, wsb, lists, kbar, qbar, dkbar, dqbar
    torch.cuda.empty_cache()
    return res


def bench_decode(w, steps, warmup, torch, B, make_inputs):
    dev = "cuda:0"
    q, k, v = make_inputs(w, dev)
    o = torch.empty_like(q)
    p = B.make_params(q, k, v, o, w.block, w.alpha, w.gamma, w.sigma, True)
    kbar = torch.empty(B.kbar_shape(p), dtype=torch.float32, device=dev)
    B.dash_kbar_compress(p, k, kbar)
    lists = B.Lists.allocate(p, dev, idx=False, tau=False)
    ws = B.alloc_workspace(p, dev)
    fn = lambda: B.dash_attn_decode(p, q, k, v, kbar, o, lists, ws)
    fn()
    torch.cuda.synchronize()
    cnt = lists.cnt.to(torch.int64)
    kept = float(cnt.sum())                                     # chunks read, incl. diagonal
    t_c = w.n_kv // w.block
    bytes_kv = kept * w.block * w.head_dim * 2 * 2
    bytes_s1 = w.batch * w.h_kv * t_c * w.head_dim * 4
    sparsity = 1.0 - float((cnt - 1).sum()) / float(w.batch * w.h_kv * ((w.n_kv - 1) // w.block))
    t = timed(fn, steps, warmup, torch)
    od = torch.empty_like(q)
    t_dense = timed(lambda: B.dense_attn(p, q, k, v, od, ws), steps, warmup, torch)
    dense_bytes = w.batch * w.h_kv * w.n_kv * w.head_dim * 2 * 2
    res = dict(us_step=t * 1e3, us_dense=t_dense * 1e3, sparsity=sparsity, bytes_kv=bytes_kv,
               bytes_stage1=bytes_s1, kv_gbs=bytes_kv / (t * 1e-3) / 1e9,
               total_gbs=(bytes_kv + bytes_s1) / (t * 1e-3) / 1e9,
               dense_gbs=dense_bytes / (t_dense * 1e-3) / 1e9)
    # the same step over sequences of different lengths (a serving batch): lengths spread evenly
    # between a quarter of the cache and the whole cache
    lens = torch.linspace(w.n_kv // 4, w.n_kv, w.batch).to(torch.int32)
    sl = lens.to(dev)
    fr = lambda: B.dash_attn_decode_ragged(p, q, k, v, kbar, sl, o, lists, ws, update_cache=True)
    fr()
    torch.cuda.synchronize()
    kept_r = float(lists.cnt.to(torch.int64).sum())
    tr = timed(fr, steps, warmup, torch)
    res["ragged"] = dict(us_step=tr * 1e3, mean_len=float(lens.float().mean()),
                         kv_gbs=kept_r * w.block * w.head_dim * 2 * 2 / (tr * 1e-3) / 1e9)
    del q, k, v, o, od, ws, lists, kbar
    torch.cuda.empty_cache()
    return res


def paper_protocol(steps, warmup, torch, B):
    """Stage-2 speed-up over the in-library dense attention on the shapes and the
    randomised masks of the paper's kernel benchmark (Sec. 5.3, App. B.3, Table 5).
    Stage 0/1 do not depend on the mask; their time on the same tensors is given
    beside it so that the speed-up can be read with and without routing."""
    from paper_2605_18753_amd.inputs import random_chunk_lists
    dev = "cuda:0"
    h_q, h_kv, d, blk = 32, 2, 128, 64
    sparsities = (0.75, 0.875, 0.9375)
    gen = torch.Generator(device=dev)
    gen.manual_seed(0)
    out = {"shape": {"h_q": h_q, "h_kv": h_kv, "head_dim": d, "block": blk, "dtype": "bf16"},
           "prefill_batch": 1, "decode_batch": 24, "prefill": {}, "decode": {}}
    for n in (16384, 32768, 65536, 98304):
        # ---- prefill, batch 1
        q = torch.randn((1, h_q, n, d), generator=gen, device=dev).bfloat16()
        k = torch.randn((1, h_kv, n, d), generator=gen, device=dev).bfloat16()
        v = torch.randn((1, h_kv, n, d), generator=gen, device=dev).bfloat16()
        o = torch.empty_like(q)
        p = B.make_params(q, k, v, o, blk)
        ws = B.alloc_workspace(p, dev)
        kbar = torch.empty(B.kbar_shape(p), dtype=torch.float32, device=dev)
        t_dense = timed(lambda: B.dense_attn(p, q, k, v, o, ws), steps, warmup, torch)
        lists = B.Lists.allocate(p, dev, idx=False, tau=False)
        t_s0 = timed(lambda: B.dash_kbar_compress(p, k, kbar), steps, 1, torch)
        t_s1 = timed(lambda: B.dash_stage1_route(p, q, kbar, lists, ws), steps, 1, torch)
        del lists
        row = {"dense_ms": t_dense, "stage0_ms": t_s0, "stage1_ms": t_s1}
        for s_ in sparsities:
            mask, cnt, bias = random_chunk_lists(1, h_kv, n, n, blk, s_, dev, seed=1)
            ls = B.Lists(mask=mask, bias=bias)
            t_s2 = timed(lambda: B.dash_stage2_attend(p, q, k, v, o, ls, ws), steps, warmup, torch)
            row[f"s{s_}"] = {"stage2_ms": t_s2, "speedup_stage2": t_dense / t_s2,
                             "speedup_with_routing": t_dense / (t_s0 + t_s1 + t_s2)}
            del mask, cnt, bias, ls
        out["prefill"][str(n)] = row
        del q, k, v, o, ws, kbar
        torch.cuda.empty_cache()
        # ---- decode, batch 24
        bd = 24
        q = torch.randn((bd, h_q, 1, d), generator=gen, device=dev).bfloat16()
        k = torch.randn((bd, h_kv, n, d), generator=gen, device=dev).bfloat16()
        v = torch.randn((bd, h_kv, n, d), generator=gen, device=dev).bfloat16()
        o = torch.empty_like(q)
        p = B.make_params(q, k, v, o, blk)
        ws = B.alloc_workspace(p, dev)
        kbar = torch.empty(B.kbar_shape(p), dtype=torch.float32, device=dev)
        B.dash_kbar_compress(p, k, kbar)
        t_dense = timed(lambda: B.dense_attn(p, q, k, v, o, ws), max(steps, 20), warmup, torch)
        lists = B.Lists.allocate(p, dev, idx=False, tau=False)
        t_s1 = timed(lambda: B.dash_stage1_route(p, q, kbar, lists, ws), max(steps, 20), 1, torch)
        del lists
        row = {"dense_us": t_dense * 1e3, "stage1_us": t_s1 * 1e3}
        for s_ in sparsities:
            mask, cnt, bias = random_chunk_lists(bd, h_kv, 1, n, blk, s_, dev, seed=2)
            ls = B.Lists(mask=mask, bias=bias)
            t_s2 = timed(lambda: B.dash_stage2_attend(p, q, k, v, o, ls, ws), max(steps, 20), warmup, torch)
            kv_bytes = float(cnt.sum()) * blk * d * 2 * 2
            row[f"s{s_}"] = {"stage2_us": t_s2 * 1e3, "speedup_stage2": t_dense / t_s2,
                             "speedup_with_routing": t_dense / (t_s1 + t_s2),
                             "kv_GBps_stage2": kv_bytes / (t_s2 * 1e-3) / 1e9}
            del mask, cnt, bias, ls
        out["decode"][str(n)] = row
        del q, k, v, o, ws, kbar
        torch.cuda.empty_cache()
    return out


def gemm_context(torch):
    """Library bf16 GEMM rate (8192^3, hipBLASLt through torch) with N(0,1) and with
    all-zero operands: how far the chip's power management lets dense bf16 MFMA
    work run on data that toggles, as context for the MFMA roofline fraction."""
    n = 8192
    out = {}
    for name in ("normal", "zeros"):
        a = torch.randn(n, n, device="cuda:0", dtype=torch.bfloat16) if name == "normal" else \
            torch.zeros(n, n, device="cuda:0", dtype=torch.bfloat16)
        b = a.t().contiguous()
        ms = timed(lambda: torch.mm(a, b), 10, 3, torch)
        out[name] = 2.0 * n ** 3 / (ms * 1e-3) / 1e12
        del a, b
    torch.cuda.empty_cache()
    return out


def cpu_baseline(w, seconds, torch, make_inputs):
    """The oracle as it stands, single thread, on a uniform sample of query rows of
    the same workload; reported in the metric's unit (dense-equivalent flops / s)."""
    import numpy as np
    from oracle import dash_oracle as orc
    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(limits=1)
    except Exception:  # pragma: no cover
        limiter = None
    ws = w.replace(batch=1, h_q=w.g_q, h_kv=1)       # one kv-head's worth of tensors
    q, k, v = make_inputs(ws, "cpu")
    qn, kn, vn = (t.float().numpy() for t in (q, k, v))
    prm = orc.DashParams(block=w.block, alpha=w.alpha, gamma=w.gamma, sigma=w.sigma, causal=w.causal)
    kbar = orc.block_mean_summaries(kn, w.block)
    rng = np.random.default_rng(0)
    t0 = time.perf_counter()
    flops, rows = 0.0, 0
    while time.perf_counter() - t0 < seconds:
        i = int(rng.integers(0, w.n_q))
        orc.dash_row(qn, kn, vn, kbar, prm, 0, 0, i)
        flops += 4.0 * w.head_dim * w.g_q * (i + 1)
        rows += 1
    dt = time.perf_counter() - t0
    if limiter is not None:
        limiter.restore_original_limits() if hasattr(limiter, "restore_original_limits") else None
    return dict(value=flops / dt / 1e12, unit="TFLOP/s", cores=1, kind="oracle",
                sample=f"{rows} uniformly drawn query rows (all {w.g_q} heads of one kv-head) of the same "
                       f"workload, {dt:.1f} s, numpy fp64, 1 thread; dense-equivalent flops of those rows / time")


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2605_18753_amd import binding as B
    from paper_2605_18753_amd.inputs import C2, C3, C5, make_inputs
    B.load_library()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    w = C2
    wd = C3
    if a.small:
        w = w.replace(n_q=4096, n_kv=4096, name="C2_small")
        wd = wd.replace(n_kv=16384, batch=4, name="C3_small")

    if a.paper_protocol:
        res = paper_protocol(a.steps, a.warmup, torch, B)
        print(json.dumps({"metric": "Stage-2 speed-up over the in-library dense attention, randomised chunk masks "
                                    "(kernel-benchmark protocol of the paper)", "unit": "x", "n_gpus": 1,
                          "data": "synthetic", "dtype": "bf16", **res}))
        return
    if a.backward_only:
        wb = C5.replace(n_q=2048, n_kv=2048, batch=1, name="C5_small") if a.small else C5
        r = bench_backward(wb, a.steps, a.warmup, torch, B, make_inputs)
        flops = 2.5 * r["f_alg"]
        print(json.dumps({"metric": "backward algorithmic TFLOP/s (5 matrix products per attended query-key pair)",
                          "value": flops / (r["ms_backward"] * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1,
                          "steps": a.steps, "warmup": a.warmup, "ms_per_step": r["ms_backward"], "dtype": "bf16",
                          "data": "synthetic", "config": {"workload": wb.name}, "ms_forward": r["ms_forward"],
                          "chunk_sparsity": r["sparsity"], "f_alg_forward": r["f_alg"]}))
        return
    if a.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    main_res = bench_prefill(w, a.steps, a.warmup, torch, B, make_inputs)
    # the gamma that lands near 75 % chunk sparsity on this generator
    w75 = w.replace(gamma=1.5)
    res75 = bench_prefill(w75, a.steps, a.warmup, torch, B, make_inputs)
    dec = None
    if not a.no_decode:
        dec = dict(gamma1=bench_decode(wd, max(a.steps, 20), a.warmup, torch, B, make_inputs),
                   gamma04=bench_decode(wd.replace(gamma=0.4), max(a.steps, 20), a.warmup, torch, B, make_inputs))
    wb = C5.replace(n_q=2048, n_kv=2048, batch=1, name="C5_small") if a.small else C5
    bwd = None if a.no_backward else bench_backward(wb, a.steps, a.warmup, torch, B, make_inputs)
    cpu = None if a.no_cpu else cpu_baseline(w, a.cpu_seconds, torch, make_inputs)
    gemm = None if a.small else gemm_context(torch)

    def tf(flops, ms):
        return flops / (ms * 1e-3) / 1e12

    value = tf(main_res["f_dense"], main_res["ms_step"])
    achieved = tf(main_res["f_alg"], main_res["ms_stage2"])
    out = {
        "metric": "prefill effective TFLOP/s (dense-equivalent causal attention flops / time of the whole "
                  "DashAttention prefill, stages 0+1+2)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": main_res["ms_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "h_q": w.h_q, "h_kv": w.h_kv, "n": w.n_q,
                   "head_dim": w.head_dim, "block": w.block, "alpha": w.alpha, "gamma": w.gamma,
                   "sigma": w.sigma, "causal": True, "offset_sigma": w.offset_sigma, "seed": w.seed},
        "roofline": {"bound": "mfma", "kernel": "s2_attend_kernel<128,false>",
                     "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": None if a.small else S2_TRAFFIC_BYTES_C2},
        "cpu_baseline": cpu,
        "extras": {
            "chunk_sparsity": main_res["sparsity"],
            "ms": {k_: main_res[k_] for k_ in ("ms_step", "ms_stage0", "ms_stage1", "ms_stage2", "ms_dense")},
            "stage0_learned": {"ms": main_res["ms_stage0_learned"],
                               "k_read_GBps": w.batch * w.h_kv * w.n_kv * w.head_dim * 2 /
                                              (main_res["ms_stage0_learned"] * 1e-3) / 1e9,
                               "block_mean_k_read_GBps": w.batch * w.h_kv * w.n_kv * w.head_dim * 2 /
                                                         (main_res["ms_stage0"] * 1e-3) / 1e9},
            "speedup_vs_dense": main_res["ms_dense"] / main_res["ms_step"],
            "stage2_speedup_vs_dense": main_res["ms_dense"] / main_res["ms_stage2"],
            "dense_tflops": tf(main_res["f_dense"], main_res["ms_dense"]),
            "dense_mfma_frac": tf(main_res["f_dense"], main_res["ms_dense"]) / MFMA_BF16_PEAK_TFLOPS,
            "stage2_exec_tflops": tf(main_res["f_exec"], main_res["ms_stage2"]),
            "stage2_exec_mfma_frac": tf(main_res["f_exec"], main_res["ms_stage2"]) / MFMA_BF16_PEAK_TFLOPS,
            "f_alg_over_f_exec": main_res["f_alg"] / main_res["f_exec"],
            "library_gemm_bf16_tflops": gemm,
            "at_75pct_sparsity": {
                "gamma": w75.gamma, "chunk_sparsity": res75["sparsity"],
                "effective_tflops": tf(res75["f_dense"], res75["ms_step"]),
                "ms": {k_: res75[k_] for k_ in ("ms_step", "ms_stage0", "ms_stage1", "ms_stage2", "ms_dense")},
                "speedup_vs_dense": res75["ms_dense"] / res75["ms_step"],
                "stage2_exec_mfma_frac": tf(res75["f_exec"], res75["ms_stage2"]) / MFMA_BF16_PEAK_TFLOPS,
                "stage2_alg_mfma_frac": tf(res75["f_alg"], res75["ms_stage2"]) / MFMA_BF16_PEAK_TFLOPS,
                "f_alg_over_f_exec": res75["f_alg"] / res75["f_exec"],
            },
            # backward of the training-shaped workload: 5 matrix products per attended (query, key)
            # pair against the forward's 2, so its flops are 2.5 x the forward's f_alg
            "backward": None if bwd is None else {
                "workload": wb.name, "ms_forward": bwd["ms_forward"], "ms_backward": bwd["ms_backward"],
                "backward_over_forward": bwd["ms_backward"] / bwd["ms_forward"],
                "ms_learned_stage0_backward": bwd["ms_summarize_backward"],
                "chunk_sparsity": bwd["sparsity"],
                "backward_alg_tflops": tf(2.5 * bwd["f_alg"], bwd["ms_backward"]),
                "backward_alg_mfma_frac": tf(2.5 * bwd["f_alg"], bwd["ms_backward"]) / MFMA_BF16_PEAK_TFLOPS,
            },
            "decode": None if dec is None else {
                "workload": wd.name,
                **{name: {"gamma": g_, "us_per_step": r["us_step"], "dense_us_per_step": r["us_dense"],
                          "chunk_sparsity": r["sparsity"], "kv_GBps": r["kv_gbs"],
                          "kv_hbm_frac": r["kv_gbs"] / HBM_PEAK_GBS, "kv_plus_stage1_GBps": r["total_gbs"],
                          "dense_GBps": r["dense_gbs"], "speedup_vs_dense": r["us_dense"] / r["us_step"],
                          "ragged_lengths": {"us_per_step": r["ragged"]["us_step"],
                                             "mean_length": r["ragged"]["mean_len"],
                                             "kv_GBps": r["ragged"]["kv_gbs"]}}
                   for name, g_, r in (("gamma_1", 1.0, dec["gamma1"]), ("gamma_0.4", 0.4, dec["gamma04"]))},
            },
        },
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
