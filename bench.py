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
  cpu_baseline  the fp64 oracle timed on a bounded row sample, on all host cores
                (worker processes started before the GPU is touched)
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
# HBM bytes per launch of the Stage-2 kernel on the headline workload cannot be measured from
# inside this script: they come from the two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) whose
# summary is committed in this file, which carries one line `traffic_json: {...}` per kernel
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "prefill_c2_hbm_traffic.md")


def traffic_from_profile(kernel, workload):
    """Scaled FETCH_SIZE + WRITE_SIZE bytes per launch from the committed summary, or None."""
    try:
        for line in open(TRAFFIC_PROFILE):
            if line.startswith("traffic_json:"):
                rec = json.loads(line[len("traffic_json:"):])
                if rec.get("kernel") == kernel and rec.get("workload") == workload:
                    return float(rec["fetch_bytes"]) + float(rec["write_bytes"])
    except (OSError, ValueError, KeyError):
        pass
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-backward", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="skip the nine-point 128k sweep")
    ap.add_argument("--only", default=None, choices=["c2-gamma1", "c2-gamma1.5", "c3-gamma1", "c3-gamma0.4"],
                    help="run one workload at one temperature and nothing else (profiling runs: the per-kernel "
                         "figures of a rocprofv3 run then belong to that configuration alone)")
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


def timed_each(fn, steps, torch):
    """Per-call ms of `steps` further calls (one event pair each): median, min, max."""
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for e0, e1 in ev:
        e0.record()
        fn()
        e1.record()
    torch.cuda.synchronize()
    t = sorted(e0.elapsed_time(e1) for e0, e1 in ev)
    return {"median": t[len(t) // 2], "min": t[0], "max": t[-1], "calls": steps}


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


def bench_prefill(w, steps, warmup, torch, B, make_inputs, sensors=None):
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
    t_all_each = timed_each(lambda: B.dash_attn_prefill(p, q, k, v, o, kbar, lists, ws), max(steps, 20), torch)
    t_s0 = timed(lambda: B.dash_kbar_compress(p, k, kbar), steps, 1, torch)
    # Stage 0 in its learned form (one summary query per kv-head), timed beside the block mean
    qbar = torch.randn((w.h_kv, w.head_dim), dtype=torch.float32, device=dev)
    kbar_l = torch.empty_like(kbar)
    t_s0l = timed(lambda: B.dash_kbar_summarize(p, k, qbar, kbar_l), steps, 1, torch)
    t_s1 = timed(lambda: B.dash_stage1_route(p, q, kbar, lists, ws), steps, 1, torch)
    od = torch.empty_like(q)
    if sensors is None:
        t_s2 = timed(lambda: B.dash_stage2_attend(p, q, k, v, o, lists, ws), steps, 1, torch)
        t_dense = timed(lambda: B.dense_attn(p, q, k, v, od, ws), steps, warmup, torch)
        sens = None
    else:
        # the box's clock / power readings while each of the two Stage-2 kernels runs alone
        t_s2, sn_s2 = sensors.during(lambda: timed(lambda: B.dash_stage2_attend(p, q, k, v, o, lists, ws), steps, 1, torch))
        t_dense, sn_d = sensors.during(lambda: timed(lambda: B.dense_attn(p, q, k, v, od, ws), steps, warmup, torch))
        sens = {"stage2_loop": sn_s2, "dense_loop": sn_d}
    res = dict(sensors=sens, ms_step_each=t_all_each, ms_step=t_all, ms_stage0=t_s0, ms_stage0_learned=t_s0l, ms_stage1=t_s1, ms_stage2=t_s2, ms_dense=t_dense, **st)
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


def paper_protocol(steps, warmup, torch, B, lengths=(16384, 32768, 65536, 98304)):
    """Stage-2 speed-up over the in-library dense attention on the shapes and the
    randomised masks of the paper's kernel benchmark (Sec. 5.2, App. B.2, Table 5).
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
    for n in lengths:
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


# ---- the oracle on the host cores -------------------------------------------------------
# Worker processes are forked before this process touches the GPU (a fork afterwards would
# duplicate a live GPU context).  Each worker holds one kv-head's worth of the workload's
# tensors (inherited through the fork), runs oracle rows drawn uniformly until its deadline
# and reports rows and dense-equivalent flops.
_ORC = {}


def _orc_worker(args):
    name, seconds, seed = args
    import numpy as np
    from oracle import dash_oracle as orc
    try:
        from threadpoolctl import threadpool_limits
        threadpool_limits(limits=1)
    except Exception:  # pragma: no cover
        pass
    w, qn, kn, vn, kbar, prm, rows_of = _ORC[name]
    rng = np.random.default_rng(seed)
    t0 = time.perf_counter()
    flops, rows = 0.0, 0
    while time.perf_counter() - t0 < seconds:
        i = int(rng.integers(rows_of[0], rows_of[1]))
        orc.dash_row(qn, kn, vn, kbar, prm, 0, 0, i)
        pos = w.n_kv - w.n_q + i
        flops += 4.0 * w.head_dim * w.g_q * ((pos + 1) if w.causal else w.n_kv)
        rows += 1
    return rows, flops, time.perf_counter() - t0


def host_cores():
    # a one-GPU machine gives this job 16 cores whatever os.cpu_count() shows
    return max(1, min(16, os.cpu_count() or 1))


def oracle_on_host(workloads, seconds):
    """Times the oracle as it stands (numpy fp64, one row at a time) on all host cores for
    every workload in `workloads` (name -> Workload), `seconds` of wall time each.  Returns
    name -> dict(rows_per_s, flops_per_s, rows, cores, seconds)."""
    import multiprocessing as mp
    import numpy as np
    from oracle import dash_oracle as orc
    from paper_2605_18753_amd.inputs import make_inputs
    cores = host_cores()
    for name, w in workloads.items():
        ws = w.replace(batch=1, h_q=w.g_q, h_kv=1)       # one kv-head's worth of tensors
        q, k, v = make_inputs(ws, "cpu")
        qn, kn, vn = (t.float().numpy() for t in (q, k, v))
        prm = orc.DashParams(block=w.block, alpha=w.alpha, gamma=w.gamma, sigma=w.sigma, causal=w.causal)
        _ORC[name] = (ws, qn, kn, vn, orc.block_mean_summaries(kn, w.block), prm, (0, ws.n_q))
    out = {}
    ctx = mp.get_context("fork")
    with ctx.Pool(cores) as pool:
        for name in workloads:
            res = pool.map(_orc_worker, [(name, seconds, 1000 + c) for c in range(cores)])
            rows = sum(r[0] for r in res)
            dt = max(r[2] for r in res)
            out[name] = dict(rows=rows, cores=cores, seconds=dt, rows_per_s=rows / dt,
                             flops_per_s=sum(r[1] for r in res) / dt)
    _ORC.clear()
    return out


def cpu_baseline(w, orc_res):
    r = orc_res[w.name]
    return dict(value=r["flops_per_s"] / 1e12, unit="TFLOP/s", cores=r["cores"], kind="oracle",
                sample=f"{r['rows']} uniformly drawn query rows (all {w.g_q} heads of one kv-head) of the same "
                       f"workload in {r['seconds']:.1f} s on {r['cores']} worker processes (numpy fp64, one thread "
                       f"each); dense-equivalent flops of those rows / wall time")


# ---- what the box reports while a kernel runs ------------------------------------------------
class Sensors:
    """Samples the GPU's engine clock and power from sysfs (hwmon) in a thread while a timing
    loop runs; fields are None where the box does not expose them to this user."""

    def __init__(self):
        import glob
        self.freq = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/freq1_input"))
        self.dpm = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        self.power = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average") +
                            glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))

    @staticmethod
    def _read(path):
        try:
            return float(open(path).read().split()[0])
        except (OSError, ValueError, IndexError):
            return None

    @staticmethod
    def _dpm_mhz(path):
        """The level marked current ('*') in a pp_dpm_sclk listing such as '1: 2100Mhz *'."""
        try:
            for line in open(path):
                if "*" in line:
                    return float(line.split(":")[1].lower().split("mhz")[0])
        except (OSError, ValueError, IndexError):
            pass
        return None

    def during(self, fn):
        """Runs fn() while sampling every 2 ms; returns (fn's result, summary dict)."""
        import threading
        f, pw, stop = [], [], threading.Event()

        def loop():
            while not stop.is_set():
                if self.freq:
                    x = self._read(self.freq[0])
                    if x:
                        f.append(x / 1e6)            # Hz -> MHz
                elif self.dpm:
                    x = self._dpm_mhz(self.dpm[0])
                    if x:
                        f.append(x)
                if self.power:
                    x = self._read(self.power[0])
                    if x:
                        pw.append(x / 1e6)           # microwatt -> W
                time.sleep(0.002)

        th = threading.Thread(target=loop, daemon=True)
        th.start()
        try:
            res = fn()
        finally:
            stop.set()
            th.join()
        mean = lambda xs: sum(xs) / len(xs) if xs else None
        return res, {"sclk_mhz_mean": mean(f), "sclk_mhz_min": min(f) if f else None, "power_w_mean": mean(pw),
                     "samples": max(len(f), len(pw))}


def microbench(torch, steps):
    """Achievable rates on this machine: streaming read of 4 GiB of HBM, and a register-fed loop of
    v_mfma_f32_32x32x16_bf16 (8 independent accumulators per wave, 2 workgroups of 4 waves per
    CU) on operands that toggle and on constant ones.  Kernels: csrc/microbench.hip."""
    import ctypes
    from paper_2605_18753_amd.build import MICROBENCH_LIB
    if not os.path.exists(MICROBENCH_LIB):
        return None
    lib = ctypes.CDLL(MICROBENCH_LIB)
    lib.dash_mb_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
    lib.dash_mb_mfma_loop.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                      ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    nbytes = 4 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0").fill_(1)
    sink = torch.zeros(4, dtype=torch.float32, device="cuda:0")
    ms = timed(lambda: lib.dash_mb_stream_read(src.data_ptr(), nbytes, sink.data_ptr(), st), max(steps, 5), 2, torch)
    out = {"stream_read_GBps": nbytes / (ms * 1e-3) / 1e9}
    del src
    torch.cuda.empty_cache()
    sens = Sensors()
    flops = ctypes.c_double(0.0)
    for name, rnd in (("random_operands", 1), ("constant_operands", 0)):
        fn = lambda: lib.dash_mb_mfma_loop(sink.data_ptr(), 512, 20000, rnd, ctypes.byref(flops), st)
        ms, sn = sens.during(lambda: timed(fn, 3, 1, torch))
        out[f"mfma_loop_tflops_{name}"] = flops.value / (ms * 1e-3) / 1e12
        out[f"mfma_loop_sensors_{name}"] = sn
    return out


def c4_sweep(torch, B, make_inputs, C4, small):
    """The long-prefill configuration at its nine (alpha, key-offset sigma) points: time of the
    whole prefill and of the dense kernel, chunk sparsity, algorithmic / executed flops."""
    rows = []
    for alpha in (1.25, 1.5, 2.0):
        for off in (0.3, 0.5, 1.0):
            w = C4.replace(alpha=alpha, offset_sigma=off)
            if small:
                w = w.replace(n_q=8192, n_kv=8192, name="C4_small")
            r = bench_prefill(w, 2, 1, torch, B, make_inputs)
            rows.append({"alpha": alpha, "offset_sigma": off, "chunk_sparsity": r["sparsity"],
                         "ms_step": r["ms_step"], "ms_stage1": r["ms_stage1"], "ms_stage2": r["ms_stage2"],
                         "ms_dense": r["ms_dense"], "speedup_vs_dense": r["ms_dense"] / r["ms_step"],
                         "f_alg_over_f_exec": r["f_alg"] / r["f_exec"],
                         "effective_tflops": r["f_dense"] / (r["ms_step"] * 1e-3) / 1e12,
                         "stage2_alg_mfma_frac": r["f_alg"] / (r["ms_stage2"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS})
    return rows


def c1_time(torch, B, make_inputs, C1, steps):
    """The fp32 single-head non-causal configuration (a correctness configuration: time only)."""
    dev = "cuda:0"
    q, k, v = make_inputs(C1, dev)
    o = torch.empty_like(q)
    p = B.make_params(q, k, v, o, C1.block, C1.alpha, C1.gamma, C1.sigma, C1.causal)
    kbar = torch.empty(B.kbar_shape(p), dtype=torch.float32, device=dev)
    lists = B.Lists.allocate(p, dev, idx=False, tau=False)
    ws = B.alloc_workspace(p, dev)
    t = timed(lambda: B.dash_attn_prefill(p, q, k, v, o, kbar, lists, ws), max(steps, 20), 3, torch)
    td = timed(lambda: B.dense_attn(p, q, k, v, o, ws), max(steps, 20), 3, torch)
    return {"workload": C1.name, "us_prefill": t * 1e3, "us_dense": td * 1e3}


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2605_18753_amd import binding as B
    from paper_2605_18753_amd.inputs import C1, C2, C3, C4, C5, make_inputs
    B.load_library()
    w = C2
    wd = C3
    if a.small:
        w = w.replace(n_q=4096, n_kv=4096, name="C2_small")
        wd = wd.replace(n_kv=16384, batch=4, name="C3_small")
    full_run = not (a.paper_protocol or a.backward_only or a.only)
    # the oracle on the host cores first: its worker processes are forked before the GPU is touched
    orc_res = None
    if full_run and not a.no_cpu:
        others = {} if a.small else {"C1": C1, "C3": wd, "C4": C4.replace(alpha=1.5, offset_sigma=0.5), "C5": C5}
        orc_res = oracle_on_host({w.name: w}, a.cpu_seconds)
        orc_res.update(oracle_on_host(others, min(3.0, a.cpu_seconds)))
    assert torch.cuda.is_available(), "bench.py needs the GPU"

    if a.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    if a.only:
        g_ = float(a.only.split("gamma")[1])
        if a.only.startswith("c2"):
            r = bench_prefill(w.replace(gamma=g_), a.steps, a.warmup, torch, B, make_inputs)
            r = {k_: r[k_] for k_ in ("ms_step", "ms_stage0", "ms_stage1", "ms_stage2", "ms_dense", "sparsity")}
        else:
            r = bench_decode(wd.replace(gamma=g_), max(a.steps, 20), a.warmup, torch, B, make_inputs)
            r = {k_: r[k_] for k_ in ("us_step", "us_dense", "sparsity", "kv_gbs")}
        print(json.dumps({"only": a.only, "steps": a.steps, **r}))
        return
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
    sens = Sensors()
    main_res = bench_prefill(w, a.steps, a.warmup, torch, B, make_inputs, sensors=sens)
    sens_main = main_res["sensors"]
    # the gamma that lands near 75 % chunk sparsity on this generator
    w75 = w.replace(gamma=1.5)
    res75 = bench_prefill(w75, a.steps, a.warmup, torch, B, make_inputs)
    sweep = None if a.no_sweep else c4_sweep(torch, B, make_inputs, C4, a.small)
    # the same configuration with queries that vary smoothly along the sequence (AR(1) over tokens, not a
    # configuration of the paper): neighbouring tokens then keep similar chunks and an MFMA tile's union shrinks
    corr = None
    if not (a.no_sweep or a.small):
        corr = {}
        for rho in (0.9, 0.97, 0.99):
            r = bench_prefill(w.replace(gamma=1.5, query_corr=rho), max(a.steps // 2, 3), 2, torch, B, make_inputs)
            corr[f"rho_{rho}"] = {"gamma": 1.5, "chunk_sparsity": r["sparsity"], "ms_step": r["ms_step"], "ms_stage2": r["ms_stage2"],
                                  "ms_dense": r["ms_dense"], "speedup_vs_dense": r["ms_dense"] / r["ms_step"],
                                  "stage2_speedup_vs_dense": r["ms_dense"] / r["ms_stage2"],
                                  "f_alg_over_f_exec": r["f_alg"] / r["f_exec"],
                                  "effective_tflops": r["f_dense"] / (r["ms_step"] * 1e-3) / 1e12}
    c1 = c1_time(torch, B, make_inputs, C1, a.steps)
    mb = None if a.small else microbench(torch, a.steps)
    # the paper's own benchmark shape (GQA group 16, randomised masks) at its 32K point; all four lengths: --paper-protocol
    pp32 = None if (a.small or a.no_sweep) else paper_protocol(a.steps, a.warmup, torch, B, lengths=(32768,))
    dec = None
    if not a.no_decode:
        dec = dict(gamma1=bench_decode(wd, max(a.steps, 20), a.warmup, torch, B, make_inputs),
                   gamma04=bench_decode(wd.replace(gamma=0.4), max(a.steps, 20), a.warmup, torch, B, make_inputs))
    wb = C5.replace(n_q=2048, n_kv=2048, batch=1, name="C5_small") if a.small else C5
    bwd = None if a.no_backward else bench_backward(wb, a.steps, a.warmup, torch, B, make_inputs)
    cpu = None if orc_res is None else cpu_baseline(w, orc_res)
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
                     "traffic": None if a.small else traffic_from_profile("s2_attend_kernel<128,false>", "C2 gamma=1"),
                     "traffic_source": os.path.relpath(TRAFFIC_PROFILE, ROOT)},
        "cpu_baseline": cpu,
        "extras": {
            "chunk_sparsity": main_res["sparsity"],
            "ms": {k_: main_res[k_] for k_ in ("ms_step", "ms_stage0", "ms_stage1", "ms_stage2", "ms_dense")},
            "stage0_learned": {"ms": main_res["ms_stage0_learned"],
                               "k_read_GBps": w.batch * w.h_kv * w.n_kv * w.head_dim * 2 /
                                              (main_res["ms_stage0_learned"] * 1e-3) / 1e9,
                               "block_mean_k_read_GBps": w.batch * w.h_kv * w.n_kv * w.head_dim * 2 /
                                                         (main_res["ms_stage0"] * 1e-3) / 1e9},
            # the same step timed call by call (20 calls after the timed loop): median / min / max in ms
            "ms_step_per_call": main_res["ms_step_each"],
            "speedup_vs_dense": main_res["ms_dense"] / main_res["ms_step"],
            "stage2_speedup_vs_dense": main_res["ms_dense"] / main_res["ms_stage2"],
            "dense_tflops": tf(main_res["f_dense"], main_res["ms_dense"]),
            "dense_mfma_frac": tf(main_res["f_dense"], main_res["ms_dense"]) / MFMA_BF16_PEAK_TFLOPS,
            "stage2_exec_tflops": tf(main_res["f_exec"], main_res["ms_stage2"]),
            "stage2_exec_mfma_frac": tf(main_res["f_exec"], main_res["ms_stage2"]) / MFMA_BF16_PEAK_TFLOPS,
            "f_alg_over_f_exec": main_res["f_alg"] / main_res["f_exec"],
            "library_gemm_bf16_tflops": gemm,
            # achievable rates on this machine (csrc/microbench.hip) and what its sensors report during the
            # headline prefill loop (engine clock, power): context for the MFMA / HBM fractions
            "microbench": mb,
            "sensors": sens_main,
            "C1_fp32_single_head": c1,
            "C4_sweep_128k": sweep,
            "paper_protocol_32k": pp32,
            "correlated_queries_32k": corr,
            # the oracle on the host cores for the other configurations: rows per second on a 3 s sample and
            # the whole configuration's time extrapolated from it (rows are independent)
            "oracle_on_host": None if orc_res is None else {
                name: {"rows_per_s": r["rows_per_s"], "cores": r["cores"], "sample_rows": r["rows"],
                       "sample_seconds": r["seconds"]} for name, r in orc_res.items()},
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
