"""Seeded synthetic inputs for the DashAttention forward path.

This module only draws random tensors; it contains none of the method's
arithmetic.  It serves the tests (which hand the same bits to the CPU oracle
and to the HIP library) and the benchmark.

Recipe (every workload): Q, K, V are i.i.d. N(0,1) drawn in fp32; every key of
KV block c of (batch b, kv-head r) gets the same additive offset vector
o[b,r,c,:] ~ N(0, offset_sigma^2), so block means differ and the entmax
router becomes sparse; the "needle" variant instead adds +needle_gain * u to
the keys of a few randomly chosen blocks, u ~ N(0, I_d) shared by all kv-heads
of a sequence.  Tensors are rounded once (RNE) to the run dtype; those bits are
the input of both sides.  Q is NOT pre-scaled: the 1/sqrt(d) factor is applied
once, inside the attention (Eq. 1 of the paper).

Draw order is fixed (Q, K, V, offsets / needles, one batch element at a time)
so a (workload, seed, device type) triple always yields the same bits.  CPU and
GPU generators produce different streams; a test that needs both sides to see
the same data copies the generated tensors, it never regenerates them.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Optional, Tuple

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    h_q: int
    h_kv: int
    n_q: int            # prefill: == n_kv ; decode: 1
    n_kv: int
    head_dim: int
    block: int
    alpha: float = 1.5
    gamma: float = 1.0
    sigma: float = 1.0
    causal: bool = True
    window: int = 0              # always-attended complete chunks before the diagonal one
    dtype: str = "bf16"          # "bf16" | "fp32"
    offset_sigma: float = 0.5    # std of the per-block key offset
    needles: int = 0             # >0: needle recipe instead of offsets
    needle_gain: float = 2.0
    query_corr: float = 0.0      # >0: queries of consecutive tokens follow an AR(1) process with this coefficient
    seed: int = 0

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)

    @property
    def g_q(self) -> int:
        return self.h_q // self.h_kv

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32


# The five configurations the build is measured / checked on.
C1 = Workload("C1_single_head_fp32", 1, 1, 1, 1024, 1024, 64, 64, causal=False,
              dtype="fp32", offset_sigma=0.5)
C2 = Workload("C2_causal_gqa_prefill_32k", 1, 32, 8, 32768, 32768, 128, 64,
              offset_sigma=0.5)
C3 = Workload("C3_causal_gqa_decode_128k", 16, 32, 8, 1, 131072, 128, 64,
              offset_sigma=0.7)
C4 = Workload("C4_long_prefill_128k", 1, 32, 8, 131072, 131072, 128, 128,
              offset_sigma=0.5)
C5 = Workload("C5_training_shaped_needles", 4, 16, 16, 8192, 8192, 128, 64,
              offset_sigma=0.0, needles=4)

NAMED = {w.name.split("_")[0]: w for w in (C1, C2, C3, C4, C5)}


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _randn(shape, gen, device) -> torch.Tensor:
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32)


def _add_block_structure(w: Workload, k: torch.Tensor, gen, device) -> None:
    """In place: add per-block offsets (or needles) to the fp32 keys of one
    batch element, k: [h_kv, n_kv, d]."""
    h_kv, n, d = k.shape
    n_blocks = (n + w.block - 1) // w.block
    if w.needles > 0:
        u = _randn((d,), gen, device)
        # distinct blocks, chosen with the same generator
        perm = torch.randperm(n_blocks, generator=gen, device=device)
        for c in perm[: w.needles].tolist():
            k[:, c * w.block:(c + 1) * w.block, :] += w.needle_gain * u
    elif w.offset_sigma > 0.0:
        off = _randn((h_kv, n_blocks, d), gen, device) * w.offset_sigma
        off = off.repeat_interleave(w.block, dim=1)[:, :n, :]
        k += off


def _correlate_tokens(x: torch.Tensor, rho: float) -> None:
    """In place, along the token axis of x [heads, tokens, d]: x_t <- rho x_{t-1} + sqrt(1 - rho^2) x_t
    (x_0 unchanged), a stationary AR(1) process with unit variance per element.  Not part of any
    configuration of the paper: its kernel benchmark draws independent masks, real queries of
    neighbouring tokens are similar; bench.py reports this variant beside the independent one."""
    n = x.shape[1]
    blk = 256
    i = torch.arange(blk, device=x.device, dtype=torch.float64)
    low = torch.tril(rho ** (i.view(-1, 1) - i.view(1, -1)).clamp(min=0)).to(torch.float32)   # rho^(i-j), j <= i
    carry_w = (rho ** (i + 1)).to(torch.float32).view(1, -1, 1)
    s = (1.0 - rho * rho) ** 0.5
    prev = None
    for t0 in range(0, n, blk):
        m = min(blk, n - t0)
        e = x[:, t0:t0 + m] * s
        if prev is None:
            e[:, 0] = x[:, 0]          # the first token keeps unit variance
        y = torch.matmul(low[:m, :m], e)
        if prev is not None:
            y += carry_w[:, :m] * prev.unsqueeze(1)
        x[:, t0:t0 + m] = y
        prev = y[:, -1].clone()


def make_inputs(w: Workload, device="cpu") -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """Return (q, k, v) in the run dtype.

    Layout: q [batch, h_q, n_q, d]; k, v [batch, h_kv, n_kv, d]; last dim
    contiguous.  For a decode workload (n_q == 1) the single query sits at
    position n_kv - 1 and k, v are the KV cache (which already holds that
    token).
    """
    device = torch.device(device)
    gen = _gen(device, w.seed)
    dt = w.torch_dtype
    q = torch.empty((w.batch, w.h_q, w.n_q, w.head_dim), dtype=dt, device=device)
    k = torch.empty((w.batch, w.h_kv, w.n_kv, w.head_dim), dtype=dt, device=device)
    v = torch.empty_like(k)
    for b in range(w.batch):
        qb = _randn((w.h_q, w.n_q, w.head_dim), gen, device)
        if w.query_corr > 0.0:
            _correlate_tokens(qb, w.query_corr)
        q[b] = qb.to(dt)
        del qb
        kb = _randn((w.h_kv, w.n_kv, w.head_dim), gen, device)
        vb = _randn((w.h_kv, w.n_kv, w.head_dim), gen, device)
        _add_block_structure(w, kb, gen, device)
        k[b] = kb.to(dt)
        v[b] = vb.to(dt)
        del kb, vb
    return q, k, v


def shrink(w: Workload, *, n: Optional[int] = None, batch: Optional[int] = None,
           h_q: Optional[int] = None, h_kv: Optional[int] = None,
           name: Optional[str] = None) -> Workload:
    """A smaller workload with the same recipe (used by parity tests that the
    oracle must finish in seconds)."""
    kw = {}
    if n is not None:
        kw["n_kv"] = n
        kw["n_q"] = 1 if w.n_q == 1 else n
    if batch is not None:
        kw["batch"] = batch
    if h_q is not None:
        kw["h_q"] = h_q
    if h_kv is not None:
        kw["h_kv"] = h_kv
    kw["name"] = name or (w.name + "_small")
    return w.replace(**kw)


def random_chunk_lists(batch: int, h_kv: int, n_q: int, n_kv: int, block: int, sparsity: float,
                       device="cpu", seed: int = 0, bias_sigma: float = 0.0):
    """Randomised attended-chunk lists in the Stage-1 output format, the stand-in
    for the kernel benchmark of the paper (App. B.2: the Stage-2 block mask is
    randomised to a target sparsity).  Query t sits at position n_kv - n_q + t;
    every complete chunk before its own is kept independently with probability
    1 - sparsity, its own (diagonal) chunk always.  Returns (mask int32
    [batch,h_kv,n_q,words], cnt int32 [batch,h_kv,n_q], bias fp32
    [batch,h_kv,n_q,t_all]): bias holds N(0, bias_sigma^2) draws for the kept
    chunks in ascending chunk order and 0 for the diagonal chunk, which comes last.
    """
    gen = _gen(device, seed)
    t_all = (n_kv + block - 1) // block
    words = (t_all + 31) // 32
    pos = torch.arange(n_q, device=device) + (n_kv - n_q)
    c_i = (pos // block).view(1, 1, n_q, 1)
    c = torch.arange(words * 32, device=device).view(1, 1, 1, -1)
    keep = torch.rand((batch, h_kv, n_q, words * 32), generator=gen, device=device) >= sparsity
    bits = (keep & (c < c_i)) | (c == c_i)
    cnt = bits.sum(-1).to(torch.int32)
    shifts = torch.arange(32, device=device, dtype=torch.int64)
    packed = (bits.view(batch, h_kv, n_q, words, 32).to(torch.int64) << shifts).sum(-1)
    mask = torch.where(packed >= 2 ** 31, packed - 2 ** 32, packed).to(torch.int32)
    bias = torch.zeros((batch, h_kv, n_q, t_all), dtype=torch.float32, device=device)
    if bias_sigma > 0.0:
        dense = torch.randn((batch, h_kv, n_q, words * 32), generator=gen, device=device) * bias_sigma
        dense = torch.where(c == c_i, torch.zeros_like(dense), dense)
        order = torch.argsort((~bits).to(torch.int8), dim=-1, stable=True)     # kept chunks first, ascending
        bias = torch.gather(dense, -1, order)[..., :t_all].contiguous()
        rank = torch.arange(t_all, device=device).view(1, 1, 1, -1)
        bias = torch.where(rank < cnt.unsqueeze(-1), bias, torch.zeros_like(bias))
    return mask, cnt, bias
