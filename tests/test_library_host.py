"""CPU-side tests of the C-ABI library: it loads, exports every symbol the header
declares, sizes its workspace, and rejects bad arguments before touching a GPU."""
import ctypes
import os
import re

import pytest

from paper_2605_18753_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def params(**kw):
    p = B.dash_params()
    base = dict(batch=1, h_q=8, h_kv=2, n_q=1024, n_kv=1024, head_dim=128, block_size=64, causal=1,
                dtype=B.DASH_BF16, alpha=1.5, gamma=1.0, sigma=1.0, scale=0.0)
    base.update(kw)
    for k, v in base.items():
        setattr(p, k, v)
    for name, heads, n in (("q_stride", p.h_q, p.n_q), ("k_stride", p.h_kv, p.n_kv),
                           ("v_stride", p.h_kv, p.n_kv), ("o_stride", p.h_q, p.n_q)):
        getattr(p, name)[:] = [heads * n * p.head_dim, n * p.head_dim, p.head_dim]
    return p


def header_functions():
    text = open(os.path.join(ROOT, "include", "dash_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b(dash_\w+|dense_attn)\s*\(", text))


def test_library_exports_every_declared_symbol():
    lib = B.load_library()
    names = header_functions()
    assert {"dash_attn_prefill", "dash_attn_decode", "dense_attn", "dash_kbar_compress",
            "dash_kbar_summarize"} <= names
    for n in names:
        assert hasattr(lib, n), n
    assert names == set(B.exported_symbols())


def test_workspace_and_list_sizes():
    p = params()
    assert B.list_stride(p) == 16 and B.mask_words(p) == 1
    n = B.workspace_bytes(p)
    rows = 2 * 1024
    assert n >= rows * 16 * 4 + rows * 4 + 2 * 16 * 3 * 128 * 2
    p2 = params(n_q=1000, n_kv=1000)          # ragged tail: 15 complete chunks + 1 partial
    assert B.list_stride(p2) == 16
    pd = params(n_q=1, n_kv=131072, batch=16, h_q=32, h_kv=8)
    assert B.list_stride(pd) == 2048 and B.mask_words(pd) == 64
    # a decode step keeps its scores on chip: the bias lists and the split-KV partials are what it needs
    assert 16 * 8 * 2048 * 4 < B.workspace_bytes(pd) < 16 * 32 * 2047 * 4


@pytest.mark.parametrize("kw,code", [
    (dict(h_q=7), -1), (dict(alpha=1.0), -1), (dict(alpha=0.5), -1), (dict(sigma=0.0), -1),
    (dict(gamma=-1.0), -1), (dict(batch=0), -1), (dict(n_q=2048), -1), (dict(causal=2), -1),
    (dict(dtype=3), -1), (dict(causal=0, n_q=1000, n_kv=1000), -1),
    (dict(window=-1), -1), (dict(window=9), -1), (dict(window=1, causal=0), -1),
    (dict(head_dim=96), -2), (dict(block_size=32), -2), (dict(h_q=64, h_kv=2), -2),
    (dict(n_q=100, n_kv=1001), -2), (dict(n_q=262144, n_kv=262144), -2),
])
def test_invalid_parameters_are_rejected(kw, code):
    lib = B.load_library()
    p = params(**kw)
    # every compute entry point rejects the same way, before any launch
    assert lib.dash_attn_prefill(ctypes.byref(p), 256, 256, 256, 256, 256, None, None, None, None, None,
                                 256, 1 << 40, None) == code
    assert lib.dash_stage1_route(ctypes.byref(p), 256, 256, None, None, None, None, None,
                                 256, 1 << 40, None) == code
    if not (kw.get("causal") == 0 and len(kw) == 3):     # ragged non-causal is fine for dense
        n = ctypes.c_size_t(0)
        assert lib.dash_attn_workspace_bytes(ctypes.byref(p), ctypes.byref(n)) == code
        assert lib.dense_attn(ctypes.byref(p), 1, 1, 1, 1, 256, 1 << 40, None) == code


def test_null_and_workspace_errors():
    lib = B.load_library()
    p = params()
    need = B.workspace_bytes(p)
    assert lib.dense_attn(ctypes.byref(p), None, 1, 1, 1, 256, need, None) == -1
    assert lib.dense_attn(ctypes.byref(p), 256, 256, 256, 256, None, need, None) == -3
    assert lib.dense_attn(ctypes.byref(p), 256, 256, 256, 256, 256, need - 1, None) == -3
    assert lib.dense_attn(ctypes.byref(p), 256, 256, 256, 256, 257, need, None) == -3     # misaligned
    assert lib.dash_attn_prefill(ctypes.byref(p), 256, 256, 256, 256, None, None, None, None, None, None,
                                 256, need, None) == -1                                  # kbar is required
    assert lib.dash_attn_decode(ctypes.byref(p), 256, 256, 256, 256, 256, None, None, None, None, None,
                                256, need, None) == -1                                   # n_q must be 1
    assert lib.dash_attn_workspace_bytes(None, None) == -1
    p.q_stride[2] = 100                                                                    # misaligned rows
    assert lib.dense_attn(ctypes.byref(p), 256, 256, 256, 256, 256, need, None) == -1


def test_summarize_argument_errors():
    lib = B.load_library()
    p = params()
    ok = (ctypes.c_int64 * 3)(0, 128, 0)
    assert lib.dash_kbar_summarize(ctypes.byref(p), 256, None, ok, 256, 0, -1, None) == -1     # no query
    assert lib.dash_kbar_summarize(ctypes.byref(p), 256, 256, None, 256, 0, -1, None) == -1    # no strides
    assert lib.dash_kbar_summarize(ctypes.byref(p), 256, 264, ok, 256, 0, -1, None) == -1      # query not 16-byte aligned
    assert lib.dash_kbar_summarize(ctypes.byref(p), 256, 256, (ctypes.c_int64 * 3)(0, 100, 0), 256, 0, -1,
                                   None) == -1                                                # stride not a multiple of 8
    assert lib.dash_kbar_summarize(ctypes.byref(p), 256, 256, (ctypes.c_int64 * 3)(0, -128, 0), 256, 0, -1,
                                   None) == -1
    assert lib.dash_kbar_summarize(ctypes.byref(p), 256, 256, ok, 256, 15, 2, None) == -1      # 16 chunks: 15..16
    assert lib.dash_kbar_summarize(ctypes.byref(p), 256, 256, ok, 256, 3, 0, None) == 0        # empty range: nothing to do
    assert lib.dash_kbar_compress(ctypes.byref(p), 256, 256, 15, 2, None) == -1


def test_ragged_decode_argument_errors():
    lib = B.load_library()
    p = params(n_q=1, n_kv=4096)
    need = B.workspace_bytes(p)
    args = (256, 256, 256, 256)
    assert lib.dash_attn_decode_ragged(ctypes.byref(p), *args, None, 1, 256, None, None, None, None, None,
                                       256, need, None) == -1                            # no lengths
    p32 = params(n_q=1, n_kv=4096, dtype=0)
    assert lib.dash_attn_decode_ragged(ctypes.byref(p32), *args, 256, 1, 256, None, None, None, None, None,
                                       256, 1 << 40, None) == -2                          # bf16 only
    pq = params(n_q=64, n_kv=4096)
    assert lib.dash_attn_decode_ragged(ctypes.byref(pq), *args, 256, 1, 256, None, None, None, None, None,
                                       256, 1 << 40, None) == -1                          # one query per sequence


def test_backward_argument_errors():
    lib = B.load_library()
    p = params()
    need = B.backward_workspace_bytes(p)
    assert need > 2 * 8 * 1024 * 4 + 8 * 1024 * 128 * 4
    ptrs = [256] * 12          # q k v d_o kbar mask bias tau dq dk dv dkbar
    for i in range(11):          # the last one (dkbar) is optional
        bad = list(ptrs)
        bad[i] = None
        assert lib.dash_attn_backward(ctypes.byref(p), *bad, 256, need, None) == -1, i
    assert lib.dash_attn_backward(ctypes.byref(p), *ptrs, None, need, None) == -3
    assert lib.dash_attn_backward(ctypes.byref(p), *ptrs, 256, need - 1, None) == -3
    assert lib.dash_attn_backward(ctypes.byref(p), *ptrs, 257, need, None) == -3
    n = ctypes.c_size_t(0)
    pu = params(n_q=512, n_kv=1024)                                 # a chunked prefill
    assert lib.dash_attn_backward_workspace_bytes(ctypes.byref(pu), ctypes.byref(n)) == -2
    assert lib.dash_attn_backward(ctypes.byref(pu), *ptrs, 256, 1 << 40, None) == -2
    assert lib.dash_attn_backward_workspace_bytes(ctypes.byref(params(dtype=0)), ctypes.byref(n)) == 0   # fp32 tensors
    assert n.value == need
    assert lib.dash_attn_backward_workspace_bytes(ctypes.byref(p), None) == -1
    big = params(h_q=16, h_kv=1, n_q=131072, n_kv=131072)          # a 16-head slice of q spans 512 MiB: fine
    assert lib.dash_attn_backward_workspace_bytes(ctypes.byref(big), ctypes.byref(n)) == 0
    far = params()
    far.q_stride[1] = 1 << 31                                       # heads 4 GiB apart: 32-bit offsets do not reach
    assert lib.dash_attn_backward_workspace_bytes(ctypes.byref(far), ctypes.byref(n)) == -2


def test_forward_rejects_slices_beyond_32_bit_offsets():
    """The bf16 kernels address one (batch, kv-head) slice of a tensor with 32-bit byte offsets:
    a token-major cache whose slice spans 2 GiB or more is refused by every forward entry point
    (fp32 tensors use 64-bit offsets and are accepted)."""
    lib = B.load_library()
    n = ctypes.c_size_t(0)
    ok = params(n_q=1, n_kv=131072, batch=16, h_q=32, h_kv=8)
    ok.k_stride[2] = ok.v_stride[2] = 8 * 128                     # [batch, token, head, d]: 268 MB per slice
    ok.k_stride[1] = ok.v_stride[1] = 128
    assert lib.dash_attn_workspace_bytes(ctypes.byref(ok), ctypes.byref(n)) == 0
    for name in ("k_stride", "v_stride", "q_stride", "o_stride"):
        wide = params(n_q=8192, n_kv=8192)
        getattr(wide, name)[2] = 1 << 18                           # 8191 * 512 KiB + 256 B >= 2 GiB
        assert lib.dash_attn_workspace_bytes(ctypes.byref(wide), ctypes.byref(n)) == -2, name
        assert lib.dash_attn_prefill(ctypes.byref(wide), 256, 256, 256, 256, 256, None, None, None, None, None,
                                     256, 1 << 40, None) == -2, name
        assert lib.dense_attn(ctypes.byref(wide), 256, 256, 256, 256, 256, 1 << 40, None) == -2, name
        assert lib.dash_stage2_attend(ctypes.byref(wide), 256, 256, 256, 256, None, None, 256, 1 << 40, None) == -2
        wide.dtype = 0                                             # fp32: plain 64-bit pointers
        getattr(wide, name)[2] = 1 << 18
        assert lib.dash_attn_workspace_bytes(ctypes.byref(wide), ctypes.byref(n)) == 0, name
    dec = params(n_q=1, n_kv=131072, batch=2, h_q=8, h_kv=2)
    dec.k_stride[2] = 1 << 14                                      # 131071 * 32 KiB >= 2 GiB
    assert lib.dash_attn_decode(ctypes.byref(dec), 256, 256, 256, 256, 256, None, None, None, None, None,
                                256, 1 << 40, None) == -2
    heads = params()
    heads.q_stride[1] = 1 << 30                                    # the 4 query heads of a kv-head 2 GiB apart
    assert lib.dash_attn_workspace_bytes(ctypes.byref(heads), ctypes.byref(n)) == -2


def test_backward_is_refused_above_the_alpha_it_is_checked_to():
    lib = B.load_library()
    n = ctypes.c_size_t(0)
    assert lib.dash_attn_backward_workspace_bytes(ctypes.byref(params(alpha=3.0)), ctypes.byref(n)) == 0
    assert lib.dash_attn_backward_workspace_bytes(ctypes.byref(params(alpha=4.0)), ctypes.byref(n)) == -2
    assert lib.dash_attn_backward(ctypes.byref(params(alpha=4.0)), *([256] * 12), 256, 1 << 40, None) == -2
    # the forward has no such limit
    assert lib.dash_attn_workspace_bytes(ctypes.byref(params(alpha=4.0)), ctypes.byref(n)) == 0


def test_the_library_reads_no_environment_variable():
    """Behaviour depends on the arguments alone: the sources call no getenv."""
    csrc = os.path.join(ROOT, "paper_2605_18753_amd", "csrc")
    for f in os.listdir(csrc):
        if f.endswith((".hip", ".h")):
            assert "getenv" not in open(os.path.join(csrc, f)).read(), f


def test_summarize_backward_argument_errors():
    lib = B.load_library()
    p = params()
    ok = (ctypes.c_int64 * 3)(0, 128, 0)
    good = [256, 256, ok, 256, 256, 256]         # k qbar strides dkbar dk dqbar
    for i in range(6):
        bad = list(good)
        bad[i] = None
        assert lib.dash_kbar_summarize_backward(ctypes.byref(p), *bad, None) == -1, i
    assert lib.dash_kbar_summarize_backward(ctypes.byref(p), 256, 264, ok, 256, 256, 256, None) == -1   # alignment
    assert lib.dash_kbar_summarize_backward(ctypes.byref(p), 256, 256, (ctypes.c_int64 * 3)(0, 100, 0), 256, 256,
                                            256, None) == -1


def test_strerror():
    lib = B.load_library()
    assert lib.dash_strerror(0) == b"ok"
    for c in (-1, -2, -3, -4, 17):
        assert len(lib.dash_strerror(c)) > 0


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asking for more must end with a message, before anything touches a GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
