"""dash_attn_decode_static (the entry point that allocates nothing: scratch inside the library)
against dash_attn_decode on a caller-provided workspace: same kernels, so the outputs and the
lists must agree bit for bit, on two calls in a row, the second on a smaller input (the scratch
keeps the first call's contents)."""
import ctypes

import pytest
import torch

from paper_2605_18753_amd import binding as B
from paper_2605_18753_amd.inputs import Workload, make_inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def one_step(w, static):
    q, k, v = (t.to(DEV) for t in make_inputs(w, "cpu"))
    o = torch.full_like(q, float("nan"))
    p = B.make_params(q, k, v, o, w.block, w.alpha, w.gamma, w.sigma, True, window=w.window)
    kbar = torch.empty(B.kbar_shape(p), dtype=torch.float32, device=DEV)
    B.dash_kbar_compress(p, k, kbar)
    lists = B.Lists.allocate(p, DEV)
    if static:
        B.dash_attn_decode_static(p, q, k, v, kbar, o, lists)
    else:
        B.dash_attn_decode(p, q, k, v, kbar, o, lists, B.alloc_workspace(p, DEV))
    torch.cuda.synchronize()
    return o, lists


@pytest.mark.parametrize("with_lists", [True, False])
def test_decode_on_the_built_in_scratch_equals_decode_on_a_workspace(with_lists):
    big = Workload("static_big", 4, 16, 4, 1, 9000, 128, 64, offset_sigma=0.7, seed=31)
    small = Workload("static_small", 2, 8, 2, 1, 1500, 128, 64, offset_sigma=0.7, seed=32, gamma=0.5)
    for w in (big, small):                       # two calls in a row, the second smaller
        want_o, want_l = one_step(w, static=False)
        if with_lists:
            got_o, got_l = one_step(w, static=True)
            for name in ("mask", "cnt", "idx", "bias", "tau"):
                assert torch.equal(getattr(got_l, name), getattr(want_l, name)), (w.name, name)
        else:
            # lists not asked for: they live in the scratch too
            q, k, v = (t.to(DEV) for t in make_inputs(w, "cpu"))
            got_o = torch.full_like(q, float("nan"))
            p = B.make_params(q, k, v, got_o, w.block, w.alpha, w.gamma, w.sigma, True)
            kbar = torch.empty(B.kbar_shape(p), dtype=torch.float32, device=DEV)
            B.dash_kbar_compress(p, k, kbar)
            B.dash_attn_decode_static(p, q, k, v, kbar, got_o, B.Lists())
            torch.cuda.synchronize()
        assert torch.isfinite(got_o.float()).all()
        assert torch.equal(got_o, want_o), w.name


def test_static_decode_rejects_what_does_not_fit():
    # 512 sequences x 8 kv-heads at 128k tokens: the bias lists alone exceed 8 MiB
    lib = B.load_library()
    p = B.dash_params()
    for k_, v_ in dict(batch=512, h_q=32, h_kv=8, n_q=1, n_kv=131072, head_dim=128, block_size=64, causal=1,
                       dtype=B.DASH_BF16, alpha=1.5, gamma=1.0, sigma=1.0, scale=0.0).items():
        setattr(p, k_, v_)
    for name, heads, n in (("q_stride", 32, 1), ("k_stride", 8, 131072), ("v_stride", 8, 131072), ("o_stride", 32, 1)):
        getattr(p, name)[:] = [heads * n * 128, n * 128, 128]
    assert B.workspace_bytes(p) > 8 << 20
    assert lib.dash_attn_decode_static(ctypes.byref(p), 256, 256, 256, 256, 256, None, None, None, None, None, None) == -3
