"""The seeded synthetic generators (no GPU): what the recipe promises about the tensors it hands to
both the oracle and the kernels."""
import numpy as np
import torch

from paper_2605_18753_amd.inputs import C1, Workload, make_inputs, random_chunk_lists


def test_same_seed_same_bits_and_block_offsets_shift_the_chunk_means():
    w = Workload("g", 1, 2, 1, 1024, 1024, 64, 64, dtype="fp32", offset_sigma=0.5, seed=3)
    q1, k1, v1 = make_inputs(w)
    q2, k2, v2 = make_inputs(w)
    assert torch.equal(q1, q2) and torch.equal(k1, k2) and torch.equal(v1, v2)
    means = k1[0, 0].view(16, 64, 64).mean(dim=1)          # [chunk, d]
    # a chunk mean of 64 N(0,1) keys has std 1/8 per element; the shared offset adds N(0, 0.25)
    assert 0.4 < means.std().item() < 0.7
    assert abs(v1.mean().item()) < 0.02 and abs(v1.std().item() - 1.0) < 0.02   # V gets no offset


def test_correlated_queries_are_a_unit_variance_ar1_process():
    rho = 0.9
    w = Workload("c", 1, 2, 1, 6000, 6000, 64, 64, dtype="fp32", query_corr=rho, seed=1)
    q, _, _ = make_inputs(w)
    x = q[0, 0].double().numpy()
    var = x.var()
    assert abs(var - 1.0) < 0.03
    for lag in (1, 2, 5):
        c = (x[lag:] * x[:-lag]).mean() / var
        assert abs(c - rho ** lag) < 0.02, (lag, c)
    assert abs((x[400:] * x[:-400]).mean()) < 0.02
    # rho = 0 is the independent recipe itself, bit for bit
    w0 = w.replace(query_corr=0.0)
    assert torch.equal(make_inputs(w0)[0], make_inputs(w0.replace(name="other"))[0])


def test_random_chunk_lists_hit_the_target_sparsity_and_keep_the_diagonal():
    mask, cnt, bias = random_chunk_lists(1, 2, 512, 4096, 64, 0.75, seed=4)
    m = mask.numpy().astype(np.uint32)
    bits = np.unpackbits(m.view(np.uint8), axis=-1, bitorder="little")[..., :64]
    pos = np.arange(512) + 4096 - 512
    diag = pos // 64
    assert all(bits[0, r, i, diag[i]] == 1 for r in range(2) for i in range(512))
    causal = sum(int(d) for d in diag) * 2                     # complete chunks before the diagonal one
    kept = int(bits.sum()) - 2 * 512
    assert abs(kept / causal - 0.25) < 0.01
    assert np.array_equal(bits.sum(-1), cnt.numpy())
    above = np.arange(64)[None, None, None, :] > diag[None, None, :, None]
    assert bits[np.broadcast_to(above, bits.shape)].sum() == 0


def test_the_single_head_configuration_is_what_it_says():
    q, k, v = make_inputs(C1)
    assert q.shape == (1, 1, 1024, 64) and k.shape == (1, 1, 1024, 64) and q.dtype == torch.float32
