"""Pins for the oracle's Stage 0 / Stage 1 / Stage 2 and the whole path.

Checked against: the plain definition (mean), Proposition 1 (literal prior
form == bias form), the limits the paper states (sigma->inf, gamma->0), a
library attention routine, and symmetry properties.
"""
import math

import numpy as np
import pytest
import torch
from scipy import special

from oracle import dash_oracle as orc


def make(seed, B=1, hq=4, hkv=2, n=200, d=16, block=16, off=0.7):
    r = np.random.default_rng(seed)
    q = r.normal(size=(B, hq, n, d))
    k = r.normal(size=(B, hkv, n, d))
    v = r.normal(size=(B, hkv, n, d))
    nb = -(-n // block)
    o = r.normal(size=(B, hkv, nb, d)) * off
    k = k + np.repeat(o, block, axis=2)[:, :, :n]
    return q, k, v


# ---------------------------------------------------------------- Stage 0
def test_block_mean_is_plain_mean_of_own_chunk():
    r = np.random.default_rng(0)
    k = r.normal(size=(2, 3, 150, 8)).astype(np.float32)
    kb = orc.block_mean_summaries(k, 32)
    assert kb.shape == (2, 3, 4, 8)           # floor(150/32) complete chunks
    for c in range(4):
        want = k[:, :, 32 * c:32 * (c + 1)].astype(np.float64).mean(axis=2)
        assert np.array_equal(kb[:, :, c], want.astype(np.float32).astype(np.float64))
    k2 = k.copy(); k2[:, :, 40] += 5.0        # only chunk 1 may change
    kb2 = orc.block_mean_summaries(k2, 32)
    assert np.array_equal(kb2[:, :, [0, 2, 3]], kb[:, :, [0, 2, 3]])
    assert not np.array_equal(kb2[:, :, 1], kb[:, :, 1])
    # constant chunk -> the constant
    assert np.array_equal(orc.block_mean_summaries(np.full((64, 4), 0.375), 64), np.full((1, 4), 0.375))


# ---------------------------------------------------------------- Stage 1
def test_gqa_average_support_is_union_and_sums_to_one():
    r = np.random.default_rng(1)
    qh = r.normal(size=(4, 16)); kb = r.normal(size=(40, 16)) * 2
    x, tau, w_hat, w = orc.route_token(qh, kb, 1.5, 1.0, 0.25)
    assert abs(w.sum() - 1.0) < 1e-12
    union = np.zeros(40, bool)
    for h in range(4):
        assert abs(w_hat[h].sum() - 1.0) < 1e-12
        union |= w_hat[h] > 0
        # scores follow the definition gamma (alpha-1) <q,kbar> scale
        assert np.allclose(x[h], 0.5 * (kb @ qh[h]) * 0.25)
        assert np.array_equal(w_hat[h] > 0, x[h] > tau[h])
    assert np.array_equal(w > 0, union)
    # group of one head reduces to plain entmax of gamma*zbar
    x1, _, _, w1 = orc.route_token(qh[:1], kb, 1.5, 0.7, 0.25)
    assert np.allclose(w1, orc.entmax(0.7 * (kb @ qh[0]) * 0.25, 1.5), atol=1e-14)


def test_prior_bias_definition():
    w = np.array([0.0, 0.5, 0.0, 0.125, 0.375])
    routed, d = orc.prior_bias(w, 4.0)
    assert routed.tolist() == [1, 3, 4]
    mu = (math.log(0.5) + math.log(0.125) + math.log(0.375)) / 3
    assert np.allclose(d, [(math.log(0.5) - mu) / 4, (math.log(0.125) - mu) / 4,
                           (math.log(0.375) - mu) / 4])
    assert abs(d.sum()) < 1e-15      # biases are centred on the routed set


# ---------------------------------------------------------------- Stage 2
@pytest.mark.parametrize("sigma", [0.5, 1.0, 10.0, 1e4])
@pytest.mark.parametrize("causal", [True, False])
def test_proposition1_literal_prior_equals_bias_form(sigma, causal):
    r = np.random.default_rng(2)
    block, d, n = 8, 8, 80
    k = r.normal(size=(n, d)); v = r.normal(size=(n, d)); qh = r.normal(size=(2, d))
    w = orc.entmax(r.normal(size=9) * 3, 1.5)            # 9 complete candidate chunks
    assert 0 < np.sum(w > 0) < 9
    diag = (72, 77) if causal else (0, 0)
    routed, bias = orc.prior_bias(w, sigma)
    a = orc.attend_bias_form(qh, k, v, 0.3, block, routed, bias, *diag)
    b = orc.attend_literal(qh, k, v, 0.3, block, w, sigma, *diag)
    assert np.allclose(a, b, rtol=0, atol=1e-12)


def test_prior_is_a_distribution_with_mass_lambda_on_routed():
    w = orc.entmax(np.array([0.1, 2.0, -1.0, 1.5, 1.7]), 1.5)
    block, n_diag = 8, 5
    routed, g_r, g_d, lam = orc.prior_literal(w, 3.0, block, n_diag)
    assert abs(block * g_r.sum() + n_diag * g_d - 1.0) < 1e-14
    assert abs(block * g_r.sum() - lam) < 1e-14
    # sigma -> inf: lambda -> |R| / (|R| + |D|) counted in tokens
    _, _, _, lam_inf = orc.prior_literal(w, 1e14, block, n_diag)
    nr = routed.size * block
    assert abs(lam_inf - nr / (nr + n_diag)) < 1e-9


def test_sigma_to_infinity_is_masked_softmax():
    q, k, v = make(3)
    prm = orc.DashParams(block=16, sigma=1e14)
    kb = orc.block_mean_summaries(k, 16)
    for iq in (37, 150, 199):
        rr = orc.dash_row(q, k, v, kb, prm, 0, 1, iq)
        keep = np.zeros(200, bool)
        for c in rr.routed:
            keep[16 * c:16 * (c + 1)] = True
        keep[rr.diag[0]:rr.diag[1]] = True
        for hh in range(2):
            z = (k[0, 1] @ q[0, 2 + hh, iq]) / 4.0
            z[~keep] = -np.inf
            want = special.softmax(z) @ v[0, 1]
            assert np.allclose(rr.o[hh], want, atol=1e-10)


def test_sigma_one_noncausal_is_weight_times_exp():
    q, k, v = make(4, n=128)
    prm = orc.DashParams(block=16, sigma=1.0, causal=False)
    kb = orc.block_mean_summaries(k, 16)
    rr = orc.dash_row(q, k, v, kb, prm, 0, 0, 5)
    assert rr.n_cand == 8 and rr.diag == (0, 0)
    wtok = np.repeat(rr.w, 16)
    for hh in range(2):
        e = wtok * np.exp((k[0, 0] @ q[0, hh, 5]) / 4.0)
        assert np.allclose(rr.o[hh], (e @ v[0, 0]) / e.sum(), atol=1e-12)


def test_dense_attention_matches_library_sdpa():
    r = np.random.default_rng(5)
    q = r.normal(size=(37, 16)); k = r.normal(size=(37, 16)); v = r.normal(size=(37, 16))
    for causal in (True, False):
        mine = orc.dense_attention(q, k, v, 0.25, causal)
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None],
            is_causal=causal, scale=0.25)[0].numpy()
        assert np.allclose(mine, ref, atol=1e-12)


def test_gamma_to_zero_recovers_dense_causal_attention():
    q, k, v = make(6, n=150)
    prm = orc.DashParams(block=16, gamma=1e-9, sigma=0.5)
    out, kb, res = orc.dash_forward_full(q, k, v, prm)
    for rr in res:
        assert rr.routed.size == rr.n_cand          # nothing pruned
        assert np.all(np.abs(rr.bias) < 1e-6)
    for h in range(4):
        want = orc.dense_attention(q[0, h], k[0, h // 2], v[0, h // 2], 0.25, True)
        assert np.allclose(out[0, h], want, atol=1e-6)


def test_first_chunk_rows_are_causal_softmax_inside_the_chunk():
    q, k, v = make(7, n=64)
    prm = orc.DashParams(block=16)
    kb = orc.block_mean_summaries(k, 16)
    rr0 = orc.dash_row(q, k, v, kb, prm, 0, 0, 0)
    assert rr0.n_cand == 0 and np.allclose(rr0.o, v[0, 0, 0][None].repeat(2, 0))
    rr = orc.dash_row(q, k, v, kb, prm, 0, 0, 11)
    want = orc.dense_attention(q[0, :2, 11], k[0, 0, :12], v[0, 0, :12], 0.25, False)
    assert np.allclose(rr.o, want, atol=1e-13)


def test_decode_position_and_candidates():
    # one query against a cache of 100 tokens, block 16: position 99, chunk 6,
    # candidates 0..5, diagonal tokens 96..99
    q, k, v = make(8, n=100)
    qd = q[:, :, 99:100]
    kb = orc.block_mean_summaries(k, 16)
    rr = orc.dash_row(qd, k, v, kb, orc.DashParams(block=16), 0, 1, 0)
    assert rr.pos == 99 and rr.n_cand == 6 and rr.diag == (96, 100)
    full = orc.dash_row(q, k, v, kb, orc.DashParams(block=16), 0, 1, 99)
    assert np.array_equal(rr.o, full.o)
    # a query at the last slot of a chunk: the whole chunk is the diagonal branch
    rr2 = orc.dash_row(q[:, :, 95:96], k[:, :, :96], v[:, :, :96],
                       orc.block_mean_summaries(k[:, :, :96], 16), orc.DashParams(block=16), 0, 0, 0)
    assert rr2.n_cand == 5 and rr2.diag == (80, 96)


def test_permuting_candidate_blocks_leaves_output_unchanged():
    q, k, v = make(9, n=200)
    prm = orc.DashParams(block=16, sigma=2.0)
    iq = 190                                      # chunk 11; candidates 0..10
    base = orc.dash_row(q, k, v, orc.block_mean_summaries(k, 16), prm, 0, 0, iq)
    perm = np.random.default_rng(0).permutation(11)
    k2, v2 = k.copy(), v.copy()
    for dst, src in enumerate(perm):
        k2[:, :, 16 * dst:16 * (dst + 1)] = k[:, :, 16 * src:16 * (src + 1)]
        v2[:, :, 16 * dst:16 * (dst + 1)] = v[:, :, 16 * src:16 * (src + 1)]
    moved = orc.dash_row(q, k2, v2, orc.block_mean_summaries(k2, 16), prm, 0, 0, iq)
    assert np.allclose(moved.o, base.o, atol=1e-12)
    assert sorted(perm[moved.routed].tolist()) == base.routed.tolist()


def test_routing_is_sparse_and_query_dependent_on_the_recipe():
    q, k, v = make(10, n=640, off=1.0)
    out, kb, res = orc.dash_forward_full(q[:, :, -40:], k, v, orc.DashParams(block=16))
    sizes = {rr.routed.size for rr in res}
    assert len(sizes) > 3                          # variable number of kept blocks
    assert all(rr.routed.size < rr.n_cand for rr in res)


# --------------------------------------------------------------------------
# Stage 0 with a learned summary query (Eq. 3; Alg. 1)
# --------------------------------------------------------------------------
def _bf16_round(x):
    """Round fp64/fp32 values to bf16 (round to nearest even) and return fp64."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def test_learned_summary_zero_query_is_block_mean_bit_for_bit():
    # Sec. 3.1: at initialisation the inner products are zero and the local softmax is uniform pooling
    rng = np.random.default_rng(11)
    k = _bf16_round(rng.standard_normal((2, 3, 200, 16)))
    a = orc.local_attention_summaries(k, np.zeros((3, 1, 16)), 64)
    b = orc.block_mean_summaries(k, 64)
    assert a.shape == (2, 3, 3, 16)
    assert np.array_equal(a, b)


def test_learned_summary_equals_library_softmax_attention_per_chunk():
    # Eq. 3 is one SDPA of the summary query over the chunk, keys as values: a library softmax and a matmul
    from scipy.special import softmax
    rng = np.random.default_rng(12)
    k = rng.standard_normal((2, 130, 8))
    qbar = rng.standard_normal((2, 2, 8)) * 2.0          # [h_kv, T_c, d]: one query per chunk (Alg. 1)
    got = orc.local_attention_summaries(k, qbar, 64)
    for r in range(2):
        for c in range(2):
            keys = k[r, c * 64:(c + 1) * 64]
            w = softmax(keys @ qbar[r, c] / np.sqrt(8.0))
            ref = (w[None, :] @ keys)[0]
            assert np.allclose(got[r, c], ref, rtol=0, atol=1e-6)   # fp32 rounding of the cache
    # a transposed operand or a sum over the wrong axis would break the shape or this value
    assert got.shape == (2, 2, 8)


def test_learned_summary_sharp_query_selects_the_best_matching_key():
    rng = np.random.default_rng(13)
    k = rng.standard_normal((1, 64, 8))
    t_star = 17
    qbar = 400.0 * k[0, t_star]                          # overwhelming weight on one key
    s = k[0] @ qbar
    assert int(np.argmax(s)) == t_star
    got = orc.local_attention_summaries(k, qbar[None, None, :], 64)
    assert np.allclose(got[0, 0], k[0, t_star].astype(np.float32), atol=1e-6)


def test_learned_summary_is_a_convex_combination_and_shift_equivariant():
    rng = np.random.default_rng(14)
    k = rng.standard_normal((3, 128, 8))
    qbar = rng.standard_normal((3, 1, 8))
    got = orc.local_attention_summaries(k, qbar, 32)
    body = k.reshape(3, 4, 32, 8)
    assert np.all(got <= body.max(axis=2) + 1e-6) and np.all(got >= body.min(axis=2) - 1e-6)
    # adding one vector u to every key shifts all scores of a chunk by <qbar,u>/sqrt(d), which the
    # softmax ignores, and shifts the summary by u
    u = rng.standard_normal(8)
    got2 = orc.local_attention_summaries(k + u, qbar, 32)
    assert np.allclose(got2, got + u, atol=2e-6)
    # the scale multiplies the logits: scale 0 is uniform pooling whatever the query
    got0 = orc.local_attention_summaries(k, qbar, 32, scale=0.0)
    assert np.allclose(got0, body.mean(axis=2), atol=1e-6)


# --------------------------------------------------------------------------
# local window of always-attended chunks (App. B.1: the diagonal block and the last block)
# --------------------------------------------------------------------------
def _window_case(seed=21, n=160, d=8, blk=16, g=2):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((g, d))
    k = rng.standard_normal((n, d)) + np.repeat(rng.standard_normal((n // blk, d)), blk, axis=0)
    v = rng.standard_normal((n, d))
    return q, k, v, orc.block_mean_summaries(k, blk)


def test_window_moves_chunks_from_the_candidates_to_the_local_branch():
    q, k, v, kb = _window_case()
    pos = 150                                              # chunk 9 of 10
    r0 = orc.dash_row_at(q, k, v, kb, orc.DashParams(block=16), pos)
    r1 = orc.dash_row_at(q, k, v, kb, orc.DashParams(block=16, window=1), pos)
    r2 = orc.dash_row_at(q, k, v, kb, orc.DashParams(block=16, window=2), pos)
    assert (r0.n_cand, r1.n_cand, r2.n_cand) == (9, 8, 7)
    assert r1.diag == (8 * 16, pos + 1) and r2.diag == (7 * 16, pos + 1)
    assert all(c < 8 for c in r1.routed) and all(c < 7 for c in r2.routed)
    # the window is capped by the start of the sequence: a query in chunk 1 with W = 2 sees tokens 0..pos
    r = orc.dash_row_at(q, k, v, kb, orc.DashParams(block=16, window=2), 20)
    assert r.n_cand == 0 and r.diag == (0, 21) and r.routed.size == 0


def test_window_rows_without_candidates_are_causal_softmax_over_the_window():
    # with nothing left to route, the row is plain causal attention over the local tokens
    q, k, v, kb = _window_case(seed=22)
    pos = 40                                               # chunk 2; W = 2 covers chunks 0 and 1
    r = orc.dash_row_at(q, k, v, kb, orc.DashParams(block=16, window=2), pos)
    ref = orc.dense_attention(q, k[:pos + 1], v[:pos + 1], 1 / np.sqrt(8.0), False)   # rows = the heads
    assert np.allclose(r.o, ref, atol=1e-12)


def test_window_equals_forcing_the_chunks_by_hand():
    # the windowed row is the bias form over (routed set of the shorter candidate list) + (window and
    # diagonal tokens at bias 0): build that from the parts and compare
    q, k, v, kb = _window_case(seed=23)
    pos = 150
    prm = orc.DashParams(block=16, window=1, sigma=2.0)
    r = orc.dash_row_at(q, k, v, kb, prm, pos)
    x, tau, _, w = orc.route_token(q, kb[:8], prm.alpha, prm.gamma, 1 / np.sqrt(8.0))
    routed, bias = orc.prior_bias(w, prm.sigma)
    o = orc.attend_bias_form(q, k, v, 1 / np.sqrt(8.0), 16, routed, bias, 8 * 16, pos + 1)
    assert np.array_equal(r.routed, routed) and np.allclose(r.o, o, atol=1e-13)
    # and it differs from the windowless row unless chunk 8 happened to be routed with bias 0
    r0 = orc.dash_row_at(q, k, v, kb, orc.DashParams(block=16, sigma=2.0), pos)
    assert np.abs(r0.o - r.o).max() > 1e-6


def test_window_gamma_to_zero_is_dense_causal_attention():
    q, k, v, kb = _window_case(seed=24)
    pos = 150
    r = orc.dash_row_at(q, k, v, kb, orc.DashParams(block=16, window=1, gamma=1e-9), pos)
    ref = orc.dense_attention(q, k[:pos + 1], v[:pos + 1], 1 / np.sqrt(8.0), False)
    assert np.allclose(r.o, ref, atol=1e-7)
