"""Pins for the oracle's multi-query (causal) form: several new tokens per request.  The single-query
oracle is pinned in test_oracle_pins.py; here the multi-query form is tied to it, to brute force and to
a library implementation of masked softmax attention."""
import math

import numpy as np
import pytest
import torch

import oracle
from test_oracle_pins import brute_force, contiguous_problem


def case(seed, B, n, Hq, Hkv, L, d):
    rng = np.random.RandomState(seed)
    q = rng.standard_normal((B, n, Hq, d)).astype(np.float32)
    K = rng.standard_normal((B, Hkv, L, d)).astype(np.float32)
    V = rng.standard_normal((B, Hkv, L, d)).astype(np.float32)
    return q, K, V


@pytest.mark.parametrize("n", [1, 2, 5])
def test_each_query_token_equals_a_single_query_problem_on_its_prefix(n):
    B, Hq, Hkv, L, d, T = 3, 4, 2, 23, 8, 8
    q, K, V = case(1, B, n, Hq, Hkv, L, d)
    kp, vp, table, _ = contiguous_problem(q[:, 0], K, V, T)
    lens = np.array([23, 9, 3], dtype=np.int32)     # request 2: fewer cached tokens than query tokens when n = 5
    out, lse = oracle.attention(q, kp, vp, table, lens, T, 0.4)
    assert out.shape == (B, n, Hq, d) and lse.shape == (B, n, Hq)
    for t in range(n):
        lens_t = np.maximum(lens - (n - 1 - t), 0).astype(np.int32)
        out_t, lse_t = oracle.attention(np.ascontiguousarray(q[:, t]), kp, vp, table, lens_t, T, 0.4)
        assert np.array_equal(out[:, t], out_t) and np.array_equal(lse[:, t], lse_t)
    if n == 5:
        # query tokens 0 and 1 of request 2 sit before the start of a 3-token cache: nothing to attend to
        assert np.all(out[2, :2] == 0) and np.all(np.isneginf(lse[2, :2])) and np.all(np.isfinite(lse[2, 2:]))


def test_brute_force_causal_tiny():
    B, n, Hq, Hkv, L, d, T = 1, 3, 2, 1, 7, 4, 4
    q, K, V = case(2, B, n, Hq, Hkv, L, d)
    kp, vp, table, lens = contiguous_problem(q[:, 0], K, V, T)
    out, lse = oracle.attention(q, kp, vp, table, lens, T, 0.7)
    for t in range(n):
        vis = L - (n - 1 - t)
        for h in range(Hq):
            ref, ref_lse = brute_force([float(x) for x in q[0, t, h]],
                                       [[float(x) for x in row] for row in K[0, 0, :vis]],
                                       [[float(x) for x in row] for row in V[0, 0, :vis]], 0.7)
            np.testing.assert_allclose(out[0, t, h], ref, rtol=1e-13, atol=1e-14)
            assert abs(lse[0, t, h] - ref_lse) < 1e-13


def test_masked_softmax_attention_via_torch():
    B, n, Hq, Hkv, L, d, T = 2, 6, 8, 2, 200, 128, 64
    q, K, V = case(3, B, n, Hq, Hkv, L, d)
    kp, vp, table, lens = contiguous_problem(q[:, 0], K, V, T)
    scale = 1.0 / math.sqrt(d)
    out, lse = oracle.attention(q, kp, vp, table, lens, T, scale, n_threads=4)
    tq = torch.from_numpy(q.astype(np.float64))                                  # [B][n][Hq][d]
    tK = torch.from_numpy(K.astype(np.float64)).repeat_interleave(Hq // Hkv, 1)  # [B][Hq][L][d]
    tV = torch.from_numpy(V.astype(np.float64)).repeat_interleave(Hq // Hkv, 1)
    s = torch.einsum("bnhd,bhld->bnhl", tq, tK) * scale
    pos = torch.arange(L)[None, None, None, :]
    limit = (L - (n - 1 - torch.arange(n)))[None, :, None, None]
    s = s.masked_fill(pos >= limit, float("-inf"))
    ref = torch.einsum("bnhl,bhld->bnhd", torch.softmax(s, -1), tV)
    np.testing.assert_allclose(out, ref.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, torch.logsumexp(s, -1).numpy(), rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("part", [1, 4, 9, 100])
def test_partition_invariant_across_the_causal_edge(part):
    B, n, Hq, Hkv, L, d, T = 2, 4, 4, 2, 37, 8, 8
    q, K, V = case(4, B, n, Hq, Hkv, L, d)
    kp, vp, table, _ = contiguous_problem(q[:, 0], K, V, T)
    lens = np.array([37, 2], dtype=np.int32)
    out, lse = oracle.attention(q, kp, vp, table, lens, T, 0.5)
    bounds = [list(range(0, int(x), part)) + [int(x)] for x in lens]
    MA, m, e, nparts = oracle.micro_attention(q, kp, vp, table, lens, T, 0.5, bounds)
    assert MA.shape[0] == int(nparts.sum()) * n * Hq
    out2, lse2 = oracle.aggregate(MA, m, e, nparts, n * Hq)
    np.testing.assert_allclose(out2.reshape(out.shape), out, rtol=1e-12, atol=1e-14)
    a, b = lse2.reshape(lse.shape), lse
    assert np.array_equal(np.isneginf(a), np.isneginf(b))
    np.testing.assert_allclose(a[np.isfinite(b)], b[np.isfinite(b)], rtol=1e-13, atol=1e-13)
