"""Pins for the oracle's IEEE-half inputs: every one of the 65536 bit patterns widens exactly as numpy widens it,
and attention over half-precision inputs equals the textbook softmax(q K^T) V on the exactly widened values."""
import numpy as np
import torch

import oracle


def test_every_half_bit_pattern_widens_exactly():
    # K holds all 65536 patterns as 512 tokens of 128 elements; q one-hot picks one element per token, and with
    # V = identity-like rows the scores themselves are observable through lse of single-token requests
    bits = np.arange(65536, dtype=np.uint16)
    halves = bits.view(np.float16)
    want = halves.astype(np.float64)
    finite = np.isfinite(want)
    T, d = 1, 128
    k_pool = halves.reshape(512, 1, T, d).copy()
    v_pool = np.ones((512, 1, T, d), dtype=np.float16)
    got = np.empty(65536, dtype=np.float64)
    # request r = one token (block r); head c has q = e_c, so lse[r][c] = 1.0 * K[r][c] exactly
    q = np.tile(np.eye(d, dtype=np.float16)[None], (512, 1, 1))        # [512][128 heads][128]
    table = np.arange(512, dtype=np.int32).reshape(512, 1)
    lens = np.ones(512, dtype=np.int32)
    # MQA: 128 q-heads share the one kv-head.  Elements that are inf/nan would poison the whole dot product, so
    # they are replaced by 0 in K for this check and compared separately below.
    k_clean = k_pool.copy()
    k_clean.reshape(-1)[~finite] = 0
    out, lse = oracle.attention(q, k_clean, v_pool, table, lens, T, 1.0)
    got = lse.reshape(-1)
    assert np.array_equal(got[finite], want[finite])
    assert np.all(out == 1.0)
    # signed zero, subnormals and the extremes by value
    for h, v in ((0x0001, 2.0 ** -24), (0x03FF, 1023 * 2.0 ** -24), (0x0400, 2.0 ** -14), (0x7BFF, 65504.0),
                 (0xFBFF, -65504.0), (0x3C00, 1.0), (0xC000, -2.0), (0x3555, 0.333251953125)):
        assert want[h] == v and got[h] == v


def test_infinite_half_inputs_propagate():
    q = np.array([[[1.0, 0.0]]], dtype=np.float16)
    k = np.array([[[[np.inf, 0.0], [1.0, 0.0]]]], dtype=np.float16)       # one block, 2 tokens
    v = np.array([[[[5.0, 6.0], [7.0, 8.0]]]], dtype=np.float16)
    out, lse = oracle.attention(q, k, v, np.zeros((1, 1), dtype=np.int32), np.array([2], dtype=np.int32), 2, 1.0)
    assert np.isposinf(lse[0, 0]) or np.isnan(lse[0, 0])                  # no cleansing of valid inputs


def test_half_attention_equals_textbook_on_widened_values():
    rng = np.random.RandomState(0)
    B, Hq, Hkv, d, T, L = 2, 4, 2, 16, 8, 37
    nb = (L + T - 1) // T
    q = rng.standard_normal((B, Hq, d)).astype(np.float16)
    k_pool = rng.standard_normal((B * nb, Hkv, T, d)).astype(np.float16)
    v_pool = rng.standard_normal((B * nb, Hkv, T, d)).astype(np.float16)
    table = rng.permutation(B * nb).astype(np.int32).reshape(B, nb)
    lens = np.array([L, L - 9], dtype=np.int32)
    out, lse = oracle.attention(q, k_pool, v_pool, table, lens, T, 0.25)
    for r in range(B):
        K = np.concatenate([k_pool[b] for b in table[r]], axis=1)[:, : lens[r]].astype(np.float64)   # [Hkv][L][d]
        V = np.concatenate([v_pool[b] for b in table[r]], axis=1)[:, : lens[r]].astype(np.float64)
        for h in range(Hq):
            g = h // (Hq // Hkv)
            s = torch.as_tensor(K[g] @ q[r, h].astype(np.float64) * 0.25)
            ref = (torch.softmax(s, 0)[None] @ torch.as_tensor(V[g]))[0].numpy()
            assert np.allclose(out[r, h], ref, rtol=1e-13, atol=1e-15)
            assert np.isclose(lse[r, h], torch.logsumexp(s, 0).item(), rtol=1e-14)


def test_mixed_half_pool_and_float_query():
    rng = np.random.RandomState(1)
    q32 = rng.standard_normal((1, 2, 8)).astype(np.float32)
    k = rng.standard_normal((2, 1, 4, 8)).astype(np.float16)
    v = rng.standard_normal((2, 1, 4, 8)).astype(np.float16)
    table = np.array([[1, 0]], dtype=np.int32)
    lens = np.array([7], dtype=np.int32)
    out, _ = oracle.attention(q32, k, v, table, lens, 4, 0.5)
    out32, _ = oracle.attention(q32, k.astype(np.float32), v.astype(np.float32), table, lens, 4, 0.5)
    assert np.array_equal(out, out32)        # widening half -> float is exact, so the two runs see the same numbers
