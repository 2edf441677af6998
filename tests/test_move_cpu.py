"""Pins for the oracle's KV block movement (move_kvcache of Algorithm 1, Section 5.3): a hand case and the
definition written as numpy indexing; and that attention over a request whose blocks were moved to other
physical blocks (table updated) is unchanged.  CPU only."""
import numpy as np

import oracle


def pools(P, Hkv, T, d, seed, dtype=np.float32):
    rng = np.random.RandomState(seed)
    return rng.standard_normal((P, Hkv, T, d)).astype(dtype), rng.standard_normal((P, Hkv, T, d)).astype(dtype)


def test_hand_case():
    ks = np.arange(3 * 1 * 2 * 2, dtype=np.float32).reshape(3, 1, 2, 2)      # block b holds 4b .. 4b+3
    vs = -ks
    kd = np.full((2, 1, 2, 2), 99.0, dtype=np.float32)
    vd = np.full((2, 1, 2, 2), 99.0, dtype=np.float32)
    oracle.move_blocks(ks, vs, kd, vd, [2], [0])
    assert kd[0].ravel().tolist() == [8.0, 9.0, 10.0, 11.0] and vd[0].ravel().tolist() == [-8.0, -9.0, -10.0, -11.0]
    assert np.all(kd[1] == 99.0) and np.all(vd[1] == 99.0)


def test_equals_numpy_indexing_and_skips_bad_ids():
    ks, vs = pools(9, 3, 4, 8, 1)
    kd, vd = pools(7, 3, 4, 8, 2)
    kd0, vd0 = kd.copy(), vd.copy()
    src = np.array([8, 0, 3, -1, 4, 9, 2], dtype=np.int32)     # -1 and 9 are outside the source pool
    dst = np.array([1, 6, 0, 2, 7, 3, 5], dtype=np.int32)      # 7 is outside the destination pool
    oracle.move_blocks(ks, vs, kd, vd, src, dst)
    good = (src >= 0) & (src < 9) & (dst >= 0) & (dst < 7)
    want_k, want_v = kd0.copy(), vd0.copy()
    want_k[dst[good]] = ks[src[good]]
    want_v[dst[good]] = vs[src[good]]
    assert np.array_equal(kd, want_k) and np.array_equal(vd, want_v)
    assert np.array_equal(kd[[2, 3, 4]], kd0[[2, 3, 4]])       # skipped or untouched destinations


def test_bf16_bits_travel_unchanged():
    rng = np.random.RandomState(3)
    ks = rng.randint(0, 65536, size=(4, 2, 3, 8)).astype(np.uint16)
    vs = rng.randint(0, 65536, size=(4, 2, 3, 8)).astype(np.uint16)
    kd = np.zeros((4, 2, 3, 8), dtype=np.uint16)
    vd = np.zeros_like(kd)
    oracle.move_blocks(ks, vs, kd, vd, [0, 1, 2, 3], [3, 2, 1, 0])
    assert np.array_equal(kd, ks[::-1]) and np.array_equal(vd, vs[::-1])


def test_attention_is_unchanged_when_blocks_move_and_the_table_follows():
    T, Hkv, d, L = 4, 2, 8, 22
    ks, vs = pools(10, Hkv, T, d, 5)
    q = np.random.RandomState(6).standard_normal((1, 4, d)).astype(np.float32)
    table = np.array([[7, 2, 9, 0, 5, 3]], dtype=np.int32)
    lens = np.array([L], dtype=np.int32)
    ref, ref_lse = oracle.attention(q, ks, vs, table, lens, T, 0.3)
    # the first four blocks go to a second pool, in another order of physical ids
    kd, vd = pools(6, Hkv, T, d, 8)
    oracle.move_blocks(ks, vs, kd, vd, table[0, :4], [5, 0, 3, 1])
    # the part that stayed and the part that moved, each as a request of its own, aggregate to the same output
    t_home = np.array([[5, 3, -1, -1, -1, -1]], dtype=np.int32)
    t_away = np.array([[5, 0, 3, 1, -1, -1]], dtype=np.int32)
    o1, m1, e1, _ = oracle.micro_attention(q, ks, vs, t_home, np.array([L - 16], dtype=np.int32), T, 0.3, [[0, L - 16]])
    o2, m2, e2, _ = oracle.micro_attention(q, kd, vd, t_away, np.array([16], dtype=np.int32), T, 0.3, [[0, 16]])
    Hq = q.shape[1]
    MA = np.stack([o1, o2], axis=1).reshape(2 * Hq, d)          # row(h, j) = 2 h + j
    m = np.stack([m1, m2], axis=1).reshape(2 * Hq)
    e = np.stack([e1, e2], axis=1).reshape(2 * Hq)
    out, lse = oracle.aggregate(MA, m, e, np.array([2], dtype=np.int32), Hq)
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-13) and np.allclose(lse, ref_lse, rtol=1e-12)
