"""CPU checks of the KV-append row: the oracle's append against an independent gather and against the
attention oracle on a directly built cache, and the host block pool's bookkeeping."""
import numpy as np
import pytest

import oracle
from paper_2401_02669_amd import distattn as da
from paper_2401_02669_amd import synth
from test_oracle_pins import contiguous_problem


@pytest.mark.parametrize("dtype", [np.float32, np.uint16])
def test_appended_cache_reads_back_as_the_token_sequence(dtype):
    B, Hkv, d, T, steps = 3, 2, 8, 4, 11
    rng = np.random.RandomState(1)
    num_phys = 12
    table = np.full((B, 4), -1, dtype=np.int32)
    ids = rng.permutation(num_phys)
    for r in range(B):
        table[r, :3] = ids[3 * r: 3 * r + 3]       # room for 12 tokens each
    poison = 0x7FC0 if dtype == np.uint16 else np.nan
    kp = np.full((num_phys, Hkv, T, d), poison, dtype=dtype)
    vp = np.full((num_phys, Hkv, T, d), poison, dtype=dtype)
    lens = np.array([0, 5, -1], dtype=np.int32)      # request 2 is an inactive slot
    # request 1 starts with 5 tokens already in place
    history_k = {0: [], 1: [], 2: []}
    history_v = {0: [], 1: [], 2: []}
    for i in range(5):
        row = rng.standard_normal((2, Hkv, d)).astype(np.float32)
        row = synth.f32_to_bf16_bits(row) if dtype == np.uint16 else row
        kp[table[1, i // T], :, i % T] = row[0]
        vp[table[1, i // T], :, i % T] = row[1]
        history_k[1].append(row[0]); history_v[1].append(row[1])
    for _ in range(steps):
        kn = rng.standard_normal((B, Hkv, d)).astype(np.float32)
        vn = rng.standard_normal((B, Hkv, d)).astype(np.float32)
        if dtype == np.uint16:
            kn, vn = synth.f32_to_bf16_bits(kn), synth.f32_to_bf16_bits(vn)
        before = lens.copy()
        oracle.append(kn, vn, kp, vp, table, lens)
        for r in range(B):
            if before[r] < 0 or before[r] >= 12:     # inactive, or no block left in the row: untouched
                assert lens[r] == before[r]
            else:
                assert lens[r] == before[r] + 1
                history_k[r].append(kn[r]); history_v[r].append(vn[r])
    assert lens[2] == -1 and lens[0] == 11 and lens[1] == 12   # request 1 hit the end of its 3 blocks
    for r in (0, 1):
        for i in range(lens[r]):                     # independent gather through the table
            assert np.array_equal(kp[table[r, i // T], :, i % T], history_k[r][i])
            assert np.array_equal(vp[table[r, i // T], :, i % T], history_v[r][i])
    # slots never written are still poison
    assert np.all(kp[table[0, 2], :, 3] == poison) or dtype == np.float32 and np.all(np.isnan(kp[table[0, 2], :, 3]))


def test_attention_over_an_appended_cache_equals_a_directly_built_one():
    B, Hq, Hkv, d, T, L = 2, 4, 2, 16, 8, 21
    rng = np.random.RandomState(2)
    K = rng.standard_normal((B, Hkv, L, d)).astype(np.float32)
    V = rng.standard_normal((B, Hkv, L, d)).astype(np.float32)
    q = rng.standard_normal((B, Hq, d)).astype(np.float32)
    kp, vp, table, lens = contiguous_problem(q, K, V, T)
    ref_out, ref_lse = oracle.attention(q, kp, vp, table, lens, T, 0.3)
    # the same tokens appended one at a time into a scattered layout
    nb = table.shape[1]
    ids = rng.permutation(B * nb + 3).astype(np.int32)
    table2 = ids[: B * nb].reshape(B, nb).copy()
    kp2 = np.full((B * nb + 3, Hkv, T, d), np.nan, dtype=np.float32)
    vp2 = np.full_like(kp2, np.nan)
    lens2 = np.zeros(B, dtype=np.int32)
    for i in range(L):
        oracle.append(np.ascontiguousarray(K[:, :, i]), np.ascontiguousarray(V[:, :, i]), kp2, vp2, table2, lens2)
    assert list(lens2) == [L, L]
    out, lse = oracle.attention(q, kp2, vp2, table2, lens2, T, 0.3)
    assert np.array_equal(out, ref_out) and np.array_equal(lse, ref_lse)


def test_block_pool_bookkeeping():
    T, maxb = 16, 8
    pool = da.BlockPool(10)
    assert pool.free_count == 10
    table = np.full((3, maxb), -1, dtype=np.int32)
    pool.grow(table[0], T, 0, 1)            # first token: one block
    assert pool.free_count == 9 and table[0, 0] >= 0 and np.all(table[0, 1:] == -1)
    pool.grow(table[0], T, 1, 16)           # still the same block
    assert pool.free_count == 9
    pool.grow(table[0], T, 16, 17)          # crosses into a second block
    assert pool.free_count == 8 and table[0, 1] >= 0 and table[0, 1] != table[0, 0]
    pool.grow(table[1], T, 0, 5 * T)        # five at once
    assert pool.free_count == 3
    used = [int(x) for x in table[table >= 0]]
    assert len(set(used)) == len(used) == 7 and all(0 <= x < 10 for x in used)
    with pytest.raises(da.DistAttnError) as e:
        pool.grow(table[2], T, 0, 4 * T)    # needs 4, only 3 free: nothing is taken
    assert e.value.status == da.DA_ERR_NO_SPACE and pool.free_count == 3 and np.all(table[2] == -1)
    with pytest.raises(da.DistAttnError) as e:
        pool.grow(table[1], T, 5 * T, 9 * T)   # beyond the table row
    assert e.value.status == da.DA_ERR_INVALID_ARG
    pool.release(table[1], T, 5 * T)
    assert pool.free_count == 8 and np.all(table[1] == -1)
    bad = np.array([table[0, 0], table[0, 0]] + [-1] * 6, dtype=np.int32)
    with pytest.raises(da.DistAttnError):
        pool.release(bad, T, 2 * T)         # duplicate id
    assert pool.free_count == 8
    pool.release(table[0], T, 17)
    assert pool.free_count == 10
    with pytest.raises(da.DistAttnError):
        pool.release(np.array([3] + [-1] * 7, dtype=np.int32), T, 1)   # block 3 is not in use
    pool.close()


def test_append_argument_checks_happen_before_any_launch():
    L = da.lib()
    assert L.da_append(None, None, None, None, None, None, None, None, None) == da.DA_ERR_INVALID_ARG
    assert L.da_block_pool_create(0, None) == da.DA_ERR_INVALID_ARG
    assert L.da_block_pool_destroy(None) == da.DA_OK
