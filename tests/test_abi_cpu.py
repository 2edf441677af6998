"""CPU-side checks of the C-ABI library: it loads, exports what the header declares, validates its
arguments before touching the GPU, and its host scheduler cuts the work sensibly.  No kernel runs here."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

from paper_2401_02669_amd import distattn as da
from paper_2401_02669_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def problem(B=2, Hq=8, Hkv=2, d=128, T=256, max_blocks=64, num_phys=256, kv=da.DA_BF16, q=da.DA_BF16,
            scale=0.088, token_stride=None):
    p = da.DaProblem()
    p.batch, p.num_q_heads, p.num_kv_heads, p.head_dim = B, Hq, Hkv, d
    p.block_tokens, p.max_blocks_per_seq, p.num_phys_blocks = T, max_blocks, num_phys
    p.kv_dtype, p.q_dtype, p.scale = kv, q, scale
    ts = d if token_stride is None else token_stride
    p.kv_token_stride, p.kv_head_stride, p.kv_block_stride = ts, ts * T, ts * T * Hkv
    return p


def test_library_exports_every_declared_symbol():
    from paper_2401_02669_amd import placement, probe
    declared = set()
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):
        header = open(os.path.join(ROOT, "include", name)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        declared |= set(re.findall(r"\b(da_[a-z_]+)\s*\(", header))
    exports = set(da.EXPORTS) | set(placement.EXPORTS) | set(probe.EXPORTS)
    assert declared == exports, declared ^ exports
    L = da.lib()
    for name in declared - set(probe.EXPORTS):
        assert hasattr(L, name), name
    for name in probe.EXPORTS:  # the measurement probes live in a library of their own
        assert hasattr(probe.lib(), name), name
        assert not hasattr(L, name), name
    assert da.status_string(da.DA_OK) == "ok"
    assert "unsupported" in da.status_string(da.DA_ERR_UNSUPPORTED)


@pytest.mark.parametrize("kwargs,status", [
    (dict(B=0), da.DA_ERR_INVALID_ARG),
    (dict(Hq=6, Hkv=4), da.DA_ERR_INVALID_ARG),
    (dict(d=64), da.DA_ERR_UNSUPPORTED),
    (dict(T=100), da.DA_ERR_UNSUPPORTED),
    (dict(T=0), da.DA_ERR_INVALID_ARG),
    (dict(kv=7), da.DA_ERR_UNSUPPORTED),
    (dict(scale=float("nan")), da.DA_ERR_INVALID_ARG),
    (dict(token_stride=100), da.DA_ERR_INVALID_ARG),
    (dict(token_stride=132), da.DA_ERR_INVALID_ARG),   # bf16 rows would start off a 16-byte boundary
    (dict(Hq=130, Hkv=1), da.DA_ERR_UNSUPPORTED),
])
def test_validation_status_codes(kwargs, status):
    p = problem(**kwargs)
    with pytest.raises(da.DistAttnError) as e:
        da.plan_schedule(p, [10] * max(p.batch, 1))
    assert e.value.status == status


def test_schedule_rejects_bad_lengths_and_null_pointers():
    p = problem()
    with pytest.raises(da.DistAttnError) as e:
        da.plan_schedule(p, [-1, 5])
    assert e.value.status == da.DA_ERR_INVALID_ARG
    with pytest.raises(da.DistAttnError) as e:
        da.plan_schedule(p, [64 * 256 + 1, 5])  # longer than the block table row can address
    assert e.value.status == da.DA_ERR_INVALID_ARG
    L = da.lib()
    assert L.da_plan_schedule(None, None, None, None, None, None, None, None, None) == da.DA_ERR_INVALID_ARG
    assert L.da_plan_create(None, None, None, None, None) == da.DA_ERR_INVALID_ARG
    assert L.da_partial(*([None] * 10)) == da.DA_ERR_INVALID_ARG
    assert L.da_combine(*([None] * 7)) == da.DA_ERR_INVALID_ARG
    assert L.da_attention(*([None] * 9), 0, None) == da.DA_ERR_INVALID_ARG
    assert L.da_workspace_bytes(None, None) == da.DA_ERR_INVALID_ARG
    assert L.da_plan_destroy(None) == da.DA_OK


def _items_per_request(p, ns, kernel):
    G = p.num_q_heads // p.num_kv_heads
    tile = 16 if kernel == da.DA_KERNEL_MFMA else min(8, 1 << max(0, math.ceil(math.log2(G))))
    return ns * p.num_kv_heads * ((G + tile - 1) // tile)


def _tiles(L, T):
    if L <= 0:
        return 0
    tpb = (T + 31) // 32
    nb = (L + T - 1) // T
    return (nb - 1) * tpb + (L - (nb - 1) * T + 31) // 32


@pytest.mark.parametrize("name", list(synth.WORKLOADS))
def test_schedule_properties_on_the_named_workloads(name):
    r = synth.recipe(name)
    rng = np.random.RandomState(synth.BASE_SEED + r["index"])
    lens = synth._lengths(r, rng)
    T = r["T"]
    nb = (lens + T - 1) // T
    nt = np.array([_tiles(int(L), T) for L in lens])
    p = problem(B=r["B"], Hq=r["Hq"], Hkv=r["Hkv"], T=T, max_blocks=int(nb.max()), num_phys=int(nb.sum()),
                kv=da.DA_F32 if r["dtype"] == "f32" else da.DA_BF16,
                q=da.DA_F32 if r["dtype"] == "f32" else da.DA_BF16)
    s = da.plan_schedule(p, lens, num_cus=256)
    ns = np.array(s["nsplits"])
    assert np.all(ns >= 1) and np.all(ns <= np.maximum(nt, 1))
    assert s["num_partials"] == int(ns.sum()) * r["Hq"]
    assert s["num_items"] == sum(_items_per_request(p, int(n), s["kernel"]) for n in ns)
    per_split = _items_per_request(p, 1, s["kernel"])
    assert s["workgroups"] % per_split == 0 and s["workgroups"] <= 256
    if name != "c1_tiny" and not name.startswith("small_"):
        # every compute unit gets its persistent workgroup ...
        assert s["workgroups"] == 256
        runs = 256 // per_split
        # ... requests are cut no more than the equal-cost runs need ...
        assert int(ns.sum()) <= r["B"] + runs - 1
        # ... every workgroup reads (nearly) the same number of tokens ...
        assert s["max_workgroup_tokens"] <= 1.02 * float(lens.sum()) / runs + 64
        # ... and partial rows (written once, read once) stay a small fraction of the KV bytes
        # (requests of a few hundred tokens are the exception: their one output row each is all there is)
        partial_bytes = 2.0 * s["num_partials"] * (128 + 2) * 4
        kv_bytes = float(lens.sum()) * r["Hkv"] * 2 * 128 * (4 if r["dtype"] == "f32" else 2)
        if name.startswith("c"):
            assert partial_bytes / kv_bytes < 0.01


def test_explicit_blocks_per_split_is_honoured():
    p = problem(B=3, max_blocks=100)
    lens = [100 * 256, 1, 0]
    s = da.plan_schedule(p, lens, blocks_per_split=1)
    assert s["nsplits"] == [100, 1, 1]
    s = da.plan_schedule(p, lens, blocks_per_split=7)
    assert s["nsplits"] == [15, 1, 1]
    s = da.plan_schedule(p, lens, blocks_per_split=1000)
    assert s["nsplits"] == [1, 1, 1]


def test_schedule_of_a_large_batch_is_cheap_and_balanced():
    import time
    rng = np.random.RandomState(0)
    lens = np.floor(np.exp(rng.uniform(np.log(16), np.log(200000), size=4096))).astype(np.int64)
    p = problem(B=4096, Hq=32, Hkv=8, T=256, max_blocks=int((lens.max() + 255) // 256), num_phys=1 << 20)
    t0 = time.perf_counter()
    for _ in range(5):
        s = da.plan_schedule(p, lens, num_cus=256)
    dt = (time.perf_counter() - t0) / 5
    assert dt < 0.02, dt   # a few hundred microseconds in practice
    assert s["workgroups"] == 256
    assert s["max_workgroup_tokens"] <= 1.03 * float(lens.sum()) / 32 + 64
    assert sum(s["nsplits"]) <= 4096 + 31


def test_a_wide_item_charges_a_split_more():
    # Mixed lengths: the runs at the end of the reading order collect the short requests.  With many columns per
    # item a split costs more (query rows, first-chunk latency, a wider merge), so those runs get fewer tokens and
    # the runs of the long requests more: the largest run grows with the width, and the total is the same.
    r = synth.recipe("c5_mixed")
    lens = synth._lengths(r, np.random.RandomState(synth.BASE_SEED + r["index"]))
    T = r["T"]
    nb = (lens + T - 1) // T
    worst = []
    for q_len in (1, 4, 16):
        p = problem(B=r["B"], Hq=r["Hq"], Hkv=r["Hkv"], T=T, max_blocks=int(nb.max()), num_phys=int(nb.sum()))
        p.q_len = q_len
        s = da.plan_schedule(p, lens, num_cus=256)
        assert s["workgroups"] == 256 and sum(s["nsplits"]) <= r["B"] + 31
        worst.append(s["max_workgroup_tokens"])
    mean = float(lens.sum()) / 32
    assert worst[0] <= 1.02 * mean + 64          # 4 columns: runs of (nearly) equal tokens
    assert worst[0] < worst[1] < worst[2] <= 1.25 * mean
