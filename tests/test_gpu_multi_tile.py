"""The bf16 kernel for 32 / 64 / 128 columns per K/V read (micro_attention_mfma_tiles.hip) under the conditions the
one-tile kernels are tested under: odd block sizes, padded token rows, plans cut for other lengths than the device
holds, block ids outside the pool, edge lengths, raw partial rows, a decode loop with appends.  Columns come from
the group size, from several query tokens per request, or both."""
import numpy as np
import pytest
import torch

import oracle
from paper_2401_02669_amd import distattn as da
from paper_2401_02669_amd import synth
from util import TOL, assert_parity, errors

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

# (Hq, Hkv, query tokens): 32, 64, 128 and 200 columns (two work items of 128)
SHAPES = [(32, 1, 1), (8, 2, 8), (16, 2, 8), (8, 1, 16), (64, 1, 2), (8, 1, 25)]


def make(lens, Hq, Hkv, n, T, seed=0, **kw):
    w = synth.make(synth.recipe("c5_mixed", B=len(lens), Hq=Hq, Hkv=Hkv, T=T, dtype="bf16", lens=list(lens), **kw), DEV)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(300 + seed)
    w["q"] = torch.randn((len(lens), n, Hq, 128), device=DEV, generator=gen).to(torch.bfloat16)
    return w


def reference(w, table=None, lens=None):
    return oracle.attention(synth.as_numpy(w["q"]), synth.as_numpy(w["k_pool"]), synth.as_numpy(w["v_pool"]),
                            w["block_table_host"] if table is None else table,
                            w["seq_lens_host"] if lens is None else lens, w["T"], w["scale"], n_threads=16)


def run(w, planned=None, table=None, **tuning):
    prob = da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"])
    plan = da.Plan(prob, planned if planned is not None else w["seq_lens_host"].tolist(), **tuning)
    desc = plan.describe()
    tab = w["block_table"] if table is None else table
    out, lse = plan.attention(w["q"], w["k_pool"], w["v_pool"], tab, w["seq_lens"])
    po, pm, pe = plan.partial(w["q"], w["k_pool"], w["v_pool"], tab, w["seq_lens"])
    out2, lse2 = plan.combine(po, pm, pe)
    torch.cuda.synchronize()
    flags = plan.error_flags()
    plan.close()
    return desc, flags, (out.cpu().numpy(), lse.cpu().numpy()), (out2.cpu().numpy(), lse2.cpu().numpy())


@pytest.mark.parametrize("T", [16, 48, 112, 1024])
@pytest.mark.parametrize("Hq,Hkv,n", SHAPES)
def test_block_sizes(T, Hq, Hkv, n):
    lens = [1000, 37, 4100, 0, n, 31, 33]
    w = make(lens, Hq, Hkv, n, T, seed=T + n)
    print("case multi-tile block size T=%d Hq=%d Hkv=%d n=%d" % (T, Hq, Hkv, n), flush=True)
    ref_out, ref_lse = reference(w)
    for bps in (0, 1, 5):
        desc, flags, fused, two = run(w, blocks_per_split=bps)
        assert desc["kernel"] == da.DA_KERNEL_MFMA and desc["head_tile"] in (32, 64, 128) and flags == 0
        for (out, lse), what in ((fused, "fused"), (two, "two calls")):
            assert_parity(out.reshape(ref_out.shape), lse.reshape(ref_lse.shape), ref_out, ref_lse, "bf16", "%s T=%d bps=%d" % (what, T, bps))


@pytest.mark.parametrize("Hq,Hkv,n", SHAPES)
def test_padded_token_rows(Hq, Hkv, n):
    # pools whose token rows are padded (stride 160 elements) inside a larger allocation full of NaN
    w = make([900, 300, 65], Hq, Hkv, n, T=64, seed=n)
    for key in ("k_pool", "v_pool"):
        big = torch.full(w[key].shape[:3] + (160,), float("nan"), dtype=w[key].dtype, device=DEV)
        big[..., :128] = w[key]
        w[key] = big[..., :128]
    assert w["k_pool"].stride(2) == 160
    ref_out, ref_lse = reference(w)
    desc, flags, fused, two = run(w)
    assert desc["head_tile"] in (32, 64, 128) and flags == 0
    assert_parity(fused[0].reshape(ref_out.shape), fused[1].reshape(ref_lse.shape), ref_out, ref_lse, "bf16", "padded rows")


@pytest.mark.parametrize("Hq,Hkv,n", SHAPES)
def test_stale_plan(Hq, Hkv, n):
    # the plan was cut for other lengths than the device holds: longer, shorter, zero, from zero
    planned = [5000, 3000, 0, 700, 64]
    actual = [5100, 1500, 90, 0, 6400]
    w = make(actual, Hq, Hkv, n, T=64, seed=2 * n)
    ref_out, ref_lse = reference(w)
    for bps in (0, 2):
        desc, flags, fused, two = run(w, planned=planned, blocks_per_split=bps)
        assert flags == 0
        for (out, lse), what in ((fused, "fused"), (two, "two calls")):
            assert_parity(out.reshape(ref_out.shape), lse.reshape(ref_lse.shape), ref_out, ref_lse, "bf16", "stale plan %s bps=%d" % (what, bps))


@pytest.mark.parametrize("Hq,Hkv,n", [(32, 1, 1), (8, 2, 8), (8, 1, 16)])
def test_bad_block_ids_are_skipped_and_flagged(Hq, Hkv, n):
    w = make([640, 640], Hq, Hkv, n, T=64, seed=9, spare_frac=0.0)
    table = w["block_table"].clone()
    table[0, 3] = w["num_phys"] + 5
    table[1, 0] = -7
    desc, flags, fused, two = run(w, table=table)
    assert flags == 1 and np.all(np.isfinite(fused[0]))
    if n == 1:
        # a skipped block contributes nothing: the same as a request whose table simply lacks that block (with one
        # query token no causal limit moves with the length)
        t2 = w["block_table_host"].copy()
        t2[0, 3:-1] = t2[0, 4:]
        t2[1, 0:-1] = t2[1, 1:]
        ref_out, ref_lse = reference(w, table=t2, lens=(w["seq_lens_host"] - 64).astype(np.int32))
        assert_parity(fused[0].reshape(ref_out.shape), fused[1].reshape(ref_lse.shape), ref_out, ref_lse, "bf16", "skipped blocks")


@pytest.mark.parametrize("Hq,Hkv,n", SHAPES)
def test_partial_rows_are_the_micro_attention_triples(Hq, Hkv, n):
    lens = [3000, 2000, 97]
    w = make(lens, Hq, Hkv, n, T=64, seed=40 + n)
    prob = da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"])
    plan = da.Plan(prob, lens, num_cus=24)
    po, pm, pe = plan.partial(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    torch.cuda.synchronize()
    bounds = []
    for r in range(len(lens)):
        b = [0]
        for j in range(plan.nsplits(r)):
            lo, hi = plan.split(r, j)
            assert lo == b[-1]
            b.append(hi)
        bounds.append(b)
    plan.close()
    assert max(len(b) for b in bounds) > 2
    MA, m, e, nparts = oracle.micro_attention(synth.as_numpy(w["q"]), synth.as_numpy(w["k_pool"]), synth.as_numpy(w["v_pool"]),
                                              w["block_table_host"], w["seq_lens_host"], w["T"], w["scale"], bounds, n_threads=16)
    po, pm, pe = (x.cpu().numpy().astype(np.float64) for x in (po, pm, pe))
    assert po.shape[0] == MA.shape[0] == int(nparts.sum()) * n * Hq
    live = np.isfinite(m)
    assert np.array_equal(np.isneginf(pm), ~live) and np.all(pe[~live] == 0) and np.all(po[~live] == 0)
    np.testing.assert_allclose(pm[live], m[live], rtol=0, atol=2e-5)   # the true maximum of the partition
    adj = np.exp(pm[live] - m[live])
    np.testing.assert_allclose(pe[live] * adj, e[live], rtol=2e-4)
    num = np.linalg.norm(po[live] * adj[:, None] - MA[live], axis=1)
    assert np.all(num <= 1e-3 * np.linalg.norm(MA[live], axis=1) + 1e-12)


@pytest.mark.parametrize("T", [1024, 4096])
@pytest.mark.parametrize("Hq,Hkv,n", [(8, 1, 4), (8, 1, 8), (8, 1, 16), (8, 2, 25)])
def test_long_runs_of_full_chunks_end_where_a_column_stops_seeing(T, Hq, Hkv, n):
    # Blocks of many chunks: one statement loops over a block's full, fully visible chunks.  The lengths put the
    # end of what every column sees (L - n + 1) into the middle of a block, on a chunk boundary, one row before and
    # one after it, and into the first chunk of a block; one request ends exactly with a block.
    lens = [2 * T + 517, 3 * T + 32 * 5 + n - 1, 3 * T + 32 * 5 + n - 2, 3 * T + 32 * 5 + n, T + n + 3, 2 * T]
    w = make(lens, Hq, Hkv, n, T, seed=T // 1024 + n)
    print("case multi-tile long runs T=%d Hq=%d Hkv=%d n=%d" % (T, Hq, Hkv, n), flush=True)
    ref_out, ref_lse = reference(w)
    for bps in (0, 1):
        desc, flags, fused, two = run(w, blocks_per_split=bps)
        assert desc["head_tile"] in (32, 64, 128) and flags == 0
        for (out, lse), what in ((fused, "fused"), (two, "two calls")):
            assert_parity(out.reshape(ref_out.shape), lse.reshape(ref_lse.shape), ref_out, ref_lse, "bf16", "%s T=%d bps=%d" % (what, T, bps))
