"""GPU parity of the multi-query (causal) form against the fp64 oracle: several new tokens per request,
every (query token, q-head) pair a column of its kv-head's group with its own causal limit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2401_02669_amd import distattn as da
from paper_2401_02669_amd import synth
from util import TOL, assert_parity, errors

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make(lens, n, Hq, Hkv, T, dtype="bf16", seed=0):
    w = synth.make(synth.recipe("c5_mixed", B=len(lens), Hq=Hq, Hkv=Hkv, T=T, dtype=dtype, lens=list(lens)), DEV)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(1000 + seed)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    w["q"] = torch.randn((len(lens), n, Hq, 128), device=DEV, generator=gen).to(tdt)
    return w


def run_both(w, **tuning):
    prob = da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"])
    plan = da.Plan(prob, w["seq_lens_host"].tolist(), **tuning)
    out, lse = plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    po, pm, pe = plan.partial(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    out2, lse2 = plan.combine(po, pm, pe)
    torch.cuda.synchronize()
    assert plan.error_flags() == 0
    return plan, (out.cpu().numpy(), lse.cpu().numpy()), (out2.cpu().numpy(), lse2.cpu().numpy()), (po, pm, pe)


def ref_of(w):
    return oracle.attention(synth.as_numpy(w["q"]), synth.as_numpy(w["k_pool"]), synth.as_numpy(w["v_pool"]),
                            w["block_table_host"], w["seq_lens_host"], w["T"], w["scale"], n_threads=16)


@pytest.mark.parametrize("n", [2, 3, 4, 16, 17])
@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (8, 2), (16, 2)])
@pytest.mark.parametrize("kernel", [da.DA_KERNEL_AUTO, da.DA_KERNEL_VALU], ids=["auto", "valu"])
def test_multi_query_matches_oracle(n, Hq, Hkv, kernel):
    lens = [700, 0, 1, n - 1, n, n + 1, 64, 65, 2049]
    w = make(lens, n, Hq, Hkv, T=64, seed=n)
    print("case multi-query n=%d Hq=%d Hkv=%d kernel=%d" % (n, Hq, Hkv, kernel), flush=True)
    ref_out, ref_lse = ref_of(w)
    for bps in (0, 3):
        plan, fused, two_step, _ = run_both(w, kernel=kernel, blocks_per_split=bps)
        plan.close()
        for (out, lse), what in ((fused, "fused"), (two_step, "two-step")):
            assert out.shape == ref_out.shape
            assert_parity(out, lse, ref_out, ref_lse, "bf16", "%s n=%d bps=%d" % (what, n, bps))
            # the last query token of the longest request sees everything; the first one misses n - 1 tokens
            for t in (0, n - 1):
                _, rel = errors(out[8, t], ref_out[8, t])
                assert rel <= TOL["bf16"]["rel_l2"]


def test_multi_query_fp32_cache():
    w = make([300, 5, 1000], 3, 4, 2, T=32, dtype="f32")
    ref_out, ref_lse = ref_of(w)
    plan, fused, two_step, _ = run_both(w)
    plan.close()
    assert_parity(fused[0], fused[1], ref_out, ref_lse, "f32", "fp32 multi-query fused")
    assert_parity(two_step[0], two_step[1], ref_out, ref_lse, "f32", "fp32 multi-query two-step")


@pytest.mark.parametrize("kernel", [da.DA_KERNEL_AUTO, da.DA_KERNEL_VALU], ids=["auto", "valu"])
def test_multi_query_partials_match_micro_attention(kernel):
    n, Hq = 4, 4
    w = make([900, 3, 130], n, Hq, 2, T=32)
    plan, _, _, (po, pm, pe) = run_both(w, kernel=kernel, blocks_per_split=2)
    bounds = []
    for r in range(w["B"]):
        b = [0]
        for j in range(plan.nsplits(r)):
            lo, hi = plan.split(r, j)
            assert lo == b[-1]
            b.append(hi)
        bounds.append(b)
    plan.close()
    MA, m, e, nparts = oracle.micro_attention(synth.as_numpy(w["q"]), synth.as_numpy(w["k_pool"]), synth.as_numpy(w["v_pool"]),
                                              w["block_table_host"], w["seq_lens_host"], w["T"], w["scale"], bounds)
    po, pm, pe = (x.cpu().numpy().astype(np.float64) for x in (po, pm, pe))
    assert po.shape[0] == MA.shape[0] == int(nparts.sum()) * n * Hq
    live = np.isfinite(m)
    assert np.array_equal(np.isneginf(pm), ~live) and np.all(pe[~live] == 0) and np.all(po[~live] == 0)
    np.testing.assert_allclose(pm[live], m[live], rtol=0, atol=2e-5)
    adj = np.exp(pm[live] - m[live])
    np.testing.assert_allclose(pe[live] * adj, e[live], rtol=2e-4)
    num = np.linalg.norm(po[live] * adj[:, None] - MA[live], axis=1)
    assert np.all(num <= 1e-3 * np.linalg.norm(MA[live], axis=1) + 1e-12)


def test_multi_query_with_one_wavefront_per_split():
    """Many short requests, three query tokens each: the wavefront-per-split walk with causal columns."""
    rng = np.random.RandomState(5)
    n = 3
    lens = [int(x) for x in rng.randint(0, 400, size=500)] + [0, 1, 2, 3, 4, 64, 65, 3000]
    w = make(lens, n, 8, 2, T=64, seed=3)
    ref_out, ref_lse = ref_of(w)
    plan, fused, two_step, _ = run_both(w, num_cus=8)
    assert plan.describe()["wavefront_splits"] == 1
    plan.close()
    for (out, lse), what in ((fused, "fused"), (two_step, "two-step")):
        assert_parity(out, lse, ref_out, ref_lse, "bf16", "wavefront splits, multi-query, " + what)


@pytest.mark.parametrize("n,Hq,Hkv", [(8, 16, 2), (8, 8, 2), (17, 16, 2), (32, 16, 2), (5, 24, 1), (128, 2, 1)])
def test_many_columns(n, Hq, Hkv):
    """32 to 256 (query token, q-head) columns per kv-head: up to four column tiles per work item, the K/V read
    repeated per 64 columns."""
    lens = [1500, 0, 1, n - 1, n, n + 1, 64, 65, 4100, 33]
    w = make(lens, n, Hq, Hkv, T=64, seed=100 + n)
    print("case many columns n=%d Hq=%d Hkv=%d" % (n, Hq, Hkv), flush=True)
    ref_out, ref_lse = ref_of(w)
    for bps, cus in ((0, 0), (0, 16), (5, 0)):
        plan, fused, two_step, _ = run_both(w, blocks_per_split=bps, num_cus=cus)
        plan.close()
        for (out, lse), what in ((fused, "fused"), (two_step, "two-step")):
            assert_parity(out, lse, ref_out, ref_lse, "bf16", "%s n=%d bps=%d cus=%d" % (what, n, bps, cus))
            for r in (0, 8):  # worst single query token of the long requests
                for t in (0, n - 1):
                    _, rel = errors(out[r, t], ref_out[r, t])
                    assert rel <= TOL["bf16"]["rel_l2"]


def test_partials_of_many_columns_report_the_true_maximum():
    n, Hq = 12, 8   # 48 columns per kv-head
    w = make([900, 3, 130, 0, 2500], n, Hq, 2, T=32, seed=77)
    plan, fused, _, (po, pm, pe) = run_both(w, blocks_per_split=2)
    ref_out, ref_lse = ref_of(w)
    assert_parity(fused[0], fused[1], ref_out, ref_lse, "bf16", "48 columns")
    bounds = []
    for r in range(w["B"]):
        b = [0]
        for j in range(plan.nsplits(r)):
            lo, hi = plan.split(r, j)
            b.append(hi)
        bounds.append(b)
    plan.close()
    MA, m, e, nparts = oracle.micro_attention(synth.as_numpy(w["q"]), synth.as_numpy(w["k_pool"]), synth.as_numpy(w["v_pool"]),
                                              w["block_table_host"], w["seq_lens_host"], w["T"], w["scale"], bounds)
    po, pm, pe = (x.cpu().numpy().astype(np.float64) for x in (po, pm, pe))
    live = np.isfinite(m)
    assert np.array_equal(np.isneginf(pm), ~live) and np.all(pe[~live] == 0) and np.all(po[~live] == 0)
    # m_j is the true maximum of the split (the kernel's held-back reference maximum must not show)
    np.testing.assert_allclose(pm[live], m[live], rtol=0, atol=2e-5)
    np.testing.assert_allclose(pe[live], e[live], rtol=3e-4)
    num = np.linalg.norm(po[live] - MA[live], axis=1)
    assert np.all(num <= 1e-3 * np.linalg.norm(MA[live], axis=1) + 1e-12)


@pytest.mark.parametrize("Hq,Hkv,n", [(64, 1, 1), (8, 2, 16), (16, 1, 8), (8, 1, 16), (32, 1, 1), (8, 2, 6), (16, 2, 20)])
def test_first_chunk_is_a_partly_visible_one(Hq, Hkv, n):
    # requests so short that the first chunk a wavefront sees is one with masked rows (the reference maximum is set
    # and rows are masked in the same chunk), for 32, 64 and 128 columns per work item
    lens = [31, 33, 1, 64, 95, 127, 4101]
    w = make(lens, n, Hq, Hkv, T=64, seed=100 + Hq + n)
    print("case short requests n=%d Hq=%d Hkv=%d" % (n, Hq, Hkv), flush=True)
    ref_out, ref_lse = ref_of(w)
    for bps in (0, 1):
        plan, fused, two_step, _ = run_both(w, blocks_per_split=bps)
        plan.close()
        for (out, lse), what in ((fused, "fused"), (two_step, "two-step")):
            assert_parity(out.reshape(ref_out.shape), lse.reshape(ref_lse.shape), ref_out, ref_lse, "bf16", "%s bps=%d" % (what, bps))


@pytest.mark.parametrize("Hq,Hkv,n,dtype,kernel", [(8, 8, 1, "bf16", da.DA_KERNEL_AUTO), (32, 1, 1, "bf16", da.DA_KERNEL_AUTO),
                                                   (8, 2, 16, "bf16", da.DA_KERNEL_AUTO), (8, 1, 16, "bf16", da.DA_KERNEL_AUTO),
                                                   (8, 2, 3, "bf16", da.DA_KERNEL_VALU), (8, 1, 2, "f32", da.DA_KERNEL_AUTO),
                                                   (4, 4, 1, "f32", da.DA_KERNEL_AUTO)])
def test_negative_score_scale(Hq, Hkv, n, dtype, kernel):
    # scores are scale * q.k for any sign of the scale: the largest score then belongs to the most negative product
    lens = [700, 0, 1, 33, 64, 2049]
    w = make(lens, n, Hq, Hkv, T=64, dtype=dtype, seed=7 + n)
    w["scale"] = -0.11
    print("case negative scale n=%d Hq=%d Hkv=%d %s kernel=%d" % (n, Hq, Hkv, dtype, kernel), flush=True)
    ref_out, ref_lse = ref_of(w)
    plan, fused, two_step, _ = run_both(w, kernel=kernel)
    plan.close()
    for (out, lse), what in ((fused, "fused"), (two_step, "two-step")):
        assert_parity(out.reshape(ref_out.shape), lse.reshape(ref_lse.shape), ref_out, ref_lse, dtype, what)
