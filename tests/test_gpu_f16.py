"""IEEE-half q / K / V through the same path: parity against the fp64 oracle for both kernel families, the
multi-query form, weights far below the half range, mixed fp32 query, and append / block movement of half rows."""
import numpy as np
import pytest
import torch

import oracle
from paper_2401_02669_amd import distattn as da
from paper_2401_02669_amd import synth
from util import assert_parity, gpu_attention, make_plan, oracle_attention

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def bits(t):
    return synth.as_numpy(t)


@pytest.mark.parametrize("name,div,over", [
    ("c2_7b", 64, dict(B=4)), ("c3_70b", 64, {}), ("c4_2m", 64, {}), ("c5_mixed", 50, {}),
    ("c5_mixed", 100, dict(Hq=24, Hkv=1)), ("c5_mixed", 100, dict(Hq=64, Hkv=1)),
])
@pytest.mark.parametrize("kernel", [da.DA_KERNEL_AUTO, da.DA_KERNEL_VALU], ids=["auto", "valu"])
def test_half_workloads_match_oracle(name, div, over, kernel):
    w = synth.make(synth.recipe(name, len_div=div, dtype="f16", **over), DEV)
    assert w["k_pool"].dtype == torch.float16 and w["q"].dtype == torch.float16
    print("case f16", name, div, over, kernel, flush=True)
    s = da.plan_schedule(da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"]), w["seq_lens_host"].tolist(), kernel=kernel)
    assert s["kernel"] == (da.DA_KERNEL_MFMA if kernel == da.DA_KERNEL_AUTO else da.DA_KERNEL_VALU)
    ref_out, ref_lse = oracle_attention(w)
    for bps in (0, 2):
        out, lse, flags = gpu_attention(w, kernel=kernel, blocks_per_split=bps)
        assert flags == 0
        max_abs, rel = assert_parity(out, lse, ref_out, ref_lse, "f16", "%s f16 bps=%d" % (name, bps))
        assert rel < 2e-5       # measured ~1e-6: half operands are exact in the products, weights carry 22 bits


def test_half_partials_match_micro_attention():
    w = synth.make(synth.recipe("c3_70b", len_div=128, dtype="f16"), DEV)
    plan = make_plan(w, blocks_per_split=1)
    po, pm, pe = plan.partial(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    torch.cuda.synchronize()
    B = w["B"]
    bounds = [[plan.split(r, j)[0] for j in range(plan.nsplits(r))] + [plan.split(r, plan.nsplits(r) - 1)[1]] for r in range(B)]
    MA, m, e, _ = oracle.micro_attention(bits(w["q"]), bits(w["k_pool"]), bits(w["v_pool"]), w["block_table_host"],
                                         w["seq_lens_host"], w["T"], w["scale"], bounds, n_threads=16)
    plan.close()
    assert np.allclose(pm.cpu().numpy(), m, rtol=0, atol=2e-5)
    assert np.allclose(pe.cpu().numpy(), e, rtol=2e-5, atol=1e-6)
    den = np.linalg.norm(MA)
    assert np.linalg.norm(po.cpu().numpy() - MA) / den < 2e-5


def test_small_weights_survive_the_half_range():
    """Every wavefront meets dominant keys first (score gap 13.8, so every later weight is 1.0e-6, below half's
    smallest normal number 6.1e-5) and then thousands of tokens whose values are large and of one sign: together they
    shift the output by 5 %.  Weights handed to the matrix cores as plain halves would be flushed or coarsely
    rounded; the kernel must keep them.  One compute unit, so that one workgroup reads the whole request."""
    T, L, d = 256, 60000, 128
    nb = (L + T - 1) // T
    k = torch.zeros((nb, 1, T, d), dtype=torch.float16, device=DEV)
    v = torch.full((nb, 1, T, d), 100.0, dtype=torch.float16, device=DEV)
    k[0, 0, 0:128, 0] = 16.0                   # q = (9.75, 0, ...), scale 1/sqrt(128): gap 156 / 11.31 = 13.79
    v[0, 0, 0:128] = -1.0                      # the first chunk of each of the 4 wavefronts holds dominant keys
    q = torch.zeros((1, 2, d), dtype=torch.float16, device=DEV)
    q[0, :, 0] = 9.75
    table = torch.arange(nb, dtype=torch.int32, device=DEV).reshape(1, nb)
    lens = torch.as_tensor([L], dtype=torch.int32, device=DEV)
    scale = 1.0 / np.sqrt(128.0)
    ref, ref_lse = oracle.attention(bits(q), bits(k), bits(v), table.cpu().numpy(), lens.cpu().numpy(), T, scale)
    tail_ref = ref[0, 0, 0] + 1.0
    assert 0.04 < tail_ref < 0.06
    for kernel in (da.DA_KERNEL_AUTO, da.DA_KERNEL_VALU):
        plan = da.Plan(da.make_problem(q, k, table, scale), [L], kernel=kernel, num_cus=1)
        assert plan.nsplits(0) == 1
        out, lse = plan.attention(q, k, v, table, lens)
        torch.cuda.synchronize()
        plan.close()
        tail_got = float(out[0, 0, 0].double()) + 1.0
        assert abs(tail_got - tail_ref) <= 2e-3 * tail_ref, (kernel, tail_got, tail_ref)
        assert_parity(out.cpu().numpy(), lse.cpu().numpy(), ref, ref_lse, "f16", "small weights")


def test_fp32_query_with_half_cache_and_multi_query():
    w = synth.make(synth.recipe("c5_mixed", len_div=200, dtype="f16", Hq=16, Hkv=4), DEV)
    w32 = dict(w)
    w32["q"] = w["q"].float()
    ref_out, ref_lse = oracle_attention(w32)
    out, lse, flags = gpu_attention(w32)         # mixed types go to the vector-ALU kernel
    assert flags == 0
    assert_parity(out, lse, ref_out, ref_lse, "f16", "fp32 q, half cache")
    # multi-query, 3 new tokens per request
    gen = torch.Generator(device=DEV)
    gen.manual_seed(2)
    wq = dict(w)
    wq["q"] = torch.randn((w["B"], 3, 16, 128), device=DEV, generator=gen).to(torch.float16)
    ref_out, ref_lse = oracle.attention(bits(wq["q"]), bits(w["k_pool"]), bits(w["v_pool"]), w["block_table_host"],
                                        w["seq_lens_host"], w["T"], w["scale"], n_threads=16)
    for kernel in (da.DA_KERNEL_AUTO, da.DA_KERNEL_VALU):
        plan = da.Plan(da.make_problem(wq["q"], w["k_pool"], w["block_table"], w["scale"]), w["seq_lens_host"].tolist(), kernel=kernel)
        out, lse = plan.attention(wq["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
        torch.cuda.synchronize()
        plan.close()
        assert_parity(out.cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, "f16", "f16 multi-query kernel=%d" % kernel)


def test_append_and_move_half_rows_bit_exact():
    T, B, Hkv = 16, 3, 2
    gen = torch.Generator(device=DEV)
    gen.manual_seed(8)
    k_pool = torch.randn((12, Hkv, T, 128), device=DEV, generator=gen).to(torch.float16)
    v_pool = torch.randn((12, Hkv, T, 128), device=DEV, generator=gen).to(torch.float16)
    table = np.arange(12, dtype=np.int32).reshape(3, 4)
    lens = np.array([5, 16, 63], dtype=np.int32)
    k_new = torch.randn((B, Hkv, 128), device=DEV, generator=gen).to(torch.float16)
    v_new = torch.randn((B, Hkv, 128), device=DEV, generator=gen).to(torch.float16)
    kp, vp, lens_ref = bits(k_pool).copy(), bits(v_pool).copy(), lens.copy()
    oracle.append(bits(k_new), bits(v_new), kp, vp, table, lens_ref)
    d_table, d_lens = torch.as_tensor(table, device=DEV), torch.as_tensor(lens, device=DEV)
    prob = da.make_problem(k_new, k_pool, d_table, 1.0)
    da.append(prob, k_new, v_new, k_pool, v_pool, d_table, d_lens)
    torch.cuda.synchronize()
    assert np.array_equal(d_lens.cpu().numpy(), lens_ref)
    assert np.array_equal(bits(k_pool).view(np.uint16), kp.view(np.uint16)) and np.array_equal(bits(v_pool).view(np.uint16), vp.view(np.uint16))
    kd = torch.zeros((5, Hkv, T, 128), dtype=torch.float16, device=DEV)
    vd = torch.zeros_like(kd)
    hk, hv = bits(kd).copy(), bits(vd).copy()
    oracle.move_blocks(bits(k_pool), bits(v_pool), hk, hv, [11, 0, 4], [2, 4, 0])
    prob_d = da.make_problem(k_new, kd, d_table, 1.0)
    da.move_blocks(prob, prob_d, k_pool, v_pool, kd, vd, torch.as_tensor([11, 0, 4], dtype=torch.int32, device=DEV),
                   torch.as_tensor([2, 4, 0], dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    assert np.array_equal(bits(kd).view(np.uint16), hk.view(np.uint16)) and np.array_equal(bits(vd).view(np.uint16), hv.view(np.uint16))


@pytest.mark.parametrize("dtype,Hq,Hkv,n", [("f16", 8, 2, 2), ("f16", 16, 1, 3), ("bf16", 8, 2, 2), ("bf16", 8, 1, 8)])
def test_chunk_invisible_to_a_column_with_strongly_negative_scores(dtype, Hq, Hkv, n):
    # every score is about -150: a column's running maximum is far below the point where exp2(-maximum) overflows.
    # Lengths 32 k + 1 put the newest token alone in the last chunk, which the earlier query tokens may not see at
    # all: that chunk has to join their sums with weight 0, not with 0 * inf.
    lens = [33, 65, 1, 97, 2049, 32 * 7 + n - 1]
    w = synth.make(synth.recipe("c5_mixed", B=len(lens), Hq=Hq, Hkv=Hkv, T=64, dtype=dtype, lens=lens), DEV)
    tdt = torch.float16 if dtype == "f16" else torch.bfloat16
    gen = torch.Generator(device=DEV)
    gen.manual_seed(5)
    w["q"] = torch.ones((len(lens), n, Hq, 128), device=DEV).to(tdt)
    k = w["k_pool"]
    noise = torch.randn(k.shape, device=DEV, generator=gen) * 0.05 - 1.2
    w["k_pool"].copy_(torch.where(torch.isnan(k.float()), k.float(), noise).to(tdt))  # the poison in unused slots stays
    w["scale"] = 1.0
    ref_out, ref_lse = oracle.attention(bits(w["q"]), bits(w["k_pool"]), bits(w["v_pool"]), w["block_table_host"],
                                        w["seq_lens_host"], w["T"], w["scale"], n_threads=16)
    assert np.all(np.isfinite(ref_out)) and ref_lse[np.isfinite(ref_lse)].max() < -100
    for kernel in (da.DA_KERNEL_AUTO, da.DA_KERNEL_VALU):
        plan = da.Plan(da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"]), w["seq_lens_host"].tolist(), kernel=kernel)
        out, lse = plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
        torch.cuda.synchronize()
        plan.close()
        assert_parity(out.cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, dtype, "%s kernel=%d" % (dtype, kernel))
