"""da_attention (MicroAttention + aggregation on one stream) against the fp64 oracle and against separate
da_partial + da_combine calls: on repeated calls through one plan, with a second query, after plan updates, with
a plan that is a few tokens stale, with short and long split lists, and in the multi-query form."""
import numpy as np
import pytest
import torch

from paper_2401_02669_amd import distattn as da
from paper_2401_02669_amd import synth
from util import assert_parity, make_plan, oracle_attention, oracle_inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def split_counts(plan, B):
    return [plan.nsplits(r) for r in range(B)]


def both_ways(plan, w, q=None, lens_dev=None):
    q = w["q"] if q is None else q
    lens_dev = w["seq_lens"] if lens_dev is None else lens_dev
    a = (q, w["k_pool"], w["v_pool"], w["block_table"], lens_dev)
    out, lse = plan.attention(*a)
    po, pm, pe = plan.partial(*a)
    out2, lse2 = plan.combine(po, pm, pe)
    torch.cuda.synchronize()
    return out, lse, out2, lse2


@pytest.mark.parametrize("name,div,over", [
    ("c3_70b", 64, {}), ("c4_2m", 64, {}), ("c5_mixed", 32, {}), ("c2_7b", 16, dict(B=3)),
    ("c1_tiny", 1, dict(B=4, lens=[4096, 333, 0, 2900])), ("c5_mixed", 50, dict(Hq=40, Hkv=8)),
])
def test_fused_call_equals_oracle_and_separate_calls(name, div, over):
    w = synth.make(synth.recipe(name, len_div=div, **over), DEV)
    plan = make_plan(w)
    ns = split_counts(plan, w["B"])
    assert max(ns) > 1, ns                 # the case under test: requests cut into several splits
    ref_out, ref_lse = oracle_attention(w)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(5)
    for rep in range(3):
        out, lse, out2, lse2 = both_ways(plan, w)
        print(name, "rep", rep, "splits", max(ns), flush=True)
        assert_parity(out.cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, w["dtype"], "%s rep %d" % (name, rep))
        # same partial rows, same weights; only the order of the sums differs
        assert torch.allclose(out, out2, rtol=2e-5, atol=2e-6)
        assert torch.allclose(lse, lse2, rtol=1e-5, atol=1e-5)
    # another query through the same plan
    q2 = torch.randn(w["q"].shape, device=DEV, generator=gen).to(w["q"].dtype)
    w2 = dict(w)
    w2["q"] = q2
    ref_out, ref_lse = oracle_attention(w2)
    out, lse, out2, lse2 = both_ways(plan, w, q=q2)
    assert_parity(out.cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, w["dtype"], name + " second query")
    assert plan.error_flags() == 0
    plan.close()


def test_after_plan_updates_and_with_a_stale_plan():
    w = synth.make(synth.recipe("c5_mixed", len_div=40), DEV)
    plan = make_plan(w)
    base = w["seq_lens_host"].astype(np.int64)
    for step, f in enumerate((1.0, 0.37, 0.9, 0.05)):
        lens = np.maximum((base * f).astype(np.int32), 1)
        plan.update(lens.tolist())
        w2 = dict(w)
        w2["seq_lens"] = torch.as_tensor(lens, device=DEV)
        ref_out, ref_lse = oracle_attention(w2, oracle_inputs(w2))
        out, lse = plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w2["seq_lens"])
        torch.cuda.synchronize()
        assert_parity(out.cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, "bf16", "update %d" % step)
        # the device lengths move on without a re-plan
        lens3 = np.maximum(lens - 7, 0).astype(np.int32)
        w3 = dict(w)
        w3["seq_lens"] = torch.as_tensor(lens3, device=DEV)
        ref_out, ref_lse = oracle_attention(w3, oracle_inputs(w3))
        out, lse = plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w3["seq_lens"])
        torch.cuda.synchronize()
        assert_parity(out.cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, "bf16", "stale %d" % step)
    plan.close()


def test_long_split_lists():
    w = synth.make(synth.recipe("c3_70b", len_div=4), DEV)
    ref_out, ref_lse = oracle_attention(w)
    plan = make_plan(w, blocks_per_split=1)
    assert max(split_counts(plan, w["B"])) > 64
    for rep in range(2):
        out, lse = plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
        torch.cuda.synchronize()
        assert_parity(out.cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, "bf16", "bps=1 rep %d" % rep)
    plan.close()
    for nblocks in (64, 65):
        w = synth.make(synth.recipe("c5_mixed", B=2, Hq=16, Hkv=4, T=32, lens=[32 * nblocks, 100]), DEV)
        ref_out, ref_lse = oracle_attention(w)
        plan = make_plan(w, blocks_per_split=1)
        assert max(split_counts(plan, 2)) == nblocks
        out, lse = plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
        torch.cuda.synchronize()
        assert_parity(out.cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, "bf16", "%d splits" % nblocks)
        plan.close()


def test_multi_query_form():
    import oracle
    lens = [9000, 4100, 37, 6000]
    w = synth.make(synth.recipe("c5_mixed", B=4, Hq=32, Hkv=8, T=64, lens=lens), DEV)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(11)
    for n in (2, 5):
        w["q"] = torch.randn((4, n, 32, 128), device=DEV, generator=gen).to(torch.bfloat16)
        prob = da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"])
        plan = da.Plan(prob, lens)
        assert max(split_counts(plan, 4)) > 1
        ref_out, ref_lse = oracle.attention(synth.as_numpy(w["q"]), synth.as_numpy(w["k_pool"]), synth.as_numpy(w["v_pool"]),
                                            w["block_table_host"], w["seq_lens_host"], w["T"], w["scale"], n_threads=16)
        for rep in range(2):
            out, lse = plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
            torch.cuda.synchronize()
            assert_parity(out.cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, "bf16", "q_len %d rep %d" % (n, rep))
        plan.close()
