"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times (default plan,
da_plan_update + da_partial + da_combine, and the fused da_attention): a seeded sample of (request,
q-head) outputs is recomputed by the fp64 oracle from the same stored K/V, through the same block table."""
import numpy as np
import pytest
import torch

import oracle
from paper_2401_02669_amd import distattn as da
from paper_2401_02669_amd import synth
from util import TOL, errors

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


# every (request, q-head) output of c2_7b, c3_70b and c4_2m; a seeded half of c5_mixed's 2048
@pytest.mark.parametrize("name,n_pairs", [("c2_7b", 512), ("c3_70b", 256), ("c4_2m", 64), ("c5_mixed", 1024)])
def test_full_size_sampled_outputs_match_oracle(name, n_pairs):
    print("case full-size %s" % name, flush=True)
    w = synth.make(synth.recipe(name), DEV)
    prob = da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"])
    lens = w["seq_lens_host"].tolist()
    plan = da.Plan(prob, lens)
    plan.update(lens)
    po, pm, pe = plan.partial(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    out, lse = plan.combine(po, pm, pe)
    out2, lse2 = plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    torch.cuda.synchronize()
    assert plan.error_flags() == 0
    plan.close()
    assert torch.isfinite(out).all() and torch.isfinite(out2).all()

    # sample: the longest and the shortest request, and a seeded draw of the rest
    rng = np.random.RandomState(99)
    if n_pairs >= w["B"] * w["Hq"]:
        pairs = np.array([[r, h] for r in range(w["B"]) for h in range(w["Hq"])], dtype=np.int32)
    else:
        rs = [int(np.argmax(w["seq_lens_host"])), int(np.argmin(w["seq_lens_host"]))]
        rs += [int(x) for x in rng.randint(0, w["B"], size=n_pairs - 2)]
        pairs = np.array([[r, int(rng.randint(0, w["Hq"]))] for r in rs], dtype=np.int32)
    host = dict(q=synth.as_numpy(w["q"]), k=synth.as_numpy(w["k_pool"]), v=synth.as_numpy(w["v_pool"]))
    ref, ref_lse = oracle.attention(host["q"], host["k"], host["v"], w["block_table_host"], w["seq_lens_host"], w["T"],
                                    w["scale"], pairs=pairs, n_threads=16)
    tol = TOL[w["dtype"]]
    for got_out, got_lse, what in ((out, lse, "partial+combine"), (out2, lse2, "fused")):
        got = got_out.cpu().numpy().astype(np.float64)[pairs[:, 0], pairs[:, 1]]
        gl = got_lse.cpu().numpy().astype(np.float64)[pairs[:, 0], pairs[:, 1]]
        max_abs, rel = errors(got, ref)
        assert max_abs <= tol["max_abs"] and rel <= tol["rel_l2"], (what, max_abs, rel)
        for i in range(len(pairs)):  # per output row as well: long requests have tiny outputs
            _, rel_i = errors(got[i], ref[i])
            assert rel_i <= tol["rel_l2"], (what, pairs[i], rel_i)
        assert np.max(np.abs(gl - ref_lse) / np.maximum(1.0, np.abs(ref_lse))) <= tol["lse"]


@pytest.mark.parametrize("name,q_len,n_pairs", [("c3_70b", 4, 384), ("c3_70b", 8, 384), ("c3_70b", 16, 384),
                                                 ("c4_2m", 4, 48), ("c5_mixed", 8, 384)])
def test_full_size_multi_query_sampled_outputs_match_oracle(name, q_len, n_pairs):
    # several query tokens per request: 32, 64 and 128 columns per K/V read (the multi-tile kernel), at full size:
    # c3_70b, one request of 2M tokens cut into many splits, and the mixed lengths (many short items per workgroup);
    # a seeded sample of (request, query token, q-head) outputs
    print("case full-size %s q_len %d" % (name, q_len), flush=True)
    w = synth.make(synth.recipe(name), DEV)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(4242)
    q = torch.randn((w["B"], q_len, w["Hq"], 128), device=DEV, generator=gen).to(w["q"].dtype)
    prob = da.make_problem(q, w["k_pool"], w["block_table"], w["scale"])
    plan = da.Plan(prob, w["seq_lens_host"].tolist())
    out, lse = plan.attention(q, w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    torch.cuda.synchronize()
    assert plan.error_flags() == 0
    plan.close()
    rng = np.random.RandomState(7 + q_len)
    vh = w["Hq"] * q_len  # virtual heads: query token * Hq + q-head
    pairs = np.array([[int(rng.randint(0, w["B"])), int(rng.randint(0, vh))] for _ in range(n_pairs - 2)]
                     + [[0, 0], [w["B"] - 1, vh - 1]], dtype=np.int32)
    ref, ref_lse = oracle.attention(synth.as_numpy(q), synth.as_numpy(w["k_pool"]), synth.as_numpy(w["v_pool"]),
                                    w["block_table_host"], w["seq_lens_host"], w["T"], w["scale"], pairs=pairs, n_threads=16)
    got = out.cpu().numpy().astype(np.float64).reshape(w["B"], vh, 128)[pairs[:, 0], pairs[:, 1]]
    gl = lse.cpu().numpy().astype(np.float64).reshape(w["B"], vh)[pairs[:, 0], pairs[:, 1]]
    tol = TOL["bf16"]
    max_abs, rel = errors(got, ref)
    assert max_abs <= tol["max_abs"] and rel <= tol["rel_l2"], (max_abs, rel)
    for i in range(len(pairs)):
        _, rel_i = errors(got[i], ref[i])
        assert rel_i <= tol["rel_l2"], (pairs[i], rel_i)
    assert np.max(np.abs(gl - ref_lse) / np.maximum(1.0, np.abs(ref_lse))) <= tol["lse"]
