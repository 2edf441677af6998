"""Seeded random small problems across the option space (operand types, group sizes, block sizes, query tokens,
split modes, kernel families, compute-unit counts, ragged lengths), each checked against the fp64 oracle through
the fused call and through da_partial + da_combine."""
import numpy as np
import pytest
import torch

import oracle
from paper_2401_02669_amd import distattn as da
from paper_2401_02669_amd import synth
from util import assert_parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def draw(seed):
    rng = np.random.RandomState(9000 + seed)
    dtype = ["bf16", "f16", "f32"][seed % 3]
    Hkv = int(rng.choice([1, 2, 3, 8]))
    G = int(rng.choice([1, 2, 4, 5, 8, 16, 20]))
    T = int(rng.choice([16, 32, 48, 64, 128, 256]))
    q_len = int(rng.choice([1, 1, 1, 2, 3, 7]))
    B = int(rng.choice([1, 2, 5, 17, 60, 300]))
    top = int(rng.choice([40, 300, 3000])) if B > 20 else int(rng.choice([100, 3000, 20000]))
    lens = [int(x) for x in rng.randint(0, top + 1, size=B)]
    lens[int(rng.randint(B))] = top                 # at least one request of the top length
    tuning = dict(blocks_per_split=int(rng.choice([0, 0, 0, 1, 3])), kernel=int(rng.choice([0, 0, 1, 2])),
                  num_cus=int(rng.choice([0, 0, 8, 40, 256])))
    return dtype, Hkv, G, T, q_len, lens, tuning


@pytest.mark.parametrize("seed", range(36))
def test_random_problem(seed):
    dtype, Hkv, G, T, q_len, lens, tuning = draw(seed)
    Hq = Hkv * G
    print("case seed=%d %s Hq=%d Hkv=%d T=%d q_len=%d B=%d max_len=%d %s" % (seed, dtype, Hq, Hkv, T, q_len, len(lens), max(lens), tuning),
          flush=True)
    w = synth.make(synth.recipe("c5_mixed", B=len(lens), Hq=Hq, Hkv=Hkv, T=T, dtype=dtype, lens=lens, index=50 + seed), DEV)
    q = w["q"]
    if q_len > 1:
        gen = torch.Generator(device=DEV)
        gen.manual_seed(seed)
        q = torch.randn((len(lens), q_len, Hq, 128), device=DEV, generator=gen).to(w["q"].dtype)
    prob = da.make_problem(q, w["k_pool"], w["block_table"], w["scale"])
    try:
        plan = da.Plan(prob, lens, **tuning)
    except da.DistAttnError as e:
        # the only legitimate refusal: the matrix-core family asked for with nothing it could run (never happens
        # here, q and the cache share a type) -- anything else is a failure
        raise AssertionError("plan refused: %s" % e)
    ref_out, ref_lse = oracle.attention(synth.as_numpy(q), synth.as_numpy(w["k_pool"]), synth.as_numpy(w["v_pool"]),
                                        w["block_table_host"], w["seq_lens_host"], T, w["scale"], n_threads=16)
    out, lse = plan.attention(q, w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    po, pm, pe = plan.partial(q, w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    out2, lse2 = plan.combine(po, pm, pe)
    torch.cuda.synchronize()
    assert plan.error_flags() == 0
    plan.close()
    assert_parity(out.cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, dtype, "seed %d fused" % seed)
    assert_parity(out2.cpu().numpy(), lse2.cpu().numpy(), ref_out, ref_lse, dtype, "seed %d two calls" % seed)
