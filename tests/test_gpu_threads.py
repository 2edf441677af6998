"""One plan shared by two host threads: the launch calls only read a plan, so two threads may enqueue
da_partial / da_combine / da_attention / da_combine_multi on it at the same time, each on its own stream with its
own outputs and workspace.  Every result of both threads is checked against the fp64 oracle.  Covers a schedule
small enough to travel in the kernel arguments and one that lives in device tables."""
import threading

import pytest
import torch

from paper_2401_02669_amd import distattn as da
from paper_2401_02669_amd import synth
from util import assert_parity, make_plan, oracle_attention

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("name,div,over", [
    ("c5_mixed", 40, {}),                                            # 64 requests: schedule in the kernel arguments
    ("c5_mixed", 200, dict(B=150, lens="loguniform", Hq=16, Hkv=4)),  # 150 requests: device tables
])
def test_two_threads_two_streams_one_plan(name, div, over):
    w = synth.make(synth.recipe(name, len_div=div, **over), DEV)
    plan = make_plan(w)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(11)
    qs = [w["q"], torch.randn(w["q"].shape, device=DEV, generator=gen).to(w["q"].dtype)]
    refs = []
    for q in qs:
        w2 = dict(w)
        w2["q"] = q
        refs.append(oracle_attention(w2))
    torch.cuda.synchronize()
    results = [[], []]
    errors = []

    def worker(i):
        try:
            torch.cuda.set_device(0)
            stream = torch.cuda.Stream()
            a = (qs[i], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
            ws = torch.empty((max(plan.workspace_bytes, 256),), dtype=torch.uint8, device=DEV)
            for rep in range(6):
                out, lse = plan.attention(*a, workspace=ws, stream=stream)
                po, pm, pe = plan.partial(*a, stream=stream)
                out2, lse2 = plan.combine(po, pm, pe, stream=stream)
                out3, lse3 = da.combine_multi([(plan, po, pm, pe)], stream=stream)
                stream.synchronize()
                results[i].append([(o.cpu().numpy(), l.cpu().numpy()) for o, l in ((out, lse), (out2, lse2), (out3, lse3))])
        except Exception as e:  # reported by the main thread
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for i in range(2):
        assert len(results[i]) == 6
        for rep, trio in enumerate(results[i]):
            for k, (o, l) in enumerate(trio):
                assert_parity(o, l, refs[i][0], refs[i][1], w["dtype"], "thread %d rep %d call %d" % (i, rep, k))
    assert plan.error_flags() == 0
    plan.close()
