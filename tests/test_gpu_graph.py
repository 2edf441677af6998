"""A decode step (da_append + da_attention) captured once in a HIP graph and replayed: every replay is checked
against the oracle, with eager work and synchronisation between replays.  The captured launches carry the plan
that was current at capture time; the device lengths grow with every replay, so all later replays run on a stale
plan and must still be exact (the last split of a request is open-ended)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2401_02669_amd import distattn as da
from paper_2401_02669_amd import synth
from util import assert_parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def bits(t):
    return synth.as_numpy(t)


@pytest.mark.parametrize("Hq,Hkv,dtype", [(8, 2, "bf16"), (4, 4, "bf16"), (2, 2, "f32")])
def test_captured_decode_step_replays_exactly(Hq, Hkv, dtype):
    T, B, steps = 32, 4, 24
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    start = np.array([700, 31, 0, 2049], dtype=np.int32)
    max_blocks = 80
    num_phys = 4 * max_blocks
    rng = np.random.RandomState(5)
    table = rng.permutation(num_phys).astype(np.int32).reshape(B, max_blocks)   # every block the loop will need
    gen = torch.Generator(device=DEV)
    gen.manual_seed(21)
    k_pool = torch.randn((num_phys, Hkv, T, 128), device=DEV, generator=gen).to(tdt)
    v_pool = torch.randn((num_phys, Hkv, T, 128), device=DEV, generator=gen).to(tdt)
    d_table = torch.as_tensor(table, device=DEV)
    d_lens = torch.as_tensor(start, device=DEV)
    # static buffers of the captured step
    q_buf = torch.zeros((B, Hq, 128), dtype=tdt, device=DEV)
    kn_buf = torch.zeros((B, Hkv, 128), dtype=tdt, device=DEV)
    vn_buf = torch.zeros((B, Hkv, 128), dtype=tdt, device=DEV)
    out = torch.zeros((B, Hq, 128), dtype=torch.float32, device=DEV)
    lse = torch.zeros((B, Hq), dtype=torch.float32, device=DEV)
    prob = da.make_problem(q_buf, k_pool, d_table, 0.088)
    plan = da.Plan(prob, (start + 1).tolist())
    ws = torch.empty((max(plan.workspace_bytes, 256) + 4096,), dtype=torch.uint8, device=DEV)
    # host mirror for the oracle
    kp, vp = bits(k_pool).copy(), bits(v_pool).copy()
    lens_ref = start.copy()

    def step():
        da.append(prob, kn_buf, vn_buf, k_pool, v_pool, d_table, d_lens)
        plan.attention(q_buf, k_pool, v_pool, d_table, d_lens, out, lse, ws)

    def feed():
        q = torch.randn((B, Hq, 128), device=DEV, generator=gen).to(tdt)
        kn = torch.randn((B, Hkv, 128), device=DEV, generator=gen).to(tdt)
        vn = torch.randn((B, Hkv, 128), device=DEV, generator=gen).to(tdt)
        q_buf.copy_(q); kn_buf.copy_(kn); vn_buf.copy_(vn)
        oracle.append(bits(kn), bits(vn), kp, vp, table, lens_ref)
        return bits(q)

    def check(q_bits, what):
        torch.cuda.synchronize()
        assert np.array_equal(d_lens.cpu().numpy(), lens_ref), what
        ref_out, ref_lse = oracle.attention(q_bits, kp, vp, table, lens_ref, T, 0.088, n_threads=8)
        assert_parity(out.cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, dtype, what)

    # one eager step first (also the warm-up that capture wants)
    qb = feed()
    step()
    check(qb, "eager step")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    qb = feed()
    with torch.cuda.graph(graph, stream=side):
        step()
    graph.replay()                       # capture records, the first replay runs the step fed above
    check(qb, "first replay")
    for s in range(steps):
        qb = feed()
        if s % 5 == 2:                   # eager work of the program's own between replays
            (k_pool[0, 0, 0] * 1.0).sum().item()
        graph.replay()
        print("replay", s, "lens", lens_ref.tolist(), flush=True)
        check(qb, "replay %d" % s)
    assert np.array_equal(bits(k_pool), kp) and np.array_equal(bits(v_pool), vp)
    assert plan.error_flags() == 0
    # a re-plan is a re-capture: the new graph carries the new schedule
    plan.update(lens_ref.tolist())
    graph2 = torch.cuda.CUDAGraph()
    qb = feed()
    with torch.cuda.graph(graph2, stream=side):
        step()
    graph2.replay()
    check(qb, "re-captured")
    qb = feed()
    graph2.replay()
    check(qb, "re-captured, second replay")
    del graph, graph2
    plan.close()
