"""Timing aid: a step (da_plan_update + da_attention) from one short request to one 2M-token request and over
batch sizes, as a table of K/V bytes, workgroups, time and read rate.  Not part of the library.
Run: python -m paper_2401_02669_amd.context_sweep"""
import ctypes

import torch

from . import distattn as da
from . import synth


def run(B, Hq, Hkv, L, T, reps=30):
    r = synth.recipe("c5_mixed", B=B, Hq=Hq, Hkv=Hkv, T=T, lens=[L] * B, spare_frac=0.0)
    w = synth.make(r, "cuda:0", poison=False)
    prob = da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"])
    lens = w["seq_lens_host"].tolist()
    plan = da.Plan(prob, lens)
    ws = torch.empty((max(plan.workspace_bytes, 256),), dtype=torch.uint8, device="cuda:0")
    out = torch.empty((B, Hq, 128), dtype=torch.float32, device="cuda:0"); lse = torch.empty((B, Hq), dtype=torch.float32, device="cuda:0")
    lens_c = (ctypes.c_int32 * B)(*lens); sp = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    def step():
        plan.update_raw(lens_c, sp)
        plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"], out, lse, ws)
    for _ in range(5): step()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps): step()
    e1.record(); torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    s = da.plan_schedule(prob, lens)
    print("| %d x %d | %d/%d | %.1f MB | %d | %.4f | %.0f | %.1f %% |" % (B, L, Hq, Hkv, w["kv_bytes"] / 1e6, s["workgroups"], ms, w["kv_bytes"] / ms / 1e6, w["kv_bytes"] / ms / 1e6 / 80), flush=True)
    plan.close()
    del w


def main():
    print("| batch x context | Hq/Hkv | K/V bytes | workgroups | step ms | GB/s | % of 8 TB/s |")
    for L in (1024, 4096, 16384, 32768, 131072, 524288, 2000000):
        run(1, 64, 8, L, 256)
    for B in (4, 16, 64):
        run(B, 64, 8, 32768, 256)
    for L in (4096, 32768, 262144):
        run(1, 32, 32, L, 256)
    # many short requests (what a lending instance serves): the same 8.6 GB in ever shorter pieces
    for B, L in ((256, 8192), (1024, 2048), (2048, 1024), (4096, 512)):
        run(B, 32, 8, L, 256)
    for B, L in ((256, 4096), (1024, 1024), (2048, 512)):
        run(B, 32, 32, L, 256)


if __name__ == "__main__":
    main()
