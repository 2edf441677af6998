"""Timing aid: what moving KV blocks on a second stream costs the attention step that runs beside it (the
experiment behind Section 7.4 "Overhead of KVCache movement", on one GPU: both streams draw on the same HBM).
Prints a table; not part of the library.  Run: python -m paper_2401_02669_amd.move_probe [--workload c3_70b]"""
import argparse
import time

import torch

from . import distattn as da
from . import synth


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="c3_70b")
    ap.add_argument("--steps", type=int, default=50)
    a = ap.parse_args()
    dev = "cuda:0"
    w = synth.make(synth.recipe(a.workload), dev, poison=False)
    T, Hkv = w["T"], w["Hkv"]
    prob = da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"])
    plan = da.Plan(prob, w["seq_lens_host"].tolist())
    ws = torch.empty((max(plan.workspace_bytes, 256),), dtype=torch.uint8, device=dev)
    out = torch.empty((w["B"], w["Hq"], 128), dtype=torch.float32, device=dev)
    lse = torch.empty((w["B"], w["Hq"]), dtype=torch.float32, device=dev)
    nmax = 256
    away_k = torch.empty((nmax,) + tuple(w["k_pool"].shape[1:]), dtype=w["k_pool"].dtype, device=dev)
    away_v = torch.empty_like(away_k)
    lay_src = prob
    lay_dst = da.make_problem(w["q"], away_k, w["block_table"], w["scale"])
    block_bytes = 2 * Hkv * T * 128 * w["k_pool"].element_size()
    mover = torch.cuda.Stream()
    main_s = torch.cuda.current_stream()

    def attention():
        plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"], out, lse, ws)

    print("| blocks moved per step | KV tokens moved per step | bytes per step | attention step ms | slowdown | move alone, GB/s (read + write) |")
    print("|---|---|---|---|---|---|")
    base = None
    for n in (0, 1, 4, 16, 64, 256):
        src = torch.arange(n, dtype=torch.int32, device=dev)
        dst = torch.arange(n, dtype=torch.int32, device=dev)
        alone = 0.0
        if n:
            for _ in range(3):
                da.move_blocks(lay_src, lay_dst, w["k_pool"], w["v_pool"], away_k, away_v, src, dst)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(20):
                da.move_blocks(lay_src, lay_dst, w["k_pool"], w["v_pool"], away_k, away_v, src, dst)
            torch.cuda.synchronize()
            alone = 2 * n * block_bytes / ((time.perf_counter() - t0) / 20) / 1e9
        def step():
            if n:
                mover.wait_stream(main_s)      # the step's move starts with the step
                with torch.cuda.stream(mover):
                    da.move_blocks(lay_src, lay_dst, w["k_pool"], w["v_pool"], away_k, away_v, src, dst, stream=mover)
            attention()

        for _ in range(10):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / a.steps * 1e3
        base = base or ms
        print("| %d | %d | %.1f MB | %.4f | %+.1f %% | %s |" % (n, n * T, n * block_bytes / 1e6, ms, 100 * (ms / base - 1),
                                                            ("%.0f" % alone) if n else "—"), flush=True)
    plan.close()


if __name__ == "__main__":
    main()
