"""Timing of the two-share (debtor / creditor) form on one GPU.

A workload's KV blocks are divided between two pools; each share gets its own plan, sized for half of
the compute units, and its own stream; the home stream aggregates both partial sets with
da_combine_multi.  Prints the time of (a) the undivided da_attention, (b) both shares one after the
other on one stream, (c) both shares on two streams at once.  On one GPU the shares compete for the
same HBM, so (c) can at best equal (a): the figure shows what the division itself costs.
Usage: python -m paper_2401_02669_amd.shares_probe [workload] [remote_fraction]
"""
import sys

import numpy as np
import torch

from paper_2401_02669_amd import distattn as da
from paper_2401_02669_amd import synth


def main():
    name = sys.argv[1] if len(sys.argv) > 1 else "c3_70b"
    frac = float(sys.argv[2]) if len(sys.argv) > 2 else 0.5
    dev = "cuda:0"
    w = synth.make(synth.recipe(name), dev, poison=False)
    T, B = w["T"], w["B"]
    lens, table = w["seq_lens_host"], w["block_table_host"]
    nb = (lens + T - 1) // T
    cus = torch.cuda.get_device_properties(0).multi_processor_count

    shares = []
    for which in (0, 1):  # 0: remote (first blocks), 1: local (the rest)
        tab = np.full_like(table, -1)
        new_lens = []
        for r in range(B):
            k = int(nb[r] * frac)
            ids = table[r, :k] if which == 0 else table[r, k: nb[r]]
            tab[r, : len(ids)] = ids
            tok_remote = min(int(lens[r]), k * T)
            new_lens.append(tok_remote if which == 0 else int(lens[r]) - tok_remote)
        shares.append(dict(table=torch.as_tensor(tab, device=dev), lens=new_lens,
                           seq_lens=torch.as_tensor(np.array(new_lens, dtype=np.int32), device=dev)))
    # (both shares read the same physical pool here: only the block tables differ, the bytes read are the same)

    def timed(fn, reps=20):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    prob = da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"])
    whole = da.Plan(prob, lens.tolist())
    ws = torch.empty((max(whole.workspace_bytes, 256),), dtype=torch.uint8, device=dev)
    out = torch.empty((B, w["Hq"], 128), dtype=torch.float32, device=dev)
    lse = torch.empty((B, w["Hq"]), dtype=torch.float32, device=dev)
    t_whole = timed(lambda: whole.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"], out, lse, ws))

    main_stream = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    plans, bufs = [], []
    for s in shares:
        p = da.make_problem(w["q"], w["k_pool"], s["table"], w["scale"])
        plan = da.Plan(p, s["lens"], num_cus=cus // 2)
        n = plan.num_partials
        plans.append(plan)
        bufs.append((torch.empty((n, 128), dtype=torch.float32, device=dev), torch.empty(n, dtype=torch.float32, device=dev),
                     torch.empty(n, dtype=torch.float32, device=dev)))
    out2, lse2 = torch.empty_like(out), torch.empty_like(lse)
    sets = [(plans[i],) + bufs[i] for i in range(2)]

    def serial():
        for i in range(2):
            plans[i].partial(w["q"], w["k_pool"], w["v_pool"], shares[i]["table"], shares[i]["seq_lens"], *bufs[i])
        da.combine_multi(sets, out2, lse2)

    def overlapped():
        side.wait_stream(main_stream)
        plans[0].partial(w["q"], w["k_pool"], w["v_pool"], shares[0]["table"], shares[0]["seq_lens"], *bufs[0], stream=side)
        plans[1].partial(w["q"], w["k_pool"], w["v_pool"], shares[1]["table"], shares[1]["seq_lens"], *bufs[1])
        main_stream.wait_stream(side)
        da.combine_multi(sets, out2, lse2)

    t_serial = timed(serial)
    t_overlap = timed(overlapped)
    torch.cuda.synchronize()
    err = float((out2 - out).abs().max())
    gb = w["kv_bytes"] / 1e9
    print("%s, %.0f %% of the blocks in the remote share, %.2f GB of K/V" % (name, 100 * frac, gb))
    print("  undivided da_attention            %.4f ms  %.0f GB/s" % (t_whole, gb / t_whole * 1e3))
    print("  two shares, one stream            %.4f ms  %.0f GB/s" % (t_serial, gb / t_serial * 1e3))
    print("  two shares, two streams           %.4f ms  %.0f GB/s" % (t_overlap, gb / t_overlap * 1e3))
    print("  max |two-share - undivided| = %.2e" % err, flush=True)
    for p in plans + [whole]:
        p.close()


if __name__ == "__main__":
    main()
