"""Timing aid: one decode token through `layers` attention layers (da_append + da_attention each, every layer with
its own KV pools), launched eagerly and replayed from one HIP graph.  Prints a table; not part of the library."""
import argparse
import ctypes
import time

import torch

from . import distattn as da
from . import synth


def run(B, L, Hq, Hkv, T, layers, reps):
    dev = "cuda:0"
    r = synth.recipe("c5_mixed", B=B, Hq=Hq, Hkv=Hkv, T=T, lens=[L] * B, spare_frac=0.02)
    ws = []
    for layer in range(layers):
        r["index"] = 100 + layer
        ws.append(synth.make(r, dev, poison=False))
    w0 = ws[0]
    prob = da.make_problem(w0["q"], w0["k_pool"], w0["block_table"], w0["scale"])
    lens = w0["seq_lens_host"].tolist()
    plans = [da.Plan(prob, lens) for _ in range(layers)]
    wsb = [torch.empty((max(p.workspace_bytes, 256),), dtype=torch.uint8, device=dev) for p in plans]
    out = torch.empty((B, Hq, 128), dtype=torch.float32, device=dev)
    lse = torch.empty((B, Hq), dtype=torch.float32, device=dev)
    kn = torch.randn((B, Hkv, 128), device=dev).to(torch.bfloat16)
    # the appended token overwrites the same slot every time: lengths are put back after each token
    saved = [w["seq_lens"].clone() for w in ws]

    def token():
        for i, w in enumerate(ws):
            da.append(prob, kn, kn, w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
            plans[i].attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"], out, lse, wsb[i])
            w["seq_lens"].copy_(saved[i])

    def timed(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e3

    eager = timed(token)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        token()
    graph = timed(g.replay)
    kv = w0["kv_bytes"] * layers
    print("| %d x %d | %d/%d | %d | %.3f | %.3f | %.0f | %.0f |" % (B, L, Hq, Hkv, layers, eager, graph, kv / eager / 1e6, kv / graph / 1e6),
          flush=True)
    for p in plans:
        p.close()


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=20)
    a = ap.parse_args()
    print("| batch x context | Hq/Hkv | layers | eager ms/token | graph ms/token | eager GB/s | graph GB/s |")
    print("|---|---|---|---|---|---|---|")
    run(1, 4096, 64, 8, 256, 32, a.reps)
    run(1, 32768, 64, 8, 256, 32, a.reps)
    run(4, 32768, 64, 8, 256, 32, a.reps)
    run(16, 32768, 64, 8, 256, 16, a.reps)
