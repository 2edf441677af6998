#!/usr/bin/env python3
"""Benchmark of the DistAttention decode hot path on one MI355X.

A step = one pass of the whole path over one batch of synthetic input already resident in HBM:
work scheduling (da_plan_update, host) -> MicroAttention (da_partial) -> aggregation (da_combine).
Prints ONE JSON line: KV-read GB/s (algorithmic KV bytes / step time), the HBM roofline of the
MicroAttention kernel (HIP events around the da_partial launch of every 4th timed step), and the
fp64 CPU oracle timed on a bounded sample of the same workload on this machine's host cores.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak


def parse_traffic(workload):
    """HBM bytes per MicroAttention launch from the committed rocprofv3 --pmc summary, if one exists."""
    path = os.path.join(ROOT, "profiles", "micro_attention_%s_pmc.txt" % workload)
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        parts = line.split()
        if len(parts) == 2 and parts[0] in ("hbm_read_bytes_per_launch", "hbm_write_bytes_per_launch"):
            vals[parts[0]] = float(parts[1])
    if "hbm_read_bytes_per_launch" not in vals:
        return None
    return vals["hbm_read_bytes_per_launch"] + vals.get("hbm_write_bytes_per_launch", 0.0)


def cpu_baseline(w, host, budget_s, threads):
    """Time the oracle (as it stands) on a sample of (request, q-head) pairs; returns (dict, pairs, ref)."""
    import numpy as np
    import oracle

    B, Hq, Hkv = w["B"], w["Hq"], w["Hkv"]
    lens = w["seq_lens_host"].astype(np.int64)
    esize = 4 if w["dtype"] == "f32" else 2
    # cost of a pair is proportional to its length: probe with the shortest non-empty request
    order = np.argsort(lens)
    probe_r = int(next((r for r in order if lens[r] > 0), order[-1]))
    t0 = time.perf_counter()
    oracle.attention(host["q"], host["k_pool"], host["v_pool"], host["block_table"], host["seq_lens"], w["T"],
                     w["scale"], pairs=np.array([[probe_r, 0]], dtype=np.int32), n_threads=1)
    per_token = (time.perf_counter() - t0) / max(1, int(lens[probe_r]))
    # deterministic sample: walk pairs spread over requests and heads until the budget is filled
    rng = np.random.RandomState(1234)
    cand = [(r, h) for r in range(B) for h in range(Hq) if lens[r] > 0]
    rng.shuffle(cand)
    want = budget_s * threads / per_token  # tokens of pair-work that fit the budget
    pairs, tok = [], 0
    for r, h in cand:
        if pairs and tok + lens[r] > want:
            continue
        pairs.append((r, h))
        tok += int(lens[r])
        if tok >= want:
            break
    pairs = np.array(pairs, dtype=np.int32)
    t0 = time.perf_counter()
    ref, ref_lse = oracle.attention(host["q"], host["k_pool"], host["v_pool"], host["block_table"], host["seq_lens"],
                                    w["T"], w["scale"], pairs=pairs, n_threads=threads)
    dt = time.perf_counter() - t0
    # a pair stands for 1/G of its kv-head's bytes (the GPU reads K/V once per group)
    G = Hq // Hkv
    sample_bytes = float(tok) * 2 * w["d"] * esize / G
    info = dict(value=sample_bytes / dt / 1e9, unit="GB/s", cores=threads, kind="oracle",
                sample="%d of %d (request, q-head) pairs, %d pair-tokens, %.1f s" % (len(pairs), B * Hq, tok, dt),
                tokens_per_s=(sample_bytes / w["kv_bytes"]) * B / dt)
    return info, pairs, ref, ref_lse


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2_7b", help="c1_tiny c2_7b c3_70b c4_2m c5_mixed")
    ap.add_argument("--len-div", type=int, default=1, help="divide every length (debug only; result is not the named workload)")
    ap.add_argument("--blocks-per-split", type=int, default=0)
    ap.add_argument("--kernel", type=int, default=0, help="0 auto, 1 VALU, 2 MFMA")
    ap.add_argument("--q-len", type=int, default=1, help="query tokens per request (1 = decode, the headline metric)")
    ap.add_argument("--cpu-budget", type=float, default=15.0, help="seconds of oracle time for cpu_baseline (0 = skip)")
    ap.add_argument("--no-parity", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives or sharding); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2401_02669_amd import distattn as da
    from paper_2401_02669_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU", file=sys.stderr)
        sys.exit(2)
    da.lib()  # fail loudly if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)

    w = synth.make(synth.recipe(args.workload, len_div=args.len_div), dev)
    if args.q_len > 1:  # multi-query form: every request brings q_len new tokens (already in the cache)
        gen = torch.Generator(device=dev)
        gen.manual_seed(4242)
        w["q"] = torch.randn((w["B"], args.q_len, w["Hq"], 128), device=dev, generator=gen).to(w["q"].dtype)
    prob = da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"])
    lens_list = w["seq_lens_host"].tolist()
    plan = da.Plan(prob, lens_list, blocks_per_split=args.blocks_per_split, kernel=args.kernel)
    sched = da.plan_schedule(prob, lens_list, blocks_per_split=args.blocks_per_split, kernel=args.kernel,
                             num_cus=torch.cuda.get_device_properties(0).multi_processor_count)
    n = plan.num_partials
    part_o = torch.empty((n, 128), dtype=torch.float32, device=dev)
    part_m = torch.empty((n,), dtype=torch.float32, device=dev)
    part_e = torch.empty((n,), dtype=torch.float32, device=dev)
    oshape = (w["B"], w["Hq"]) if args.q_len <= 1 else (w["B"], args.q_len, w["Hq"])
    out = torch.empty(oshape + (128,), dtype=torch.float32, device=dev)
    lse = torch.empty(oshape, dtype=torch.float32, device=dev)
    lens_c = (ctypes.c_int32 * w["B"])(*lens_list)
    stream = torch.cuda.current_stream()
    sptr = ctypes.c_void_p(stream.cuda_stream)
    args_partial = (w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"], part_o, part_m, part_e)

    def step(e0=None, e1=None):
        plan.update_raw(lens_c, sptr)
        if e0 is not None:
            e0.record(stream)
        plan.partial(*args_partial)
        if e1 is not None:
            e1.record(stream)
        plan.combine(part_o, part_m, part_e, out, lse)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # HIP events bracket the MicroAttention launch of every 4th timed step (an event pair costs a few
    # microseconds of stream time, which would otherwise show up in every step)
    ev = {i: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for i in range(0, args.steps, 4)}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(*ev.get(i, (None, None)))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kern_ms = sum(a.elapsed_time(b) for a, b in ev.values()) / len(ev)
    assert plan.error_flags() == 0

    # the fused convenience call, for reference (same kernels; single-split requests skip the aggregation)
    ws = torch.empty((max(plan.workspace_bytes, 256),), dtype=torch.uint8, device=dev)
    out2 = torch.empty_like(out)
    lse2 = torch.empty_like(lse)
    for _ in range(3):
        plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"], out2, lse2, ws)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(args.steps):
        plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"], out2, lse2, ws)
    torch.cuda.synchronize()
    fused_ms = (time.perf_counter() - t2) * 1e3 / args.steps

    kv_bytes = float(w["kv_bytes"])
    value = kv_bytes / (ms_per_step * 1e-3) / 1e9
    achieved = kv_bytes / (kern_ms * 1e-3) / 1e9
    result = {
        "metric": "kv_read_hbm_GBps", "value": round(value, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w["name"], "q_len": args.q_len, "kv_storage": w["dtype"], "kv_layout": "[block][K|V][kv_head][token][dim], one pool" if w["recipe"].get("kv_layout", "adjacent") == "adjacent" else "two pools [block][kv_head][token][dim]", "batch": w["B"], "q_heads": w["Hq"], "kv_heads": w["Hkv"], "head_dim": 128,
                   "block_tokens": w["T"], "tokens_total": int(w["seq_lens_host"].sum()),
                   "max_len": int(w["seq_lens_host"].max()), "kv_bytes": int(kv_bytes),
                   "work_items": sched["num_items"], "workgroups": sched["workgroups"], "partials": sched["num_partials"],
                   "kernel": sched["kernel"]},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "decode_tokens_per_s_per_layer": round(w["B"] * max(1, args.q_len) / (ms_per_step * 1e-3), 1),
        "fused_da_attention_ms": round(fused_ms, 4),
        "roofline": {"bound": "hbm", "kernel": "micro_attention", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "kernel_ms": round(kern_ms, 4),
                     "traffic": parse_traffic(args.workload)},
    }

    if args.cpu_budget > 0 and args.q_len <= 1:
        host = dict(q=synth.as_numpy(w["q"]), k_pool=synth.as_numpy(w["k_pool"]), v_pool=synth.as_numpy(w["v_pool"]),
                    block_table=w["block_table_host"], seq_lens=w["seq_lens_host"])
        threads = min(16, len(os.sched_getaffinity(0)))
        info, pairs, ref, ref_lse = cpu_baseline(w, host, args.cpu_budget, threads)
        result["cpu_baseline"] = {k: (round(v, 4) if isinstance(v, float) else v) for k, v in info.items()}
        if not args.no_parity:
            got = out.cpu().numpy().astype(np.float64)[pairs[:, 0], pairs[:, 1]]
            got2 = out2.cpu().numpy().astype(np.float64)[pairs[:, 0], pairs[:, 1]]
            den = np.linalg.norm(ref)
            result["parity_on_sample"] = {
                "max_abs": float(np.abs(got - ref).max()), "rel_l2": float(np.linalg.norm(got - ref) / den),
                "fused_max_abs": float(np.abs(got2 - ref).max()), "pairs": int(len(pairs)),
                # worst single (request, q-head) pair, so that short requests are not hidden by long ones
                "worst_pair_rel_l2": float(np.max(np.linalg.norm(got - ref, axis=-1) / np.maximum(np.linalg.norm(ref, axis=-1), 1e-300)))}
    # KV append (the step before attention in a decode iteration), timed apart from the attention step:
    # the last token of every request is rewritten in place, so the cache contents are left as they were
    k_new = torch.stack([w["k_pool"][int(w["block_table_host"][r, (L - 1) // w["T"]]), :, (L - 1) % w["T"]]
                         if L > 0 else torch.zeros_like(w["k_pool"][0, :, 0]) for r, L in enumerate(lens_list)])
    v_new = torch.stack([w["v_pool"][int(w["block_table_host"][r, (L - 1) // w["T"]]), :, (L - 1) % w["T"]]
                         if L > 0 else torch.zeros_like(w["v_pool"][0, :, 0]) for r, L in enumerate(lens_list)])
    lens_m1 = torch.as_tensor([L - 1 for L in lens_list], dtype=torch.int32, device=dev)  # empty requests: -1 = inactive
    tmp = lens_m1.clone()
    def timed(fn, reps=50):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a0.record(stream)
        for _ in range(reps):
            fn()
        a1.record(stream)
        torch.cuda.synchronize()
        return a0.elapsed_time(a1) / reps

    # back-to-back launches; the length reset that every append needs is timed alone and subtracted
    t_reset = timed(lambda: tmp.copy_(lens_m1))
    t_both = timed(lambda: (tmp.copy_(lens_m1), da.append(prob, k_new, v_new, w["k_pool"], w["v_pool"], w["block_table"], tmp)))
    assert torch.equal(tmp, w["seq_lens"])
    result["append_us"] = round(max(t_both - t_reset, 0.0) * 1e3, 2)
    # the other rows of the path, each alone: host time of a re-plan (no stream work for small schedules) and
    # the aggregation launch back to back (its stream time includes the launch floor of a few microseconds)
    h0 = time.perf_counter()
    for _ in range(200):
        plan.update_raw(lens_c, sptr)
    torch.cuda.synchronize()
    result["plan_update_host_us"] = round((time.perf_counter() - h0) / 200 * 1e6, 2)
    result["combine_us"] = round(timed(lambda: plan.combine(part_o, part_m, part_e, out, lse)) * 1e3, 2)
    h0 = time.perf_counter()
    for _ in range(20):
        da.Plan(prob, lens_list, blocks_per_split=args.blocks_per_split, kernel=args.kernel).close()
    torch.cuda.synchronize()
    result["plan_create_host_us"] = round((time.perf_counter() - h0) / 20 * 1e6, 1)
    # what a pure streaming read of the same K pool sustains on this GPU right now (non-temporal loads, no
    # arithmetic): the practical ceiling next to the 8 TB/s peak.  Skipped for cache-sized pools.
    pool_bytes = w["k_pool"].numel() * w["k_pool"].element_size()
    if pool_bytes >= (1 << 30):
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        best = 0.0
        for variant in (3, 4):
            for seg in (256 << 10, 1 << 20):
                for wgs in (256, 512):
                    t_probe = timed(lambda: da.probe_read(w["k_pool"], seg, wgs, variant, sink), reps=5)
                    best = max(best, pool_bytes / (t_probe * 1e-3) / 1e9)
        result["read_ceiling"] = {"GBps": round(best, 1), "probe": "da_probe_read over k_pool, best of 8 launch shapes",
                                  "value_frac": round(value / best, 4), "kernel_frac": round(achieved / best, 4)}
    props = torch.cuda.get_device_properties(0)
    result["device"] = {"name": props.name, "compute_units": props.multi_processor_count,
                        "hbm_GiB": round(props.total_memory / 2 ** 30, 1), "arch": getattr(props, "gcnArchName", "")}
    plan.close()
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
