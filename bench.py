#!/usr/bin/env python3
"""Benchmark of the DistAttention decode hot path on one MI355X.

A step = one pass of the whole path over one batch of synthetic input already resident in HBM:
work scheduling (da_plan_update, host) -> MicroAttention (da_partial) -> aggregation (da_combine).
Every timed step is bracketed by HIP events on the launch stream (before da_partial, between the two launches,
after da_combine); a workload's step time is the MEDIAN of the timed steps, and its roofline figure is the
algorithmic K/V bytes over the median MicroAttention time.

With no --workload the four large workloads (c2_7b, c3_70b, c4_2m, c5_mixed: 32K to 2M tokens of context) run one
after the other, plus c1_tiny for latency.  ONE JSON line is printed; its value / roofline / cpu_baseline are
those of the SLOWEST of the four (lowest KV-read GB/s), and `per_workload` carries every workload's own figures,
including parity on a sample against the fp64 CPU oracle, which is timed on the host cores in the same run.
The run fails (exit status 1) if any sampled output misses the parity bar.

--workload <name> runs one named recipe of synth.WORKLOADS; --workload ctx_sweep / short_sweep time the rows of a
sweep through the fused call; --calibrate-copy runs plain copies of a known size (the kernel whose hardware
traffic counters scale those of the attention kernels) and exits.
"""
import argparse
import ctypes
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak
LARGE = ["c2_7b", "c3_70b", "c4_2m", "c5_mixed"]
PARITY_BAR = {"bf16": (2e-3, 1e-3), "f16": (2e-3, 1e-3), "f32": (1e-5, 1e-5)}  # (max-abs, rel-L2) against the oracle


def traffic_from_profile(workload):
    """HBM bytes per MicroAttention launch from the committed rocprofv3 --pmc summary of this workload, if any.
    A stored figure from separate counter runs of the same command, not something this run measures."""
    import glob
    found = sorted(glob.glob(os.path.join(ROOT, "profiles", "micro_attention_*_%s.txt" % workload)))
    if not found:
        return None, None
    path = found[0]
    rel = os.path.relpath(path, ROOT)
    vals = {}
    for line in open(path):
        parts = line.split()
        if len(parts) == 2 and parts[0] in ("hbm_read_bytes_per_launch", "hbm_write_bytes_per_launch"):
            vals[parts[0]] = float(parts[1])
    if "hbm_read_bytes_per_launch" not in vals:
        return None, None
    return vals["hbm_read_bytes_per_launch"] + vals.get("hbm_write_bytes_per_launch", 0.0), rel


def cpu_baseline(w, host, budget_s, threads, q_len):
    """Time the oracle (as it stands) on a sample of (request, q-head) pairs; returns (dict, pairs, ref, ref_lse)."""
    import numpy as np
    import oracle

    B, Hq, Hkv = w["B"], w["Hq"], w["Hkv"]
    lens = w["seq_lens_host"].astype(np.int64)
    esize = 4 if w["dtype"] == "f32" else 2
    kw = {}  # (the oracle takes the number of query tokens from q's shape)
    # cost of a pair is proportional to its length: probe with a request of median length (a very short one
    # would measure the call, not the tokens)
    order = [r for r in np.argsort(lens) if lens[r] > 0] or [0]
    probe_r = int(order[len(order) // 2])
    t0 = time.perf_counter()
    oracle.attention(host["q"], host["k_pool"], host["v_pool"], host["block_table"], host["seq_lens"], w["T"],
                     w["scale"], pairs=np.array([[probe_r, 0]], dtype=np.int32), n_threads=1, **kw)
    per_token = (time.perf_counter() - t0) / max(1, int(lens[probe_r]))
    # deterministic sample: walk pairs spread over requests and heads until the budget is filled
    rng = np.random.RandomState(1234)
    cand = [(r, h) for r in range(B) for h in range(Hq * q_len) if lens[r] > 0]
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
    use = min(threads, len(pairs))
    t0 = time.perf_counter()
    ref, ref_lse = oracle.attention(host["q"], host["k_pool"], host["v_pool"], host["block_table"], host["seq_lens"],
                                    w["T"], w["scale"], pairs=pairs, n_threads=use, **kw)
    dt = time.perf_counter() - t0
    # a pair stands for 1/G of its kv-head's bytes (the GPU reads K/V once per group)
    G = Hq // Hkv
    sample_bytes = float(tok) * 2 * w["d"] * esize / G
    info = dict(value=sample_bytes / dt / 1e9, unit="GB/s", cores=use, kind="oracle",
                sample="%d of %d (request, q-head) pairs, %d pair-tokens, %.1f s" % (len(pairs), B * Hq * q_len, tok, dt),
                seconds=round(dt, 6), tokens_per_s=(sample_bytes / w["kv_bytes"]) * B / dt)
    return info, pairs, ref, ref_lse


def median_ms(pairs):
    return statistics.median(a.elapsed_time(b) for a, b in pairs)


def build_workload(recipe, dev, q_len, arena=None):
    import torch
    from paper_2401_02669_amd import synth

    w = synth.make(recipe, dev, kv_storage=arena)
    if q_len > 1:  # multi-query form: every request brings q_len new tokens (already in the cache)
        gen = torch.Generator(device=dev)
        gen.manual_seed(4242)
        w["q"] = torch.randn((w["B"], q_len, w["Hq"], 128), device=dev, generator=gen).to(w["q"].dtype)
    return w


def run_workload(recipe, args, dev, threads, arena=None):
    """Times one workload; returns its result dict (and whether parity held)."""
    import numpy as np
    import torch
    from paper_2401_02669_amd import distattn as da
    from paper_2401_02669_amd import probe, synth

    t_begin = time.perf_counter()
    w = build_workload(recipe, dev, args.q_len, arena)
    name = w["name"]
    prob = da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"])
    lens_list = w["seq_lens_host"].tolist()
    tune = dict(blocks_per_split=args.blocks_per_split, kernel=args.kernel)
    plan = da.Plan(prob, lens_list, **tune)
    sched = da.plan_schedule(prob, lens_list, num_cus=torch.cuda.get_device_properties(0).multi_processor_count, **tune)
    desc = plan.describe()
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

    def step(ev=None):
        plan.update_raw(lens_c, sptr)
        if ev:
            ev[0].record(stream)
        plan.partial(*args_partial)
        if ev:
            ev[1].record(stream)
        plan.combine(part_o, part_m, part_e, out, lse)
        if ev:
            ev[2].record(stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    step_ms = median_ms([(e[0], e[2]) for e in evs])
    partial_ms = median_ms([(e[0], e[1]) for e in evs])
    combine_ms = median_ms([(e[1], e[2]) for e in evs])
    assert plan.error_flags() == 0

    # the fused convenience call (same kernels; single-split requests skip the aggregation), timed the same way
    ws = torch.empty((max(plan.workspace_bytes, 256),), dtype=torch.uint8, device=dev)
    out2 = torch.empty_like(out)
    lse2 = torch.empty_like(lse)
    fused_args = (w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"], out2, lse2, ws)
    for _ in range(3):
        plan.attention(*fused_args)
    fev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    for i in range(args.steps):
        plan.update_raw(lens_c, sptr)
        fev[i][0].record(stream)
        plan.attention(*fused_args)
        fev[i][1].record(stream)
    torch.cuda.synchronize()
    fused_ms = median_ms(fev)

    kv_bytes = float(w["kv_bytes"])
    value = kv_bytes / (step_ms * 1e-3) / 1e9
    achieved = kv_bytes / (partial_ms * 1e-3) / 1e9
    lens_np = w["seq_lens_host"].astype(np.float64)
    traffic, traffic_file = traffic_from_profile(name) if args.q_len <= 1 else (None, None)
    res = {
        "workload": name, "value": round(value, 1), "unit": "GB/s", "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "ms_per_step": round(step_ms, 4), "ms_per_step_wall_mean": round(wall_ms, 4),
        "da_partial_ms": round(partial_ms, 4), "da_combine_ms": round(combine_ms, 4),
        "fused_da_attention_ms": round(fused_ms, 4), "fused_GBps": round(kv_bytes / (fused_ms * 1e-3) / 1e9, 1),
        "decode_tokens_per_s_per_layer": round(w["B"] * max(1, args.q_len) / (step_ms * 1e-3), 1),
        "config": {"workload": name, "q_len": args.q_len, "kv_storage": w["dtype"], "accumulate": "f32",
                   "kv_layout": "[block][K|V][kv_head][token][dim], one pool" if w["recipe"].get("kv_layout", "adjacent") == "adjacent" else "two pools [block][kv_head][token][dim]",
                   "batch": w["B"], "q_heads": w["Hq"], "kv_heads": w["Hkv"], "head_dim": 128, "block_tokens": w["T"],
                   "kv_bytes": int(kv_bytes), "work_items": sched["num_items"], "workgroups": sched["workgroups"],
                   "partials": sched["num_partials"], "kernel": sched["kernel"], "columns_per_item": desc["head_tile"],
                   "wavefront_splits": desc["wavefront_splits"]},
        "lengths": {"sum": int(lens_np.sum()), "min": int(lens_np.min()), "max": int(lens_np.max()),
                    "mean": round(float(lens_np.mean()), 1), "sd": round(float(lens_np.std()), 1)},
        "roofline": {"bound": "hbm", "kernel": "micro_attention", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "kernel_ms": round(partial_ms, 4),
                     "traffic": traffic,
                     "traffic_source": ("%s (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, stored; not measured by this run)" % traffic_file) if traffic_file else None},
    }

    ok = True
    if args.cpu_budget > 0:
        # host copies for the oracle, made without a temporary on the device: the one allocation behind both
        # pools is copied as it is and the oracle reads its K and V halves in place
        if w["kv_pool"] is not None:
            host_kv = synth.as_numpy(w["kv_pool"])
            host_k, host_v = host_kv[:, 0], host_kv[:, 1]
        else:
            host_k, host_v = synth.as_numpy(w["k_pool"]), synth.as_numpy(w["v_pool"])
        host = dict(q=synth.as_numpy(w["q"]), k_pool=host_k, v_pool=host_v,
                    block_table=w["block_table_host"], seq_lens=w["seq_lens_host"])
        one_thread = name.startswith("c1_tiny")  # latency case: the oracle's single-thread time is the figure asked for
        info, pairs, ref, ref_lse = cpu_baseline(w, host, args.cpu_budget, 1 if one_thread else threads, args.q_len)
        res["cpu_baseline"] = {k: (round(v, 4) if isinstance(v, float) else v) for k, v in info.items()}
        if not args.no_parity:
            flat = (w["B"], -1, 128)
            got = out.cpu().numpy().astype(np.float64).reshape(flat)[pairs[:, 0], pairs[:, 1]]
            got2 = out2.cpu().numpy().astype(np.float64).reshape(flat)[pairs[:, 0], pairs[:, 1]]
            den = np.linalg.norm(ref)
            par = {"max_abs": float(np.abs(got - ref).max()), "rel_l2": float(np.linalg.norm(got - ref) / den),
                   "fused_max_abs": float(np.abs(got2 - ref).max()),
                   "fused_rel_l2": float(np.linalg.norm(got2 - ref) / den), "pairs": int(len(pairs)),
                   # worst single (request, q-head) pair, so that short requests are not hidden by long ones
                   "worst_pair_rel_l2": float(np.max(np.linalg.norm(got - ref, axis=-1) / np.maximum(np.linalg.norm(ref, axis=-1), 1e-300)))}
            bar_abs, bar_rel = PARITY_BAR[w["dtype"]]
            par["bar"] = {"max_abs": bar_abs, "rel_l2": bar_rel}
            par["ok"] = bool(np.all(np.isfinite(got)) and np.all(np.isfinite(got2)) and par["max_abs"] <= bar_abs and
                             par["rel_l2"] <= bar_rel and par["fused_max_abs"] <= bar_abs and par["fused_rel_l2"] <= bar_rel)
            ok = par["ok"]
            res["parity_on_sample"] = par
        del host

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

    if args.q_len <= 1:
        # KV append (the step before attention in a decode iteration), timed apart from the attention step:
        # the last token of every request is rewritten in place, so the cache contents are left as they were
        bt, T = w["block_table_host"], w["T"]
        ids = torch.as_tensor([int(bt[r, (L - 1) // T]) if L > 0 else 0 for r, L in enumerate(lens_list)], device=dev)
        slots = torch.as_tensor([(L - 1) % T if L > 0 else 0 for L in lens_list], device=dev)
        k_new = w["k_pool"][ids, :, slots].contiguous()
        v_new = w["v_pool"][ids, :, slots].contiguous()
        lens_m1 = torch.as_tensor([L - 1 for L in lens_list], dtype=torch.int32, device=dev)  # empty requests: -1 = inactive
        tmp = lens_m1.clone()
        # back-to-back launches; the length reset that every append needs is timed alone and subtracted
        t_reset = timed(lambda: tmp.copy_(lens_m1))
        t_both = timed(lambda: (tmp.copy_(lens_m1), da.append(prob, k_new, v_new, w["k_pool"], w["v_pool"], w["block_table"], tmp)))
        assert torch.equal(tmp, w["seq_lens"])
        res["append_us"] = round(max(t_both - t_reset, 0.0) * 1e3, 2)
    # host time of a re-plan and of making a plan
    h0 = time.perf_counter()
    for _ in range(200):
        plan.update_raw(lens_c, sptr)
    torch.cuda.synchronize()
    res["plan_update_host_us"] = round((time.perf_counter() - h0) / 200 * 1e6, 2)
    h0 = time.perf_counter()
    for _ in range(10):
        da.Plan(prob, lens_list, **tune).close()
    torch.cuda.synchronize()
    res["plan_create_host_us"] = round((time.perf_counter() - h0) / 10 * 1e6, 1)
    # what a pure streaming read of the same K pool sustains on this GPU right now (a probe kernel of this
    # repository with non-temporal loads and no arithmetic): a reference point, not a hardware limit
    pool_bytes = w["k_pool"].numel() * w["k_pool"].element_size()
    if pool_bytes >= (1 << 30) and not args.no_probe:
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        best = 0.0
        for variant in (3, 4):
            for seg in (256 << 10, 1 << 20):
                for wgs in (256, 512):
                    t_probe = timed(lambda: probe.probe_read(w["k_pool"], seg, wgs, variant, sink), reps=5)
                    best = max(best, pool_bytes / (t_probe * 1e-3) / 1e9)
        res["stream_read_probe"] = {"GBps": round(best, 1), "what": "da_probe_read over k_pool, best of 8 launch shapes",
                                    "kernel_over_probe": round(achieved / best, 4)}
    res["wall_s"] = round(time.perf_counter() - t_begin, 1)
    plan.close()
    return res, ok


def run_sweep(sweep, args, dev):
    """Rows of a sweep through the fused call (da_plan_update + da_attention per step), median of HIP-event step times."""
    import torch
    from paper_2401_02669_amd import distattn as da
    from paper_2401_02669_amd import synth

    rows = []
    stream = torch.cuda.current_stream()
    sptr = ctypes.c_void_p(stream.cuda_stream)
    # one allocation for the pools of every row (see main)
    arena = torch.empty((max(synth.pool_bytes(rec) for _, rec in synth.SWEEPS[sweep]) + 4096,), dtype=torch.uint8, device=dev)
    for row_name, rec in synth.SWEEPS[sweep]:
        r = dict(rec)
        r["name"], r["len_div"] = row_name, 1
        w = synth.make(r, dev, poison=False, kv_storage=arena)
        prob = da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"])
        lens_list = w["seq_lens_host"].tolist()
        plan = da.Plan(prob, lens_list, kernel=args.kernel)
        desc = plan.describe()
        sched = da.plan_schedule(prob, lens_list, kernel=args.kernel)
        ws = torch.empty((max(plan.workspace_bytes, 256),), dtype=torch.uint8, device=dev)
        out = torch.empty((w["B"], w["Hq"], 128), dtype=torch.float32, device=dev)
        lse = torch.empty((w["B"], w["Hq"]), dtype=torch.float32, device=dev)
        lens_c = (ctypes.c_int32 * w["B"])(*lens_list)
        a = (w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"], out, lse, ws)
        for _ in range(max(3, args.warmup)):
            plan.update_raw(lens_c, sptr)
            plan.attention(*a)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
        torch.cuda.synchronize()
        for i in range(args.steps):
            ev[i][0].record(stream)
            plan.update_raw(lens_c, sptr)  # a large schedule's table upload is part of the step
            plan.attention(*a)
            ev[i][1].record(stream)
        torch.cuda.synchronize()
        ms = median_ms(ev)
        assert plan.error_flags() == 0
        gbps = w["kv_bytes"] / (ms * 1e-3) / 1e9
        rows.append({"row": row_name, "batch": w["B"], "context": int(w["seq_lens_host"].max()), "q_heads": w["Hq"],
                     "kv_heads": w["Hkv"], "kv_bytes": int(w["kv_bytes"]), "workgroups": sched["workgroups"],
                     "wavefront_splits": desc["wavefront_splits"], "ms_per_step": round(ms, 4), "GBps": round(gbps, 1),
                     "pct_of_hbm_peak": round(100.0 * gbps / HBM_PEAK_GBPS, 2)})
        print("# %s" % json.dumps(rows[-1]), file=sys.stderr, flush=True)
        plan.close()
        del w, a, ws, out, lse
    return rows


def calibrate_copy(args, dev):
    """Plain copies of a known size: under `rocprofv3 --pmc FETCH_SIZE` (or WRITE_SIZE) the counter's reading for
    copy_probe_kernel against the known bytes gives the factor that scales the attention kernels' readings."""
    import torch
    from paper_2401_02669_amd import probe

    n = int(args.calibrate_gib * (1 << 30)) // 4
    src = torch.arange(n, dtype=torch.int32, device=dev)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(3):
        probe.probe_copy(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(dst[:4096], src[:4096]) and torch.equal(dst[-4096:], src[-4096:])
    print(json.dumps({"calibrate_copy": {"kernel": "copy_probe_kernel", "bytes_read_per_copy": n * 4,
                                         "bytes_written_per_copy": n * 4, "copies": 3}}), flush=True)


def probe_writes(args, dev):
    """What small result writes cost a read stream, by write pattern (da_probe_read_write): 8 GiB read as 256 KiB
    items (512 tokens of one kv-head, bf16 K + V) by 1024 wavefronts, 2 KiB of result per item (4 q-heads)."""
    import torch
    from paper_2401_02669_amd import probe

    total, item, frag, wgs = 8 << 30, 256 << 10, 2048, 256
    src = torch.full((total // 4,), 0x01020304, dtype=torch.int32, device=dev)
    dst = torch.zeros((total // item * frag // 4,), dtype=torch.int32, device=dev)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream()
    rows = []
    per_wave = total // item // (wgs * 4)
    for what, burst, stag in (("no writes", 0, 0), ("after every item", 1, 0), ("every 4 items", 4, 0),
                              ("every 16 items", 16, 0), ("every 16 items, each wavefront at its own phase", 16, 1),
                              ("once, after the last read", per_wave, 0), ("no writes", 0, 0)):
        best = None
        for _ in range(6):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            probe.probe_read_write(src, dst, item, frag, wgs, burst, stag, sink)
            e1.record(stream)
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
        rows.append({"writes": what, "burst_items": burst, "staggered": stag, "ms": round(best, 4),
                     "read_GBps": round(total / best / 1e6, 1), "pct_of_hbm_peak": round(total / best / 1e6 / 80, 2)})
    print(json.dumps({"probe_writes": {"read_bytes": total, "item_bytes": item, "result_bytes_per_item": frag,
                                       "written_bytes": total // item * frag, "rows": rows}}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="all",
                    help="all (c2_7b c3_70b c4_2m c5_mixed + c1_tiny), names of synth.WORKLOADS (comma-separated), ctx_sweep, short_sweep")
    ap.add_argument("--len-div", type=int, default=1, help="divide every length (debug only; result is not the named workload)")
    ap.add_argument("--blocks-per-split", type=int, default=0)
    ap.add_argument("--kernel", type=int, default=0, help="0 auto, 1 VALU, 2 MFMA")
    ap.add_argument("--q-len", type=int, default=1, help="query tokens per request (1 = decode, the headline metric)")
    ap.add_argument("--cpu-budget", type=float, default=5.0, help="seconds of oracle time per workload for cpu_baseline (0 = skip)")
    ap.add_argument("--no-parity", action="store_true")
    ap.add_argument("--no-probe", action="store_true", help="skip the streaming-read probe")
    ap.add_argument("--no-arena", action="store_true", help="allocate every workload's pools afresh instead of placing them in one up-front allocation")
    ap.add_argument("--calibrate-copy", action="store_true")
    ap.add_argument("--probe-writes", action="store_true", help="time a read stream with result writes in several patterns and exit")
    ap.add_argument("--calibrate-gib", type=float, default=4.0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives or sharding); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    if args.steps < 1:
        ap.error("--steps must be >= 1")

    import torch
    from paper_2401_02669_amd import distattn as da
    from paper_2401_02669_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU", file=sys.stderr)
        sys.exit(2)
    da.lib()  # fail loudly if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)
    props = torch.cuda.get_device_properties(0)
    device = {"name": props.name, "compute_units": props.multi_processor_count,
              "hbm_GiB": round(props.total_memory / 2 ** 30, 1), "arch": getattr(props, "gcnArchName", "")}
    threads = min(16, len(os.sched_getaffinity(0)))

    if args.calibrate_copy:
        calibrate_copy(args, dev)
        return
    if args.probe_writes:
        probe_writes(args, dev)
        return

    base = {"metric": "kv_read_hbm_GBps", "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "timing": "median over the timed steps of HIP-event step times on the launch stream"}

    if args.workload in synth.SWEEPS:
        rows = run_sweep(args.workload, args, dev)
        big = [r for r in rows if r["kv_bytes"] >= (1 << 29)] or rows
        low = min(big, key=lambda r: r["GBps"])
        base.update({"value": low["GBps"], "ms_per_step": low["ms_per_step"],
                     "config": {"workload": args.workload, "row": low["row"], "step": "da_plan_update + da_attention",
                                "value_is": "lowest row of at least 0.5 GB"},
                     "rows": rows, "device": device})
        print(json.dumps(base), flush=True)
        return

    names = LARGE + ["c1_tiny"] if args.workload == "all" else args.workload.split(",")
    # KV memory is allocated once, before anything else, and every workload's pools are placed in it, as in an
    # engine that reserves its KV space at start-up.  (Pools allocated after other allocations of the process
    # have come and gone read several percent slower on this GPU.)
    recipes = [synth.recipe(name, len_div=args.len_div) for name in names]
    arena = None
    if not args.no_arena:
        arena = torch.empty((max(synth.pool_bytes(r) for r in recipes) + 4096,), dtype=torch.uint8, device=dev)
    per, all_ok = {}, True
    for name, rec in zip(names, recipes):
        res, ok = run_workload(rec, args, dev, threads, arena)
        per[name] = res
        all_ok = all_ok and ok
        print("# %s: %.4f ms/step, %.1f GB/s, roofline frac %.4f, parity %s" % (
            name, res["ms_per_step"], res["value"], res["roofline"]["frac"],
            res.get("parity_on_sample", {}).get("ok", "not checked")), file=sys.stderr, flush=True)
        # (no torch.cuda.empty_cache() here: returning large blocks to the driver in the middle of a process
        # left every later launch several percent slower on this GPU; torch re-uses what it holds)

    ranked = [n for n in names if n in LARGE] or names
    head = per[min(ranked, key=lambda n: per[n]["value"])]
    base.update({"value": head["value"], "ms_per_step": head["ms_per_step"], "dtype": head["config"]["kv_storage"],
                 "config": dict(head["config"], headline="lowest KV-read GB/s of %s" % ", ".join(ranked)),
                 "pct_of_hbm_peak": head["pct_of_hbm_peak"],
                 "decode_tokens_per_s_per_layer": head["decode_tokens_per_s_per_layer"],
                 "roofline": head["roofline"]})
    if "cpu_baseline" in head:
        base["cpu_baseline"] = head["cpu_baseline"]
    if "parity_on_sample" in head:
        base["parity_on_sample"] = head["parity_on_sample"]
    base["parity_ok"] = all_ok
    if "c1_tiny" in per:
        c1 = per["c1_tiny"]
        base["c1_tiny_latency"] = {"step_us": round(c1["ms_per_step"] * 1e3, 2), "fused_us": round(c1["fused_da_attention_ms"] * 1e3, 2),
                                   "oracle_single_thread_us": round(c1.get("cpu_baseline", {}).get("seconds", 0.0) * 1e6, 1)}
    base["per_workload"] = per
    base["device"] = device
    print(json.dumps(base), flush=True)
    if not all_ok:
        print("bench.py: PARITY FAILED on a sampled output (see parity_on_sample)", file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
