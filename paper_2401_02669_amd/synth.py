"""Seeded synthetic decode-attention workloads.

Input plumbing only: random q / K / V pools, block tables and sequence lengths
with the shapes of the five benchmark workloads (and scaled-down twins).  No
attention arithmetic lives here; both the HIP library's tests and the CPU
oracle's tests draw their inputs from this module.

The paper evaluates on conversation and long-document traces (Section 7.1,
Table 1) that are not available; these generators stand in for them, taking
only the length ranges from that table (a few tokens up to 2000K).

Layout produced: K and V pools ``[num_phys_blocks][Hkv][T][d]``, by default the two halves of one allocation
``[num_phys_blocks][2][Hkv][T][d]`` (a block's K and V adjacent; ``kv_layout="separate"`` gives two allocations),
``block_table`` int32 ``[B][max_blocks]`` with -1 past a request's last block,
``seq_lens`` int32 ``[B]``.  Unused physical blocks and the unused tail of a
partial last block are filled with NaN ("poison"): they must never influence a
result.
"""
import math

import numpy as np
import torch

BASE_SEED = 20240102

# name -> recipe.  "lens" is a list, an int (every request) or "loguniform".
WORKLOADS = {
    "c1_tiny": dict(index=0, B=1, Hq=1, Hkv=1, d=128, T=256, dtype="f32", lens=4096,
                    shuffle=False, spare_frac=0.0, outlier_frac=0.0),
    "c2_7b": dict(index=1, B=16, Hq=32, Hkv=32, d=128, T=256, dtype="bf16", lens=32768,
                  shuffle=True, spare_frac=0.02, outlier_frac=0.0),
    "c3_70b": dict(index=2, B=4, Hq=64, Hkv=8, d=128, T=512, dtype="bf16", lens=262144,
                   shuffle=True, spare_frac=0.02, outlier_frac=0.01),
    "c4_2m": dict(index=3, B=1, Hq=64, Hkv=8, d=128, T=1024, dtype="bf16", lens=2_000_000,
                  shuffle=True, spare_frac=0.02, outlier_frac=0.0),
    "c5_mixed": dict(index=4, B=64, Hq=32, Hkv=8, d=128, T=256, dtype="bf16", lens="loguniform",
                     len_range=(16, 1_000_000), shuffle=True, spare_frac=0.02, outlier_frac=0.0),
}


def _uniform(index, B, L, Hq, Hkv, T=256, dtype="bf16"):
    """B requests of L tokens each, shuffled block table, no spare blocks."""
    return dict(index=index, B=B, Hq=Hq, Hkv=Hkv, d=128, T=T, dtype=dtype, lens=L, shuffle=True, spare_frac=0.0,
                outlier_frac=0.0)


# Further named, seeded recipes: regimes off the five headline workloads that the measurements cover.
WORKLOADS.update({
    # the same 8.6 GB of K/V in ever shorter requests (what an instance that hosts many conversations serves)
    "short_4096x512": _uniform(10, 4096, 512, 32, 8),
    "short_2048x1024": _uniform(11, 2048, 1024, 32, 8),
    "short_1024x2048": _uniform(12, 1024, 2048, 32, 8),
    "short_256x8192": _uniform(13, 256, 8192, 32, 8),
    "short_mha_2048x512": _uniform(14, 2048, 512, 32, 32),
    "short_mha_1024x1024": _uniform(15, 1024, 1024, 32, 32),
    "short_mha_256x4096": _uniform(16, 256, 4096, 32, 32),
    # small totals (0.5 GB): two launches and ramp / tail weigh in
    "small_1x131072": _uniform(20, 1, 131072, 64, 8),
    "small_4x32768": _uniform(21, 4, 32768, 64, 8),
    # fp32 caches: MHA goes to the vector-ALU kernel, a query group to the fp32 matrix-core kernel
    "f32_mha_16x16384": _uniform(30, 16, 16384, 32, 32, dtype="f32"),
    "f32_gqa_4x131072": _uniform(31, 4, 131072, 64, 8, T=512, dtype="f32"),
})

# Sweeps: lists of (row name, recipe) that bench.py --workload <sweep> times row by row.
SWEEPS = {
    # from one short request to one 2M-token request, and over batch sizes at 32K (GQA 64/8, T = 256)
    "ctx_sweep": [("%dx%d" % (B, L), _uniform(40 + i, B, L, 64, 8)) for i, (B, L) in enumerate(
        [(1, 1024), (1, 4096), (1, 16384), (1, 32768), (1, 131072), (4, 32768), (1, 524288), (16, 32768),
         (1, 2000000), (64, 32768)])],
    "short_sweep": [(n, WORKLOADS[n]) for n in (
        "short_256x8192", "short_1024x2048", "short_2048x1024", "short_4096x512", "short_mha_256x4096",
        "short_mha_1024x1024", "short_mha_2048x512")],
}


def recipe(name, len_div=1, **overrides):
    """Recipe of a named workload; ``len_div`` > 1 gives the scaled-down twin (lengths / len_div)."""
    r = dict(WORKLOADS[name])
    r["name"] = name if len_div == 1 else "%s/%d" % (name, len_div)
    r["len_div"] = len_div
    r.update(overrides)
    return r


def _lengths(r, rng):
    lens = r["lens"]
    B = r["B"]
    if isinstance(lens, str):
        lo, hi = r["len_range"]
        u = rng.uniform(math.log(lo), math.log(hi), size=B)
        out = np.clip(np.floor(np.exp(u)), lo, hi).astype(np.int64)
    elif isinstance(lens, int):
        out = np.full((B,), lens, dtype=np.int64)
    else:
        out = np.asarray(lens, dtype=np.int64)
        assert out.shape == (B,)
    div = r.get("len_div", 1)
    if div > 1:
        out = np.maximum(out // div, np.minimum(out, 1))
    return out


def pool_bytes(r):
    """Bytes of K pool + V pool that ``make(r)`` allocates (or takes from ``kv_storage``)."""
    rng = np.random.RandomState(BASE_SEED + r["index"])
    nb = (_lengths(r, rng) + r["T"] - 1) // r["T"]
    used = int(nb.sum())
    num_phys = max(1, used + int(math.ceil(used * r["spare_frac"])))
    return num_phys * 2 * r["Hkv"] * r["T"] * r["d"] * (4 if r["dtype"] == "f32" else 2)


def make(r, device="cpu", poison=True, kv_storage=None):
    """Build the tensors of recipe ``r`` on ``device``.  Returns a dict of torch tensors + metadata.

    ``kv_storage``: optional 1-D uint8 tensor on ``device`` of at least ``pool_bytes(r)`` bytes to place the pools
    in (an engine allocates its KV memory once and keeps it; a caller that builds several workloads in one process
    can do the same)."""
    seed = BASE_SEED + r["index"]
    rng = np.random.RandomState(seed)
    B, Hq, Hkv, d, T = r["B"], r["Hq"], r["Hkv"], r["d"], r["T"]
    tdtype = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[r["dtype"]]
    lens = _lengths(r, rng)
    nb = (lens + T - 1) // T
    used = int(nb.sum())
    num_phys = max(1, used + int(math.ceil(used * r["spare_frac"])))
    ids = rng.permutation(num_phys) if r["shuffle"] else np.arange(num_phys)
    max_blocks = max(1, int(nb.max()))
    table = np.full((B, max_blocks), -1, dtype=np.int32)
    pos = 0
    for i in range(B):
        table[i, : nb[i]] = ids[pos: pos + nb[i]]
        pos += nb[i]

    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    def storage(shape, first_byte=0):
        if kv_storage is None:
            return torch.empty(shape, dtype=tdtype, device=device)
        nbytes = int(np.prod(shape)) * tdtype.itemsize
        assert kv_storage.dtype == torch.uint8 and kv_storage.numel() >= first_byte + nbytes
        return kv_storage[first_byte: first_byte + nbytes].view(tdtype).view(shape)

    if r.get("kv_layout", "adjacent") == "adjacent":
        # one allocation [P][2][Hkv][T][d]: the K rows and the V rows of a block lie next to each other
        kv_pool = storage((num_phys, 2, Hkv, T, d))
        k_pool, v_pool = kv_pool[:, 0], kv_pool[:, 1]
    else:
        kv_pool = None
        k_pool = storage((num_phys, Hkv, T, d))
        v_pool = storage((num_phys, Hkv, T, d), first_byte=k_pool.numel() * tdtype.itemsize)
    chunk = max(1, (64 << 20) // (Hkv * T * d))  # ~64M elements of fp32 scratch at a time
    for lo in range(0, num_phys, chunk):
        hi = min(num_phys, lo + chunk)
        shape = (hi - lo, Hkv, T, d)
        kf = torch.randn(shape, dtype=torch.float32, device=device, generator=gen)
        if r["outlier_frac"] > 0.0:
            # a seeded Bernoulli per key row; selected rows are scaled by 8 before rounding
            pick = torch.rand(shape[:3], dtype=torch.float32, device=device, generator=gen) < r["outlier_frac"]
            kf = torch.where(pick.unsqueeze(-1), kf * 8.0, kf)
        k_pool[lo:hi] = kf.to(tdtype)
        del kf
        v_pool[lo:hi] = torch.randn(shape, dtype=torch.float32, device=device, generator=gen).to(tdtype)
    q = torch.randn((B, Hq, d), dtype=torch.float32, device=device, generator=gen).to(tdtype)

    if poison:
        nan = float("nan")
        unused = ids[used:]
        if len(unused):
            idx = torch.as_tensor(np.ascontiguousarray(unused), device=device, dtype=torch.long)
            k_pool[idx] = nan
            v_pool[idx] = nan
        for i in range(B):
            tail = int(lens[i] % T)
            if nb[i] > 0 and tail != 0:
                pb = int(table[i, nb[i] - 1])
                k_pool[pb, :, tail:, :] = nan
                v_pool[pb, :, tail:, :] = nan

    return dict(
        name=r["name"], recipe=r, q=q, k_pool=k_pool, v_pool=v_pool,
        kv_pool=kv_pool,  # the one allocation behind both pools ([P][2][Hkv][T][d]) or None
        block_table=torch.as_tensor(table, device=device),
        seq_lens=torch.as_tensor(lens.astype(np.int32), device=device),
        seq_lens_host=lens.astype(np.int32), block_table_host=table,
        B=B, Hq=Hq, Hkv=Hkv, d=d, T=T, dtype=r["dtype"], num_phys=num_phys,
        max_blocks=max_blocks, scale=1.0 / math.sqrt(d),
        kv_bytes=int(lens.sum()) * Hkv * 2 * d * (4 if r["dtype"] == "f32" else 2),
    )


def as_numpy(t):
    """Host numpy view of a tensor; bf16 becomes uint16 bit patterns (what the oracle reads), half stays float16."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def f32_to_bf16_bits(x):
    """Round fp32 numpy values to bf16 (nearest-even, via torch) and return the uint16 bit patterns."""
    t = torch.as_tensor(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


# ---- cluster states for the placement scheduler (Section 5.3) ---------------------------------------
def natn_time_table(max_batch, weight_bytes=403e6, flops_per_token=0.403e9, hbm_bytes_per_s=7.0e12,
                    flops_per_s=1.2e15, fixed_s=20e-6):
    """Synthetic stand-in for the measured non-attention time of one layer at batch sizes 0..max_batch.

    A two-regime curve: the layer's weights are read once per step whatever the batch, and the arithmetic grows with
    the batch.  Defaults are a 4096-wide layer (12 h^2 parameters in bf16).  Entry 0 is 0 (an idle instance).
    """
    t = [0.0]
    for b in range(1, max_batch + 1):
        t.append(fixed_s + max(weight_bytes / hbm_bytes_per_s, b * flops_per_token / flops_per_s))
    return t


def attention_rate(kv_heads=32, head_dim=128, kv_elem_bytes=2, kv_read_bytes_per_s=7.0e12):
    """g of Section 5.3 in tokens per second for one layer, from a measured KV-read rate of the MicroAttention kernel."""
    return kv_read_bytes_per_s / (2 * kv_heads * head_dim * kv_elem_bytes)


def make_cluster(seed, num_instances=32, block_tokens=256, capacity_blocks=2048, max_batch=256):
    """Seeded cluster state: a mix of long-request, short-request, idle and middling instances.

    Returns ``(model, instances)`` as plain dicts / lists of Python numbers:
    model = {num_layers, block_tokens, attn_tokens_per_s, t_natn}; an instance = {req_tokens, req_remote_blocks,
    hosted_blocks, capacity_blocks, waiting, admit_blocks}.  Lengths follow the ranges of Table 1 (a few tokens up to
    2000K; longer than one instance can hold means part of the request is already remote).
    """
    rng = np.random.default_rng(BASE_SEED + 7919 * (seed + 1))
    model = dict(num_layers=32, block_tokens=block_tokens, attn_tokens_per_s=attention_rate(),
                 t_natn=natn_time_table(max_batch))
    cap_tokens = capacity_blocks * block_tokens
    instances = []
    for _ in range(num_instances):
        kind = rng.choice(4, p=[0.3, 0.45, 0.1, 0.15])
        cap = int(capacity_blocks * rng.choice([1.0, 1.0, 0.5]))
        remote = None
        hosted = 0
        if kind == 0:      # one long request filling most of the memory, few short ones beside it
            long_len = int(rng.uniform(0.6, 1.6) * cap * block_tokens)
            lens = [long_len] + [int(x) for x in rng.integers(16, 2000, size=int(rng.integers(0, 4)))]
            blocks = [-(-s // block_tokens) for s in lens]
            over = max(0, sum(blocks) - cap)
            remote = [over + int(rng.integers(0, 8)) if over else 0] + [0] * (len(lens) - 1)
            waiting, admit = int(rng.integers(0, 64)), int(rng.integers(1, 9))
        elif kind == 1:    # many short requests, memory to spare
            lens = [int(x) for x in rng.integers(16, 4000, size=int(rng.integers(8, min(max_batch, 120))))]
            waiting, admit = int(rng.integers(0, 4)), int(rng.integers(1, 9))
            hosted = int(rng.integers(0, 2)) * int(rng.integers(0, cap // 8))
        elif kind == 2:    # idle
            lens, waiting, admit = [], 0, 0
        else:              # a handful of medium requests
            lens = [int(x) for x in np.exp(rng.uniform(np.log(1000), np.log(cap_tokens // 8), size=int(rng.integers(1, 12))))]
            waiting, admit = int(rng.integers(0, 16)), int(rng.integers(1, 17))
        used = sum(-(-s // block_tokens) for s in lens) - (sum(remote) if remote else 0) + hosted
        if used > cap:     # keep the state consistent: never more than the capacity in use
            hosted = max(0, hosted - (used - cap))
            used = sum(-(-s // block_tokens) for s in lens) - (sum(remote) if remote else 0) + hosted
            if used > cap:
                lens = lens[:1]
                remote = remote[:1] if remote else None
                used = -(-lens[0] // block_tokens) - (remote[0] if remote else 0)
                if used > cap:
                    remote = [(remote[0] if remote else 0) + used - cap]
        instances.append(dict(req_tokens=lens, req_remote_blocks=remote if remote else [0] * len(lens),
                              hosted_blocks=hosted, capacity_blocks=cap, waiting=waiting, admit_blocks=admit))
    return model, instances
