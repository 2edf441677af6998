"""Seeded synthetic decode-attention workloads.

Input plumbing only: random q / K / V pools, block tables and sequence lengths
with the shapes of the five benchmark workloads (and scaled-down twins).  No
attention arithmetic lives here; both the HIP library's tests and the CPU
oracle's tests draw their inputs from this module.

The paper evaluates on conversation and long-document traces (Section 7.1,
Table 1) that are not available; these generators stand in for them, taking
only the length ranges from that table (a few tokens up to 2000K).

Layout produced: K and V pools ``[num_phys_blocks][Hkv][T][d]`` (contiguous),
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


def make(r, device="cpu", poison=True):
    """Build the tensors of recipe ``r`` on ``device``.  Returns a dict of torch tensors + metadata."""
    seed = BASE_SEED + r["index"]
    rng = np.random.RandomState(seed)
    B, Hq, Hkv, d, T = r["B"], r["Hq"], r["Hkv"], r["d"], r["T"]
    tdtype = torch.float32 if r["dtype"] == "f32" else torch.bfloat16
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
    k_pool = torch.empty((num_phys, Hkv, T, d), dtype=tdtype, device=device)
    v_pool = torch.empty_like(k_pool)
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
        block_table=torch.as_tensor(table, device=device),
        seq_lens=torch.as_tensor(lens.astype(np.int32), device=device),
        seq_lens_host=lens.astype(np.int32), block_table_host=table,
        B=B, Hq=Hq, Hkv=Hkv, d=d, T=T, dtype=r["dtype"], num_phys=num_phys,
        max_blocks=max_blocks, scale=1.0 / math.sqrt(d),
        kv_bytes=int(lens.sum()) * Hkv * 2 * d * (4 if r["dtype"] == "f32" else 2),
    )


def as_numpy(t):
    """Host numpy view of a tensor; bf16 becomes uint16 bit patterns (what the oracle reads)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def f32_to_bf16_bits(x):
    """Round fp32 numpy values to bf16 (nearest-even, via torch) and return the uint16 bit patterns."""
    t = torch.as_tensor(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()
