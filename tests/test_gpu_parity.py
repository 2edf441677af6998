"""GPU parity: the HIP library (through its C ABI) against the fp64 CPU oracle, element by element,
on seeded workloads small enough for the oracle yet spanning many tiles, ragged tails and all the
degenerate cases."""
import numpy as np
import pytest
import torch

import oracle
from paper_2401_02669_amd import distattn as da
from paper_2401_02669_amd import synth
from util import TOL, assert_parity, errors, gpu_attention, make_plan, oracle_attention, oracle_inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def note(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ the five workloads, scaled down
SCALED = [
    ("c1_tiny", 1, {}),
    ("c2_7b", 16, {}),
    ("c3_70b", 64, {}),
    ("c4_2m", 100, {}),
    ("c5_mixed", 50, {}),
]


@pytest.mark.parametrize("name,div,over", SCALED, ids=[s[0] for s in SCALED])
@pytest.mark.parametrize("kernel", [da.DA_KERNEL_AUTO, da.DA_KERNEL_VALU], ids=["auto", "valu"])
def test_scaled_workloads_match_oracle(name, div, over, kernel):
    w = synth.make(synth.recipe(name, len_div=div, **over), DEV)
    note("case %s kernel=%d lens[min,max]=%d,%d" % (w["name"], kernel, w["seq_lens_host"].min(), w["seq_lens_host"].max()))
    ref_out, ref_lse = oracle_attention(w)
    out, lse, flags = gpu_attention(w, kernel=kernel)
    assert flags == 0
    assert_parity(out, lse, ref_out, ref_lse, w["dtype"], w["name"])
    # per-request bar, so that short requests are not hidden behind long ones
    for r in range(w["B"]):
        _, rel = errors(out[r], ref_out[r])
        assert rel <= TOL[w["dtype"]]["rel_l2"], "request %d rel-L2 %.3e" % (r, rel)


# ------------------------------------------------------------------ raw partials, Eq. 2 literally
@pytest.mark.parametrize("bps", [0, 1, 3])
@pytest.mark.parametrize("name,div", [("c1_tiny", 1), ("c5_mixed", 200), ("c3_70b", 128)])
@pytest.mark.parametrize("kernel", [da.DA_KERNEL_AUTO, da.DA_KERNEL_VALU], ids=["auto", "valu"])
def test_partials_match_micro_attention(name, div, bps, kernel):
    w = synth.make(synth.recipe(name, len_div=div), DEV)
    note("case %s bps=%d kernel=%d" % (w["name"], bps, kernel))
    plan = make_plan(w, blocks_per_split=bps, kernel=kernel)
    po, pm, pe = plan.partial(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    out, lse = plan.combine(po, pm, pe)
    torch.cuda.synchronize()
    T = w["T"]
    bounds = []
    for r in range(w["B"]):
        L = int(w["seq_lens_host"][r])
        b = [0]
        for j in range(plan.nsplits(r)):
            lo, hi = plan.split(r, j)
            assert lo == b[-1] and lo <= hi <= L
            if bps > 0 and L > 0:
                assert lo == min(L, j * bps * T) and hi == min(L, (j + 1) * bps * T)  # whole blocks, as asked
            b.append(hi)
        assert b[-1] == L
        bounds.append(b)
    h = oracle_inputs(w)
    MA, m, e, nparts = oracle.micro_attention(h["q"], h["k_pool"], h["v_pool"], h["block_table"], h["seq_lens"],
                                              T, w["scale"], bounds, n_threads=16)
    assert plan.num_partials == MA.shape[0]
    po, pm, pe = po.cpu().numpy().astype(np.float64), pm.cpu().numpy().astype(np.float64), pe.cpu().numpy().astype(np.float64)
    tight = w["dtype"] == "f32"
    live = np.isfinite(m)
    assert np.array_equal(np.isneginf(pm), ~live)
    assert np.all(pe[~live] == 0) and np.all(po[~live] == 0)
    np.testing.assert_allclose(pm[live], m[live], rtol=0, atol=2e-5 if tight else 2e-5)
    # e_j and MA_j are relative to m_j: remove the (tiny) difference of the two maxima before comparing
    adj = np.exp(pm[live] - m[live])
    np.testing.assert_allclose(pe[live] * adj, e[live], rtol=2e-5 if tight else 2e-4)
    num = np.linalg.norm(po[live] * adj[:, None] - MA[live], axis=1)
    den = np.linalg.norm(MA[live], axis=1)
    assert np.all(num <= (1e-5 if tight else 1e-3) * den + 1e-12)
    # and their aggregation is the plain result
    ref_out, ref_lse = oracle_attention(w, h)
    assert_parity(out.cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, w["dtype"], w["name"])
    plan.close()


# ------------------------------------------------------------------ degenerate and ragged shapes
def custom(lens, Hq, Hkv, T, dtype="bf16", shuffle=True, **kw):
    return synth.recipe("c5_mixed", B=len(lens), Hq=Hq, Hkv=Hkv, T=T, dtype=dtype, lens=list(lens), shuffle=shuffle, **kw)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("kernel", [da.DA_KERNEL_AUTO, da.DA_KERNEL_VALU], ids=["auto", "valu"])
def test_edge_lengths(dtype, kernel):
    T = 64
    lens = [0, 1, T - 1, T, T + 1, 2, 5 * T + 7, 0, 33, 16 * T]
    w = synth.make(custom(lens, Hq=4, Hkv=2, T=T, dtype=dtype), DEV)
    note("case edge_lengths %s kernel=%d" % (dtype, kernel))
    ref_out, ref_lse = oracle_attention(w)
    for bps in (0, 1, 2):
        out, lse, flags = gpu_attention(w, blocks_per_split=bps, kernel=kernel)
        assert flags == 0
        assert np.all(out[0] == 0) and np.all(np.isneginf(lse[0])) and np.all(out[7] == 0)
        assert_parity(out, lse, ref_out, ref_lse, dtype, "edge bps=%d" % bps)


@pytest.mark.parametrize("G", [1, 2, 3, 4, 5, 8, 16, 24, 32, 64])
@pytest.mark.parametrize("kernel", [da.DA_KERNEL_AUTO, da.DA_KERNEL_VALU], ids=["auto", "valu"])
def test_group_sizes(G, kernel):
    w = synth.make(custom([700, 129, 2048], Hq=2 * G, Hkv=2, T=128), DEV)
    note("case group G=%d kernel=%d" % (G, kernel))
    ref_out, ref_lse = oracle_attention(w)
    out, lse, flags = gpu_attention(w, kernel=kernel)
    assert flags == 0
    assert_parity(out, lse, ref_out, ref_lse, "bf16", "G=%d" % G)


@pytest.mark.parametrize("G", [2, 3, 8, 16, 24])
def test_fp32_groups_on_the_matrix_cores(G):
    lens = [700, 129, 0, 2048, 1, 31, 33]
    w = synth.make(custom(lens, Hq=2 * G, Hkv=2, T=64, dtype="f32"), DEV)
    note("case fp32 group G=%d" % G)
    prob = da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"])
    assert da.plan_schedule(prob, lens)["kernel"] == da.DA_KERNEL_MFMA
    ref_out, ref_lse = oracle_attention(w)
    for bps in (0, 1, 3):
        out, lse, flags = gpu_attention(w, blocks_per_split=bps)
        assert flags == 0
        assert_parity(out, lse, ref_out, ref_lse, "f32", "fp32 G=%d bps=%d" % (G, bps))
    out, lse, flags = gpu_attention(w, kernel=da.DA_KERNEL_VALU)
    assert_parity(out, lse, ref_out, ref_lse, "f32", "fp32 G=%d valu" % G)


def test_fp32_scaled_gqa_workload_with_outlier_keys():
    w = synth.make(synth.recipe("c3_70b", len_div=64, dtype="f32"), DEV)
    ref_out, ref_lse = oracle_attention(w)
    out, lse, flags = gpu_attention(w)
    assert flags == 0
    assert_parity(out, lse, ref_out, ref_lse, "f32", "c3_70b/64 fp32")


@pytest.mark.parametrize("T", [16, 48, 112, 1024])
@pytest.mark.parametrize("G", [1, 4])
def test_block_sizes_give_the_same_answer(T, G):
    lens = [1000, 37, 4100]
    w = synth.make(custom(lens, Hq=2 * G, Hkv=2, T=T), DEV)
    note("case block size T=%d G=%d" % (T, G))
    ref_out, ref_lse = oracle_attention(w)
    for bps in (0, 1, 5):
        out, lse, flags = gpu_attention(w, blocks_per_split=bps)
        assert flags == 0
        assert_parity(out, lse, ref_out, ref_lse, "bf16", "T=%d bps=%d" % (T, bps))


def test_mixed_query_dtype_and_strided_pool():
    w = synth.make(custom([900, 300], Hq=8, Hkv=2, T=64), DEV)
    # fp32 query over bf16 K/V
    w["q"] = w["q"].float() + 0.001
    # pools whose token rows are padded (stride 160 elements) inside a larger allocation
    for key in ("k_pool", "v_pool"):
        big = torch.full(w[key].shape[:3] + (160,), float("nan"), dtype=w[key].dtype, device=DEV)
        big[..., :128] = w[key]
        w[key] = big[..., :128]
    assert w["k_pool"].stride(2) == 160
    h = dict(q=synth.as_numpy(w["q"]), k_pool=synth.as_numpy(w["k_pool"]), v_pool=synth.as_numpy(w["v_pool"]),
             block_table=w["block_table_host"], seq_lens=w["seq_lens_host"])
    ref_out, ref_lse = oracle_attention(w, h)
    for kernel in (da.DA_KERNEL_AUTO, da.DA_KERNEL_VALU):
        out, lse, flags = gpu_attention(w, kernel=kernel)
        assert_parity(out, lse, ref_out, ref_lse, "bf16", "mixed/strided kernel=%d" % kernel)


def test_softmax_range_stress():
    # 5 % of the keys scaled x8 and a large score scale: block maxima differ by far more than 88,
    # so most partial weights underflow to exactly 0 in fp32 - and the result must still be right
    w = synth.make(custom([3000, 800], Hq=8, Hkv=1, T=64, outlier_frac=0.05), DEV)
    w["scale"] = 1.0
    ref_out, ref_lse = oracle_attention(w)
    for bps in (1, 4):
        out, lse, _ = gpu_attention(w, blocks_per_split=bps)
        # near one-hot softmax: outputs are O(1) value rows, keep the same absolute bar
        assert_parity(out, lse, ref_out, ref_lse, "bf16", "range stress bps=%d" % bps)


def test_deterministic_and_plan_update():
    w = synth.make(synth.recipe("c5_mixed", len_div=100), DEV)
    plan = make_plan(w)
    a, la = plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    b, lb = plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(la, lb)
    # shorter lengths through the same plan object
    lens2 = np.maximum(w["seq_lens_host"] // 3, 1).astype(np.int32)
    w2 = dict(w)
    w2["seq_lens"] = torch.as_tensor(lens2, device=DEV)
    plan.update(lens2.tolist())
    c, lc = plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w2["seq_lens"])
    torch.cuda.synchronize()
    h = oracle_inputs(w2)
    ref_out, ref_lse = oracle_attention(w2, h)
    assert_parity(c.cpu().numpy(), lc.cpu().numpy(), ref_out, ref_lse, "bf16", "after update")
    plan.close()


def test_many_small_requests_share_workgroups():
    # hundreds of short requests: most workgroups walk several requests, a few requests are cut
    rng = np.random.RandomState(3)
    lens = [int(x) for x in rng.randint(0, 300, size=600)] + [5000, 7777]
    w = synth.make(custom(lens, Hq=8, Hkv=8, T=32), DEV)
    ref_out, ref_lse = oracle_attention(w)
    for kernel in (da.DA_KERNEL_VALU, da.DA_KERNEL_MFMA):
        out, lse, flags = gpu_attention(w, kernel=kernel)
        assert flags == 0
        assert_parity(out, lse, ref_out, ref_lse, "bf16", "many small, kernel=%d" % kernel)
        for r in (0, 17, 599, 600, 601):
            _, rel = errors(out[r], ref_out[r])
            assert rel <= TOL["bf16"]["rel_l2"]


def test_more_head_groups_than_workgroup_slots():
    # Hkv * head tiles = 1024 > 256 persistent slots: one run per (kv-head, head tile), requests never split
    w = synth.make(custom([100, 37], Hq=128 * 64, Hkv=128, T=16), DEV)
    prob = da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"])
    s = da.plan_schedule(prob, w["seq_lens_host"].tolist(), kernel=da.DA_KERNEL_VALU)
    assert s["workgroups"] == 1024 and s["nsplits"] == [1, 1]
    ref_out, ref_lse = oracle_attention(w)
    for kernel in (da.DA_KERNEL_VALU, da.DA_KERNEL_AUTO):
        out, lse, flags = gpu_attention(w, kernel=kernel)
        assert_parity(out, lse, ref_out, ref_lse, "bf16", "many heads kernel=%d" % kernel)


def test_plan_update_grows_its_tables():
    T = 16
    w = synth.make(custom([6400, 6400, 6400, 6400], Hq=2, Hkv=2, T=T), DEV)
    short = [16, 16, 16, 16]
    prob = da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"])
    plan = da.Plan(prob, short, blocks_per_split=1)     # 4 splits in all
    assert plan.num_partials == 4 * 2
    plan.update(w["seq_lens_host"].tolist())            # 1600 splits: more than the tables were made for
    assert plan.num_partials == 1600 * 2
    out, lse = plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    torch.cuda.synchronize()
    ref_out, ref_lse = oracle_attention(w)
    assert_parity(out.cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, "bf16", "grown plan")
    plan.close()


def test_stale_plan_still_gives_exact_results():
    # the plan was cut for other lengths than the device holds: longer, shorter, zero, from zero
    T = 64
    planned = [5000, 3000, 0, 700, 64]
    actual = [5100, 1500, 90, 0, 6400]
    w = synth.make(custom(actual, Hq=8, Hkv=2, T=T), DEV)
    ref_out, ref_lse = oracle_attention(w)
    prob = da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"])
    for kernel in (da.DA_KERNEL_VALU, da.DA_KERNEL_MFMA):
        for bps in (0, 2):
            plan = da.Plan(prob, planned, blocks_per_split=bps, kernel=kernel)
            out, lse = plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
            po, pm, pe = plan.partial(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
            out2, lse2 = plan.combine(po, pm, pe)
            torch.cuda.synchronize()
            assert plan.error_flags() == 0
            plan.close()
            assert_parity(out.cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, "bf16", "stale plan fused")
            assert_parity(out2.cpu().numpy(), lse2.cpu().numpy(), ref_out, ref_lse, "bf16", "stale plan two-step")


def test_bad_block_ids_are_skipped_and_flagged():
    w = synth.make(custom([640, 640], Hq=2, Hkv=2, T=64, spare_frac=0.0), DEV)
    table = w["block_table"].clone()
    table[0, 3] = w["num_phys"] + 5
    table[1, 0] = -7
    plan = make_plan(w)
    out, lse = plan.attention(w["q"], w["k_pool"], w["v_pool"], table, w["seq_lens"])
    torch.cuda.synchronize()
    assert plan.error_flags() == 1
    assert plan.error_flags() == 0  # reading clears it
    assert torch.isfinite(out).all()
    # a skipped block contributes nothing: the same as a request whose table simply lacks that block
    t2 = w["block_table_host"].copy()
    t2[0, 3:-1] = t2[0, 4:]
    t2[1, 0:-1] = t2[1, 1:]
    h = oracle_inputs(w)
    h["block_table"] = t2
    h["seq_lens"] = (w["seq_lens_host"] - 64).astype(np.int32)
    ref_out, ref_lse = oracle_attention(w, h)
    assert_parity(out.cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, "bf16", "skipped blocks")
    plan.close()


def test_combine_alone_on_hand_made_partials():
    B, Hq, d = 2, 3, 128
    rng = np.random.RandomState(5)
    w = synth.make(custom([64 * 6, 64 * 2], Hq=Hq, Hkv=3, T=64), DEV)
    plan = make_plan(w, blocks_per_split=2)  # nsplits = [3, 1]
    assert [plan.nsplits(0), plan.nsplits(1)] == [3, 1]
    n = plan.num_partials
    MA = rng.standard_normal((n, d))
    m = rng.standard_normal(n) * 30
    e = rng.uniform(0.5, 50.0, n)
    m[1] = -np.inf   # an empty split in the middle of request 0, head 0
    e[1] = 0.0
    MA[1] = 0.0
    ref_out, ref_lse = oracle.aggregate(MA, m, e, np.array([3, 1], dtype=np.int32), Hq)
    t = lambda a: torch.as_tensor(a, dtype=torch.float32, device=DEV)
    out, lse = plan.combine(t(MA), t(m), t(e))
    torch.cuda.synchronize()
    # inputs were rounded to fp32 on the way in
    MAf, mf, ef = (np.asarray(a, dtype=np.float32).astype(np.float64) for a in (MA, m, e))
    ref_out, ref_lse = oracle.aggregate(MAf, mf, ef, np.array([3, 1], dtype=np.int32), Hq)
    np.testing.assert_allclose(out.cpu().numpy(), ref_out, rtol=2e-5, atol=1e-6)
    np.testing.assert_allclose(lse.cpu().numpy(), ref_lse, rtol=1e-6, atol=1e-5)
    plan.close()


def test_workspace_and_argument_errors_on_device():
    w = synth.make(custom([500], Hq=2, Hkv=1, T=64), DEV)
    plan = make_plan(w, blocks_per_split=1)
    small = torch.empty((16,), dtype=torch.uint8, device=DEV)
    with pytest.raises(da.DistAttnError) as e:
        plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"], workspace=small)
    assert e.value.status == da.DA_ERR_WORKSPACE
    with pytest.raises(da.DistAttnError) as e:
        plan.partial(None, w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"],
                     part_o=small, part_m=small, part_e=small)
    assert e.value.status == da.DA_ERR_INVALID_ARG
    plan.close()


@pytest.mark.parametrize("Hq,Hkv,dtype", [(2, 2, "bf16"), (8, 2, "bf16"), (8, 2, "f16"), (32, 2, "bf16")])
def test_many_short_requests_one_wavefront_per_split(Hq, Hkv, dtype):
    """Hundreds of short requests per run: each wavefront takes whole splits and writes its result from registers.
    Few compute units, so that a run holds enough splits for that mode; lengths include empty, one token, block
    edges, and a few long requests that are cut across runs."""
    rng = np.random.RandomState(11)
    lens = [int(x) for x in rng.randint(0, 700, size=700)] + [0, 1, 63, 64, 65, 128, 5000, 9000]
    w = synth.make(custom(lens, Hq=Hq, Hkv=Hkv, T=64, dtype=dtype), DEV)
    note("case wavefront splits Hq=%d Hkv=%d %s" % (Hq, Hkv, dtype))
    ref_out, ref_lse = oracle_attention(w)
    plan = make_plan(w, num_cus=8)
    d = plan.describe()
    assert d["kernel"] == da.DA_KERNEL_MFMA and d["head_tile"] == 16 and d["wavefront_splits"] == (1 if Hq // Hkv <= 16 else 0)
    out, lse = plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    po, pm, pe = plan.partial(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    out2, lse2 = plan.combine(po, pm, pe)
    torch.cuda.synchronize()
    assert plan.error_flags() == 0
    # (a group of 16 columns and more costs a split so much that these plans leave every request whole)
    assert max(plan.nsplits(r) for r in range(len(lens))) > 1 or Hq // Hkv >= 16
    plan.close()
    assert_parity(out.cpu().numpy(), lse.cpu().numpy(), ref_out, ref_lse, dtype, "wavefront splits, fused")
    assert_parity(out2.cpu().numpy(), lse2.cpu().numpy(), ref_out, ref_lse, dtype, "wavefront splits, two calls")
    # the same problem with the workgroup-shared walk (all compute units: too few splits per run for the other mode)
    plan = make_plan(w)
    assert plan.describe()["wavefront_splits"] == 0
    out3, lse3 = plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    torch.cuda.synchronize()
    plan.close()
    assert_parity(out3.cpu().numpy(), lse3.cpu().numpy(), ref_out, ref_lse, dtype, "shared walk")
