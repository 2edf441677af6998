"""Shared helpers of the GPU parity tests: run the HIP library and the CPU oracle on one workload."""
import numpy as np
import torch

import oracle
from paper_2401_02669_amd import distattn as da
from paper_2401_02669_amd import synth

# Tolerances of the parity bar.  bf16 K/V with fp32 accumulation: max-abs 2e-3 and relative L2 1e-3
# against the fp64 oracle; fp32 K/V: 1e-5 on both.
TOL = {"bf16": dict(max_abs=2e-3, rel_l2=1e-3, lse=1e-4), "f32": dict(max_abs=1e-5, rel_l2=1e-5, lse=2e-5)}
TOL["f16"] = TOL["bf16"]  # IEEE half K/V: the 16-bit bar (half carries three more mantissa bits than bf16)


def errors(got, ref):
    got = np.asarray(got, dtype=np.float64)
    diff = got - ref
    den = float(np.linalg.norm(ref))
    return float(np.max(np.abs(diff))) if diff.size else 0.0, (float(np.linalg.norm(diff)) / den if den > 0 else 0.0)


def oracle_inputs(w):
    """Host copies of a workload's tensors in the form the oracle reads (bf16 as uint16 bits)."""
    return dict(q=synth.as_numpy(w["q"]), k_pool=synth.as_numpy(w["k_pool"]), v_pool=synth.as_numpy(w["v_pool"]),
                block_table=w["block_table"].cpu().numpy(), seq_lens=w["seq_lens"].cpu().numpy())


def oracle_attention(w, host=None, pairs=None, n_threads=16):
    h = host or oracle_inputs(w)
    return oracle.attention(h["q"], h["k_pool"], h["v_pool"], h["block_table"], h["seq_lens"], w["T"], w["scale"],
                            pairs=pairs, n_threads=n_threads)


def make_plan(w, **tuning):
    prob = da.make_problem(w["q"], w["k_pool"], w["block_table"], w["scale"])
    lens = w["seq_lens"].cpu().tolist()
    return da.Plan(prob, lens, **tuning)


def gpu_attention(w, **tuning):
    plan = make_plan(w, **tuning)
    out, lse = plan.attention(w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    torch.cuda.synchronize()
    flags = plan.error_flags()
    plan.close()
    return out.cpu().numpy(), lse.cpu().numpy(), flags


def assert_parity(got_out, got_lse, ref_out, ref_lse, dtype, what=""):
    tol = TOL[dtype]
    assert np.all(np.isfinite(got_out)), what + ": non-finite output"
    max_abs, rel_l2 = errors(got_out, ref_out)
    assert max_abs <= tol["max_abs"], "%s: max-abs %.3e > %.1e" % (what, max_abs, tol["max_abs"])
    assert rel_l2 <= tol["rel_l2"], "%s: rel-L2 %.3e > %.1e" % (what, rel_l2, tol["rel_l2"])
    finite = np.isfinite(ref_lse)
    assert np.array_equal(np.isneginf(got_lse), np.isneginf(ref_lse)), what + ": lse -inf pattern"
    if finite.any():
        err = np.max(np.abs(got_lse[finite] - ref_lse[finite]) / np.maximum(1.0, np.abs(ref_lse[finite])))
        assert err <= tol["lse"], "%s: lse error %.3e" % (what, err)
    return max_abs, rel_l2
