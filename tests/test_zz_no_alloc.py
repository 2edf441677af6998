"""da_attention_noalloc (partials in the library's fixed device array, no workspace argument, nothing allocated)
against da_attention and the fp64 oracle, through the C ABI: two calls in a row, the second with a smaller input
(the array still holds the first call's partial rows), then a plan too large for the array."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2401_02669_amd import distattn as da
from paper_2401_02669_amd import synth
from util import assert_parity, make_plan, oracle_attention

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SCRATCH_BYTES = 8 << 20  # DA_NOALLOC_SCRATCH_BYTES


def run_both(w):
    plan = make_plan(w)
    assert max(plan.nsplits(r) for r in range(w["B"])) > 1     # partial rows are really used
    assert plan.workspace_bytes <= SCRATCH_BYTES
    a = (w["q"], w["k_pool"], w["v_pool"], w["block_table"], w["seq_lens"])
    ref_out, ref_lse = plan.attention(*a)
    out = torch.full_like(ref_out, float("nan"))
    lse = torch.full_like(ref_lse, float("nan"))
    stream = torch.cuda.current_stream()
    st = da.lib().da_attention_noalloc(plan._h, *[ctypes.c_void_p(t.data_ptr()) for t in a],
                                       ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(lse.data_ptr()),
                                       ctypes.c_void_p(stream.cuda_stream))
    assert st == da.DA_OK, da.status_string(st)
    torch.cuda.synchronize()
    assert plan.error_flags() == 0
    plan.close()
    return out, lse, ref_out, ref_lse


def test_two_calls_in_a_row_the_second_smaller():
    first = synth.make(synth.recipe("c5_mixed", len_div=16), DEV)          # 64 ragged requests, many splits
    second = synth.make(synth.recipe("c3_70b", len_div=256, B=2), DEV)     # fewer, shorter: fewer partial rows
    for tag, w in (("first", first), ("second (smaller)", second)):
        print("da_attention_noalloc", tag, w["name"], flush=True)
        out, lse, ref_out, ref_lse = run_both(w)
        # same kernels, same partial rows: the two entry points agree bit for bit
        assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse), tag
        o_ref, l_ref = oracle_attention(w)
        assert_parity(out.cpu().numpy(), lse.cpu().numpy(), o_ref, l_ref, w["dtype"], "noalloc " + tag)


def test_a_plan_beyond_the_fixed_array_is_rejected():
    # one partial per block: 20000 blocks x 8 heads x 520 B of partial rows > 8 MiB
    p = da.DaProblem()
    p.batch, p.num_q_heads, p.num_kv_heads, p.head_dim = 1, 8, 8, 128
    p.block_tokens, p.max_blocks_per_seq, p.num_phys_blocks = 16, 20000, 20000
    p.kv_dtype = p.q_dtype = da.DA_BF16
    p.scale = 0.1
    p.kv_token_stride, p.kv_head_stride, p.kv_block_stride = 128, 128 * 16, 128 * 16 * 8
    p.q_len = 1
    plan = da.Plan(p, [20000 * 16], blocks_per_split=1)
    assert plan.workspace_bytes > SCRATCH_BYTES
    dummy = torch.zeros(4096, dtype=torch.float32, device=DEV)
    ptr = ctypes.c_void_p(dummy.data_ptr())
    st = da.lib().da_attention_noalloc(plan._h, ptr, ptr, ptr, ptr, ptr, ptr, None, None)
    assert st == da.DA_ERR_WORKSPACE           # rejected on the host, nothing launched
    plan.close()
