"""Static checks of the hand-scheduled chunk statements (csrc/gen_tiles_asm.py).

The hardware does not interlock a matrix product against the vector instructions around it, and vector loads land
in their registers whenever they come back; the generator orders the instructions so that
  * a product reads a register a vector instruction wrote two issue slots earlier at the soonest,
  * a vector instruction reads a product's result only after two further products have gone out (each waits for the
    matrix pipe, so the one before it has been written by then),
  * nothing reads or overwrites the target of a load that has not been waited for, and no load overwrites a register
    that an instruction of the same pass still has to read,
  * a select follows its compare, and a conversion its exponential, with the wait states the compiler would put.
This test walks every statement body as the not-taken path through it, twice in a row (what the second pass finds
outstanding is what the first one left), and checks those rules instruction by instruction."""
import os
import re
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2401_02669_amd", "csrc")
sys.path.insert(0, CSRC)
import gen_tiles_asm as g  # noqa: E402


def regs(tok):
    """Registers named by one operand: ('v', n) / ('a', n)."""
    m = re.fullmatch(r"-?([va])(\d+)", tok)
    if m:
        return [(m.group(1), int(m.group(2)))]
    m = re.fullmatch(r"([va])\[(\d+):(\d+)\]", tok)
    if m:
        return [(m.group(1), n) for n in range(int(m.group(2)), int(m.group(3)) + 1)]
    return []


def parse(ins):
    """(op, written registers, read registers, writes vcc, reads vcc)"""
    op, _, rest = ins.partition(" ")
    toks = [t.strip() for t in rest.split(",")] if rest else []
    toks = [t.split()[0] if t else t for t in toks]   # drops modifiers such as "offset:64 nt"
    if op.startswith("s_") or not toks:
        return op, [], [], False, False
    if op.startswith("v_cmp"):
        return op, [], [r for t in toks[1:] for r in regs(t)], True, False
    dst = regs(toks[0])
    src = [r for t in toks[1:] for r in regs(t)]
    return op, dst, src, False, "vcc" in toks[1:]


def hot_path(ins):
    """The instructions a pass executes when no rare branch is taken (the branches themselves stay, as issue slots)."""
    out = []
    for i in ins:
        if i.startswith("s_branch 39f") or i.startswith("s_sub_u32 %s" % g.RUN_N):
            break
        if not i.endswith(":"):
            out.append(i)
    return out


def check(ins, what):
    stream = hot_path(ins) * 2
    slot = 0            # issue slots so far (an s_nop k takes k + 1)
    products = 0
    written_at = {}     # register -> (slot of the vector instruction that wrote it last, was it an exponential)
    product_at = {}     # register -> number of products out when a product wrote it last
    outstanding = []    # loads not yet known to be back: lists of registers, oldest first
    vcc_at = -99
    for i in stream:
        op, dst, src, wvcc, rvcc = parse(i)
        if op == "s_nop":
            slot += int(i.split()[1]) + 1
            continue
        if op == "s_waitcnt":
            m = re.search(r"vmcnt\((\d+)\)", i)
            if m:
                keep = int(m.group(1))
                outstanding = outstanding[len(outstanding) - keep:] if keep else []
            slot += 1
            continue
        pending = {r for ld in outstanding for r in ld}
        # (a load may target a register that an older load still targets: loads come back in order)
        for r in src + ([] if op.startswith("global_load") else dst):
            assert r not in pending, "%s: %r touches %s%d before its load is waited for" % (what, i, r[0], r[1])
        if op.startswith("global_load"):
            outstanding.append(dst)
        elif op.startswith("v_mfma"):
            for r in src:
                if r in written_at:
                    gap = slot - written_at[r][0] - 1
                    assert gap >= 2, "%s: %r reads %s%d %d slots after its write" % (what, i, r[0], r[1], gap)
                assert r not in product_at or r in dst, "%s: %r takes a product's result as an operand" % (what, i)
            products += 1
            for r in dst:
                product_at[r] = products
                written_at.pop(r, None)
        else:
            for r in src:
                if r in product_at:
                    later = products - product_at[r]
                    assert later >= 2, "%s: %r reads %s%d with %d products behind it" % (what, i, r[0], r[1], later)
                if r in written_at and written_at[r][1]:
                    assert slot - written_at[r][0] - 1 >= 1, "%s: %r reads an exponential at once" % (what, i)
            if rvcc:
                assert slot - vcc_at - 1 >= 2, "%s: %r follows its compare too closely" % (what, i)
            if wvcc:
                vcc_at = slot
            for r in dst:
                written_at[r] = (slot, op.startswith("v_exp"))
                product_at.pop(r, None)
        slot += 1
    # what a pass leaves behind is what the next one assumes may be outstanding
    assert len(outstanding) <= len(g.OLD_K), what
    return True


VARIANTS = [(t, m, r) for t in (2, 4) for m, r in ((False, False), (True, False), (False, True))]


@pytest.mark.parametrize("tiles,masked,run", VARIANTS)
def test_chunk_statement_keeps_the_distances(tiles, masked, run):
    for nt in (" nt", ""):
        assert check(g.body(tiles, masked, nt, run=run), "tiles %d masked %d run %d" % (tiles, masked, run))


def test_request_statement_keeps_the_distances():
    assert check(g.request_body(" nt"), "request")


def test_the_checks_find_a_planted_mistake():
    ins = g.body(4, False, " nt")
    # a product moved right behind the conversion that writes its operand
    k = next(n for n, i in enumerate(ins) if i.startswith("v_cvt_pk_bf16_f32 v%d," % (g.PH(0) + 3)))
    bad = ins[:k + 1] + [x for x in ins[k + 1:] if not x.startswith("s_nop")]
    first_pv = next(n for n, i in enumerate(bad) if n > k and i.startswith("v_mfma") and "v[%d:%d]" % (g.PH(0), g.PH(0) + 3) in i)
    bad = bad[:k + 1] + [bad[first_pv]] + bad[k + 1:first_pv] + bad[first_pv + 1:]
    with pytest.raises(AssertionError):
        check(bad, "planted")
    # a score read right behind the last product that writes it
    ins = g.body(4, False, " nt")
    last_qk0 = max(n for n, i in enumerate(ins) if i.startswith("v_mfma") and i.split()[1].startswith("v[%d:" % g.S(0, 4)))
    reader = next(n for n, i in enumerate(ins) if i.startswith("v_max3_f32") and "v%d," % g.S(0, 4) in i + ",")
    bad = ins[:last_qk0 + 1] + [ins[reader]] + ins[last_qk0 + 1:reader] + ins[reader + 1:]
    with pytest.raises(AssertionError):
        check(bad, "planted")
