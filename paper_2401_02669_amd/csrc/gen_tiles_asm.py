"""Writes tiles_asm.h: the per-chunk instruction streams of the multi-tile matrix-core MicroAttention kernel.

The kernel (micro_attention_mfma_tiles.hip) serves 32, 64 or 128 columns from one K/V read; at that width a chunk's
vector-ALU and matrix work, not memory, decide the speed, and what the compiler makes of the same arithmetic written
in C++ (it shuttles the accumulators between the two halves of the register file on every chunk, and keeps matrix
and vector work apart) takes twice the cycles.  A chunk is therefore written out instruction by instruction here,
over a fixed register map:

  accumulation registers (only the statements below touch them)
    a[0:127]    O^T accumulators, tile t at a[32t:32t+31], dimension group n at +4n
    a[128:191]  Q^T operands, tile t, k-step s at a[128+16t+4s:+3]
    a[192:223]  K rows of the chunk being processed (then requested again for the next), load j at a[192+4j:+3]
    a[224:239]  exp-sums, tile t at a[224+4t:+3] (a row of ones times P^T: all four registers hold the sum)
    a[240:243]  bf16 ones
  vector registers above the kernel's own allocation limit of 96
    v[96:127]   scores, tile t at v[96+8t:+7] (tokens 4g+i, then 16+4g+i of lane group g)
    v[128:159]  V rows as loaded, load j at v[128+4j:+3]
    v[160:191]  V^T operands: even dims at v[160+4w:+3], odd dims at v[176+4w:+3]
    v[192:207]  weights of a tile as bf16 pairs, two buffers of (high 4, low 4)
    v[208:223]  temporaries
    v[224:235]  per tile: lane's running maximum m, reference maximum mref, and nmu = -mref (0 while mref = -inf)
    v[236:245]  the lane's byte offsets of its 8 V loads and 2 groups of K loads inside a full chunk
    v[246:247]  clamps for a chunk whose last rows are not valid

Order of a chunk statement (chunk i; the K rows of i were requested by the statement before, the V^T operands of its
dimension groups 0 and 1 built there):
    K.Q^T of tile 0; behind its products the V^T operands of groups 2 and 3, then the requests for the V rows of i+1
    K.Q^T of the other tiles, K register by K register, each register requested again (chunk i+1) after its last
           product; behind them: maximum, (rarely) rescale and the weights' high parts of tile 0
    tile after tile: V^T.P^T of tile t with the high parts of its weights, then with the low parts (and the ones row);
           behind them: the low parts of tile t's weights, (t = 0: maxima and rescale of all other tiles,) the
           weights' high parts of tile t+1; behind the last tile's products the V^T operands of groups 0 and 1 of i+1
How many vector instructions go behind one product follows from measured issue costs (see interleave).

Run `python gen_tiles_asm.py` after changing it; the header it writes is committed beside it.
"""
import os

HERE = os.path.dirname(os.path.abspath(__file__))

MFMA = "v_mfma_f32_16x16x32_bf16"
CAP = 96  # the kernel's own code is compiled for v[0:95]


def a4(i):
    return "a[%d:%d]" % (i, i + 3)


def v4(i):
    return "v[%d:%d]" % (i, i + 3)


def ACC(t, n):
    return 32 * t + 4 * n


def QOP(t, s):
    return 128 + 16 * t + 4 * s


def KOP(j):
    return 192 + 4 * j


def ESUM(t):
    return 224 + 4 * t


ONES = 240


def S(t, i):
    return 96 + 8 * t + i


def VR(j, w):
    return 128 + 4 * j + w


def VE(w):
    return 160 + 4 * w


def VO(w):
    return 176 + 4 * w


def PH(b):
    return 192 + 8 * b


def PL(b):
    return 196 + 8 * b


def T(i):
    return 208 + i


def M(t):
    return 224 + t


def MREF(t):
    return 228 + t


def NMU(t):
    return 232 + t


def VOFF(j):
    return 236 + j


def KOFF(g):
    return 244 + g


VCL, KCL = 246, 247
K_ORDER = (0, 4, 1, 5, 2, 6, 3, 7)  # K loads alternate between the chunk's two 16-row halves
OLD_K = ["K%d" % j for j in K_ORDER]  # what may be outstanding when a statement starts, oldest first


def v_row(j):
    return 16 * (j >> 2) + (j & 3)   # lane group g reads tokens 16 * (j / 4) + 4 g + j % 4 with its V load j


# ---------------------------------------------------------------------------------------------- pieces

def set_offsets():
    """The lane's offsets inside a full chunk, from the lane constants."""
    out = ["v_mad_u32_u24 v%d, %d, %%[rb], %%[vlane]" % (VOFF(j), v_row(j)) for j in range(8)]
    out += ["v_mov_b32_e32 v%d, %%[klane]" % KOFF(0), "v_mad_u32_u24 v%d, 16, %%[rb], %%[klane]" % KOFF(1)]
    return out


def clamp_offsets():
    """For a chunk whose last valid row comes before row 31: rows past it re-read it."""
    out = ["v_add_u32_e32 v%d, %%[last], %%[ln16]" % VCL, "v_add_u32_e32 v%d, %%[last], %%[lg16]" % KCL]
    out += ["v_min_u32_e32 v%d, v%d, v%d" % (VOFF(j), VOFF(j), VCL) for j in range(8)]
    out += ["v_min_u32_e32 v%d, v%d, v%d" % (KOFF(g), KOFF(g), KCL) for g in range(2)]
    return out


def k_load(j, nt):
    off = (" offset:%d" % (64 * (j % 4))) if j % 4 else ""
    return ("load", "K%d" % j, "global_load_dwordx4 %s, v%d, %%[kbase]%s%s" % (a4(KOP(j)), KOFF(j // 4), off, nt))


def v_load(j, nt):
    return ("load", "V%d" % j, "global_load_dwordx4 %s, v%d, %%[vbase]%s" % (v4(VR(j, 0)), VOFF(j), nt))


def qk(t, j):
    half, s = j // 4, j % 4
    dst = v4(S(t, 4 * half))
    return "%s %s, %s, %s, %s" % (MFMA, dst, a4(KOP(j)), a4(QOP(t, s)), "0" if s == 0 else dst)


def perms_of_group(w):
    """V^T operands of dimension group w (the four registers of its even and of its odd operand; a register pairs
    the tokens of two V loads)."""
    out = [("need", "V%d" % j) for j in range(8)]
    for t in range(4):
        out.append("v_perm_b32 v%d, v%d, v%d, %%[sel_lo]" % (VE(w) + t, VR(2 * t + 1, w), VR(2 * t, w)))
        out.append("v_perm_b32 v%d, v%d, v%d, %%[sel_hi]" % (VO(w) + t, VR(2 * t + 1, w), VR(2 * t, w)))
    return out


def mask_tile(t):
    """Scores of rows this lane's column may not see become -inf; rs = rows seen - 4 * lane group."""
    out = ["v_mov_b32_e32 v%d, 0xff800000" % T(15)]
    for i in range(8):
        row = i if i < 4 else 16 + (i - 4)
        out += ["v_cmp_lt_i32_e32 vcc, %d, %%[rs%d]" % (row, t), "s_nop 1",
                "v_cndmask_b32_e32 v%d, v%d, v%d, vcc" % (S(t, i), T(15), S(t, i))]
    return out


def max_tile(t, d):
    """Lane maximum of the tile's 8 scores into m; d := m - mref (more than 16: the weights would run away).
    Temporaries 12 and 13."""
    s = [S(t, i) for i in range(8)]
    return ["v_max3_f32 v%d, v%d, v%d, v%d" % (T(12), s[0], s[1], s[2]),
            "v_max3_f32 v%d, v%d, v%d, v%d" % (T(13), s[3], s[4], s[5]),
            "v_max3_f32 v%d, v%d, v%d, v%d" % (T(12), T(12), s[6], s[7]),
            "v_max_f32_e32 v%d, v%d, v%d" % (T(12), T(12), T(13)),
            "v_mul_f32_e32 v%d, %%[c2], v%d" % (T(12), T(12)),
            "v_max_f32_e32 v%d, v%d, v%d" % (M(t), M(t), T(12)),
            "v_sub_f32_e32 v%d, v%d, v%d" % (d, M(t), MREF(t))]


def weights_head(t, b):
    """exp2(score * c2 - reference) for tile t (temporaries 0..7) and its bf16 high parts (weight buffer b)."""
    out = []
    for i in range(8):
        out.append("v_fma_f32 v%d, v%d, %%[c2], v%d" % (T(i), S(t, i), NMU(t)))
    for i in range(8):
        out.append("v_exp_f32_e32 v%d, v%d" % (T(i), T(i)))
    for k in range(4):
        out.append("v_cvt_pk_bf16_f32 v%d, v%d, v%d" % (PH(b) + k, T(2 * k), T(2 * k + 1)))
    return out + ["s_nop 1"]   # the tile's products may follow at once: they read a register two slots after its write


def weights_low(b):
    """What the high parts leave of the weights in temporaries 0..7: w - high, with the high parts widened again by
    a shift / a mask (temporaries 8..11), as bf16.  (A bf16 dot product would do it in one instruction per weight,
    but it runs on the matrix pipe and waits for every product in flight.)"""
    out = []
    for k in range(4):
        e, o = T(8 + 2 * (k % 2)), T(9 + 2 * (k % 2))
        out.append("v_lshlrev_b32_e32 v%d, 16, v%d" % (e, PH(b) + k))
        out.append("v_and_b32_e32 v%d, 0xffff0000, v%d" % (o, PH(b) + k))
        out.append("v_sub_f32_e32 v%d, v%d, v%d" % (T(2 * k), T(2 * k), e))
        out.append("v_sub_f32_e32 v%d, v%d, v%d" % (T(2 * k + 1), T(2 * k + 1), o))
    for k in range(4):
        if k == 3:
            out.append(("mark", "low%d" % b))   # travels with the instruction after it: the last one
        out.append("v_cvt_pk_bf16_f32 v%d, v%d, v%d" % (PL(b) + k, T(2 * k), T(2 * k + 1)))
    return out


def pv_mfmas(t, b):
    """O^T += V^T . P^T of tile t and the ones row: the products with the high parts of the weights, then (once the
    low parts are there) those with the low parts.  Returns the products and, per dimension group w, after how many
    of them the group's V^T operands may be overwritten."""
    out = ["%s %s, %s, %s, %s" % (MFMA, a4(ESUM(t)), a4(ONES), v4(PH(b)), a4(ESUM(t)))]
    for w in range(4):
        out.append("%s %s, %s, %s, %s" % (MFMA, a4(ACC(t, 2 * w)), v4(VE(w)), v4(PH(b)), a4(ACC(t, 2 * w))))
        out.append("%s %s, %s, %s, %s" % (MFMA, a4(ACC(t, 2 * w + 1)), v4(VO(w)), v4(PH(b)), a4(ACC(t, 2 * w + 1))))
    out.append(("wait", "low%d" % b))
    out.append("%s %s, %s, %s, %s" % (MFMA, a4(ESUM(t)), a4(ONES), v4(PL(b)), a4(ESUM(t))))
    free_after = {}
    for w in range(4):
        out.append("%s %s, %s, %s, %s" % (MFMA, a4(ACC(t, 2 * w)), v4(VE(w)), v4(PL(b)), a4(ACC(t, 2 * w))))
        out.append("%s %s, %s, %s, %s" % (MFMA, a4(ACC(t, 2 * w + 1)), v4(VO(w)), v4(PL(b)), a4(ACC(t, 2 * w + 1))))
        free_after[w] = 10 + 2 * (w + 1)   # products issued by then
    return out, free_after


def rescale_tile(t, label):
    """The column maximum over its four lanes; when it has left the reference by more than 16, the reference
    moves up to it and the sums and accumulators of the tile are rescaled.  Temporaries 0..14."""
    out = ["ds_bpermute_b32 v%d, %%[bp16], v%d" % (T(0), M(t)), "s_waitcnt lgkmcnt(0)",
           "v_max_f32_e32 v%d, v%d, v%d" % (T(0), T(0), M(t)),
           "ds_bpermute_b32 v%d, %%[bp32], v%d" % (T(1), T(0)), "s_waitcnt lgkmcnt(0)",
           "v_max_f32_e32 v%d, v%d, v%d" % (T(0), T(0), T(1)),
           "v_sub_f32_e32 v%d, v%d, v%d" % (T(1), T(0), MREF(t)),
           "v_sub_f32_e32 v%d, v%d, v%d" % (T(2), MREF(t), T(0)),
           "v_exp_f32_e32 v%d, v%d" % (T(2), T(2)),
           "v_cmp_lt_f32_e32 vcc, 0x41800000, v%d" % T(1),
           "s_nop 1",
           "v_cndmask_b32_e32 v%d, 1.0, v%d, vcc" % (T(2), T(2)),
           "v_cndmask_b32_e32 v%d, v%d, v%d, vcc" % (MREF(t), MREF(t), T(0)),
           "s_mov_b64 s[100:101], vcc",
           "s_nop 1",
           "v_cmp_neq_f32_e32 vcc, 0xff800000, v%d" % MREF(t),
           "s_nop 1",
           "v_cndmask_b32_e64 v%d, 0, -v%d, vcc" % (NMU(t), MREF(t)),
           "s_mov_b64 vcc, s[100:101]",
           "s_cbranch_vccz %sf" % label]
    regs = [ACC(t, n) + i for n in range(8) for i in range(4)] + [ESUM(t) + i for i in range(4)]
    for g in range(0, len(regs), 12):
        grp = regs[g:g + 12]
        out += ["v_accvgpr_read_b32 v%d, a%d" % (T(3 + k), r) for k, r in enumerate(grp)]
        out += ["v_mul_f32_e32 v%d, v%d, v%d" % (T(3 + k), T(2), T(3 + k)) for k in range(len(grp))]
        out += ["v_accvgpr_write_b32 a%d, v%d" % (r, T(3 + k)) for k, r in enumerate(grp)]
    out.append("%s:" % label)
    return out


# ---------------------------------------------------------------------------------------------- streams

# Issue cost of an instruction in cycles, measured on one wavefront per SIMD: a vector instruction 4.55 (exp2 8.1),
# a scalar one 4.05; a matrix product occupies its pipe for 16 and the issue for 6.6 of them, so that what is issued
# beside it is free up to about 9.4 cycles per product and delays the next product beyond that.
SHADOW, OVERDRAFT = 9.4, 1.0


def issue_cost(x):
    if isinstance(x, tuple) and x[0] == "load":
        return 8.0
    if not isinstance(x, str) or x.endswith(":"):
        return 0.0
    op = x.split()[0]
    if op == "s_nop":
        return max(4.05, float(x.split()[1]) + 1.0)
    if op.startswith("v_exp"):
        return 8.1
    if op.startswith("ds_") or op.startswith("global_"):
        return 8.0
    return 4.55 if op.startswith("v_") else 4.05


def units(stream):
    """Markers (tuples) travel with the instruction after them, a label with the instruction before it (a branch
    out of the stream comes back to the label right behind it: nothing may come between the two)."""
    def instr(y):   # a load is an instruction that resolve_waits still has to see
        return (isinstance(y, str) and not y.endswith(":")) or (isinstance(y, tuple) and y[0] == "load")
    out, cur = [], []
    for n, x in enumerate(stream):
        cur.append(x)
        label_next = n + 1 < len(stream) and isinstance(stream[n + 1], str) and stream[n + 1].endswith(":")
        if (instr(x) or (isinstance(x, str) and x.endswith(":"))) and not label_next and any(instr(y) for y in cur):
            out.append(cur)
            cur = []
    if cur:
        out.append(cur)
    return out


def interleave(major, minor):
    """The minor stream in the shadow of the major stream's matrix products: after each product as many of its
    instructions as the product's 16 cycles leave room for; what is left of either stream follows.
    ("mark", x) in the minor stream and ("wait", x) in the major one: the major stream goes on past the wait only
    when the minor one has passed the mark (and two more issue slots: a matrix product may read a register two
    slots after a vector instruction wrote it).  ("after", n) in the minor stream: not before n products of the
    major stream are out."""
    a, b = units(major), units(minor)
    out, k, products, passed, since = [], 0, 0, set(), 99

    def emit_minor():
        nonlocal k, since
        for x in b[k]:
            if isinstance(x, tuple) and x[0] == "mark":
                passed.add(x[1])
                since = -1   # the marked instruction comes next
            elif not (isinstance(x, tuple) and x[0] == "after"):
                out.append(x)
                if (isinstance(x, str) and not x.endswith(":")) or (isinstance(x, tuple) and x[0] == "load"):
                    since += 1
        k += 1

    def blocked():
        return any(isinstance(x, tuple) and x[0] == "after" and products < x[1] for x in b[k])

    for u in a:
        for x in u:
            if isinstance(x, tuple) and x[0] == "wait":
                while x[1] not in passed:
                    assert k < len(b) and not blocked(), x
                    emit_minor()
                if since < 2:
                    out.append("s_nop %d" % (1 - since))   # 2 - since issue slots
                    since = 2
            else:
                out.append(x)
                if isinstance(x, str) and not x.endswith(":"):
                    since += 1
        if not any(isinstance(x, str) and x.startswith("v_mfma") for x in u):
            continue
        products += 1
        room = SHADOW
        while k < len(b) and not blocked():
            c = sum(issue_cost(x) for x in b[k])
            if c > room + OVERDRAFT:
                break
            emit_minor()
            room -= c
    while k < len(b):
        emit_minor()
    return out


def resolve_waits(stream, old_queue):
    """Turns need / load markers into s_waitcnt vmcnt(n).  Vector loads return in order; when the stream starts, the
    loads named in old_queue (oldest first) may all be outstanding.  A need means the newest load of that name (none
    if it is not among those that may be outstanding); needs that follow one another become one wait."""
    queue = list(old_queue)
    done = 0                  # this many from the front are known to have returned
    want = 0                  # ... and this many must have before the next instruction
    out = []
    for x in stream:
        if isinstance(x, tuple) and x[0] == "need":
            if x[1] in queue:   # otherwise it has come back long ago
                want = max(want, len(queue) - queue[::-1].index(x[1]))
            continue
        if want > done:
            assert len(queue) - want <= 63
            out.append("s_waitcnt vmcnt(%d)" % (len(queue) - want))
            done = want
        if isinstance(x, str):
            out.append(x)
        else:
            out.append(x[2])
            queue.append(x[1])
    assert want <= done
    return out, queue[done:]


def offsets_prologue():
    """Offsets for the chunk about to be requested: the full-chunk ones, clamped in place when it is not full."""
    return ["s_cmp_eq_u32 %[full], 0", "s_cbranch_scc1 20f", "21:"]


def offsets_epilogue():
    return ["s_cmp_eq_u32 %[full], 0", "s_cbranch_scc1 22f", "23:"]


def offsets_out_of_line():
    return ["20:"] + clamp_offsets() + ["s_branch 21b", "22:"] + set_offsets() + ["s_branch 23b"]


def still_out(queue):
    """What a statement leaves outstanding must be what the next one assumes: K loads only, the newest ones."""
    assert queue == OLD_K[len(OLD_K) - len(queue):], queue
    return True


def request_body(nt):
    """All 16 loads of a chunk and the first half of its V^T operands (the second half of those before them first,
    as every statement does)."""
    s = perms_of_group(2) + perms_of_group(3)
    s += [v_load(j, nt) for j in range(8)] + [k_load(j, nt) for j in K_ORDER]
    s += perms_of_group(0) + perms_of_group(1)
    ins, left = resolve_waits(s, OLD_K)
    assert still_out(left)
    return offsets_prologue() + ins + offsets_epilogue() + ["s_branch 29f"] + offsets_out_of_line() + ["29:"]


RUN_KB, RUN_VB, RUN_N = "s[96:97]", "s[98:99]", "s95"  # scalar registers of a run statement: row pointers, chunks left


def body(tiles, masked, nt, run=False):
    """One chunk; with run, a loop over chunks whose successors are all full and lie `step` bytes apart.

    Matrix products and vector instructions share the issue: a product needs 6.6 cycles of it and 16 of its pipe, so
    every product should have two vector instructions (one exp2) behind it.  The products of a chunk come in the
    order K.Q^T of tile 0, K.Q^T of the other tiles, then per tile V^T.P^T with the high parts of the weights and
    V^T.P^T with their low parts; behind them run, in this order: the V^T operands of dimension groups 2 and 3
    (left over from the statement before), the requests for the next V rows, maximum / rescale / weights of tile 0,
    and per tile t: low parts of tile t's weights, (t = 0: maxima and rescale of all other tiles,) weights of tile
    t + 1; behind the last tile's products the V^T operands of groups 0 and 1 of the next chunk."""
    ins = ["60:"] if run else offsets_prologue()
    # ---- K.Q^T: tile 0, then the other tiles K register by K register (each asked for again after its last product)
    major = []
    for j in K_ORDER:
        major += [("need", "K%d" % j), qk(0, j)]
    for j in K_ORDER:
        major += [qk(t, j) for t in range(1, tiles)] + [k_load(j, nt)]
    minor = perms_of_group(2) + perms_of_group(3)
    minor += [v_load(j, nt) for j in range(8)]
    minor += [("after", 10)]   # tile 0's last scores are written when two more products have gone out
    if masked:
        minor += mask_tile(0)
    minor += max_tile(0, T(14))
    minor += ["v_cmp_lt_f32_e32 vcc, 0x41800000, v%d" % T(14), "s_cbranch_vccnz 30f", "31:"]
    minor += weights_head(0, 0)
    first, queue = resolve_waits(interleave(major, minor), OLD_K)
    ins += first
    if run:   # all requests of the iteration are out: on to the rows of the next one
        assert not masked
        for pair in (RUN_KB, RUN_VB):
            lo, hi = pair[2:pair.index(":")], pair[pair.index(":") + 1:-1]
            ins += ["s_add_u32 s%s, s%s, %%[step]" % (lo, lo), "s_addc_u32 s%s, s%s, 0" % (hi, hi)]
    else:
        ins += offsets_epilogue()
    # ---- tile after tile: V^T.P^T; behind it the low parts of its own weights, then what the next tile needs ------
    for t in range(tiles):
        pv, free_after = pv_mfmas(t, t % 2)
        side = weights_low(t % 2)
        if t == 0:
            side += [("after", 2)]   # the last scores of the other tiles are written
            for u in range(1, tiles):
                if masked:
                    side += mask_tile(u)
                side += max_tile(u, T(14) if u == 1 else T(12))
                if u > 1:
                    side += ["v_max_f32_e32 v%d, v%d, v%d" % (T(14), T(14), T(12))]
            side += ["v_cmp_lt_f32_e32 vcc, 0x41800000, v%d" % T(14), "s_cbranch_vccnz 32f", "33:"]
        if t + 1 < tiles:
            side += weights_head(t + 1, (t + 1) % 2)
            ins += interleave(pv, side)
        else:
            # the last tile's products free the V^T operands group by group; the next chunk's are built behind them
            for w in range(2):
                side += [("after", free_after[w])] + perms_of_group(w)
            last, queue = resolve_waits(interleave(pv, side), queue)
            ins += last
    # what is rare lies behind the stream (a taken branch costs about 70 cycles: a loop has one per iteration)
    rare = ["30:"] + rescale_tile(0, "34") + ["s_branch 31b", "32:"]
    for u in range(1, tiles):
        rare += rescale_tile(u, "3%d" % (4 + u))
    rare += ["s_branch 33b"]
    if run:
        ins += ["s_sub_u32 %s, %s, 1" % (RUN_N, RUN_N), "s_cmp_lg_u32 %s, 0" % RUN_N, "s_cbranch_scc1 60b", "s_branch 39f"]
        ins += rare + ["39:"]
        ins = [i.replace("%[kbase]", RUN_KB).replace("%[vbase]", RUN_VB) for i in ins]
        ins = ["s_mov_b64 %s, %%[kbase]" % RUN_KB, "s_mov_b64 %s, %%[vbase]" % RUN_VB, "s_mov_b32 %s, %%[n]" % RUN_N] + ins
    else:
        ins += ["s_branch 39f"] + rare + offsets_out_of_line() + ["39:"]
    assert still_out(queue)
    return ins


def check(ins):
    """Every marker resolved, every label defined once, every branch pointing the way it says."""
    labels = [i[:-1] for i in ins if i.endswith(":")]
    assert len(labels) == len(set(labels)), labels
    for n, i in enumerate(ins):
        assert isinstance(i, str), i
        if i.startswith("s_cbranch") or i.startswith("s_branch"):
            tgt = i.split()[-1]
            assert tgt[:-1] in labels, i
            pos = ins.index(tgt[:-1] + ":")
            assert (tgt[-1] == "f") == (pos > n), i
            # a branch out of the stream comes back to the label right behind it
            if i.split()[-1] in ("30f", "32f", "20f", "22f"):
                assert ins[n + 1].endswith(":"), (i, ins[n + 1])
    return ins


def c_string(ins):
    return "\n".join('        "%s\\n"' % i for i in ins)


LOAD_OPS = ('[vbase] "s"(nl.vb), [kbase] "s"(nl.kb), [last] "s"(nl.last), [full] "s"(nl.full), [rb] "s"(lc.rb), '
            '[vlane] "v"(lc.vlane), [klane] "v"(lc.klane), [ln16] "v"(lc.ln16), [lg16] "v"(lc.lg16), '
            '[sel_lo] "s"(sel_lo), [sel_hi] "s"(sel_hi)')


def emit():
    h = []
    h.append("// Generated by gen_tiles_asm.py (same directory); do not edit by hand.  Instruction streams of the multi-tile")
    h.append("// matrix-core MicroAttention kernel over a fixed register map, which the generator's header describes.")
    h.append("#pragma once")
    h.append("#include <hip/hip_runtime.h>")
    h.append("#include <stdint.h>")
    h.append("")
    h.append("namespace da {")
    h.append("namespace tiles_asm {")
    h.append("")
    h.append("// vector registers from this one up, and the whole accumulation file, belong to the statements below")
    h.append("constexpr int kFirstOwnVgpr = %d;" % CAP)
    h.append("")
    h.append("// what a statement needs to request a chunk's V and K rows (all wavefront-uniform) ...")
    h.append("struct NextLoads {")
    h.append("    const char *vb, *kb;   // first row of the chunk in the V / K pool")
    h.append("    uint32_t last;         // byte offset of the chunk's last valid row (rows past it re-read it)")
    h.append("    uint32_t full;         // 1: all 32 rows are valid")
    h.append("};")
    h.append("// ... and what never changes: K: the lane reads rows ln and 16 + ln, bytes [64 s + 16 g, +16) of k-step s;")
    h.append("// V: rows 16 * (j / 4) + 4 g + j % 4 for its load j, bytes [16 ln, +16)  (g = lane / 16, ln = lane % 16)")
    h.append("struct LaneConstants {")
    h.append("    uint32_t rb;           // bytes from one token row to the next (wavefront-uniform)")
    h.append("    uint32_t vlane, klane; // 4 g * rb + 16 ln;  ln * rb + 16 g")
    h.append("    uint32_t ln16, lg16;   // 16 ln; 16 g")
    h.append("};")
    h.append("")
    h.append("// once per wavefront: bf16 ones, the lane's load offsets; names the highest registers of both files so that the")
    h.append("// kernel is given them")
    h.append("__device__ __forceinline__ void init(const LaneConstants &lc)")
    h.append("{")
    h.append("    asm volatile(")
    h.append(c_string(["v_mov_b32_e32 v255, 0x3f803f80"] + ["v_accvgpr_write_b32 a%d, v255" % (ONES + i) for i in range(4)]
                      + ["v_accvgpr_write_b32 a255, v255"] + set_offsets()))
    h.append('        :: [rb] "s"(lc.rb), [vlane] "v"(lc.vlane), [klane] "v"(lc.klane) : "v255", "a255");')
    h.append("}")
    h.append("")
    for tiles in (2, 4):
        qregs = [QOP(t, s) + i for t in range(tiles) for s in range(4) for i in range(4)]
        # the query rows asked for by load_q are there; a negative scale flips their signs (exact)
        ins = ["s_waitcnt vmcnt(0)", "s_cmp_eq_u32 %[qsign], 0", "s_cbranch_scc1 1f"]
        for r in qregs:
            ins += ["v_accvgpr_read_b32 v%d, a%d" % (T(0), r), "v_xor_b32_e32 v%d, %%[qsign], v%d" % (T(0), T(0)),
                    "v_accvgpr_write_b32 a%d, v%d" % (r, T(0))]
        ins += ["1:"]
        ins += ["v_accvgpr_write_b32 a%d, 0" % r for r in list(range(0, 32 * tiles)) + [ESUM(t) + i for t in range(tiles) for i in range(4)]]
        for t in range(tiles):
            ins += ["v_mov_b32_e32 v%d, 0xff800000" % M(t), "v_mov_b32_e32 v%d, 0xff800000" % MREF(t), "v_mov_b32_e32 v%d, 0" % NMU(t)]
        h.append("// start of an item for %d tiles: its query rows have arrived (qsign = 0x80008000 flips their signs, 0 leaves" % tiles)
        h.append("// them); accumulators and exp-sums := 0, maxima := -inf")
        h.append("__device__ __forceinline__ void begin_item_%d(uint32_t qsign)" % tiles)
        h.append("{")
        h.append("    asm volatile(")
        h.append(c_string(ins))
        h.append('        :: [qsign] "s"(qsign) : "scc", "memory");')
        h.append("}")
        h.append("")
        # query rows straight into the accumulation registers
        ins = ["v_accvgpr_write_b32 a%d, 0" % r for r in qregs]
        ins += ["s_mov_b64 s[100:101], exec"]
        for t in range(tiles):
            ins += ["s_mov_b64 exec, %%[live%d]" % t]
            ins += ["global_load_dwordx4 %s, %%[row%d], off%s" % (a4(QOP(t, s)), t, (" offset:%d" % (64 * s)) if s else "") for s in range(4)]
        ins += ["s_mov_b64 exec, s[100:101]"]
        h.append("// Q^T operands of an item's %d tiles: the lane's column reads bytes [64 s, +16) from `row` on for k-step s (the" % tiles)
        h.append("// lane group's slice is part of the address); lanes outside `live` get zeros.  The loads are waited for by")
        h.append("// begin_item_%d, not here." % tiles)
        rows = ", ".join("const void *row%d" % t for t in range(tiles))
        lives = ", ".join("uint64_t live%d" % t for t in range(tiles))
        h.append("__device__ __forceinline__ void load_q_%d(%s, %s)" % (tiles, rows, lives))
        h.append("{")
        h.append("    asm volatile(")
        h.append(c_string(ins))
        h.append("        :: " + ", ".join('[row%d] "v"(row%d)' % (t, t) for t in range(tiles)) + ", "
                 + ", ".join('[live%d] "s"(live%d)' % (t, t) for t in range(tiles)))
        h.append('        : "s100", "s101", "memory");')
        h.append("}")
        h.append("")
    h.append("// accumulator of tile t, dimension group n (four registers)")
    h.append("template <int t, int n>")
    h.append("__device__ __forceinline__ void read_acc(float &x0, float &x1, float &x2, float &x3)")
    h.append("{")
    first = True
    for t in range(4):
        for n in range(8):
            r = ACC(t, n)
            h.append("    %sif constexpr (t == %d && n == %d)" % ("" if first else "else ", t, n))
            h.append('        asm volatile("v_accvgpr_read_b32 %%0, a%d\\n v_accvgpr_read_b32 %%1, a%d\\n v_accvgpr_read_b32 %%2, a%d\\n v_accvgpr_read_b32 %%3, a%d\\n"'
                     % (r, r + 1, r + 2, r + 3))
            h.append('                     : "=v"(x0), "=v"(x1), "=v"(x2), "=v"(x3));')
            first = False
    h.append("}")
    h.append("")
    h.append("// of tile t: the lane's running maximum, the reference maximum, the column's exp-sum over all tokens so far")
    h.append("// (relative to the reference; the same in the column's four lanes)")
    h.append("template <int t>")
    h.append("__device__ __forceinline__ void read_state(float &m, float &mref, float &esum)")
    h.append("{")
    first = True
    for t in range(4):
        h.append("    %sif constexpr (t == %d)" % ("" if first else "else ", t))
        h.append('        asm volatile("v_mov_b32_e32 %%0, v%d\\n v_mov_b32_e32 %%1, v%d\\n v_accvgpr_read_b32 %%2, a%d\\n" : "=v"(m), "=v"(mref), "=v"(esum));'
                 % (M(t), MREF(t), ESUM(t)))
        first = False
    h.append("}")
    h.append("")
    h.append("// matrix results may be read by other instructions 8 issue slots after the product at the earliest")
    h.append('__device__ __forceinline__ void settle() { asm volatile("s_nop 7\\n s_nop 7" ::: ); }')
    h.append("")
    h.append("// Requests the V and K rows of a chunk and builds its V^T operands: before a wavefront's first chunk, and in place")
    h.append("// of the chunk statement for a chunk slot without valid rows (`nl` then describes the chunk after it).")
    h.append("// NT: non-temporal loads (rows that no other wavefront reads).")
    h.append("template <bool NT>")
    h.append("__device__ __forceinline__ void request_chunk(const NextLoads &nl, const LaneConstants &lc)")
    h.append("{")
    h.append("    const uint32_t sel_lo = 0x05040100u, sel_hi = 0x07060302u;")
    for nt in (True, False):
        h.append("    %sif constexpr (%sNT)" % ("" if nt else "else ", "" if nt else "!"))
        h.append("    asm volatile(")
        h.append(c_string(check(request_body(" nt" if nt else ""))))
        h.append("        :: " + LOAD_OPS)
        h.append('        : "vcc", "scc");')
    h.append("}")
    h.append("")
    for tiles in (2, 4):
        for masked in (False, True):
            name = "chunk_%d%s" % (tiles, "_masked" if masked else "")
            h.append("// One 32-token chunk for %d column tiles%s: scores, maxima, (rarely) the rescale, weights, V^T.P^T; requests"
                     % (tiles, ", some rows masked (rs = rows the lane's column sees - 4 * lane group)" if masked else ""))
            h.append("// the rows of the next chunk (`nl`) and builds its V^T operands.")
            args = "float c2, const NextLoads &nl, const LaneConstants &lc, uint32_t bp16, uint32_t bp32"
            if masked:
                args += ", const int (&rs)[%d]" % tiles
            h.append("template <bool NT>")
            h.append("__device__ __forceinline__ void %s(%s)" % (name, args))
            h.append("{")
            h.append("    const uint32_t sel_lo = 0x05040100u, sel_hi = 0x07060302u;")
            ops = '[c2] "s"(c2), [bp16] "v"(bp16), [bp32] "v"(bp32), ' + LOAD_OPS
            if masked:
                ops += ", " + ', '.join('[rs%d] "v"(rs[%d])' % (t, t) for t in range(tiles))
            for nt in (True, False):
                if tiles == 2 and not nt:
                    h.append("    else static_assert(NT, \"two tiles: non-temporal loads only\");")
                    continue
                h.append("    %sif constexpr (%sNT)" % ("" if nt else "else ", "" if nt else "!"))
                h.append("    asm volatile(")
                h.append(c_string(check(body(tiles, masked, " nt" if nt else ""))))
                h.append("        :: " + ops)
                h.append('        : "vcc", "scc", "s100", "s101");')
            h.append("}")
            h.append("")
    for tiles in (2, 4):
        h.append("// n chunks of 32 tokens one after the other for %d column tiles, none with a masked row; iteration i requests" % tiles)
        h.append("// the rows `nl` + i * step bytes, all of them full chunks (the rows of the chunk after the one it processes).")
        h.append("template <bool NT>")
        h.append("__device__ __forceinline__ void chunk_%d_run(float c2, const NextLoads &nl, const LaneConstants &lc, uint32_t bp16, uint32_t bp32, uint32_t n, uint32_t step)" % tiles)
        h.append("{")
        h.append("    const uint32_t sel_lo = 0x05040100u, sel_hi = 0x07060302u;")
        ops = ('[c2] "s"(c2), [bp16] "v"(bp16), [bp32] "v"(bp32), [n] "s"(n), [step] "s"(step), '
               '[vbase] "s"(nl.vb), [kbase] "s"(nl.kb), [sel_lo] "s"(sel_lo), [sel_hi] "s"(sel_hi)')
        for nt in (True, False):
            if tiles == 2 and not nt:
                h.append("    else static_assert(NT, \"two tiles: non-temporal loads only\");")
                continue
            h.append("    %sif constexpr (%sNT)" % ("" if nt else "else ", "" if nt else "!"))
            h.append("    asm volatile(")
            h.append(c_string(check(body(tiles, False, " nt" if nt else "", run=True))))
            h.append("        :: " + ops)
            h.append('        : "vcc", "scc", "s100", "s101", "s95", "s96", "s97", "s98", "s99");')
        h.append("}")
        h.append("")
    h.append("}  // namespace tiles_asm")
    h.append("}  // namespace da")
    return "\n".join(h) + "\n"


if __name__ == "__main__":
    with open(os.path.join(HERE, "tiles_asm.h"), "w") as f:
        f.write(emit())
