"""Writes tiles_asm.h: the per-chunk instruction streams of the multi-tile matrix-core MicroAttention kernel.

The kernel (micro_attention_mfma_tiles.hip) serves 32 or 64 columns from one K/V read; at that width a chunk's
vector-ALU work decides the speed, and the compiler's register allocation (it shuttles the accumulators between the
two halves of the register file on every chunk) more than doubles it.  The chunk body is therefore written out
instruction by instruction here, with a fixed register map:

  accumulation registers (only the statements below touch them)
    a[0:127]    O^T accumulators, tile t at a[32t:32t+31], dimension group n at +4n
    a[128:191]  Q^T operands, tile t, k-step s at a[128+16t+4s:+3]
    a[192:255]  K rows, two buffers of 32: load j of buffer b at a[192+32b+4j:+3]
  vector registers above the kernel's own allocation limit of 96
    v[96:127]   scores, tile t at v[96+8t:+7] (tokens 4g+i, then 16+4g+i of lane group g)
    v[128:191]  V rows as loaded, two buffers of 32: load j of buffer b at v[128+32b+4j:+3]
    v[192:223]  V^T operands: even dims at v[192+4w:+3], odd dims at v[208+4w:+3]
    v[224:239]  weights of a tile as bf16 pairs, two buffers of (high 4, low 4)
    v[240:255]  temporaries

Chunks alternate between the two K / V buffers along a wavefront's whole chunk stream: the statement for a chunk
in buffer b finds its rows there (requested two chunks ago), and requests the rows of the chunk after the next
into the registers it has just used, so that a request has two chunk periods to return in.

Run `python gen_tiles_asm.py` after changing it; the header it writes is committed beside it.
"""
import os

HERE = os.path.dirname(os.path.abspath(__file__))

MFMA = "v_mfma_f32_16x16x32_bf16"


def a4(i):
    return "a[%d:%d]" % (i, i + 3)


def v4(i):
    return "v[%d:%d]" % (i, i + 3)


def ACC(t, n):
    return 32 * t + 4 * n


def QOP(t, s):
    return 128 + 16 * t + 4 * s


def KOP(b, j):
    return 192 + 32 * b + 4 * j


CAP = 96                                # the kernel's own code is compiled for v[0:95]
S = lambda t, i: 96 + 8 * t + i         # noqa: E731  score i (0..7) of tile t
VR = lambda b, j, w: 128 + 32 * b + 4 * j + w   # noqa: E731  dword w of V load j of buffer b
VE = lambda w: 192 + 4 * w              # noqa: E731
VO = lambda w: 208 + 4 * w              # noqa: E731
PH = lambda b: 224 + 8 * b              # noqa: E731
PL = lambda b: 228 + 8 * b              # noqa: E731
T = lambda i: 240 + i                   # noqa: E731


def interleave(major, minor, per):
    """major[0], `per` of minor, major[1], ... ; what is left of either stream follows."""
    out, k = [], 0
    for ins in major:
        out.append(ins)
        out += minor[k:k + per]
        k += per
    out += minor[k:]
    return out


K_ORDER = (0, 4, 1, 5, 2, 6, 3, 7)  # K loads alternate between the chunk's two 16-row halves


# Byte offsets of a lane's loads inside the chunk being requested, computed in the temporaries during the first
# phase (which has no other use for them): a row past the chunk's last valid one is replaced by that last row.
KOFF = (T(12), T(13))   # the lane's K rows ln and 16 + ln
VCLAMP, KCLAMP = T(14), T(15)


def offsets_preamble():
    return ["v_add_u32_e32 v%d, %%[last], %%[ln16]" % VCLAMP,
            "v_add_u32_e32 v%d, %%[last], %%[lg16]" % KCLAMP,
            "v_min_u32_e32 v%d, %%[klane], v%d" % (KOFF[0], KCLAMP),
            "v_mad_u32_u24 v%d, 16, %%[rb], %%[klane]" % KOFF[1],
            "v_min_u32_e32 v%d, v%d, v%d" % (KOFF[1], KOFF[1], KCLAMP)]


def k_load(b, j):
    off = (" offset:%d" % (64 * (j % 4))) if j % 4 else ""
    return ("load", "K%d" % j, "global_load_dwordx4 %s, v%d, %%[kbase]%s nt" % (a4(KOP(b, j)), KOFF[j // 4], off))


def v_offset(j):
    row = 16 * (j >> 2) + (j & 3)   # lane group g reads tokens 16 * (j / 4) + 4 g + j % 4
    return ["v_mad_u32_u24 v%d, %d, %%[rb], %%[vlane]" % (T(j % 2), row), "v_min_u32_e32 v%d, v%d, v%d" % (T(j % 2), T(j % 2), VCLAMP)]


def v_load(b, j):
    return ("load", "V%d" % j, "global_load_dwordx4 %s, v%d, %%[vbase] nt" % (v4(VR(b, j, 0)), T(j % 2)))


def qk_stream(tiles, b):
    """K . Q^T for all tiles, K register by K register: each is needed just before its first product and requested
    again (for the next chunk) right after its last.  An accumulator comes up again 2 * tiles products later."""
    out = []
    for j in K_ORDER:
        half, s = j // 4, j % 4
        out.append(("need", "K%d" % j))
        for t in range(tiles):
            dst = v4(S(t, 4 * half))
            out.append("%s %s, %s, %s, %s" % (MFMA, dst, a4(KOP(b, j)), a4(QOP(t, s)), "0" if s == 0 else dst))
        out.append(k_load(b, j))
    return out


def perm_stream(b):
    """V^T operands from the V rows, load pair by load pair: a pair is requested again as soon as it has been used."""
    out = []
    for t in range(4):
        out += [("need", "V%d" % (2 * t)), ("need", "V%d" % (2 * t + 1))]
        for w in range(4):
            out.append("v_perm_b32 v%d, v%d, v%d, %%[sel_lo]" % (VE(w) + t, VR(b, 2 * t + 1, w), VR(b, 2 * t, w)))
            out.append("v_perm_b32 v%d, v%d, v%d, %%[sel_hi]" % (VO(w) + t, VR(b, 2 * t + 1, w), VR(b, 2 * t, w)))
        out += v_offset(2 * t) + v_offset(2 * t + 1) + [v_load(b, 2 * t), v_load(b, 2 * t + 1)]
    return out


def merge_streams(major, minor):
    """One instruction of each in turn (markers travel with the instruction after them); leftovers follow."""
    def units(stream):
        out, cur = [], []
        for x in stream:
            cur.append(x)
            if isinstance(x, str):
                out.append(cur)
                cur = []
        if cur:
            out.append(cur)
        return out
    a, b = units(major), units(minor)
    out = []
    for k in range(max(len(a), len(b))):
        if k < len(a):
            out += a[k]
        if k < len(b):
            out += b[k]
    return out


def first_phase(tiles, b):
    return offsets_preamble() + merge_streams(qk_stream(tiles, b), perm_stream(b))


def load_order(tiles):
    return [x[1] for x in first_phase(tiles, 0) if isinstance(x, tuple) and x[0] == "load"]


def resolve_waits(stream, tiles):
    """Turns need / load markers into s_waitcnt vmcnt(n).  Vector loads return in order; when this stream starts, the
    16 loads of this chunk (issued two statements ago, in load_order) and after them the 16 of the next chunk (issued
    by the previous statement) may all be outstanding."""
    order = load_order(tiles)
    done = -1      # loads of the previous statement up to this index are known to have returned
    issued = 0     # loads issued by this statement so far
    out = []
    for x in stream:
        if isinstance(x, str):
            out.append(x)
        elif x[0] == "load":
            out.append(x[2])
            issued += 1
        else:
            pos = order.index(x[1])
            if pos > done:
                out.append("s_waitcnt vmcnt(%d)" % (len(order) - 1 - pos + len(order) + issued))
                done = pos
    return out


def loads(tiles, b):
    """The 16 loads into buffer b alone (and their offsets), in the order the chunk statements issue them."""
    out = offsets_preamble()
    for x in first_phase(tiles, b):
        if isinstance(x, tuple) and x[0] == "load":
            if x[1][0] == "V":
                out += v_offset(int(x[1][1:]))
            out.append(x[2])
    return out


def mask_tile(t):
    """Scores of rows this lane's column may not see become -inf; rs = rows seen - 4 * lane group."""
    out = []
    for i in range(8):
        row = i if i < 4 else 16 + (i - 4)
        out += ["v_cmp_lt_i32_e32 vcc, %d, %%[rs%d]" % (row, t), "s_nop 1",
                "v_cndmask_b32_e32 v%d, v%d, v%d, vcc" % (S(t, i), T(15), S(t, i))]
    return out


def max_tile(t):
    s = [S(t, i) for i in range(8)]
    return ["v_max3_f32 v%d, v%d, v%d, v%d" % (T(0), s[0], s[1], s[2]),
            "v_max3_f32 v%d, v%d, v%d, v%d" % (T(1), s[3], s[4], s[5]),
            "v_max3_f32 v%d, v%d, v%d, v%d" % (T(0), T(0), s[6], s[7]),
            "v_max_f32_e32 v%d, v%d, v%d" % (T(0), T(0), T(1)),
            "v_mul_f32_e32 v%d, %%[c2], v%d" % (T(0), T(0)),
            "v_max_f32_e32 %%[m%d], %%[m%d], v%d" % (t, t, T(0)),
            "v_sub_f32_e32 v%d, %%[m%d], %%[mref%d]" % (T(4 + t), t, t)]


def weights_tile(t, b):
    """exp2(score * c2 - reference), split into bf16 high and low parts, for tile t into weight buffer b."""
    out = []
    for i in range(8):
        out.append("v_fma_f32 v%d, v%d, %%[c2], %%[nmu%d]" % (T(i), S(t, i), t))
    for i in range(8):
        out.append("v_exp_f32_e32 v%d, v%d" % (T(i), T(i)))
    for k in range(4):
        out.append("v_cvt_pk_bf16_f32 v%d, v%d, v%d" % (PH(b) + k, T(2 * k), T(2 * k + 1)))
    for i in range(8):
        out.append("v_add_f32_e32 %%[e%d], %%[e%d], v%d" % (t, t, T(i)))
    # what the high parts leave: w - high, one dot product per weight (high pair . (-1, 0) + w, high pair . (0, -1) + w)
    for k in range(4):
        out.append("v_dot2_f32_bf16 v%d, v%d, %%[neg_lo], v%d" % (T(8 + 2 * k), PH(b) + k, T(2 * k)))
        out.append("v_dot2_f32_bf16 v%d, v%d, %%[neg_hi], v%d" % (T(9 + 2 * k), PH(b) + k, T(2 * k + 1)))
    for k in range(4):
        out.append("v_cvt_pk_bf16_f32 v%d, v%d, v%d" % (PL(b) + k, T(8 + 2 * k), T(9 + 2 * k)))
    return out


def pv_mfmas(t, b):
    out = []
    for p in (PH(b), PL(b)):
        for w in range(4):
            out.append("%s %s, %s, %s, %s" % (MFMA, a4(ACC(t, 2 * w)), v4(VE(w)), v4(p), a4(ACC(t, 2 * w))))
            out.append("%s %s, %s, %s, %s" % (MFMA, a4(ACC(t, 2 * w + 1)), v4(VO(w)), v4(p), a4(ACC(t, 2 * w + 1))))
    return out


def rescale_tile(t, label):
    """The column maximum over its four lanes; when it has left the reference by more than 16, the reference
    moves up to it and the sums and accumulators of the tile are rescaled."""
    out = ["ds_bpermute_b32 v%d, %%[bp16], %%[m%d]" % (T(0), t), "s_waitcnt lgkmcnt(0)",
           "v_max_f32_e32 v%d, v%d, %%[m%d]" % (T(0), T(0), t),
           "ds_bpermute_b32 v%d, %%[bp32], v%d" % (T(1), T(0)), "s_waitcnt lgkmcnt(0)",
           "v_max_f32_e32 v%d, v%d, v%d" % (T(0), T(0), T(1)),
           "v_sub_f32_e32 v%d, v%d, %%[mref%d]" % (T(1), T(0), t),
           "v_sub_f32_e32 v%d, %%[mref%d], v%d" % (T(2), t, T(0)),
           "v_exp_f32_e32 v%d, v%d" % (T(2), T(2)),
           "v_cmp_lt_f32_e32 vcc, 0x41800000, v%d" % T(1),
           "s_nop 1",
           "v_cndmask_b32_e32 v%d, 1.0, v%d, vcc" % (T(2), T(2)),
           "v_cndmask_b32_e32 %%[mref%d], %%[mref%d], v%d, vcc" % (t, t, T(0)),
           "s_mov_b64 s[100:101], vcc",
           "s_nop 1",
           "v_cmp_neq_f32_e32 vcc, 0xff800000, %%[mref%d]" % t,
           "s_nop 1",
           "v_cndmask_b32_e64 %%[nmu%d], 0, -%%[mref%d], vcc" % (t, t),
           "s_mov_b64 vcc, s[100:101]",
           "s_cbranch_vccz %sf" % label]
    out.append("v_mul_f32_e32 %%[e%d], v%d, %%[e%d]" % (t, T(2), t))
    regs = [ACC(t, n) + i for n in range(8) for i in range(4)]
    for g in range(0, len(regs), 12):
        grp = regs[g:g + 12]
        out += ["v_accvgpr_read_b32 v%d, a%d" % (T(3 + k), r) for k, r in enumerate(grp)]
        out += ["v_mul_f32_e32 v%d, v%d, v%d" % (T(3 + k), T(2), T(3 + k)) for k in range(len(grp))]
        out += ["v_accvgpr_write_b32 a%d, v%d" % (r, T(3 + k)) for k, r in enumerate(grp)]
    out.append("%s:" % label)
    return out


def body(tiles, masked, buf):
    ins = resolve_waits(first_phase(tiles, buf), tiles)
    ins += ["s_nop 7"]  # the last scores settle
    if masked:
        ins += ["s_nop 3", "v_mov_b32_e32 v%d, 0xff800000" % T(15)]
        for t in range(tiles):
            ins += mask_tile(t)
    for t in range(tiles):
        ins += max_tile(t)
    d = [T(4 + t) for t in range(tiles)]
    if tiles == 4:
        ins += ["v_max3_f32 v%d, v%d, v%d, v%d" % (T(0), d[0], d[1], d[2]), "v_max_f32_e32 v%d, v%d, v%d" % (T(0), T(0), d[3])]
    else:
        ins += ["v_max_f32_e32 v%d, v%d, v%d" % (T(0), d[0], d[1])]
    ins += ["v_cmp_lt_f32_e32 vcc, 0x41800000, v%d" % T(0), "s_cbranch_vccnz 10f", "11:"]
    ins += weights_tile(0, 0)
    for t in range(tiles):
        nxt = weights_tile(t + 1, (t + 1) % 2) if t + 1 < tiles else []
        ins += interleave(pv_mfmas(t, t % 2), nxt, 3)
    ins += ["s_branch 19f", "10:"]
    for t in range(tiles):
        ins += rescale_tile(t, "1%d" % (2 + t))
    ins += ["s_branch 11b", "19:"]
    return ins


def c_string(ins):
    return "\n".join('        "%s\\n"' % i for i in ins)


def state_ops(tiles):
    return ', '.join('[m%d] "+v"(m[%d]), [mref%d] "+v"(mref[%d]), [nmu%d] "+v"(nmu[%d]), [e%d] "+v"(e[%d])' % (t, t, t, t, t, t, t, t)
                     for t in range(tiles))


LOAD_OPS = ('[vbase] "s"(nl.vb), [kbase] "s"(nl.kb), [last] "s"(nl.last), [rb] "s"(lc.rb), [vlane] "v"(lc.vlane), [klane] "v"(lc.klane), '
            '[ln16] "v"(lc.ln16), [lg16] "v"(lc.lg16)')


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
    h.append("// what a statement needs to request a chunk's V and K rows: wavefront-uniform ...")
    h.append("struct NextLoads {")
    h.append("    const char *vb, *kb;   // first row of the chunk in the V / K pool")
    h.append("    uint32_t last;         // byte offset of the chunk's last valid row (rows past it re-read it)")
    h.append("};")
    h.append("// ... and what never changes: K: the lane reads rows ln and 16 + ln, bytes [64 s + 16 g, +16) of k-step s;")
    h.append("// V: rows 16 * (j / 4) + 4 g + j % 4 for its load j, bytes [16 ln, +16)  (g = lane / 16, ln = lane % 16)")
    h.append("struct LaneConstants {")
    h.append("    uint32_t rb;           // bytes from one token row to the next (wavefront-uniform)")
    h.append("    uint32_t vlane, klane; // 4 g * rb + 16 ln;  ln * rb + 16 g")
    h.append("    uint32_t ln16, lg16;   // 16 ln; 16 g")
    h.append("};")
    h.append("")
    h.append("// names the highest registers of both files so that the kernel is given them")
    h.append("__device__ __forceinline__ void init()")
    h.append("{")
    h.append('    asm volatile("v_mov_b32 v255, 0\\n v_accvgpr_write_b32 a255, v255\\n" ::: "v255", "a255");')
    h.append("}")
    h.append("")
    for tiles in (2, 4):
        regs = list(range(0, 32 * tiles))
        h.append("// accumulators of %d tiles := 0" % tiles)
        h.append("__device__ __forceinline__ void zero_%d()" % tiles)
        h.append("{")
        h.append("    asm volatile(")
        h.append(c_string(["v_accvgpr_write_b32 a%d, 0" % r for r in regs]))
        h.append("        ::: );")
        h.append("}")
        h.append("")
    h.append("// Q^T operand of tile t, k-step s (four registers)")
    h.append("template <int t, int s>")
    h.append("__device__ __forceinline__ void set_q(uint32_t x0, uint32_t x1, uint32_t x2, uint32_t x3)")
    h.append("{")
    first = True
    for t in range(4):
        for s in range(4):
            q = QOP(t, s)
            h.append("    %sif constexpr (t == %d && s == %d)" % ("" if first else "else ", t, s))
            h.append('        asm volatile("v_accvgpr_write_b32 a%d, %%0\\n v_accvgpr_write_b32 a%d, %%1\\n v_accvgpr_write_b32 a%d, %%2\\n v_accvgpr_write_b32 a%d, %%3\\n"'
                     % (q, q + 1, q + 2, q + 3))
            h.append('                     "s_nop 1\\n" :: "v"(x0), "v"(x1), "v"(x2), "v"(x3));')
            first = False
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
    h.append("// matrix results may be read by other instructions 8 issue slots after the product at the earliest")
    h.append('__device__ __forceinline__ void settle() { asm volatile("s_nop 7\\n s_nop 7" ::: ); }')
    h.append("")
    for tiles in (2, 4):
        h.append("// requests the V and K rows of a chunk into buffer `buf` (the first two chunks of a wavefront, or when a")
        h.append("// chunk slot is skipped), in the order the chunk statements for %d tiles request them" % tiles)
        h.append("template <int buf>")
        h.append("__device__ __forceinline__ void issue_loads_%d(const NextLoads &nl, const LaneConstants &lc)" % tiles)
        h.append("{")
        for b in (0, 1):
            h.append("    %sif constexpr (buf == %d)" % ("" if b == 0 else "else ", b))
            h.append("    asm volatile(")
            h.append(c_string(loads(tiles, b)))
            h.append("        :: " + LOAD_OPS + ");")
        h.append("}")
        h.append("")
    for tiles in (2, 4):
        for masked in (False, True):
            name = "chunk_%d%s" % (tiles, "_masked" if masked else "")
            h.append("// One 32-token chunk (its rows in buffer `buf`) for %d column tiles%s: scores, maxima, (rarely) the rescale,"
                     % (tiles, ", some rows masked" if masked else ""))
            h.append("// weights, V^T.P^T; requests the rows of the chunk after the next into `buf`.  m: lane's running maximum; mref:")
            h.append("// reference maximum; nmu: -mref, or 0 while mref = -inf; e: lane's exp-sum.")
            args = ("float (&m)[%d], float (&mref)[%d], float (&nmu)[%d], float (&e)[%d], float c2, const NextLoads &nl, const LaneConstants &lc, uint32_t bp16, uint32_t bp32"
                    % (tiles, tiles, tiles, tiles))
            if masked:
                args += ", const int (&rs)[%d]" % tiles
            h.append("template <int buf>")
            h.append("__device__ __forceinline__ void %s(%s)" % (name, args))
            h.append("{")
            h.append("    const uint32_t sel_lo = 0x05040100u, sel_hi = 0x07060302u;")
            h.append("    const uint32_t neg_lo = 0x0000bf80u, neg_hi = 0xbf800000u;  // bf16 pairs (-1, 0) and (0, -1)")
            ops = '[c2] "s"(c2), [sel_lo] "s"(sel_lo), [sel_hi] "s"(sel_hi), [neg_lo] "s"(neg_lo), [neg_hi] "s"(neg_hi), [bp16] "v"(bp16), [bp32] "v"(bp32), ' + LOAD_OPS
            if masked:
                ops += ", " + ', '.join('[rs%d] "v"(rs[%d])' % (t, t) for t in range(tiles))
            for b in (0, 1):
                h.append("    %sif constexpr (buf == %d)" % ("" if b == 0 else "else ", b))
                h.append("    asm volatile(")
                h.append(c_string(body(tiles, masked, b)))
                h.append("        : " + state_ops(tiles))
                h.append("        : " + ops)
                h.append('        : "vcc", "scc", "s100", "s101");')
            h.append("}")
            h.append("")
    h.append("}  // namespace tiles_asm")
    h.append("}  // namespace da")
    return "\n".join(h) + "\n"


if __name__ == "__main__":
    with open(os.path.join(HERE, "tiles_asm.h"), "w") as f:
        f.write(emit())
