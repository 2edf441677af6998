// MicroAttention on the matrix cores, for q / K / V in one 16-bit type (bf16 or IEEE half), any group size
// (Section 4, m_j / e_j equation and Eq. 2; Section 3: the q-heads of a GQA group share one K/V read).
//
// A work item is a run of tokens of one (request, kv-head) and a tile of up to 16 q-heads of its
// group.  The launch is persistent: each workgroup (4 wavefronts) walks its items one after the
// other, and the first K chunk and the query of the next item are requested before the current
// item's partial result is merged and written, so the memory pipe never drains between items.
// Each wavefront walks 32-token chunks on its own:
//
//   S  = K  . Q^T   v_mfma_f32_16x16x32_bf16 / _f16, A = 16 token rows of K (16 B of a row per lane, loaded
//                   straight from HBM in operand layout), B = Q^T (head = lane % 16).  bf16 x bf16
//                   products are exact and summed in fp32.
//   P  = exp2(S * scale*log2e - m), running m / e per head (head = lane % 16 in every step).
//   O^T += V^T . P^T  A = V^T: a lane loads the same 16-byte column slice of 8 token rows (so a load
//                   instruction fetches whole 256-byte rows) and interleaves them in registers with
//                   v_perm_b32; B = P^T, which is exactly how the lane already holds P.  P is split
//                   into bf16 high + low parts (two MFMAs) so that it keeps 16 bits of mantissa.
//
// The columns of a work item are (query token, q-head) pairs of the kv-head's group: q-heads for
// plain decode, query tokens x q-heads in the multi-query form, where each column also has its own
// causal limit.  A work item serves TILES (1, 2 or 4) tiles of 16 columns from one K/V read (bf16 with more than
// one tile has a kernel of its own, micro_attention_mfma_tiles.hip; here more than one tile is IEEE half).  Columns
// past the group carry q = 0 and are never written.
#include <hip/hip_runtime.h>

#include "../../include/distattn.h"
#include "item_walk.h"
#include "kernel_params.h"
#include "mfma_16bit.h"

namespace da {
namespace {

using namespace mfma16bit;

// Result rows of a wavefront that owns whole items, held back in shared memory and written out kStageRows at a
// time (and at the end of the wavefront's items).  On this GPU a store that reaches memory in the middle of the read
// stream costs the reads around it far more than its bytes: one output row per (request, q-head) written as
// it is produced took 14 % off the read rate for 512-token requests, the same rows written in a few large
// bursts a third of that, and rows written after the last read next to nothing.
constexpr int kStageRows = 70;               // rows per wavefront: 4 x 70 x (528 + 32) bytes = 153 KB of the CU's 160 KB
constexpr int kStagePitch = kHeadDim + 4;    // floats per staged row; the pad spreads 16 rows over all banks
struct OutStage {
    float o[kStageRows][kStagePitch];
    float *o_dst[kStageRows];                // where the row goes (out or part_o)
    float *s_dst[kStageRows][2];             // where its two scalars go: (lse, -) or (part_m, part_e); may be null
    float s[kStageRows][2];
};

// Writes the first `count` staged rows of a wavefront to memory: two 512-byte rows per store instruction.
__device__ __forceinline__ void flush_stage(OutStage &st, int count, int lane)
{
    // rows were staged by other lanes of this wavefront: keep the compiler from moving the reads above those writes
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    for (int r0 = 0; r0 < count; r0 += 2) {
        const int r = r0 + (lane >> 5);
        if (r < count) {
            const float4 v = *(const float4 *)&st.o[r][4 * (lane & 31)];
            *(float4 *)(st.o_dst[r] + 4 * (lane & 31)) = v;
        }
    }
    for (int r = lane; r < count; r += 64) {
#pragma unroll
        for (int k = 0; k < 2; ++k)
            if (st.s_dst[r][k]) *st.s_dst[r][k] = st.s[r][k];
    }
}

// WAVE_ITEMS: for runs of many short splits.  Each wavefront then takes whole splits of the run (wavefront w the
// splits w, w + 4, ...) instead of a quarter of every split's chunks: no merge across wavefronts, no barriers, the
// result goes from registers to memory.
template <int TILES, bool F16, bool WAVE_ITEMS>
__global__ __launch_bounds__(kWaves * 64) void micro_attention_mfma_kernel(const MicroParams p)
{
    constexpr int COLS = kHeadTile * TILES;  // columns per work item
    constexpr int W = WAVE_ITEMS ? 1 : kWaves;  // wavefronts that share an item's chunks
    // Shared memory.  Wavefronts that share items: cross-wavefront merge buffers (one barrier after they are
    // written, one after they are read).  Wavefronts that own items: each wavefront's result rows wait here and
    // go to memory many at a time (see OutStage).
    constexpr size_t kLdsBytes = WAVE_ITEMS ? sizeof(OutStage) * kWaves : sizeof(MergeBuffers<COLS>);
    __shared__ __align__(16) char lds_raw[kLdsBytes];
    MergeBuffers<COLS> &mb = *(MergeBuffers<COLS> *)lds_raw;
    float (&lds_m)[kWaves][COLS] = mb.m;
    float (&lds_e)[kWaves][COLS] = mb.e;
    float (&lds_o)[kWaves][COLS][kHeadDim] = mb.o;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int lg = lane >> 4;   // lane group: k-slice of the MFMA operands
    const int ln = lane & 15;   // token row (K operand) / head (Q, P operands, results)

    const char *kbase = (const char *)p.k_pool;
    const char *vbase = (const char *)p.v_pool;
    const uint32_t row_bytes = (uint32_t)p.stride_token * 2u;
    // K: lane reads token (16*mb + ln), bytes [64*ks + 16*lg, +16) of the row
    const uint32_t k_lane_off = (uint32_t)ln * row_bytes + lg * 16;
    // V: lane reads token (16*(jj/4) + 4*lg + jj%4), bytes [16*ln, +16) of the row
    const uint32_t v_lane_off = (uint32_t)(4 * lg) * row_bytes + ln * 16;
    // scores come out of the matrix cores unscaled; |scale| * log2(e) is applied inside the exponent's fused
    // multiply-add (never 0, so that a masked -inf stays -inf) and a negative scale by flipping the sign bits of
    // the query as it is loaded, which is exact
    const float c2 = fmaxf(fabsf(p.scale_log2e), 1.17549435e-38f);
    const uint32_t q_sign = p.scale_log2e < 0.0f ? 0x80008000u : 0u;

    // Every step issues 8 K loads and 8 V loads whatever the chunk: rows past the valid ones re-read
    // the last valid row (their scores are masked), so the loads need no branches.
    const uint32_t k_full[2] = {k_lane_off, k_lane_off + 16u * row_bytes};
    uint32_t v_full[8];
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) v_full[jj] = v_lane_off + (uint32_t)(16 * (jj >> 2) + (jj & 3)) * row_bytes;
    auto load_k = [&](const Fetch &f, u32x4 (&dst)[8]) {
        const char *base = kbase + f.off * 2;
        const uint32_t clamp_off = (uint32_t)f.last * row_bytes + lg * 16;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
            const uint32_t off = k_full[mb] < clamp_off ? k_full[mb] : clamp_off;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) dst[mb * 4 + ks] = load16_stream(base + off + ks * 64);
        }
    };
    auto load_v = [&](const Fetch &f, u32x4 (&dst)[8]) {
        const char *base = vbase + f.off * 2;
        const uint32_t clamp_off = (uint32_t)f.last * row_bytes + ln * 16;
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            const uint32_t off = v_full[jj] < clamp_off ? v_full[jj] : clamp_off;
            dst[jj] = load16_stream(base + off);
        }
    };
    // Q^T operand of an item: column (query token, q-head) = ln, k-slice lg of each of the 4 k-steps
    // (zero for columns past the group); also the number of tokens that column may see (causal limit)
    auto load_q = [&](const ItemInfo &it, u32x4 (&dst)[TILES][4], int (&visible)[TILES]) {
#pragma unroll
        for (int tl = 0; tl < TILES; ++tl) {
            const Column col = column_of(p, it.ht * COLS + tl * kHeadTile + ln, it.kvh, it.L);
            const bool live = it.valid && col.live;
            // columns past the group carry q = 0 and are never written: they take no part in the masking decision
            visible[tl] = col.live ? col.visible : (1 << 30);
            const uint16_t *q = (const uint16_t *)p.q + ((int64_t)it.r * p.q_len * p.Hq + col.vh) * kHeadDim;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                dst[tl][ks] = u32x4{0u, 0u, 0u, 0u};
                if (live) dst[tl][ks] = *(const u32x4 *)(q + ks * 32 + lg * 8) ^ q_sign;
            }
        }
    };

    // this workgroup's run of splits and its (kv-head, head tile)
    const int run = blockIdx.x / p.per_split;
    const int combo = blockIdx.x - run * p.per_split;
    const int kvh = combo / p.head_tiles;
    const int ht = combo - kvh * p.head_tiles;
    int e_begin, e_end;
    run_bounds(p, run, e_begin, e_end);
    int round = 0;
    int staged = 0;  // result rows this wavefront holds in shared memory (wavefronts that own items)
    const int e_first = WAVE_ITEMS ? e_begin + wave : e_begin;  // this wavefront's first split and its stride
    constexpr int e_step = WAVE_ITEMS ? kWaves : 1;
    const int cw = WAVE_ITEMS ? 0 : wave;                       // which of an item's chunk slots are this wavefront's
    ItemInfo it = decode_item<kChunk>(p, e_first, e_end, kvh, ht);
    Chunk cur = first_chunk<kChunk>(p, it, cw, lane);
    u32x4 kr[8], vr[8], qreg[TILES][4];
    int visible[TILES], visible_next[TILES];  // causal limits of this lane's columns, for the current / next item
    load_k(fetch_of(cur), kr);
    load_q(it, qreg, visible);

    while (it.valid) {
        float m[TILES];      // running maximum of column ln's scores, base-2 units (half: all lane groups agree;
                             // bf16: this lane's own tokens only, joined across the lane groups at the end)
        float mref[TILES];   // bf16: the maximum the weights and sums are currently taken against (all lane groups agree)
        float e[TILES];      // this lane's share of the exp-sum (its 8 tokens per chunk)
        f32x4 acc[TILES][8]; // O^T: acc[tl][n][i] = O[column ln of tile tl][dim 32*lg + 8*i + n]
#pragma unroll
        for (int tl = 0; tl < TILES; ++tl) {
            m[tl] = kNegInf;
            mref[tl] = kNegInf;
            e[tl] = 0.0f;
#pragma unroll
            for (int n = 0; n < 8; ++n) acc[tl][n] = f32x4{0.f, 0.f, 0.f, 0.f};
        }

        // the item after this one is looked up early, so that its first K chunk can be requested
        // before this item's result is merged
        ++round;
        const ItemInfo nit = decode_item<kChunk>(p, e_first + round * e_step, e_end, kvh, ht);
        const Chunk ncur = first_chunk<kChunk>(p, nit, cw, lane);

        // every step issues 8 V loads and 8 K loads; kr always holds the K rows of `cur`
        const bool idle = !cur.valid;  // this wavefront has no chunk in the item
        while (cur.valid) {
            load_v(fetch_of(cur), vr);
            const Chunk nxt = next_chunk<kChunk, W>(p, it, cur, lane);
            const Fetch kf_next = fetch_of(nxt.valid ? nxt : ncur);  // nothing left at all: row 0 of the pool

            // S[token 16*mb + 4*lg + i][column ln] for mb = 0, 1 and every column tile
            f32x4 s0[TILES], s1[TILES];
#pragma unroll
            for (int tl = 0; tl < TILES; ++tl) {
                s0[tl] = f32x4{0.f, 0.f, 0.f, 0.f};
                s1[tl] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
                for (int tl = 0; tl < TILES; ++tl) {
                    s0[tl] = mfma16<F16>(kr[ks], qreg[tl][ks], s0[tl]);
                    s1[tl] = mfma16<F16>(kr[4 + ks], qreg[tl][ks], s1[tl]);
                }
            }
            load_k(kf_next, kr);
            if (cur.lim <= 0) {  // a chunk slot without valid tokens contributes nothing
                cur = nxt;
                continue;
            }

            u32x4 ph[TILES], pl[TILES];  // P^T operands: 8 tokens of this lane group, column ln; high and low 16-bit parts
            u32x4 ve[4], vo[4];          // V^T operands of the chunk
            float beta[TILES];           // half only: what the chunk's product is multiplied by when it joins acc
#pragma unroll
            for (int tl = 0; tl < TILES; ++tl) {
                // raw scores of this lane's 8 tokens; rows past the valid or visible tokens masked out.  A chunk
                // that every column of the tile sees in full (all but the last of a request) skips the masking.
                float s[8];
                const int rows_seen = min(cur.lim, visible[tl] - cur.tok0);
                if (__builtin_amdgcn_ballot_w64(rows_seen < kChunk) == 0) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        s[i] = s0[tl][i];
                        s[4 + i] = s1[tl][i];
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        s[i] = (4 * lg + i < rows_seen) ? s0[tl][i] : kNegInf;
                        s[4 + i] = (16 + 4 * lg + i < rows_seen) ? s1[tl][i] : kNegInf;
                    }
                }
                float cm = s[0];
#pragma unroll
                for (int i = 1; i < 8; ++i) cm = fmaxf(cm, s[i]);
                float sum = 0.0f;
                if constexpr (F16) {
                    cm = fmaxf(cm, __shfl_xor(cm, 16));
                    cm = fmaxf(cm, __shfl_xor(cm, 32));
                    cm *= c2;  // base-2 units from here on
                    const float mn = fmaxf(m[tl], cm);
                    // Half has a narrow exponent: weights are taken against the chunk's own maximum, so the largest
                    // is 1, and the chunk's product is rescaled by beta when it joins acc.
                    const float mu = (mn == kNegInf) ? 0.0f : mn;
                    const float alpha = fast_exp2(m[tl] - mu);
                    m[tl] = mn;
                    const float ref = (cm == kNegInf) ? 0.0f : cm;
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        s[i] = fast_exp2(fmaf(s[i], c2, -ref));
                        sum += s[i];
                    }
                    // a chunk with nothing visible for this column joins with weight 0 (not exp2(-mu), which
                    // overflows for strongly negative maxima and would turn its zero sums into NaN)
                    beta[tl] = (cm == kNegInf) ? 0.0f : fast_exp2(ref - mu);
                    e[tl] = fmaf(e[tl], alpha, sum * beta[tl]);
                    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
                        for (int n = 0; n < 8; ++n) acc[tl][n] *= alpha;
                    }
                } else {
                    // bf16 has fp32's exponent range: weights are taken against mref, the reference maximum that the
                    // four lanes of a column share; m is the lane's own running maximum (its 8 tokens per chunk).
                    // No lane's weights may pass 2^kLazyRescale: when a lane's maximum has left mref that far behind
                    // (also: the first chunk with a visible token), the column maximum is found across the lanes and
                    // acc, e are rescaled to it.  Otherwise the chunk needs no cross-lane step at all.
                    cm *= c2;  // base-2 units from here on
                    m[tl] = fmaxf(m[tl], cm);
                    if (__builtin_amdgcn_ballot_w64(m[tl] > mref[tl] + kLazyRescale) != 0) {
                        float mc = m[tl];
                        mc = fmaxf(mc, __shfl_xor(mc, 16));
                        mc = fmaxf(mc, __shfl_xor(mc, 32));
                        const bool grow = mc > mref[tl] + kLazyRescale;
                        const float alpha = grow ? fast_exp2(mref[tl] - mc) : 1.0f;  // 0 when nothing was seen yet
                        mref[tl] = grow ? mc : mref[tl];
                        e[tl] *= alpha;
#pragma unroll
                        for (int n = 0; n < 8; ++n) acc[tl][n] *= alpha;
                    }
                    const float mu = (mref[tl] == kNegInf) ? 0.0f : mref[tl];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        s[i] = fast_exp2(fmaf(s[i], c2, -mu));
                        sum += s[i];
                    }
                    beta[tl] = 1.0f;
                    e[tl] += sum;
                }
                uint32_t h[4], l[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) Weights<F16>::split(s[2 * t], s[2 * t + 1], h[t], l[t]);
                ph[tl] = u32x4{h[0], h[1], h[2], h[3]};
                pl[tl] = u32x4{l[0], l[1], l[2], l[3]};

                // V^T operands, built once per chunk after the first tile's softmax (V has had that long to arrive):
                // even dim 2w: low halves; odd dim 2w+1: high halves; (token 2t, token 2t+1) per register
                if (tl == 0) {
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        const uint32_t d0 = vr[0][w], d1 = vr[1][w], d2 = vr[2][w], d3 = vr[3][w];
                        const uint32_t d4 = vr[4][w], d5 = vr[5][w], d6 = vr[6][w], d7 = vr[7][w];
                        ve[w] = u32x4{__builtin_amdgcn_perm(d1, d0, 0x05040100u), __builtin_amdgcn_perm(d3, d2, 0x05040100u),
                                      __builtin_amdgcn_perm(d5, d4, 0x05040100u), __builtin_amdgcn_perm(d7, d6, 0x05040100u)};
                        vo[w] = u32x4{__builtin_amdgcn_perm(d1, d0, 0x07060302u), __builtin_amdgcn_perm(d3, d2, 0x07060302u),
                                      __builtin_amdgcn_perm(d5, d4, 0x07060302u), __builtin_amdgcn_perm(d7, d6, 0x07060302u)};
                    }
                }
                // O^T += V^T . P^T for this tile, 8 MFMA dimension groups (group n takes dims 8*m + n, m = MFMA
                // row); issued here so that the matrix pipe works on it while the vector ALU does the next tile's softmax
                if constexpr (F16) {
                    f32x4 part[8];  // the chunk's own V^T . P^T, weights relative to the chunk maximum
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        part[2 * w] = mfma16<F16>(ve[w], ph[tl], f32x4{0.f, 0.f, 0.f, 0.f});
                        part[2 * w] = mfma16<F16>(ve[w], pl[tl], part[2 * w]);
                        part[2 * w + 1] = mfma16<F16>(vo[w], ph[tl], f32x4{0.f, 0.f, 0.f, 0.f});
                        part[2 * w + 1] = mfma16<F16>(vo[w], pl[tl], part[2 * w + 1]);
                    }
                    const float b = beta[tl] * Weights<F16>::kUnscale;
#pragma unroll
                    for (int n = 0; n < 8; ++n) acc[tl][n] += part[n] * b;
                } else {
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        acc[tl][2 * w] = mfma16<F16>(ve[w], ph[tl], acc[tl][2 * w]);
                        acc[tl][2 * w] = mfma16<F16>(ve[w], pl[tl], acc[tl][2 * w]);
                        acc[tl][2 * w + 1] = mfma16<F16>(vo[w], ph[tl], acc[tl][2 * w + 1]);
                        acc[tl][2 * w + 1] = mfma16<F16>(vo[w], pl[tl], acc[tl][2 * w + 1]);
                    }
                }
            }
            cur = nxt;
        }
        // the last step above requested the first K chunk of the next item
        if (idle) load_k(fetch_of(ncur), kr);
        load_q(nit, qreg, visible_next);
        if constexpr (!F16) {
            // sums and accumulator are relative to mref: bring them to the true maximum m (over the column's four lanes)
#pragma unroll
            for (int tl = 0; tl < TILES; ++tl) {
                m[tl] = fmaxf(m[tl], __shfl_xor(m[tl], 16));
                m[tl] = fmaxf(m[tl], __shfl_xor(m[tl], 32));
                const float f = (m[tl] == kNegInf) ? 1.0f : fast_exp2(mref[tl] - m[tl]);
                if (__builtin_amdgcn_ballot_w64(f != 1.0f) != 0) {
                    e[tl] *= f;
#pragma unroll
                    for (int n = 0; n < 8; ++n) acc[tl][n] *= f;
                }
            }
        }

        if constexpr (WAVE_ITEMS) {
            // ---- the wavefront owns the item: its rows (normalised, or as a partial) wait in shared memory ----
            OutStage &st = ((OutStage *)lds_raw)[wave];
            const bool direct = p.direct_out && it.ns == 1;
            int live_cols = p.cols - it.ht * COLS;
            live_cols = live_cols > COLS ? COLS : live_cols;
            if (staged + live_cols > kStageRows) {
                flush_stage(st, staged, lane);
                staged = 0;
            }
#pragma unroll
            for (int tl = 0; tl < TILES; ++tl) {
                float et = e[tl];
                et += __shfl_xor(et, 16);
                et += __shfl_xor(et, 32);
                const int c = tl * kHeadTile + ln;  // column inside the item
                const Column col = column_of(p, it.ht * COLS + c, it.kvh, it.L);
                if (!col.live) continue;
                const float m_nat = m[tl] * kLn2;  // base-2 -> natural-log score units (-inf stays -inf)
                const float f = direct ? ((et > 0.0f) ? 1.0f / et : 0.0f) : 1.0f;
                const int sr = staged + c;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float *dst = &st.o[sr][32 * lg + 8 * i];
                    *(float4 *)dst = make_float4(acc[tl][0][i] * f, acc[tl][1][i] * f, acc[tl][2][i] * f, acc[tl][3][i] * f);
                    *(float4 *)(dst + 4) = make_float4(acc[tl][4][i] * f, acc[tl][5][i] * f, acc[tl][6][i] * f, acc[tl][7][i] * f);
                }
                if (lg == 0) {
                    if (direct) {
                        const int64_t orow = (int64_t)it.r * p.q_len * p.Hq + col.vh;
                        st.o_dst[sr] = p.out + orow * kHeadDim;
                        st.s_dst[sr][0] = p.lse ? p.lse + orow : nullptr;
                        st.s_dst[sr][1] = nullptr;
                        st.s[sr][0] = (et > 0.0f) ? m_nat + __logf(et) : kNegInf;
                    } else {
                        const int64_t prow = it.row_base + (int64_t)col.vh * it.ns + it.j;
                        st.o_dst[sr] = p.part_o + prow * kHeadDim;
                        st.s_dst[sr][0] = p.part_m + prow;
                        st.s_dst[sr][1] = p.part_e + prow;
                        st.s[sr][0] = m_nat;
                        st.s[sr][1] = et;
                    }
                }
            }
            staged += live_cols;
            if (!nit.valid) {  // the wavefront's last item: everything still held goes out
                flush_stage(st, staged, lane);
                staged = 0;
            }
        } else {
            // ---- wavefront result: exp-sum over the lane groups; m is already common -----------------
    #pragma unroll
            for (int tl = 0; tl < TILES; ++tl) {
                float et = e[tl];
                et += __shfl_xor(et, 16);
                et += __shfl_xor(et, 32);
                const int c = tl * kHeadTile + ln;  // column inside the item
                if (it.ht * COLS + c < p.cols) {
                    if (lg == 0) {
                        lds_m[wave][c] = m[tl];
                        lds_e[wave][c] = et;
                    }
    #pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        float *dst = &lds_o[wave][c][32 * lg + 8 * i];
                        *(float4 *)dst = make_float4(acc[tl][0][i], acc[tl][1][i], acc[tl][2][i], acc[tl][3][i]);
                        *(float4 *)(dst + 4) = make_float4(acc[tl][4][i], acc[tl][5][i], acc[tl][6][i], acc[tl][7][i]);
                    }
                }
            }
            __syncthreads();

            // ---- merge the wavefronts and write the item's result -------------------------------------
            const bool direct = p.direct_out && it.ns == 1;
            int heads = p.cols - it.ht * COLS;
            heads = heads > COLS ? COLS : heads;
            for (int idx = tid; idx < heads * kHeadDim; idx += kWaves * 64) {
                const int g = idx / kHeadDim, col = idx % kHeadDim;
                float M = lds_m[0][g];
    #pragma unroll
                for (int w = 1; w < kWaves; ++w) M = fmaxf(M, lds_m[w][g]);
                const float mu = (M == kNegInf) ? 0.0f : M;
                float o = 0.0f, E = 0.0f;
    #pragma unroll
                for (int w = 0; w < kWaves; ++w) {
                    const float wgt = fast_exp2(lds_m[w][g] - mu);
                    o = fmaf(lds_o[w][g][col], wgt, o);
                    E = fmaf(lds_e[w][g], wgt, E);
                }
                const int vh = column_of(p, it.ht * COLS + g, it.kvh, it.L).vh;
                const float m_nat = M * kLn2;  // base-2 -> natural-log score units (-inf stays -inf)
                if (direct) {
                    const int64_t orow = (int64_t)it.r * p.q_len * p.Hq + vh;
                    p.out[orow * kHeadDim + col] = (E > 0.0f) ? o / E : 0.0f;
                    if (col == 0 && p.lse) p.lse[orow] = (E > 0.0f) ? m_nat + __logf(E) : kNegInf;
                } else {
                    const int64_t prow = it.row_base + (int64_t)vh * it.ns + it.j;
                    p.part_o[prow * kHeadDim + col] = o;
                    if (col == 0) {
                        p.part_m[prow] = m_nat;
                        p.part_e[prow] = E;
                    }
                }
            }
            __syncthreads();  // the merge buffers are free again
        }
#pragma unroll
        for (int tl = 0; tl < TILES; ++tl) visible[tl] = visible_next[tl];
        it = nit;
        cur = ncur;
    }
}

template <bool F16>
hipError_t launch_tiles(const MicroParams &p, int grid, hipStream_t stream)
{
    if (p.head_tile == kHeadTile && p.wave_items)
        hipLaunchKernelGGL((micro_attention_mfma_kernel<1, F16, true>), dim3((unsigned)grid), dim3(kWaves * 64), 0, stream, p);
    else if (p.wave_items)
        return hipErrorInvalidValue;
    else if (p.head_tile == kHeadTile)
        hipLaunchKernelGGL((micro_attention_mfma_kernel<1, F16, false>), dim3((unsigned)grid), dim3(kWaves * 64), 0, stream, p);
    else if (!F16)
        return hipErrorInvalidValue;  // bf16 with more than one column tile: micro_attention_mfma_tiles.hip
    else if (p.head_tile == 2 * kHeadTile)
        hipLaunchKernelGGL((micro_attention_mfma_kernel<2, true, false>), dim3((unsigned)grid), dim3(kWaves * 64), 0, stream, p);
    else if (p.head_tile == 4 * kHeadTile)
        hipLaunchKernelGGL((micro_attention_mfma_kernel<4, true, false>), dim3((unsigned)grid), dim3(kWaves * 64), 0, stream, p);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace

hipError_t launch_micro_attention_mfma_tiles(const MicroParams &p, int grid, hipStream_t stream);

// q, K and V share one 16-bit type (bf16 or IEEE half); head_tile is 16, 32 or 64.
hipError_t launch_micro_attention_mfma(const MicroParams &p, int grid, hipStream_t stream)
{
    if (grid < 1 || p.q_dtype != p.kv_dtype) return hipErrorInvalidValue;
    // bf16 with more than one column tile has a kernel of its own (micro_attention_mfma_tiles.hip)
    if (p.kv_dtype == DA_BF16 && p.head_tile > kHeadTile && !p.wave_items) return launch_micro_attention_mfma_tiles(p, grid, stream);
    if (p.kv_dtype == DA_BF16) return launch_tiles<false>(p, grid, stream);
    if (p.kv_dtype == DA_F16) return launch_tiles<true>(p, grid, stream);
    return hipErrorInvalidValue;
}

}  // namespace da
