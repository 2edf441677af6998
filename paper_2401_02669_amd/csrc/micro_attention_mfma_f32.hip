// MicroAttention on the matrix cores for fp32 q / K / V with a query group (Section 4, m_j / e_j equation and
// Eq. 2; Section 3: the q-heads of a GQA group share one K/V read).
//
// Same persistent skeleton as the 16-bit matrix-core kernel (one 4-wavefront workgroup per CU walks its run of
// splits; each wavefront walks 32-token chunks; the first K chunk and the query of the next item are requested
// before the current item is merged), with v_mfma_f32_16x16x4_f32: fp32 operands, one float per lane per
// instruction, contraction length 4.  A work item serves one tile of 16 columns.
//
//   S = K . Q^T    the contraction runs over the 128 head dimensions in 32 instructions.  A lane (token row ln,
//                  lane group lg) loads bytes [64 m + 16 lg, +16) of its K row for m = 0..7, straight from HBM; the
//                  float i of that piece is the A operand of instruction (m, i), so the instruction's contraction
//                  index lg stands for dimension 16 m + 4 lg + i.  Q^T is held the same way (column ln).
//   O^T += V^T . P^T  contraction over the chunk's tokens, 4 per instruction: instruction (hb, i) takes tokens
//                  16 hb + 4 lg + i, which is exactly how a lane already holds its weights (B operand: no data
//                  movement).  A lane loads, of those 8 token rows, the two 16-byte pieces [256 hh + 16 ln, +16):
//                  float j of piece hh is the A operand of dimension group (hh, j), whose MFMA row ln stands for
//                  dimension 64 hh + 4 ln + j.
//
// All arithmetic is fp32 (products and sums inside the matrix cores, softmax on the vector ALU).
#include <hip/hip_runtime.h>

#include "../../include/distattn.h"
#include "item_walk.h"
#include "kernel_params.h"

namespace da {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr float kNegInf = -__builtin_inff();
constexpr float kLn2 = 0.69314718055994530942f;
constexpr int kCols = 16;    // columns per work item (MFMA N dimension)
constexpr int kChunk = 32;   // tokens per wavefront step
constexpr int kWaves = 4;    // wavefronts per workgroup

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// 16-byte streaming load (K and V are read exactly once)
__device__ __forceinline__ f32x4 load16_stream(const char *p) { return __builtin_nontemporal_load((const f32x4 *)p); }

__device__ __forceinline__ f32x4 mfma_f32(float a, float b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

__global__ __launch_bounds__(kWaves * 64) void micro_attention_mfma_f32_kernel(const MicroParams p)
{
    // cross-wavefront merge buffers (one barrier after they are written, one after they are read)
    __shared__ float lds_m[kWaves][kCols];
    __shared__ float lds_e[kWaves][kCols];
    __shared__ float lds_o[kWaves][kCols][kHeadDim];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int lg = lane >> 4;   // lane group: contraction index of the MFMA operands
    const int ln = lane & 15;   // token row (K operand) / dimension row (V operand) / column (Q, P, results)

    const char *kbase = (const char *)p.k_pool;
    const char *vbase = (const char *)p.v_pool;
    const uint32_t row_bytes = (uint32_t)p.stride_token * 4u;
    const float c2 = p.scale_log2e;

    // Every step issues 16 K loads and 16 V loads whatever the chunk: rows past the valid ones re-read the last
    // valid row (their scores are masked), so the loads need no branches.
    // K: lane reads token 16 hb + ln, bytes [64 m + 16 lg, +16)
    const uint32_t k_full[2] = {(uint32_t)ln * row_bytes + lg * 16, (uint32_t)(16 + ln) * row_bytes + lg * 16};
    // V: lane reads token 16 hb + 4 lg + i, bytes [256 hh + 16 ln, +16)
    uint32_t v_full[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) v_full[t] = (uint32_t)(16 * (t >> 2) + 4 * lg + (t & 3)) * row_bytes + ln * 16;
    auto load_k = [&](const Fetch &f, f32x4 (&dst)[16]) {
        const char *base = kbase + f.off * 4;
        const uint32_t clamp_off = (uint32_t)f.last * row_bytes + lg * 16;
#pragma unroll
        for (int hb = 0; hb < 2; ++hb) {
            const uint32_t off = k_full[hb] < clamp_off ? k_full[hb] : clamp_off;
#pragma unroll
            for (int m = 0; m < 8; ++m) dst[hb * 8 + m] = load16_stream(base + off + m * 64);
        }
    };
    auto load_v = [&](const Fetch &f, f32x4 (&dst)[16]) {
        const char *base = vbase + f.off * 4;
        const uint32_t clamp_off = (uint32_t)f.last * row_bytes + ln * 16;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const uint32_t off = v_full[t] < clamp_off ? v_full[t] : clamp_off;
            dst[2 * t] = load16_stream(base + off);
            dst[2 * t + 1] = load16_stream(base + off + 256);
        }
    };
    // Q^T operand of an item: column ln, floats [16 m + 4 lg, +4) for m = 0..7 (zero for columns past the group);
    // also the number of tokens that column may see (causal limit)
    auto load_q = [&](const ItemInfo &it, f32x4 (&dst)[8], int &visible) {
        const Column col = column_of(p, it.ht * kCols + ln, it.kvh, it.L);
        const bool live = it.valid && col.live;
        visible = live ? col.visible : 0;
        const float *q = (const float *)p.q + ((int64_t)it.r * p.q_len * p.Hq + col.vh) * kHeadDim;
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            dst[m] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (live) dst[m] = *(const f32x4 *)(q + 16 * m + 4 * lg);
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
    ItemInfo it = decode_item<kChunk>(p, e_begin, e_end, kvh, ht);
    Chunk cur = first_chunk<kChunk>(p, it, wave, lane);
    f32x4 kr[16], vr[16], qreg[8];
    int visible, visible_next;  // causal limit of this lane's column, for the current / next item
    load_k(fetch_of(cur), kr);
    load_q(it, qreg, visible);

    while (it.valid) {
        float m = kNegInf;  // running maximum of column ln's scores, base-2 units (all lane groups agree)
        float e = 0.0f;     // this lane's share of the exp-sum (its 8 tokens per chunk)
        f32x4 acc[8];       // O^T: acc[4 hh + j][i] = O[column ln][dim 64 hh + 16 lg + 4 i + j]
#pragma unroll
        for (int n = 0; n < 8; ++n) acc[n] = f32x4{0.f, 0.f, 0.f, 0.f};

        // the item after this one is looked up early, so that its first K chunk can be requested
        // before this item's result is merged
        ++round;
        const ItemInfo nit = decode_item<kChunk>(p, e_begin + round, e_end, kvh, ht);
        const Chunk ncur = first_chunk<kChunk>(p, nit, wave, lane);

        // every step issues 16 V loads and 16 K loads; kr always holds the K rows of `cur`
        const bool idle = !cur.valid;  // this wavefront has no chunk in the item
        while (cur.valid) {
            load_v(fetch_of(cur), vr);
            const Chunk nxt = next_chunk<kChunk, kWaves>(p, it, cur, lane);
            const Fetch kf_next = fetch_of(nxt.valid ? nxt : ncur);  // nothing left at all: row 0 of the pool

            // S[token 16 hb + 4 lg + i][column ln] for hb = 0, 1
            // (four short accumulation chains per score instead of one of 32 steps: less rounding build-up when
            // the products are large, and independent instructions for the matrix pipe)
            f32x4 s0, s1;
            {
                f32x4 a0[4], a1[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    a0[c] = f32x4{0.f, 0.f, 0.f, 0.f};
                    a1[c] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int mm = 0; mm < 8; ++mm) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        a0[i] = mfma_f32(kr[mm][i], qreg[mm][i], a0[i]);
                        a1[i] = mfma_f32(kr[8 + mm][i], qreg[mm][i], a1[i]);
                    }
                }
                s0 = (a0[0] + a0[1]) + (a0[2] + a0[3]);
                s1 = (a1[0] + a1[1]) + (a1[2] + a1[3]);
            }
            load_k(kf_next, kr);
            if (cur.lim <= 0) {  // a chunk slot without valid tokens contributes nothing
                cur = nxt;
                continue;
            }

            // scores in base-2 units (scale * log2(e) applied); rows past the valid or visible tokens masked out
            float s[8];
            const int rows_seen = min(cur.lim, visible - cur.tok0);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                s[i] = (4 * lg + i < rows_seen) ? s0[i] * c2 : kNegInf;
                s[4 + i] = (16 + 4 * lg + i < rows_seen) ? s1[i] * c2 : kNegInf;
            }
            float cm = s[0];
#pragma unroll
            for (int i = 1; i < 8; ++i) cm = fmaxf(cm, s[i]);
            cm = fmaxf(cm, __shfl_xor(cm, 16));
            cm = fmaxf(cm, __shfl_xor(cm, 32));
            const float mn = fmaxf(m, cm);
            const float mu = (mn == kNegInf) ? 0.0f : mn;
            const float alpha = fast_exp2(m - mu);
            m = mn;
            float sum = 0.0f;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                s[i] = fast_exp2(s[i] - mu);
                sum += s[i];
            }
            e = fmaf(e, alpha, sum);
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
                for (int n = 0; n < 8; ++n) acc[n] *= alpha;
            }

            // O^T += V^T . P^T: instruction (t, hh, j) contracts over tokens 16 (t / 4) + 4 lg + t % 4
#pragma unroll
            for (int t = 0; t < 8; ++t) {
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[4 * hh + j] = mfma_f32(vr[2 * t + hh][j], s[t], acc[4 * hh + j]);
                }
            }
            cur = nxt;
        }
        // the last step above requested the first K chunk of the next item
        if (idle) load_k(fetch_of(ncur), kr);
        load_q(nit, qreg, visible_next);

        // ---- wavefront result: exp-sum over the lane groups; m is already common -----------------
        float et = e;
        et += __shfl_xor(et, 16);
        et += __shfl_xor(et, 32);
        if (it.ht * kCols + ln < p.cols) {
            if (lg == 0) {
                lds_m[wave][ln] = m;
                lds_e[wave][ln] = et;
            }
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    *(float4 *)&lds_o[wave][ln][64 * hh + 16 * lg + 4 * i] =
                        make_float4(acc[4 * hh][i], acc[4 * hh + 1][i], acc[4 * hh + 2][i], acc[4 * hh + 3][i]);
            }
        }
        __syncthreads();

        // ---- merge the wavefronts and write the item's result -------------------------------------
        const bool direct = p.direct_out && it.ns == 1;
        int heads = p.cols - it.ht * kCols;
        heads = heads > kCols ? kCols : heads;
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
            const int vh = column_of(p, it.ht * kCols + g, it.kvh, it.L).vh;
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
        visible = visible_next;
        it = nit;
        cur = ncur;
    }
}

}  // namespace

// fp32 q and fp32 pools; head_tile is 16.
hipError_t launch_micro_attention_mfma_f32(const MicroParams &p, int grid, hipStream_t stream)
{
    if (grid < 1 || p.q_dtype != DA_F32 || p.kv_dtype != DA_F32 || p.head_tile != kCols) return hipErrorInvalidValue;
    hipLaunchKernelGGL(micro_attention_mfma_f32_kernel, dim3((unsigned)grid), dim3(kWaves * 64), 0, stream, p);
    return hipGetLastError();
}

}  // namespace da
