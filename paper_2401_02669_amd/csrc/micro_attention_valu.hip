// MicroAttention on the fp32 vector ALU (Section 4, m_j / e_j equation and Eq. 2).
//
// A work item is a run of tokens of one (request, kv-head) and up to GT columns of that kv-head's
// group (q-heads for plain decode; query tokens x q-heads, each with a causal limit, otherwise).  The launch is persistent: each workgroup (4 wavefronts) walks its items one after the
// other and requests the next item's first K chunk before merging and writing the current item's
// result.  Wavefront w takes chunks w, w + 4, ... of the item.  A load instruction fetches 1 KiB of
// consecutive K (or V) bytes: RPL whole token rows, LPR lanes per row, 16 bytes per lane.  Each
// lane multiplies its 16-byte slice with the matching slice of q; a DPP all-reduce over the LPR
// lanes of the row yields the score.  Every row position of every wavefront keeps its own running
// (m, e, o) in base-2 units; they are merged once, at the end of the item.
#include <hip/hip_runtime.h>

#include "../../include/distattn.h"
#include "item_walk.h"
#include "kernel_params.h"

namespace da {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float as_f(uint32_t u) { return __builtin_bit_cast(float, u); }

// 16-byte streaming load: K and V are read exactly once, so the non-temporal hint keeps them from
// displacing anything in the caches (measurably faster than a plain load on this GPU).
__device__ __forceinline__ u32x4 load16_stream(const char *p) { return __builtin_nontemporal_load((const u32x4 *)p); }

template <int CTRL>
__device__ __forceinline__ float dpp_move(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}

// Sum over the 16 lanes of a DPP row, result in every lane of the row.
__device__ __forceinline__ float row16_sum(float x)
{
    x += dpp_move<0xB1>(x);   // quad_perm [1,0,3,2]
    x += dpp_move<0x4E>(x);   // quad_perm [2,3,0,1]
    x += dpp_move<0x124>(x);  // row_ror:4
    x += dpp_move<0x128>(x);  // row_ror:8
    return x;
}

// Sum over 32 lanes (two DPP rows), result in every lane.
__device__ __forceinline__ float row32_sum(float x)
{
    x = row16_sum(x);
    // swap with the lane 16 away inside each half-wave (ds_swizzle bit mode: and 0x1F, or 0, xor 0x10)
    x += __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, x), 0x401F));
    return x;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// two IEEE halves in one register -> two floats (exact, subnormals included)
__device__ __forceinline__ void half2_to_float(uint32_t w, float &lo, float &hi)
{
    const f16x2 h = __builtin_bit_cast(f16x2, w);
    lo = (float)h[0];
    hi = (float)h[1];
}

template <int KV>
struct Slice;  // a lane's 16 bytes of one token row; KV = da_dtype of the pools
template <>
struct Slice<DA_F16> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void unpack(const u32x4 &r, float (&f)[8])
    {
        half2_to_float(r.x, f[0], f[1]);
        half2_to_float(r.y, f[2], f[3]);
        half2_to_float(r.z, f[4], f[5]);
        half2_to_float(r.w, f[6], f[7]);
    }
};
template <>
struct Slice<DA_BF16> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void unpack(const u32x4 &r, float (&f)[8])
    {
        f[0] = as_f(r.x << 16); f[1] = as_f(r.x & 0xFFFF0000u);
        f[2] = as_f(r.y << 16); f[3] = as_f(r.y & 0xFFFF0000u);
        f[4] = as_f(r.z << 16); f[5] = as_f(r.z & 0xFFFF0000u);
        f[6] = as_f(r.w << 16); f[7] = as_f(r.w & 0xFFFF0000u);
    }
};
template <>
struct Slice<DA_F32> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void unpack(const u32x4 &r, float (&f)[4])
    {
        f[0] = as_f(r.x); f[1] = as_f(r.y); f[2] = as_f(r.z); f[3] = as_f(r.w);
    }
};

constexpr float kNegInf = -__builtin_inff();
constexpr float kLn2 = 0.69314718055994530942f;
constexpr int kWaves = 4;  // wavefronts per workgroup

// KV: da_dtype of the K/V pools.  GT: q-heads per item.  NL: load instructions per chunk.
template <int KV, int GT, int NL>
__global__ __launch_bounds__(kWaves * 64) void micro_attention_valu_kernel(const MicroParams p)
{
    constexpr int EPL = Slice<KV>::N;  // elements per lane
    constexpr int LPR = kHeadDim / EPL;    // lanes per token row: 16 (16-bit types) or 32 (fp32)
    constexpr int RPL = 64 / LPR;          // token rows per load instruction: 4 or 2
    constexpr int CH = NL * RPL;           // tokens per chunk (divides the 32-token tile)
    constexpr int ESIZE = KV == DA_F32 ? 4 : 2;
    static_assert(kTile % CH == 0, "a chunk must divide the scheduling tile");

    // cross-wavefront merge buffers, two sets used alternately by consecutive items
    __shared__ float lds_m[2][kWaves][GT];
    __shared__ float lds_e[2][kWaves][GT];
    __shared__ float lds_o[2][kWaves][GT][kHeadDim];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int row = lane / LPR;   // token row inside a load
    const int colc = lane % LPR;  // 16-byte column chunk

    const char *kbase = (const char *)p.k_pool;
    const char *vbase = (const char *)p.v_pool;
    const uint32_t row_bytes = (uint32_t)p.stride_token * ESIZE;
    const uint32_t lane_off = (uint32_t)row * row_bytes + colc * 16;
    const uint32_t load_step = (uint32_t)RPL * row_bytes;
    // byte offset of this lane's 16 bytes in load jj of a full chunk; partial chunks clamp to the last valid row
    uint32_t full_off[NL];
#pragma unroll
    for (int jj = 0; jj < NL; ++jj) full_off[jj] = lane_off + jj * load_step;
    auto load_rows = [&](const char *pool, const Fetch &f, u32x4 (&dst)[NL]) {
        const char *base = pool + f.off * ESIZE;
        const uint32_t clamp_off = (uint32_t)f.last * row_bytes + colc * 16;
#pragma unroll
        for (int jj = 0; jj < NL; ++jj) {
            const uint32_t off = full_off[jj] < clamp_off ? full_off[jj] : clamp_off;
            dst[jj] = load16_stream(base + off);
        }
    };
    // this lane's slice of the item's queries, pre-scaled to base-2 units (zero for columns past the group),
    // and the number of tokens each column may see (causal limit of its query token)
    auto load_q = [&](const ItemInfo &it, float (&qf)[GT][EPL], int (&visible)[GT]) {
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            const Column col = column_of(p, it.ht * GT + g, it.kvh, it.L);
            const bool live = it.valid && col.live;
            visible[g] = live ? col.visible : 0;
            const int64_t qoff = ((int64_t)it.r * p.q_len * p.Hq + col.vh) * kHeadDim + colc * EPL;
            float x[EPL];
            if (p.q_dtype != DA_F32) {
                uint32_t w[EPL / 2];
                const uint32_t *src = (const uint32_t *)((const uint16_t *)p.q + qoff);
#pragma unroll
                for (int c = 0; c < EPL / 2; ++c) w[c] = src[c];
#pragma unroll
                for (int c = 0; c < EPL / 2; ++c) {
                    if (p.q_dtype == DA_BF16) {
                        x[2 * c] = as_f(w[c] << 16);
                        x[2 * c + 1] = as_f(w[c] & 0xFFFF0000u);
                    } else {
                        half2_to_float(w[c], x[2 * c], x[2 * c + 1]);
                    }
                }
            } else {
                const float *src = (const float *)p.q + qoff;
#pragma unroll
                for (int c = 0; c < EPL; ++c) x[c] = src[c];
            }
#pragma unroll
            for (int c = 0; c < EPL; ++c) qf[g][c] = live ? x[c] * p.scale_log2e : 0.0f;
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
    ItemInfo it = decode_item<CH>(p, e_begin, e_end, kvh, ht);
    Chunk cur = first_chunk<CH>(p, it, wave, lane);
    u32x4 kr[NL], vr[NL];
    float qf[GT][EPL];
    int visible[GT], visible_next[GT];  // causal limits of the columns, for the current / next item
    load_rows(kbase, fetch_of(cur), kr);
    load_q(it, qf, visible);

    while (it.valid) {
        float m[GT], e[GT], o[GT][EPL];
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            m[g] = kNegInf;
            e[g] = 0.0f;
#pragma unroll
            for (int c = 0; c < EPL; ++c) o[g][c] = 0.0f;
        }

        // the item after this one is looked up early, so that its first K chunk can be requested
        // before this item's result is merged
        const int buf = round & 1;
        ++round;
        const ItemInfo nit = decode_item<CH>(p, e_begin + round, e_end, kvh, ht);
        const Chunk ncur = first_chunk<CH>(p, nit, wave, lane);

        // every step issues NL V loads and NL K loads; kr always holds the K rows of `cur`
        const bool idle = !cur.valid;  // this wavefront has no chunk in the item
        while (cur.valid) {
            load_rows(vbase, fetch_of(cur), vr);
            const Chunk nxt = next_chunk<CH, kWaves>(p, it, cur, lane);
            const Fetch kf_next = fetch_of(nxt.valid ? nxt : ncur);  // nothing left at all: row 0 of the pool

            // scores of the chunk's rows, base-2 units
            float s[NL][GT];
            int rows_seen[GT];  // rows of this chunk each column may see
#pragma unroll
            for (int g = 0; g < GT; ++g) rows_seen[g] = min(cur.lim, visible[g] - cur.tok0);
#pragma unroll
            for (int jj = 0; jj < NL; ++jj) {
                float kf[EPL];
                Slice<KV>::unpack(kr[jj], kf);
#pragma unroll
                for (int g = 0; g < GT; ++g) {
                    float acc = 0.0f;
#pragma unroll
                    for (int c = 0; c < EPL; ++c) acc = fmaf(qf[g][c], kf[c], acc);
                    acc = (LPR == 16) ? row16_sum(acc) : row32_sum(acc);
                    s[jj][g] = (jj * RPL + row < rows_seen[g]) ? acc : kNegInf;
                }
            }
            load_rows(kbase, kf_next, kr);

            if (cur.lim > 0) {  // (a chunk slot without valid tokens contributes nothing)
                // online softmax update of this row position's running state
#pragma unroll
                for (int g = 0; g < GT; ++g) {
                    float cm = s[0][g];
#pragma unroll
                    for (int jj = 1; jj < NL; ++jj) cm = fmaxf(cm, s[jj][g]);
                    const float mn = fmaxf(m[g], cm);
                    const float mu = (mn == kNegInf) ? 0.0f : mn;
                    const float alpha = fast_exp2(m[g] - mu);
                    m[g] = mn;
                    float sum = 0.0f;
#pragma unroll
                    for (int jj = 0; jj < NL; ++jj) {
                        s[jj][g] = fast_exp2(s[jj][g] - mu);
                        sum += s[jj][g];
                    }
                    e[g] = e[g] * alpha + sum;
#pragma unroll
                    for (int c = 0; c < EPL; ++c) o[g][c] *= alpha;
                }
#pragma unroll
                for (int jj = 0; jj < NL; ++jj) {
                    float vf[EPL];
                    Slice<KV>::unpack(vr[jj], vf);
#pragma unroll
                    for (int g = 0; g < GT; ++g)
#pragma unroll
                        for (int c = 0; c < EPL; ++c) o[g][c] = fmaf(s[jj][g], vf[c], o[g][c]);
                }
            }
            cur = nxt;
        }
        // the last step above requested the first K chunk of the next item
        if (idle) load_rows(kbase, fetch_of(ncur), kr);
        load_q(nit, qf, visible_next);

        // ---- merge the RPL row positions of the wavefront --------------------------------------
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                const float mo = __shfl_xor(m[g], off);
                const float eo = __shfl_xor(e[g], off);
                const float mn = fmaxf(m[g], mo);
                const float mu = (mn == kNegInf) ? 0.0f : mn;
                const float a = fast_exp2(m[g] - mu), b = fast_exp2(mo - mu);
                e[g] = e[g] * a + eo * b;
#pragma unroll
                for (int c = 0; c < EPL; ++c) o[g][c] = o[g][c] * a + __shfl_xor(o[g][c], off) * b;
                m[g] = mn;
            }
        }
        if (lane < LPR) {
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                if (lane == 0) {
                    lds_m[buf][wave][g] = m[g];
                    lds_e[buf][wave][g] = e[g];
                }
#pragma unroll
                for (int c = 0; c < EPL; ++c) lds_o[buf][wave][g][colc * EPL + c] = o[g][c];
            }
        }
        __syncthreads();

        // ---- merge the wavefronts and write the item's result ---------------------------------
        const bool direct = p.direct_out && it.ns == 1;
        for (int idx = tid; idx < GT * kHeadDim; idx += kWaves * 64) {
            const int g = idx / kHeadDim, col = idx % kHeadDim;
            const Column cc = column_of(p, it.ht * GT + g, it.kvh, it.L);
            if (!cc.live) continue;
            float M = lds_m[buf][0][g];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) M = fmaxf(M, lds_m[buf][w][g]);
            const float mu = (M == kNegInf) ? 0.0f : M;
            float acc = 0.0f, E = 0.0f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                const float wgt = fast_exp2(lds_m[buf][w][g] - mu);
                acc = fmaf(lds_o[buf][w][g][col], wgt, acc);
                E = fmaf(lds_e[buf][w][g], wgt, E);
            }
            if (direct) {
                const int64_t orow = (int64_t)it.r * p.q_len * p.Hq + cc.vh;
                p.out[orow * kHeadDim + col] = (E > 0.0f) ? acc / E : 0.0f;
                if (col == 0 && p.lse) p.lse[orow] = (E > 0.0f) ? M * kLn2 + __logf(E) : kNegInf;
            } else {
                const int64_t prow = it.row_base + (int64_t)cc.vh * it.ns + it.j;
                p.part_o[prow * kHeadDim + col] = acc;
                if (col == 0) {
                    p.part_m[prow] = M * kLn2;  // back to natural-log units (-inf stays -inf)
                    p.part_e[prow] = E;
                }
            }
        }
#pragma unroll
        for (int g = 0; g < GT; ++g) visible[g] = visible_next[g];
        it = nit;
        cur = ncur;
    }
}

template <int KV, int GT, int NL>
hipError_t launch_one(const MicroParams &p, int grid, hipStream_t stream)
{
    hipLaunchKernelGGL((micro_attention_valu_kernel<KV, GT, NL>), dim3((unsigned)grid), dim3(kWaves * 64), 0, stream, p);
    return hipGetLastError();
}

template <int KV>
hipError_t launch_for(const MicroParams &p, int grid, hipStream_t stream)
{
    switch (p.head_tile) {
    case 1: return launch_one<KV, 1, 8>(p, grid, stream);
    case 2: return launch_one<KV, 2, 8>(p, grid, stream);
    case 4: return launch_one<KV, 4, 4>(p, grid, stream);
    case 8: return launch_one<KV, 8, 2>(p, grid, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

// head_tile must be 1, 2, 4 or 8.
hipError_t launch_micro_attention_valu(const MicroParams &p, int grid, hipStream_t stream)
{
    if (grid < 1) return hipErrorInvalidValue;
    switch (p.kv_dtype) {
    case DA_F32: return launch_for<DA_F32>(p, grid, stream);
    case DA_BF16: return launch_for<DA_BF16>(p, grid, stream);
    case DA_F16: return launch_for<DA_F16>(p, grid, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace da
