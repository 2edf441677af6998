// MicroAttention on the fp32 vector ALU (Section 4, m_j / e_j equation and Eq. 2).
//
// One workgroup (8 wavefronts) owns one work item: a run of KV blocks of one (request, kv-head)
// and up to GT q-heads of that kv-head's group.  A wavefront load instruction fetches 1 KiB of
// consecutive K (or V) bytes: RPL whole token rows, LPR lanes per row, 16 bytes per lane.  Each
// lane multiplies its 16-byte slice with the matching slice of q; a DPP all-reduce over the LPR
// lanes of the row yields the score.  Every row position of every wavefront keeps its own running
// (m, e, o) in base-2 units; they are merged once, at the end of the item.
#include <hip/hip_runtime.h>

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

template <bool BF16>
struct Slice;  // a lane's 16 bytes of one token row
template <>
struct Slice<true> {
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
struct Slice<false> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void unpack(const u32x4 &r, float (&f)[4])
    {
        f[0] = as_f(r.x); f[1] = as_f(r.y); f[2] = as_f(r.z); f[3] = as_f(r.w);
    }
};

constexpr float kNegInf = -__builtin_inff();
constexpr float kLn2 = 0.69314718055994530942f;

// KVBF16: K/V storage is bf16 (else fp32).  GT: q-heads per item.  NL: load instructions per chunk.
template <bool KVBF16, int GT, int NL>
__global__ __launch_bounds__(kThreads) void micro_attention_valu_kernel(const MicroParams p)
{
    constexpr int EPL = Slice<KVBF16>::N;  // elements per lane
    constexpr int LPR = kHeadDim / EPL;    // lanes per token row: 16 (bf16) or 32 (fp32)
    constexpr int RPL = 64 / LPR;          // token rows per load instruction: 4 or 2
    constexpr int CH = NL * RPL;           // tokens per chunk
    constexpr int ESIZE = KVBF16 ? 2 : 4;

    __shared__ float lds_m[kWavesPerGroup][GT];
    __shared__ float lds_e[kWavesPerGroup][GT];
    __shared__ float lds_o[kWavesPerGroup][GT][kHeadDim];

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int row = lane / LPR;   // token row inside a load
    const int colc = lane % LPR;  // 16-byte column chunk

    // ---- which work item -------------------------------------------------------------------
    const int item = blockIdx.x;
    int lo = 0, hi = p.B;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (p.item_prefix[mid] <= item) lo = mid; else hi = mid;
    }
    const int r = p.order[lo];
    const int local = item - p.item_prefix[lo];
    const int ns = p.nsplits[r];
    const int per_split = p.Hkv * p.head_tiles;
    const int j = local / per_split;
    const int rem = local - j * per_split;
    const int kvh = rem / p.head_tiles;
    const int ht = rem - kvh * p.head_tiles;

    const int T = p.T;
    int L = p.seq_lens[r];
    L = L < 0 ? 0 : L;
    const int64_t cap = (int64_t)p.max_blocks * T;
    if ((int64_t)L > cap) L = (int)cap;
    const int nb = (L + T - 1) / T;
    const int b0 = (int)(((int64_t)j * nb) / ns);
    const int b1 = (int)(((int64_t)(j + 1) * nb) / ns);

    // ---- q slice of this lane, pre-scaled to base-2 units -----------------------------------
    float qf[GT][EPL];
#pragma unroll
    for (int g = 0; g < GT; ++g) {
        const int hl = ht * GT + g;
        const bool live = hl < p.G;
        const int64_t qoff = ((int64_t)r * p.Hq + (int64_t)kvh * p.G + (live ? hl : 0)) * kHeadDim + colc * EPL;
#pragma unroll
        for (int c = 0; c < EPL; ++c) {
            float x;
            if (p.q_bf16)
                x = as_f((uint32_t)((const uint16_t *)p.q)[qoff + c] << 16);
            else
                x = ((const float *)p.q)[qoff + c];
            qf[g][c] = live ? x * p.scale_log2e : 0.0f;
        }
    }

    float m[GT], e[GT], o[GT][EPL];
#pragma unroll
    for (int g = 0; g < GT; ++g) {
        m[g] = kNegInf;
        e[g] = 0.0f;
#pragma unroll
        for (int c = 0; c < EPL; ++c) o[g][c] = 0.0f;
    }

    // ---- chunk walk: chunk n of the split = block b0 + n / cpb, position n % cpb ---------------
    const int cpb = (T + CH - 1) / CH;
    const int nchunks = (b1 - b0) * cpb;
    const char *kbase = (const char *)p.k_pool;
    const char *vbase = (const char *)p.v_pool;
    const int64_t lane_off = ((int64_t)row * p.stride_token + colc * EPL) * ESIZE;
    const int64_t load_step = (int64_t)RPL * p.stride_token * ESIZE;

    struct Chunk {
        int n, blk, cib;   // chunk number, logical block, chunk inside the block
        int lim;           // valid tokens from the chunk's first row on (<= 0: none)
        int64_t off;       // byte offset of (row 0, column 0) of this lane's first load
    };
    auto locate = [&](Chunk &c) {
        c.lim = 0;
        c.off = 0;
        if (c.n >= nchunks) return;
        const int pb = p.block_table[(int64_t)r * p.max_blocks + c.blk];
        const int first = c.cib * CH;
        int valid = L - c.blk * T;
        valid = (valid > T ? T : valid) - first;
        if ((unsigned)pb >= (unsigned)p.num_phys) {
            if (lane == 0) atomicOr(p.err_flag, 1);
            valid = 0;
        }
        c.lim = valid;
        c.off = ((int64_t)pb * p.stride_block + (int64_t)kvh * p.stride_head + (int64_t)first * p.stride_token) * ESIZE +
                lane_off;
    };
    auto advance = [&](Chunk c) {
        c.n += kWavesPerGroup;
        c.cib += kWavesPerGroup;
        while (c.cib >= cpb) {
            c.cib -= cpb;
            c.blk += 1;
        }
        locate(c);
        return c;
    };
    auto load_rows = [&](const char *base, const Chunk &c, u32x4 (&dst)[NL]) {
#pragma unroll
        for (int jj = 0; jj < NL; ++jj) {
            dst[jj] = u32x4{0u, 0u, 0u, 0u};
            if (jj * RPL + row < c.lim) dst[jj] = load16_stream(base + c.off + jj * load_step);
        }
    };

    Chunk cur;
    cur.n = wave;
    cur.blk = b0 + wave / cpb;
    cur.cib = wave % cpb;
    locate(cur);

    u32x4 kr[NL], vr[NL];
    if (cur.n < nchunks) load_rows(kbase, cur, kr);

    while (cur.n < nchunks) {
        load_rows(vbase, cur, vr);
        const Chunk nxt = advance(cur);

        // scores of the chunk's rows, base-2 units
        float s[NL][GT];
#pragma unroll
        for (int jj = 0; jj < NL; ++jj) {
            float kf[EPL];
            Slice<KVBF16>::unpack(kr[jj], kf);
            const bool valid = jj * RPL + row < cur.lim;
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                float acc = 0.0f;
#pragma unroll
                for (int c = 0; c < EPL; ++c) acc = fmaf(qf[g][c], kf[c], acc);
                acc = (LPR == 16) ? row16_sum(acc) : row32_sum(acc);
                s[jj][g] = valid ? acc : kNegInf;
            }
        }
        if (nxt.n < nchunks) load_rows(kbase, nxt, kr);

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
            Slice<KVBF16>::unpack(vr[jj], vf);
#pragma unroll
            for (int g = 0; g < GT; ++g)
#pragma unroll
                for (int c = 0; c < EPL; ++c) o[g][c] = fmaf(s[jj][g], vf[c], o[g][c]);
        }
        cur = nxt;
    }

    // ---- merge the RPL row positions of the wavefront ------------------------------------------
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
                lds_m[wave][g] = m[g];
                lds_e[wave][g] = e[g];
            }
#pragma unroll
            for (int c = 0; c < EPL; ++c) lds_o[wave][g][colc * EPL + c] = o[g][c];
        }
    }
    __syncthreads();

    // ---- merge the wavefronts and write the item's result -------------------------------------
    const bool direct = p.direct_out && ns == 1;
    for (int idx = tid; idx < GT * kHeadDim; idx += kThreads) {
        const int g = idx / kHeadDim, col = idx % kHeadDim;
        const int hl = ht * GT + g;
        if (hl >= p.G) continue;
        float M = lds_m[0][g];
#pragma unroll
        for (int w = 1; w < kWavesPerGroup; ++w) M = fmaxf(M, lds_m[w][g]);
        const float mu = (M == kNegInf) ? 0.0f : M;
        float acc = 0.0f, E = 0.0f;
#pragma unroll
        for (int w = 0; w < kWavesPerGroup; ++w) {
            const float wgt = fast_exp2(lds_m[w][g] - mu);
            acc = fmaf(lds_o[w][g][col], wgt, acc);
            E = fmaf(lds_e[w][g], wgt, E);
        }
        const int h = kvh * p.G + hl;
        if (direct) {
            const int64_t orow = (int64_t)r * p.Hq + h;
            p.out[orow * kHeadDim + col] = (E > 0.0f) ? acc / E : 0.0f;
            if (col == 0 && p.lse) p.lse[orow] = (E > 0.0f) ? M * kLn2 + __logf(E) : kNegInf;
        } else {
            const int64_t prow = p.row_base[r] + (int64_t)h * ns + j;
            p.part_o[prow * kHeadDim + col] = acc;
            if (col == 0) {
                p.part_m[prow] = M * kLn2;  // back to natural-log units (-inf stays -inf)
                p.part_e[prow] = E;
            }
        }
    }
}

template <bool KVBF16, int GT, int NL>
hipError_t launch_one(const MicroParams &p, int64_t num_items, hipStream_t stream)
{
    hipLaunchKernelGGL((micro_attention_valu_kernel<KVBF16, GT, NL>), dim3((unsigned)num_items), dim3(kThreads), 0, stream, p);
    return hipGetLastError();
}

}  // namespace

// head_tile must be 1, 2, 4 or 8.
hipError_t launch_micro_attention_valu(const MicroParams &p, bool kv_bf16, int64_t num_items, hipStream_t stream)
{
    if (num_items <= 0) return hipSuccess;
    switch (p.head_tile) {
    case 1: return kv_bf16 ? launch_one<true, 1, 8>(p, num_items, stream) : launch_one<false, 1, 8>(p, num_items, stream);
    case 2: return kv_bf16 ? launch_one<true, 2, 8>(p, num_items, stream) : launch_one<false, 2, 8>(p, num_items, stream);
    case 4: return kv_bf16 ? launch_one<true, 4, 4>(p, num_items, stream) : launch_one<false, 4, 4>(p, num_items, stream);
    case 8: return kv_bf16 ? launch_one<true, 8, 2>(p, num_items, stream) : launch_one<false, 8, 2>(p, num_items, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace da
