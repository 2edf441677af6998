// Aggregation of MicroAttention partials (Section 4, m_g / e_g equation and Eq. 3).
//
// One workgroup of 256 threads per (request, q-head, column slice).  Pass 1 finds m_g over the
// partial maxima; pass 2 accumulates e_j w_j and MA_j w_j with w_j = exp(m_j - m_g), rows spread
// over the thread rows of the workgroup, float4 columns over its thread columns.  The partials may
// come in several sets (one per KV share of the batch, e.g. local and remote blocks of a request);
// the sum runs over all of them.
#include <hip/hip_runtime.h>

#include <cstddef>

#include "kernel_params.h"

namespace da {
namespace {

constexpr int kCombineThreads = 256;
constexpr float kNegInf = -__builtin_inff();

// SLICES in {1, 4}: SLICES == 1 -> 32 float4 columns x 8 rows; SLICES == 4 -> 8 float4 columns x 32 rows.
template <int SLICES>
__global__ __launch_bounds__(kCombineThreads) void combine_kernel(const CombineParams p)
{
    constexpr int COLS4 = (kHeadDim / 4) / SLICES;   // float4 columns per workgroup
    constexpr int ROWS = kCombineThreads / COLS4;    // partial rows in flight per step
    __shared__ float red[kCombineThreads / 64];
    __shared__ float4 acc_lds[ROWS][COLS4];
    __shared__ float e_lds[ROWS];

    const int tid = threadIdx.x;
    const int pair = blockIdx.x / SLICES;
    const int slice = blockIdx.x % SLICES;
    const int r = pair / p.Hq;
    const int h = pair % p.Hq;
    // per-set split count and first partial row of request r (a set may carry them in the kernel arguments)
    int ns_of[kMaxPartialSets];
    int64_t base_of[kMaxPartialSets];
    int total = 0;
#pragma unroll
    for (int s = 0; s < kMaxPartialSets; ++s) {
        ns_of[s] = 0;
        base_of[s] = 0;
        if (s < p.num_sets) {
            if (p.set[s].nsplits == nullptr) {
                // read from the kernel-argument segment itself (CombineParams is the only argument)
                typedef const char __attribute__((address_space(4))) * kernarg_ptr;
                const kernarg_ptr ka = (kernarg_ptr)__builtin_amdgcn_kernarg_segment_ptr();
                ns_of[s] = ((const int32_t __attribute__((address_space(4))) *)(ka + offsetof(CombineParams, inline_nsplits)))[s * kInlineBatch + r];
                base_of[s] = ((const int64_t __attribute__((address_space(4))) *)(ka + offsetof(CombineParams, inline_row_base)))[s * kInlineBatch + r];
            } else {
                ns_of[s] = p.set[s].nsplits[r];
                base_of[s] = p.set[s].row_base[r];
            }
        }
        total += ns_of[s];
    }
    if (p.skip_single && p.num_sets == 1 && total == 1) return;

    // pass 1: m_g
    float mg = kNegInf;
#pragma unroll
    for (int s = 0; s < kMaxPartialSets; ++s) {
        if (s >= p.num_sets) break;
        const int ns = ns_of[s];
        const float *pm = p.set[s].part_m + base_of[s] + (int64_t)h * ns;
        for (int j = tid; j < ns; j += kCombineThreads) mg = fmaxf(mg, pm[j]);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mg = fmaxf(mg, __shfl_xor(mg, off));
    if ((tid & 63) == 0) red[tid >> 6] = mg;
    __syncthreads();
    mg = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float mu = (mg == kNegInf) ? 0.0f : mg;

    // pass 2: weighted sums
    const int c4 = tid % COLS4;
    const int rw = tid / COLS4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float eg = 0.0f;
#pragma unroll
    for (int s = 0; s < kMaxPartialSets; ++s) {
        if (s >= p.num_sets) break;
        const int ns = ns_of[s];
        const int64_t row0 = base_of[s] + (int64_t)h * ns;
        const float *pm = p.set[s].part_m + row0;
        const float *pe = p.set[s].part_e + row0;
        const float4 *po = (const float4 *)(p.set[s].part_o + row0 * kHeadDim) + slice * COLS4 + c4;
        for (int j = rw; j < ns; j += ROWS) {
            const float mj = pm[j];
            const float w = (mj == kNegInf) ? 0.0f : __expf(mj - mu);
            const float4 v = po[(int64_t)j * (kHeadDim / 4)];
            eg = fmaf(pe[j], w, eg);
            acc.x = fmaf(v.x, w, acc.x);
            acc.y = fmaf(v.y, w, acc.y);
            acc.z = fmaf(v.z, w, acc.z);
            acc.w = fmaf(v.w, w, acc.w);
        }
    }
    acc_lds[rw][c4] = acc;
    if (c4 == 0) e_lds[rw] = eg;
    __syncthreads();
    if (tid < COLS4) {
        float4 a = acc_lds[0][tid];
        float e = e_lds[0];
        for (int i = 1; i < ROWS; ++i) {
            const float4 b = acc_lds[i][tid];
            a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
            e += e_lds[i];
        }
        const bool live = e > 0.0f;
        const float inv = live ? 1.0f / e : 0.0f;
        float4 o = live ? make_float4(a.x * inv, a.y * inv, a.z * inv, a.w * inv) : make_float4(0.f, 0.f, 0.f, 0.f);
        ((float4 *)(p.out + (int64_t)pair * kHeadDim))[slice * COLS4 + tid] = o;
        if (p.lse && slice == 0 && tid == 0) p.lse[pair] = live ? mg + __logf(e) : kNegInf;
    }
}

}  // namespace

hipError_t launch_combine(const CombineParams &p, hipStream_t stream)
{
    const int64_t pairs = (int64_t)p.B * p.Hq;
    if (pairs <= 0) return hipSuccess;
    if (p.col_slices == 4)
        hipLaunchKernelGGL(combine_kernel<4>, dim3((unsigned)(pairs * 4)), dim3(kCombineThreads), 0, stream, p);
    else
        hipLaunchKernelGGL(combine_kernel<1>, dim3((unsigned)pairs), dim3(kCombineThreads), 0, stream, p);
    return hipGetLastError();
}

}  // namespace da
