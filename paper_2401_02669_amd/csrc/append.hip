// KV append: the K and V rows of one newly generated token per request join the paged block layout
// (Section 4: the cache is sliced along the sequence dimension so that new tokens are grouped into
// the sub-blocks as they are produced).
//
// One workgroup per request: wavefront w copies kv-heads w, w + 4, ...; inside a wavefront lanes
// 0..31 carry the K row and lanes 32..63 the V row, 16 bytes per lane.  The request's length is read
// once by every thread before a barrier and incremented by one thread after it.
#include <hip/hip_runtime.h>

#include "../../include/distattn.h"
#include "kernel_params.h"

namespace da {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct AppendParams {
    const char *k_new;
    const char *v_new;
    char *k_pool;
    char *v_pool;
    const int32_t *block_table;
    int32_t *seq_lens;
    int32_t *err_flags;  // may be null
    int32_t Hkv, T, max_blocks, num_phys;
    int32_t row_bytes;   // head_dim * element size: 256 or 512
    int64_t stride_block_b, stride_head_b, stride_token_b;  // bytes
};

__global__ __launch_bounds__(256) void append_kernel(const AppendParams p)
{
    const int r = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int L = p.seq_lens[r];
    __syncthreads();  // every thread holds L before anyone may change it
    if (L < 0) return;  // inactive slot
    const int blk = L / p.T, slot = L - blk * p.T;
    int err = 0;
    int pb = 0;
    if (blk >= p.max_blocks) {
        err = 2;  // the block table row is full
    } else {
        pb = p.block_table[(int64_t)r * p.max_blocks + blk];
        if ((unsigned)pb >= (unsigned)p.num_phys) err = 1;  // no valid block for this position
    }
    if (err) {
        if (threadIdx.x == 0 && p.err_flags) atomicOr(p.err_flags, err);
        return;
    }
    const int chunks = p.row_bytes >> 4;  // 16-byte pieces of a row: 16 (bf16) or 32 (fp32)
    const bool is_v = lane >= 32;
    const int piece = lane & 31;
    if (piece < chunks) {
        const char *src = is_v ? p.v_new : p.k_new;
        char *pool = is_v ? p.v_pool : p.k_pool;
        for (int g = wave; g < p.Hkv; g += 4) {
            const u32x4 v = *(const u32x4 *)(src + ((int64_t)r * p.Hkv + g) * p.row_bytes + piece * 16);
            *(u32x4 *)(pool + (int64_t)pb * p.stride_block_b + (int64_t)g * p.stride_head_b +
                       (int64_t)slot * p.stride_token_b + piece * 16) = v;
        }
    }
    if (threadIdx.x == 0) p.seq_lens[r] = L + 1;
}

}  // namespace
}  // namespace da

extern "C" da_status da_append(const da_problem *problem, const void *k_new, const void *v_new, void *k_pool,
                               void *v_pool, const int32_t *block_table, int32_t *seq_lens, int32_t *err_flags,
                               void *stream)
{
    if (!problem || !k_new || !v_new || !k_pool || !v_pool || !block_table || !seq_lens) return DA_ERR_INVALID_ARG;
    const da_problem &q = *problem;
    if (q.batch < 1 || q.num_kv_heads < 1 || q.block_tokens < 1 || q.max_blocks_per_seq < 1 || q.num_phys_blocks < 1)
        return DA_ERR_INVALID_ARG;
    if (q.head_dim != 128 || (q.kv_dtype < DA_F32 || q.kv_dtype > DA_F16)) return DA_ERR_UNSUPPORTED;
    const int64_t esize = q.kv_dtype == DA_F32 ? 4 : 2;
    if (q.kv_token_stride < q.head_dim || q.kv_head_stride < 0 || q.kv_block_stride < 0) return DA_ERR_INVALID_ARG;
    if ((q.kv_token_stride * esize) % 16 || (q.kv_head_stride * esize) % 16 || (q.kv_block_stride * esize) % 16)
        return DA_ERR_INVALID_ARG;
    if (((uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)k_pool | (uintptr_t)v_pool) & 15) return DA_ERR_INVALID_ARG;
    da::AppendParams p;
    p.k_new = (const char *)k_new;
    p.v_new = (const char *)v_new;
    p.k_pool = (char *)k_pool;
    p.v_pool = (char *)v_pool;
    p.block_table = block_table;
    p.seq_lens = seq_lens;
    p.err_flags = err_flags;
    p.Hkv = q.num_kv_heads;
    p.T = q.block_tokens;
    p.max_blocks = q.max_blocks_per_seq;
    p.num_phys = q.num_phys_blocks;
    p.row_bytes = (int32_t)(q.head_dim * esize);
    p.stride_block_b = q.kv_block_stride * esize;
    p.stride_head_b = q.kv_head_stride * esize;
    p.stride_token_b = q.kv_token_stride * esize;
    hipLaunchKernelGGL(da::append_kernel, dim3((unsigned)q.batch), dim3(256), 0, (hipStream_t)stream, p);
    return hipGetLastError() == hipSuccess ? DA_OK : DA_ERR_HIP;
}
