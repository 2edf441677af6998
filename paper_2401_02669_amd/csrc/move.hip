// KV block movement: whole blocks of K and V go from one pair of pools to another (Section 5.3, move_kvcache of
// Algorithm 1; Section 5.2: a debtor places part of a request's KV cache in a creditor's memory, and the copy runs
// beside the model's own work).
//
// A workgroup copies 64 token rows of one (block pair, kv-head), K and V, 16 bytes per lane: a row is 16 (bf16) or
// 32 (fp32) lanes wide, so a 256-thread pass covers 16 or 8 rows.  Pure copy, bound by HBM read + write.
#include <hip/hip_runtime.h>

#include "../../include/distattn.h"

namespace da {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMoveRows = 64;  // token rows per workgroup

struct MoveParams {
    const char *k_src;
    const char *v_src;
    char *k_dst;
    char *v_dst;
    const int32_t *src_ids;
    const int32_t *dst_ids;
    int32_t *err_flags;  // may be null
    int32_t Hkv, T, num_src, num_dst;
    int32_t lanes_per_row;  // row bytes / 16
    int64_t src_block_b, src_head_b, src_token_b;  // byte strides
    int64_t dst_block_b, dst_head_b, dst_token_b;
};

__global__ __launch_bounds__(256) void move_blocks_kernel(const MoveParams p)
{
    const int pair = blockIdx.x / p.Hkv;
    const int g = blockIdx.x - pair * p.Hkv;
    const int a = p.src_ids[pair], b = p.dst_ids[pair];
    if ((unsigned)a >= (unsigned)p.num_src || (unsigned)b >= (unsigned)p.num_dst) {
        if (threadIdx.x == 0 && g == 0 && blockIdx.y == 0 && p.err_flags) atomicOr(p.err_flags, 1);
        return;
    }
    const int piece = threadIdx.x % p.lanes_per_row;
    const int row_in_pass = threadIdx.x / p.lanes_per_row;
    const int rows_per_pass = 256 / p.lanes_per_row;
    const int64_t src0 = (int64_t)a * p.src_block_b + (int64_t)g * p.src_head_b + piece * 16;
    const int64_t dst0 = (int64_t)b * p.dst_block_b + (int64_t)g * p.dst_head_b + piece * 16;
    const int s_end = min(p.T, (int)(blockIdx.y + 1) * kMoveRows);
    for (int s = blockIdx.y * kMoveRows + row_in_pass; s < s_end; s += rows_per_pass) {
        const int64_t from = src0 + (int64_t)s * p.src_token_b, to = dst0 + (int64_t)s * p.dst_token_b;
        const u32x4 k = *(const u32x4 *)(p.k_src + from);
        const u32x4 v = *(const u32x4 *)(p.v_src + from);
        *(u32x4 *)(p.k_dst + to) = k;
        *(u32x4 *)(p.v_dst + to) = v;
    }
}

bool layout_ok(const da_problem &q, int64_t esize)
{
    if (q.num_kv_heads < 1 || q.block_tokens < 1 || q.num_phys_blocks < 1) return false;
    if (q.kv_token_stride < q.head_dim || q.kv_head_stride < 0 || q.kv_block_stride < 0) return false;
    return !((q.kv_token_stride * esize) % 16 || (q.kv_head_stride * esize) % 16 || (q.kv_block_stride * esize) % 16);
}

}  // namespace
}  // namespace da

extern "C" da_status da_move_blocks(const da_problem *src_layout, const da_problem *dst_layout, const void *k_src,
                                    const void *v_src, void *k_dst, void *v_dst, const int32_t *src_ids,
                                    const int32_t *dst_ids, int32_t num_blocks, int32_t *err_flags, void *stream)
{
    if (!src_layout || !dst_layout || !k_src || !v_src || !k_dst || !v_dst || num_blocks < 0) return DA_ERR_INVALID_ARG;
    if (num_blocks > 0 && (!src_ids || !dst_ids)) return DA_ERR_INVALID_ARG;
    const da_problem &a = *src_layout, &b = *dst_layout;
    if (a.head_dim != 128 || b.head_dim != 128) return DA_ERR_UNSUPPORTED;
    if (a.kv_dtype < DA_F32 || a.kv_dtype > DA_F16) return DA_ERR_UNSUPPORTED;
    if (a.kv_dtype != b.kv_dtype || a.num_kv_heads != b.num_kv_heads || a.block_tokens != b.block_tokens)
        return DA_ERR_INVALID_ARG;
    const int64_t esize = a.kv_dtype == DA_F32 ? 4 : 2;
    if (!da::layout_ok(a, esize) || !da::layout_ok(b, esize)) return DA_ERR_INVALID_ARG;
    if (((uintptr_t)k_src | (uintptr_t)v_src | (uintptr_t)k_dst | (uintptr_t)v_dst) & 15) return DA_ERR_INVALID_ARG;
    if (num_blocks == 0) return DA_OK;
    if ((int64_t)num_blocks * a.num_kv_heads > 0x7fffffffLL) return DA_ERR_INVALID_ARG;
    da::MoveParams p;
    p.k_src = (const char *)k_src;
    p.v_src = (const char *)v_src;
    p.k_dst = (char *)k_dst;
    p.v_dst = (char *)v_dst;
    p.src_ids = src_ids;
    p.dst_ids = dst_ids;
    p.err_flags = err_flags;
    p.Hkv = a.num_kv_heads;
    p.T = a.block_tokens;
    p.num_src = a.num_phys_blocks;
    p.num_dst = b.num_phys_blocks;
    p.lanes_per_row = (int32_t)(a.head_dim * esize / 16);
    p.src_block_b = a.kv_block_stride * esize;
    p.src_head_b = a.kv_head_stride * esize;
    p.src_token_b = a.kv_token_stride * esize;
    p.dst_block_b = b.kv_block_stride * esize;
    p.dst_head_b = b.kv_head_stride * esize;
    p.dst_token_b = b.kv_token_stride * esize;
    const dim3 grid((unsigned)(num_blocks * a.num_kv_heads), (unsigned)((a.block_tokens + da::kMoveRows - 1) / da::kMoveRows));
    hipLaunchKernelGGL(da::move_blocks_kernel, grid, dim3(256), 0, (hipStream_t)stream, p);
    return hipGetLastError() == hipSuccess ? DA_OK : DA_ERR_HIP;
}
