// Arguments shared by the MicroAttention and aggregation kernels (device side of the C ABI).
#pragma once
#include <stdint.h>

namespace da {

constexpr int kHeadDim = 128;    // only head_dim supported
constexpr int kTile = 32;        // scheduling granule in tokens: splits begin and end on tiles of a block

// One MicroAttention launch.  A work item is a (request, split, kv-head, head tile): the split's
// tokens are read once and serve the head tile's q-heads.  The launch is persistent: workgroup b
// handles items b, b + gridDim.x, ... (odd rounds mirrored) of the item list.
struct MicroParams {
    const void *q;
    const void *k_pool;
    const void *v_pool;
    const int32_t *block_table;
    const int32_t *seq_lens;
    float *part_o;
    float *part_m;
    float *part_e;
    float *out;  // used only for requests with one split when direct_out != 0
    float *lse;  // may be null
    const int32_t *order;        // [B] request ids, processing order
    const int32_t *item_prefix;  // [B+1] first work item of order[i]
    const int32_t *nsplits;      // [B] by request id
    const int64_t *row_base;     // [B] by request id: first partial row of the request
    int32_t *err_flag;
    int32_t B, Hq, Hkv, G, T, max_blocks, num_phys;
    int32_t head_tile;          // q-heads served per work item
    int32_t head_tiles;         // ceil(G / head_tile)
    int32_t q_bf16;
    int32_t direct_out;
    int32_t num_items;
    int32_t fixed_split_tiles;  // > 0: split j = tiles [j*f, (j+1)*f); 0: split j = tiles [j*nt/ns, (j+1)*nt/ns)
    int64_t stride_block, stride_head, stride_token;  // elements
    float scale_log2e;          // scale * log2(e): scores are kept in base-2 units inside the kernels
};

struct CombineParams {
    const float *part_o;
    const float *part_m;
    const float *part_e;
    float *out;
    float *lse;  // may be null
    const int32_t *nsplits;
    const int64_t *row_base;
    int32_t B, Hq;
    int32_t skip_single;  // requests with one split were already normalised by the MicroAttention kernel
    int32_t col_slices;   // workgroups per (request, q-head), each owning 128 / col_slices columns
};

}  // namespace da
