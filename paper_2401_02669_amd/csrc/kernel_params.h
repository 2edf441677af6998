// Arguments shared by the MicroAttention and aggregation kernels (device side of the C ABI).
#pragma once
#include <stdint.h>

namespace da {

constexpr int kHeadDim = 128;    // only head_dim supported
constexpr int kTile = 32;        // scheduling granule in tokens: splits begin and end on tiles of a block

// One split of one request (host-made, 32 bytes: one scalar load on the device).
struct SplitEntry {
    int32_t r;         // request
    int32_t j;         // split index inside the request
    int32_t t0, t1;    // tiles [t0, t1) of the request
    int32_t ns;        // splits of the request
    int32_t pad;
    int64_t row_base;  // first partial row of the request
};

// Small schedules travel inside the kernel arguments instead of through device tables, which saves
// the table upload (a copy engine round trip on the stream) on every re-plan.
constexpr int kInlineEntries = 96;
constexpr int kInlineRuns = 64;
constexpr int kInlineBatch = 64;

// One MicroAttention launch.  A work item is a (split, kv-head, head tile): the split's tokens are
// read once and serve the head tile's q-heads.  The launch is persistent: workgroup b reads, for
// (kv-head, head tile) number b % per_split, the splits entries[range_start[m] .. range_start[m+1])
// with m = b / per_split, one after the other.
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
    const SplitEntry *entries;   // every split of every request, in reading order; null: inline_entries
    const int32_t *range_start;  // [ranges + 1]; null: inline_range_start
    int32_t *err_flag;
    int32_t B, Hq, Hkv, G, T, max_blocks, num_phys;
    int32_t head_tile;          // columns served per work item
    int32_t head_tiles;         // ceil(cols / head_tile)
    int32_t q_dtype;            // da_dtype of q
    int32_t kv_dtype;           // da_dtype of the pools
    int32_t direct_out;
    int32_t wave_items;         // each wavefront takes whole splits of the run (runs of many short splits)
    int32_t per_split;          // Hkv * head_tiles
    int32_t q_len;              // query tokens per request
    int32_t cols;               // (query token, q-head) columns per kv-head: q_len * G
    int64_t stride_block, stride_head, stride_token;  // elements
    float scale_log2e;          // scale * log2(e): scores are kept in base-2 units inside the kernels
    int32_t inline_range_start[kInlineRuns + 1];
    SplitEntry inline_entries[kInlineEntries];
};

constexpr int kMaxPartialSets = 4;

// Partials of one MicroAttention launch (one KV share of the batch) as the aggregation reads them.
struct PartialSet {
    const float *part_o;
    const float *part_m;
    const float *part_e;
    const int32_t *nsplits;   // [B] of the plan that made them; null: CombineParams::inline_* of this set
    const int64_t *row_base;  // [B]
};

struct CombineParams {
    PartialSet set[kMaxPartialSets];
    int32_t num_sets;
    float *out;
    float *lse;  // may be null
    int32_t B, Hq;  // Hq counts virtual heads (q_len * num_q_heads)
    int32_t skip_single;  // requests with one split were already normalised by the MicroAttention kernel
    int32_t col_slices;   // workgroups per (request, q-head), each owning 128 / col_slices columns
    int32_t inline_nsplits[kMaxPartialSets][kInlineBatch];
    int64_t inline_row_base[kMaxPartialSets][kInlineBatch];
};

}  // namespace da
