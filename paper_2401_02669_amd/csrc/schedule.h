// Host-side work scheduling: how the KV blocks of every request are cut into MicroAttention splits.
#pragma once
#include <stdint.h>

#include <vector>

#include "../../include/distattn.h"

namespace da {

struct Schedule {
    int32_t kernel = DA_KERNEL_VALU;  // da_kernel actually used
    int32_t head_tile = 1;            // q-heads served by one work item
    int32_t head_tiles = 1;           // work items per (split, kv-head)
    int32_t blocks_per_split = 1;     // target run length in blocks
    int32_t max_nsplits = 1;
    int64_t num_items = 0;
    int64_t num_partials = 0;
    std::vector<int32_t> nblocks;      // [B] by request id: ceil(len / block_tokens)
    std::vector<int32_t> nsplits;      // [B] by request id, >= 1
    std::vector<int32_t> order;        // [B] request ids, longest first
    std::vector<int32_t> item_prefix;  // [B+1] over `order`
    std::vector<int64_t> row_base;     // [B] by request id
};

// Validates `problem` (DA_ERR_INVALID_ARG / DA_ERR_UNSUPPORTED) without touching the GPU.
da_status validate_problem(const da_problem &problem);

// Fills `s` for the given lengths.  num_cus > 0.
da_status make_schedule(const da_problem &problem, const int32_t *seq_lens_host, const da_tuning &tuning,
                        int32_t num_cus, Schedule &s);

}  // namespace da
