// Host-side work scheduling: how the cached tokens of every request are cut into MicroAttention splits.
#pragma once
#include <stdint.h>

#include <vector>

#include "../../include/distattn.h"

namespace da {

constexpr int kTileTokens = 32;  // scheduling granule: splits start and end on 32-token tiles of a block

struct Schedule {
    int32_t kernel = DA_KERNEL_VALU;  // da_kernel actually used
    int32_t head_tile = 1;            // q-heads served by one work item
    int32_t head_tiles = 1;           // work items per (split, kv-head)
    int32_t waves = 8;                // wavefronts per MicroAttention workgroup
    int32_t fixed_split_tiles = 0;    // > 0: every split is this many tiles (last one shorter); 0: balanced cut
    int32_t max_nsplits = 1;
    int32_t grid = 1;                 // persistent workgroups of the MicroAttention launch
    int64_t num_items = 0;
    int64_t num_partials = 0;
    std::vector<int32_t> ntiles;       // [B] by request id: tiles holding valid tokens
    std::vector<int32_t> nsplits;      // [B] by request id, >= 1
    std::vector<int32_t> order;        // [B] request ids, largest items first
    std::vector<int32_t> item_prefix;  // [B+1] over `order`
    std::vector<int64_t> row_base;     // [B] by request id
};

// Validates `problem` (DA_ERR_INVALID_ARG / DA_ERR_UNSUPPORTED) without touching the GPU.
da_status validate_problem(const da_problem &problem);

// Tiles of a request of L tokens: whole blocks hold ceil(T / 32) tiles, the last block only those with valid tokens.
int64_t tiles_of(int64_t L, int32_t block_tokens);
// First token of tile t.
int64_t tile_first_token(int64_t t, int32_t block_tokens);
// Split j of a request with nt tiles and ns splits covers tiles [first, last).
void split_tiles(int64_t nt, int32_t ns, int32_t fixed_split_tiles, int32_t j, int64_t *first, int64_t *last);

// Fills `s` for the given lengths.  num_cus > 0.
da_status make_schedule(const da_problem &problem, const int32_t *seq_lens_host, const da_tuning &tuning,
                        int32_t num_cus, Schedule &s);

}  // namespace da
