// Host-side work scheduling: how the cached tokens of every request are cut into MicroAttention splits
// and which persistent workgroup reads which of them.
#pragma once
#include <stdint.h>

#include <vector>

#include "../../include/distattn.h"
#include "kernel_params.h"

namespace da {

constexpr int kTileTokens = 32;  // scheduling granule: splits start and end on 32-token tiles of a block

struct Schedule {
    int32_t kernel = DA_KERNEL_VALU;  // da_kernel actually used
    int32_t head_tile = 1;            // q-heads served by one work item
    int32_t head_tiles = 1;           // work items per (split, kv-head)
    int32_t waves = 4;                // wavefronts per MicroAttention workgroup
    int32_t wave_items = 0;           // 1: each wavefront takes whole splits of its run (many short splits)
    int32_t ranges = 1;               // consecutive runs of splits; range m is read by workgroups m*P .. m*P+P-1
    int32_t grid = 1;                 // workgroups of the MicroAttention launch = ranges * P, P = Hkv * head_tiles
    int32_t max_nsplits = 1;
    int64_t num_items = 0;            // (split, kv-head, head tile) work items
    int64_t num_partials = 0;
    std::vector<int32_t> ntiles;       // [B] tiles holding valid tokens
    std::vector<int32_t> nsplits;      // [B] >= 1
    std::vector<int64_t> row_base;     // [B]
    std::vector<int32_t> first_entry;  // [B] index of the request's split 0 in `entries` (its splits are consecutive)
    std::vector<SplitEntry> entries;   // every split of every request, in reading order
    std::vector<int32_t> range_start;  // [ranges + 1] first entry of each range
};

// Validates `problem` (DA_ERR_INVALID_ARG / DA_ERR_UNSUPPORTED) without touching the GPU.
da_status validate_problem(const da_problem &problem);

// Tiles of a request of L tokens: whole blocks hold ceil(T / 32) tiles, the last block only those with valid tokens.
int64_t tiles_of(int64_t L, int32_t block_tokens);
// First token of tile t.
int64_t tile_first_token(int64_t t, int32_t block_tokens);

// Fills `s` for the given lengths.  num_cus > 0.
da_status make_schedule(const da_problem &problem, const int32_t *seq_lens_host, const da_tuning &tuning,
                        int32_t num_cus, Schedule &s);

}  // namespace da
