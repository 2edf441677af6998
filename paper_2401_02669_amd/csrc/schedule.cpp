// Work scheduling for DistAttention decode (host arithmetic only).
//
// Section 5.3, Eq. 5 prices attention by the total number of cached tokens, and Section 3 allows a
// sequence to be partitioned at any length.  So the unit of balance is the token, not the request:
// each request's blocks are cut into nsplits near-equal runs, every (run, kv-head, head tile) is one
// work item of the MicroAttention launch, and items are issued longest request first so that the
// last items to start are the shortest.
#include "schedule.h"

#include <algorithm>
#include <cmath>
#include <numeric>

namespace da {

namespace {
constexpr int kResidentGroupsPerCu = 2;  // 8-wave MicroAttention workgroups resident per compute unit
constexpr int kItemsPerSlot = 32;        // wanted items per resident workgroup: keeps the tail short
constexpr double kPartialBudget = 0.015; // partial write + read traffic allowed, relative to KV bytes
}

da_status validate_problem(const da_problem &p)
{
    if (p.batch < 1 || p.num_q_heads < 1 || p.num_kv_heads < 1 || p.max_blocks_per_seq < 1 ||
        p.num_phys_blocks < 1 || p.block_tokens < 1 || p.head_dim < 1)
        return DA_ERR_INVALID_ARG;
    if (p.num_q_heads % p.num_kv_heads != 0) return DA_ERR_INVALID_ARG;
    if (!std::isfinite(p.scale)) return DA_ERR_INVALID_ARG;
    if ((p.kv_dtype != DA_F32 && p.kv_dtype != DA_BF16) || (p.q_dtype != DA_F32 && p.q_dtype != DA_BF16))
        return DA_ERR_UNSUPPORTED;
    if (p.head_dim != 128) return DA_ERR_UNSUPPORTED;
    if (p.block_tokens % 16 != 0) return DA_ERR_UNSUPPORTED;
    if (p.num_q_heads / p.num_kv_heads > 64) return DA_ERR_UNSUPPORTED;
    const int64_t esize = p.kv_dtype == DA_BF16 ? 2 : 4;
    if (p.kv_token_stride < p.head_dim || p.kv_head_stride < 0 || p.kv_block_stride < 0) return DA_ERR_INVALID_ARG;
    if ((p.kv_token_stride * esize) % 16 || (p.kv_head_stride * esize) % 16 || (p.kv_block_stride * esize) % 16)
        return DA_ERR_INVALID_ARG;
    if ((int64_t)p.max_blocks_per_seq * p.block_tokens > INT32_MAX) return DA_ERR_INVALID_ARG;
    return DA_OK;
}

da_status make_schedule(const da_problem &p, const int32_t *seq_lens_host, const da_tuning &tuning,
                        int32_t num_cus, Schedule &s)
{
    da_status st = validate_problem(p);
    if (st != DA_OK) return st;
    if (!seq_lens_host || num_cus < 1) return DA_ERR_INVALID_ARG;
    if (tuning.blocks_per_split < 0 || tuning.kernel < DA_KERNEL_AUTO || tuning.kernel > DA_KERNEL_MFMA)
        return DA_ERR_INVALID_ARG;

    const int B = p.batch, T = p.block_tokens;
    const int G = p.num_q_heads / p.num_kv_heads;

    // kernel family and head tile
    int kernel = tuning.kernel;
    const bool mfma_ok = p.kv_dtype == DA_BF16 && p.q_dtype == DA_BF16;
    if (kernel == DA_KERNEL_AUTO) kernel = (G > 1 && mfma_ok) ? DA_KERNEL_MFMA : DA_KERNEL_VALU;
    if (kernel == DA_KERNEL_MFMA && !mfma_ok) return DA_ERR_UNSUPPORTED;
    s.kernel = kernel;
    if (kernel == DA_KERNEL_MFMA) {
        s.head_tile = 16;
    } else {
        s.head_tile = 1;
        while (s.head_tile < G && s.head_tile < 8) s.head_tile *= 2;
    }
    s.head_tiles = (G + s.head_tile - 1) / s.head_tile;

    // blocks per request
    std::vector<int64_t> nb(B);
    int64_t total_blocks = 0;
    for (int r = 0; r < B; ++r) {
        int64_t L = seq_lens_host[r];
        if (L < 0) return DA_ERR_INVALID_ARG;
        if (L > (int64_t)p.max_blocks_per_seq * T) return DA_ERR_INVALID_ARG;
        nb[r] = (L + T - 1) / T;
        total_blocks += nb[r];
    }

    // run length: long enough that partial traffic stays inside its budget, short enough that
    // every resident workgroup sees many items
    int64_t bps = tuning.blocks_per_split;
    if (bps == 0) {
        const double esize = p.kv_dtype == DA_BF16 ? 2.0 : 4.0;
        const int heads_per_item = std::min(G, s.head_tile);
        const double partial_bytes = 2.0 * heads_per_item * (p.head_dim + 2) * 4.0;
        const double token_bytes = 2.0 * p.head_dim * esize;
        const int64_t min_tokens = (int64_t)std::ceil(partial_bytes / (kPartialBudget * token_bytes));
        const int64_t bps_min = std::max<int64_t>(1, (min_tokens + T - 1) / T);
        const int64_t units = total_blocks * p.num_kv_heads * s.head_tiles;
        const int64_t want_items = (int64_t)num_cus * kResidentGroupsPerCu * kItemsPerSlot;
        const int64_t bps_fill = std::max<int64_t>(1, units / want_items);
        // a nearly idle GPU (few units) prefers parallelism over partial traffic
        bps = units < (int64_t)num_cus * kResidentGroupsPerCu * 4 ? 1 : std::max(bps_min, std::min(bps_fill, 4 * bps_min));
    }
    s.blocks_per_split = (int32_t)std::min<int64_t>(bps, INT32_MAX);

    s.nblocks.resize(B);
    for (int r = 0; r < B; ++r) s.nblocks[r] = (int32_t)nb[r];
    s.nsplits.assign(B, 1);
    s.row_base.assign(B, 0);
    s.max_nsplits = 1;
    int64_t rows = 0;
    for (int r = 0; r < B; ++r) {
        const int64_t n = std::max<int64_t>(1, (nb[r] + bps - 1) / bps);
        s.nsplits[r] = (int32_t)n;
        s.max_nsplits = std::max<int32_t>(s.max_nsplits, (int32_t)n);
        s.row_base[r] = rows;
        rows += n * p.num_q_heads;
    }
    s.num_partials = rows;

    s.order.resize(B);
    std::iota(s.order.begin(), s.order.end(), 0);
    std::stable_sort(s.order.begin(), s.order.end(), [&](int a, int b) { return nb[a] > nb[b]; });
    s.item_prefix.assign(B + 1, 0);
    int64_t items = 0;
    for (int i = 0; i < B; ++i) {
        s.item_prefix[i] = (int32_t)items;
        items += (int64_t)s.nsplits[s.order[i]] * p.num_kv_heads * s.head_tiles;
        if (items > INT32_MAX) return DA_ERR_UNSUPPORTED;
    }
    s.item_prefix[B] = (int32_t)items;
    s.num_items = items;
    return DA_OK;
}

}  // namespace da
