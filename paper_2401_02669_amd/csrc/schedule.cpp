// Work scheduling for DistAttention decode (host arithmetic only).
//
// Section 5.3, Eq. 5 prices attention by the total number of cached tokens, and Section 3 allows a
// sequence to be partitioned at any length.  So the unit of balance is the token, not the request or
// the block: every request is cut, on 32-token tile boundaries, into nsplits near-equal splits whose
// size is the same across the whole batch; each (split, kv-head, head tile) is one work item.  The
// MicroAttention launch is persistent: `grid` workgroups (two per compute unit) each take items
// b, b + grid, ... of the size-sorted list, so when the item count is a multiple of the grid every
// workgroup reads the same number of bytes and there is no tail.
#include "schedule.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <numeric>

namespace da {

namespace {
constexpr int kGroupsPerCu = 2;          // persistent MicroAttention workgroups per compute unit
constexpr int kMaxItemsPerGroup = 8;     // more, smaller items only add partial rows
constexpr double kPartialBudget = 0.01;  // partial write + read traffic allowed, relative to KV bytes
}

int64_t tiles_of(int64_t L, int32_t T)
{
    if (L <= 0) return 0;
    const int64_t tpb = (T + kTileTokens - 1) / kTileTokens;
    const int64_t nb = (L + T - 1) / T;
    const int64_t tail = L - (nb - 1) * T;
    return (nb - 1) * tpb + (tail + kTileTokens - 1) / kTileTokens;
}

int64_t tile_first_token(int64_t t, int32_t T)
{
    const int64_t tpb = (T + kTileTokens - 1) / kTileTokens;
    return (t / tpb) * T + (t % tpb) * kTileTokens;
}

void split_tiles(int64_t nt, int32_t ns, int32_t fixed, int32_t j, int64_t *first, int64_t *last)
{
    if (fixed > 0) {
        *first = std::min<int64_t>(nt, (int64_t)j * fixed);
        *last = std::min<int64_t>(nt, (int64_t)(j + 1) * fixed);
    } else {
        *first = (int64_t)j * nt / ns;
        *last = ((int64_t)j + 1) * nt / ns;
    }
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
    if (p.kv_token_stride * esize > (1 << 20)) return DA_ERR_UNSUPPORTED;  // lane offsets are 32-bit
    if ((int64_t)p.max_blocks_per_seq * p.block_tokens > INT32_MAX / 2) return DA_ERR_INVALID_ARG;
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
    const int64_t tpb = (T + kTileTokens - 1) / kTileTokens;

    // kernel family, head tile, workgroup size
    int kernel = tuning.kernel;
    const bool mfma_ok = p.kv_dtype == DA_BF16 && p.q_dtype == DA_BF16;
    if (kernel == DA_KERNEL_AUTO) kernel = (G > 1 && mfma_ok) ? DA_KERNEL_MFMA : DA_KERNEL_VALU;
    if (kernel == DA_KERNEL_MFMA && !mfma_ok) return DA_ERR_UNSUPPORTED;
    s.kernel = kernel;
    if (kernel == DA_KERNEL_MFMA) {
        s.head_tile = 16;
        s.waves = 4;
    } else {
        s.head_tile = 1;
        while (s.head_tile < G && s.head_tile < 8) s.head_tile *= 2;
        s.waves = 4;
    }
    s.head_tiles = (G + s.head_tile - 1) / s.head_tile;
    const int64_t per_split = (int64_t)p.num_kv_heads * s.head_tiles;  // items per (request, split)

    // tiles per request
    s.ntiles.resize(B);
    int64_t total_tiles = 0;
    for (int r = 0; r < B; ++r) {
        const int64_t L = seq_lens_host[r];
        if (L < 0 || L > (int64_t)p.max_blocks_per_seq * T) return DA_ERR_INVALID_ARG;
        s.ntiles[r] = (int32_t)tiles_of(L, T);
        total_tiles += s.ntiles[r];
    }

    const int64_t slots = (int64_t)num_cus * kGroupsPerCu;
    s.nsplits.assign(B, 1);
    s.fixed_split_tiles = 0;
    if (tuning.blocks_per_split > 0) {
        // caller's choice: every split is exactly this many blocks (1 = one partial per block)
        const int64_t fixed = std::min<int64_t>((int64_t)tuning.blocks_per_split * tpb, INT32_MAX);
        s.fixed_split_tiles = (int32_t)fixed;
        for (int r = 0; r < B; ++r) s.nsplits[r] = (int32_t)std::max<int64_t>(1, (s.ntiles[r] + fixed - 1) / fixed);
    } else {
        // item size (tiles), the same for the whole batch: at least one tile per wavefront and enough
        // tokens that the item's partial rows (written once, read once) stay inside their budget;
        // beyond that, at most kMaxItemsPerGroup items per persistent workgroup.
        const double esize = p.kv_dtype == DA_BF16 ? 2.0 : 4.0;
        const int heads_per_item = std::min(G, s.head_tile);
        const double partial_bytes = 2.0 * heads_per_item * (p.head_dim + 2) * 4.0;
        const double tile_bytes = 2.0 * p.head_dim * esize * kTileTokens;
        const int64_t t_min = std::max<int64_t>(s.waves, (int64_t)std::ceil(partial_bytes / (kPartialBudget * tile_bytes)));
        const int64_t units = total_tiles * per_split;  // (tile, kv-head, head tile) units of work
        const int64_t kmax = getenv("DA_EXP_KMAX") ? atoi(getenv("DA_EXP_KMAX")) : kMaxItemsPerGroup;  // EXPERIMENT
        const int64_t k = std::max<int64_t>(1, std::min<int64_t>(kmax, units / (slots * t_min)));
        double t_star = std::max<double>((double)units / (double)(k * slots), (double)s.waves);
        if (units >= slots * t_min) t_star = std::max<double>(t_star, (double)t_min);
        int64_t sum_ns = 0;
        for (int r = 0; r < B; ++r) {
            const int64_t n = std::max<int64_t>(1, std::min<int64_t>(std::max<int64_t>(1, s.ntiles[r]), (int64_t)std::llround(s.ntiles[r] / t_star)));
            s.nsplits[r] = (int32_t)n;
            sum_ns += n;
        }
        // make the item count a multiple of the grid when the batch is big enough: adjust the split
        // counts of the requests that change their item size least
        const int64_t q = slots / std::gcd(slots, per_split);
        if (sum_ns * per_split > slots && B <= 1024 && q > 1) {
            const int64_t rem = sum_ns % q;
            int64_t delta = rem == 0 ? 0 : (rem * 2 <= q ? -rem : q - rem);  // splits to add (+) or drop (-)
            for (int guard = 0; delta != 0 && guard < 4096; ++guard) {
                int best = -1;
                double best_cost = 0.0;
                for (int r = 0; r < B; ++r) {
                    const int64_t n = s.nsplits[r], nn = n + (delta > 0 ? 1 : -1);
                    if (nn < 1 || nn > s.ntiles[r] || s.ntiles[r] / nn < s.waves) continue;
                    // relative change of this request's item size
                    const double cost = std::fabs((double)n / (double)nn - 1.0);
                    if (best < 0 || cost < best_cost) { best = r; best_cost = cost; }
                }
                if (best < 0) break;
                s.nsplits[best] += delta > 0 ? 1 : -1;
                delta += delta > 0 ? -1 : 1;
            }
        }
    }

    s.row_base.assign(B, 0);
    s.max_nsplits = 1;
    int64_t rows = 0;
    for (int r = 0; r < B; ++r) {
        s.max_nsplits = std::max<int32_t>(s.max_nsplits, s.nsplits[r]);
        s.row_base[r] = rows;
        rows += (int64_t)s.nsplits[r] * p.num_q_heads;
    }
    s.num_partials = rows;

    // items in order of decreasing size, so that each round of the persistent grid holds like-sized items
    std::vector<double> item_tiles(B);
    for (int r = 0; r < B; ++r) item_tiles[r] = (double)s.ntiles[r] / s.nsplits[r];
    s.order.resize(B);
    std::iota(s.order.begin(), s.order.end(), 0);
    std::stable_sort(s.order.begin(), s.order.end(), [&](int a, int b) { return item_tiles[a] > item_tiles[b]; });
    s.item_prefix.assign(B + 1, 0);
    int64_t items = 0;
    for (int i = 0; i < B; ++i) {
        s.item_prefix[i] = (int32_t)items;
        items += (int64_t)s.nsplits[s.order[i]] * per_split;
        if (items > INT32_MAX / 2) return DA_ERR_UNSUPPORTED;
    }
    s.item_prefix[B] = (int32_t)items;
    s.num_items = items;
    const int64_t gmult = getenv("DA_EXP_GRIDMULT") ? atoi(getenv("DA_EXP_GRIDMULT")) : 1;  // EXPERIMENT
    s.grid = (int32_t)std::max<int64_t>(1, std::min<int64_t>(items, slots * gmult));
    return DA_OK;
}

}  // namespace da
