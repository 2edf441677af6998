// Work scheduling for DistAttention decode (host arithmetic only).
//
// Section 5.3, Eq. 5 prices attention by the total number of cached tokens, and Section 3 allows a
// sequence to be partitioned at any length.  So the unit of balance is the token, not the request or
// the block.  The tiles (32 tokens) of all requests are laid end to end, longest request first, and
// that stream is cut into `ranges` runs of equal cost; a cut that falls inside a request splits it
// there.  Every kv-head (and head tile) is read by its own set of `ranges` persistent workgroups, one
// per run, so all workgroups of the launch read the same number of bytes, each request is split no
// more than the balance needs, and all heads of a request share the same split boundaries.
#include "schedule.h"

#include <algorithm>
#include <cmath>
#include <numeric>

namespace da {

namespace {
constexpr int kGroupsPerCu = 1;          // persistent MicroAttention workgroups per compute unit (measured: 2 is 1-2 % slower)
constexpr int64_t kMinRunTiles = 8;      // shortest run worth a workgroup: two tiles per wavefront
constexpr int kWaveItemsMinPerRun = 32;  // splits per run from which a wavefront takes whole splits ...
constexpr int kWaveItemsMaxTiles = 128;  // ... if a split holds no more than this many tiles on average

// Fixed cost of one split, in tiles (what a workgroup would have read meanwhile): look-ups, the query rows, the first
// chunk's latency, merge and result rows.  It grows with the columns a work item serves (an item of two 32-token
// chunks takes a workgroup about 2 us at 4 columns, 6 us at 32, 9 us at 64, 12 us at 128); measured on the
// mixed-length workload (64 requests, 16 to 866 514 tokens), where the runs that collect the short requests
// otherwise end last: 4 columns 4..16 alike, 16 and 32 columns flat over 8..40, 64 and 128 columns best at 24..32.
int64_t split_cost_tiles(int cols) { return cols <= 8 ? 4 : cols <= 32 ? 16 : 28; }
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

da_status validate_problem(const da_problem &p)
{
    if (p.batch < 1 || p.num_q_heads < 1 || p.num_kv_heads < 1 || p.max_blocks_per_seq < 1 ||
        p.num_phys_blocks < 1 || p.block_tokens < 1 || p.head_dim < 1)
        return DA_ERR_INVALID_ARG;
    if (p.num_q_heads % p.num_kv_heads != 0) return DA_ERR_INVALID_ARG;
    if (!std::isfinite(p.scale)) return DA_ERR_INVALID_ARG;
    if (p.kv_dtype < DA_F32 || p.kv_dtype > DA_F16 || p.q_dtype < DA_F32 || p.q_dtype > DA_F16) return DA_ERR_UNSUPPORTED;
    if (p.head_dim != 128) return DA_ERR_UNSUPPORTED;
    if (p.block_tokens % 16 != 0) return DA_ERR_UNSUPPORTED;
    if (p.num_q_heads / p.num_kv_heads > 64) return DA_ERR_UNSUPPORTED;
    if (p.q_len < 0) return DA_ERR_INVALID_ARG;
    if (p.q_len > 128) return DA_ERR_UNSUPPORTED;
    const int64_t esize = p.kv_dtype == DA_F32 ? 4 : 2;
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
    const int q_len = p.q_len > 0 ? p.q_len : 1;
    const int G = (p.num_q_heads / p.num_kv_heads) * q_len;  // (query token, q-head) columns per kv-head
    const int64_t tpb = (T + kTileTokens - 1) / kTileTokens;
    const int64_t split_cost = split_cost_tiles(G);

    // kernel family, head tile, workgroup size
    int kernel = tuning.kernel;
    const bool mfma_ok = p.q_dtype == p.kv_dtype;  // one type throughout
    // 16-bit q and K/V go to the matrix-core kernel whatever the group size: even with one live column per tile it
    // streams about 1 % faster than the vector-ALU kernel.  fp32 goes there when a group shares the K/V read
    // (the vector ALU cannot keep up with 8 q-heads per kv-head); alone, the vector-ALU kernel is as fast.
    if (kernel == DA_KERNEL_AUTO)
        kernel = (mfma_ok && (p.kv_dtype != DA_F32 || G > 1)) ? DA_KERNEL_MFMA : DA_KERNEL_VALU;
    if (kernel == DA_KERNEL_MFMA && !mfma_ok) return DA_ERR_UNSUPPORTED;
    s.kernel = kernel;
    s.waves = 4;
    if (kernel == DA_KERNEL_MFMA) {
        // one, two or four 16-column matrix-core tiles per K/V read (fp32: one); bf16: eight, four each for
        // two pairs of wavefronts that read the same chunks
        s.head_tile = p.kv_dtype == DA_F32 ? 16 : (G > 64 && p.kv_dtype == DA_BF16) ? 128 : G > 32 ? 64 : G > 16 ? 32 : 16;
    } else {
        s.head_tile = 1;
        while (s.head_tile < G && s.head_tile < 8) s.head_tile *= 2;
    }
    s.head_tiles = (G + s.head_tile - 1) / s.head_tile;
    const int64_t P = (int64_t)p.num_kv_heads * s.head_tiles;  // workgroups that read the same splits

    // tiles per request; reading order = longest first
    s.ntiles.resize(B);
    int64_t total_tiles = 0;
    for (int r = 0; r < B; ++r) {
        const int64_t L = seq_lens_host[r];
        if (L < 0 || L > (int64_t)p.max_blocks_per_seq * T) return DA_ERR_INVALID_ARG;
        s.ntiles[r] = (int32_t)tiles_of(L, T);
        total_tiles += s.ntiles[r];
    }
    std::vector<int32_t> order(B);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return s.ntiles[a] > s.ntiles[b]; });

    // cut positions (tile index inside the request) per request, in reading order
    std::vector<std::vector<int32_t>> cuts(B);
    const int64_t slots = (int64_t)num_cus * kGroupsPerCu;
    int64_t ranges = std::max<int64_t>(1, slots / P);
    std::vector<int64_t> range_first_tile;  // auto mode: stream position where each range begins
    if (tuning.blocks_per_split > 0) {
        // caller's choice: every split is exactly this many blocks (1 = one partial per block)
        const int64_t f = std::min<int64_t>((int64_t)tuning.blocks_per_split * tpb, INT32_MAX);
        for (int r = 0; r < B; ++r)
            for (int64_t t = f; t < s.ntiles[r]; t += f) cuts[r].push_back((int32_t)t);
    } else {
        // Big batches get one run per compute unit, and their partial rows are then a fraction of a
        // percent of the KV bytes.  A small batch is latency-bound (one workgroup streams only a few
        // tens of GB/s), so it is spread over as many compute units as have at least a few tiles to read,
        // whatever that costs in partial rows.
        ranges = std::max<int64_t>(1, std::min<int64_t>(ranges, total_tiles / kMinRunTiles));
        // equal-cost cut of the stream; a request costs its tiles plus a fixed amount per split
        const double total_cost = (double)total_tiles + (double)split_cost * B;
        int64_t m = 1;          // next boundary to place
        double cost_before = 0; // cost of the requests before the current one
        for (int i = 0; i < B && m < ranges; ++i) {
            const int r = order[i];
            const double cost_end = cost_before + split_cost + s.ntiles[r];
            while (m < ranges) {
                const double x = total_cost * (double)m / (double)ranges;
                if (x >= cost_end) break;
                int64_t t = (int64_t)std::llround(x - cost_before - split_cost);
                t = std::max<int64_t>(0, std::min<int64_t>(t, s.ntiles[r]));
                const int64_t prev = cuts[r].empty() ? 0 : cuts[r].back();
                // keep splits at least one tile per wavefront long; a boundary that would fall too close
                // to the previous one or to an end of the request moves to that end (no split there)
                if (t - prev >= s.waves && s.ntiles[r] - t >= s.waves) cuts[r].push_back((int32_t)t);
                ++m;
            }
            cost_before = cost_end;
        }
    }

    // splits, partial rows, entries in reading order
    s.nsplits.assign(B, 1);
    s.row_base.assign(B, 0);
    s.first_entry.assign(B, 0);
    s.max_nsplits = 1;
    int64_t rows = 0;
    for (int r = 0; r < B; ++r) {
        s.nsplits[r] = (int32_t)cuts[r].size() + 1;
        s.max_nsplits = std::max(s.max_nsplits, s.nsplits[r]);
        s.row_base[r] = rows;
        rows += (int64_t)s.nsplits[r] * p.num_q_heads * q_len;
    }
    s.num_partials = rows;
    s.entries.clear();
    for (int i = 0; i < B; ++i) {
        const int r = order[i];
        s.first_entry[r] = (int32_t)s.entries.size();
        for (int j = 0; j < s.nsplits[r]; ++j) {
            SplitEntry e;
            e.r = r;
            e.j = j;
            e.t0 = j == 0 ? 0 : cuts[r][j - 1];
            e.t1 = j + 1 == s.nsplits[r] ? s.ntiles[r] : cuts[r][j];
            e.ns = s.nsplits[r];
            e.pad = 0;
            e.row_base = s.row_base[r];
            s.entries.push_back(e);
        }
    }
    if ((int64_t)s.entries.size() * P > INT32_MAX / 2) return DA_ERR_UNSUPPORTED;
    s.num_items = (int64_t)s.entries.size() * P;

    // runs of consecutive entries of equal cost (in auto mode this reproduces the cuts made above)
    const int64_t E = (int64_t)s.entries.size();
    ranges = std::max<int64_t>(1, std::min<int64_t>(ranges, E));
    double total_cost = 0;
    for (const SplitEntry &e : s.entries) total_cost += split_cost + (e.t1 - e.t0);
    s.range_start.assign(1, 0);
    double acc = 0;
    for (int64_t i = 0; i < E; ++i) {
        const double c = split_cost + (s.entries[i].t1 - s.entries[i].t0);
        const int64_t m = (int64_t)s.range_start.size();  // boundary being looked for
        // start a new run before entry i when the boundary lies nearer to its start than to its end,
        // while leaving at least one entry for every run still to come
        if (m < ranges && i > s.range_start.back() &&
            (acc + 0.5 * c >= total_cost * (double)m / (double)ranges || E - i <= ranges - m))
            s.range_start.push_back((int32_t)i);
        acc += c;
    }
    s.ranges = (int32_t)s.range_start.size();
    s.range_start.push_back((int32_t)E);
    s.grid = (int32_t)(s.ranges * P);
    // Many short splits per run: a wavefront takes whole splits (no merge across wavefronts, no barriers).  Needs
    // enough splits per run that dealing them to four wavefronts comes out even.
    s.wave_items = kernel == DA_KERNEL_MFMA && p.kv_dtype != DA_F32 && s.head_tile == 16 &&
                   E >= (int64_t)kWaveItemsMinPerRun * s.ranges && total_tiles <= (int64_t)kWaveItemsMaxTiles * E;
    return DA_OK;
}

}  // namespace da
