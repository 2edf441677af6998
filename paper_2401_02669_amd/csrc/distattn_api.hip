// C ABI of the DistAttention decode library: argument checks, plan objects, kernel launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstring>
#include <mutex>
#include <new>

#include "../../include/distattn.h"
#include "kernel_params.h"
#include "schedule.h"

namespace da {
hipError_t launch_micro_attention_valu(const MicroParams &p, int grid, hipStream_t stream);
hipError_t launch_micro_attention_mfma(const MicroParams &p, int grid, hipStream_t stream);
hipError_t launch_micro_attention_mfma_f32(const MicroParams &p, int grid, hipStream_t stream);
hipError_t launch_combine(const CombineParams &p, hipStream_t stream);
}  // namespace da

// Partial results of da_attention_noalloc.  Every GPU the library runs on holds its own copy of this array, at its
// own address, until the process ends; host code reaches it only through the address hipGetSymbolAddress returns
// for the current device (the array's name is not a device address on the host side).
constexpr size_t kScratchBytes = DA_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];  // per device: address of `scratch` there (null: not asked yet)
std::mutex g_scratch_mutex;

// Address of `scratch` on the current device; asked once per device.
da_status scratch_of_current_device(void **ptr)
{
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) return DA_ERR_HIP;
    if (device < 0 || device >= kMaxDevices) return DA_ERR_UNSUPPORTED;
    void *p = g_scratch_ptr[device].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        p = g_scratch_ptr[device].load(std::memory_order_relaxed);
        if (!p) {
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DA_ERR_HIP;
            g_scratch_ptr[device].store(p, std::memory_order_release);
        }
    }
    *ptr = p;
    return DA_OK;
}

constexpr int kRing = 4;  // pinned staging slots for table uploads

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Device tables of a plan: [error flag | range_start | nsplits | row_base | entries], sized for a capacity.
// Everything behind the error flag is uploaded in one copy that ends with the last used entry.
struct TableLayout {
    size_t err, range_start, nsplits, row_base, entries, total;
    TableLayout(size_t cap_entries, size_t cap_ranges, size_t batch)
    {
        size_t off = 0;
        err = off;         off = align_up(off + sizeof(int32_t), 32);
        range_start = off; off = align_up(off + sizeof(int32_t) * (cap_ranges + 1), 32);
        nsplits = off;     off = align_up(off + sizeof(int32_t) * batch, 32);
        row_base = off;    off = align_up(off + sizeof(int64_t) * batch, 32);
        entries = off;     off = align_up(off + sizeof(da::SplitEntry) * cap_entries, 32);
        total = off;
    }
};

}  // namespace

struct da_plan {
    da_problem problem;
    da_tuning tuning;
    int32_t num_cus;
    da::Schedule sched;
    std::vector<int32_t> lens;  // host lengths the schedule was made from
    size_t cap_entries = 0, cap_ranges = 0;
    bool inline_ok = false;    // the schedule is small enough to travel in the kernel arguments (then the device
                               // tables are not kept current; otherwise every create / update uploads them)
    char *dev = nullptr;       // device tables (+ error flag at layout.err)
    char *stage[kRing] = {};   // pinned host staging
    hipEvent_t ev[kRing] = {};
    bool ev_pending[kRing] = {};
    int ring = 0;
};

namespace {

TableLayout layout_of(const da_plan *pl) { return TableLayout(pl->cap_entries, pl->cap_ranges, pl->problem.batch); }

void release_tables(da_plan *pl)
{
    for (int i = 0; i < kRing; ++i) {
        if (pl->ev_pending[i]) (void)hipEventSynchronize(pl->ev[i]);
        pl->ev_pending[i] = false;
        if (pl->stage[i]) (void)hipHostFree(pl->stage[i]);
        pl->stage[i] = nullptr;
    }
    if (pl->dev) (void)hipFree(pl->dev);
    pl->dev = nullptr;
}

// (Re)allocates the tables so that the current schedule fits, with room to grow.
da_status reserve_tables(da_plan *pl, hipStream_t stream)
{
    const size_t need_e = pl->sched.entries.size(), need_r = (size_t)pl->sched.ranges;
    if (pl->dev && need_e <= pl->cap_entries && need_r <= pl->cap_ranges) return DA_OK;
    int32_t pending_err = 0;  // a flag raised under the old tables survives the move to the new ones
    if (pl->dev) {
        if (hipStreamSynchronize(stream) != hipSuccess) return DA_ERR_HIP;  // earlier launches still read them
        if (hipMemcpy(&pending_err, pl->dev + layout_of(pl).err, sizeof pending_err, hipMemcpyDeviceToHost) != hipSuccess)
            return DA_ERR_HIP;
    }
    release_tables(pl);
    pl->cap_entries = need_e * 2 + 1024;
    pl->cap_ranges = std::max<size_t>(need_r * 2, 1024);
    const TableLayout lay = layout_of(pl);
    bool ok = hipMalloc((void **)&pl->dev, lay.total) == hipSuccess;
    for (int i = 0; ok && i < kRing; ++i) ok = hipHostMalloc((void **)&pl->stage[i], lay.total, hipHostMallocDefault) == hipSuccess;
    // blocking copy: the flag word is in place before any launch that follows, on whatever stream
    const int32_t flag_init[8] = {pending_err, 0, 0, 0, 0, 0, 0, 0};
    ok = ok && hipMemcpy(pl->dev + lay.err, flag_init, sizeof flag_init, hipMemcpyHostToDevice) == hipSuccess;
    return ok ? DA_OK : DA_ERR_HIP;
}

// Small schedules travel in the kernel arguments of every launch that needs them.
bool fits_inline(const da_plan *pl)
{
    return pl->sched.entries.size() <= (size_t)da::kInlineEntries && pl->sched.ranges <= da::kInlineRuns &&
           pl->problem.batch <= da::kInlineBatch;
}

da_status upload(da_plan *pl, hipStream_t stream)
{
    da_status st = reserve_tables(pl, stream);
    if (st != DA_OK) return st;
    const int B = pl->problem.batch;
    const TableLayout lay = layout_of(pl);
    const int slot = pl->ring;
    pl->ring = (pl->ring + 1) % kRing;
    if (pl->ev_pending[slot]) {
        if (hipEventSynchronize(pl->ev[slot]) != hipSuccess) return DA_ERR_HIP;
        pl->ev_pending[slot] = false;
    }
    char *h = pl->stage[slot];
    const da::Schedule &s = pl->sched;
    std::memcpy(h + lay.entries, s.entries.data(), sizeof(da::SplitEntry) * s.entries.size());
    std::memcpy(h + lay.range_start, s.range_start.data(), sizeof(int32_t) * s.range_start.size());
    std::memcpy(h + lay.nsplits, s.nsplits.data(), sizeof(int32_t) * B);
    std::memcpy(h + lay.row_base, s.row_base.data(), sizeof(int64_t) * B);
    const size_t end = lay.entries + sizeof(da::SplitEntry) * s.entries.size();
    if (hipMemcpyAsync(pl->dev + lay.range_start, h + lay.range_start, end - lay.range_start, hipMemcpyHostToDevice,
                       stream) != hipSuccess)
        return DA_ERR_HIP;
    if (hipEventRecord(pl->ev[slot], stream) != hipSuccess) return DA_ERR_HIP;
    pl->ev_pending[slot] = true;
    return DA_OK;
}

// After a (re-)plan: upload now, or leave it to the kernel arguments.  Everything a launch call needs is in place
// when this returns, so the launch calls only read the plan.
da_status publish(da_plan *pl, hipStream_t stream)
{
    pl->inline_ok = fits_inline(pl);
    if (pl->inline_ok && pl->dev) return DA_OK;  // (the first call still allocates, for the error flag)
    return upload(pl, stream);
}

void fill_micro(const da_plan *pl, da::MicroParams &mp)
{
    const da_problem &p = pl->problem;
    const TableLayout lay = layout_of(pl);
    if (pl->inline_ok) {
        mp.entries = nullptr;
        mp.range_start = nullptr;
        std::memcpy(mp.inline_entries, pl->sched.entries.data(), sizeof(da::SplitEntry) * pl->sched.entries.size());
        std::memcpy(mp.inline_range_start, pl->sched.range_start.data(), sizeof(int32_t) * pl->sched.range_start.size());
    } else {
        mp.entries = (const da::SplitEntry *)(pl->dev + lay.entries);
        mp.range_start = (const int32_t *)(pl->dev + lay.range_start);
    }
    mp.err_flag = (int32_t *)(pl->dev + lay.err);
    mp.B = p.batch;
    mp.Hq = p.num_q_heads;
    mp.Hkv = p.num_kv_heads;
    mp.G = p.num_q_heads / p.num_kv_heads;
    mp.T = p.block_tokens;
    mp.max_blocks = p.max_blocks_per_seq;
    mp.num_phys = p.num_phys_blocks;
    mp.head_tile = pl->sched.head_tile;
    mp.head_tiles = pl->sched.head_tiles;
    mp.per_split = p.num_kv_heads * pl->sched.head_tiles;
    mp.wave_items = pl->sched.wave_items;
    mp.q_len = p.q_len > 0 ? p.q_len : 1;
    mp.cols = mp.q_len * mp.G;
    mp.q_dtype = p.q_dtype;
    mp.kv_dtype = p.kv_dtype;
    mp.stride_block = p.kv_block_stride;
    mp.stride_head = p.kv_head_stride;
    mp.stride_token = p.kv_token_stride;
    mp.scale_log2e = p.scale * 1.4426950408889634f;
}

da_status launch_micro(const da_plan *pl, const da::MicroParams &mp, hipStream_t stream)
{
    hipError_t e = hipErrorInvalidValue;
    if (pl->sched.kernel == DA_KERNEL_VALU)
        e = da::launch_micro_attention_valu(mp, pl->sched.grid, stream);
    else if (pl->sched.kernel == DA_KERNEL_MFMA)
        e = pl->problem.kv_dtype == DA_F32 ? da::launch_micro_attention_mfma_f32(mp, pl->sched.grid, stream)
                                           : da::launch_micro_attention_mfma(mp, pl->sched.grid, stream);
    return e == hipSuccess ? DA_OK : DA_ERR_HIP;
}

// Partial set number `i` of an aggregation launch.  A small plan's two tables travel in the kernel arguments, a
// large plan's were uploaded when it was made.
void fill_set(const da_plan *pl, const float *part_o, const float *part_m, const float *part_e, da::CombineParams &cp,
              int i)
{
    da::PartialSet &ps = cp.set[i];
    ps.part_o = part_o;
    ps.part_m = part_m;
    ps.part_e = part_e;
    if (pl->inline_ok) {
        ps.nsplits = nullptr;
        ps.row_base = nullptr;
        std::memcpy(cp.inline_nsplits[i], pl->sched.nsplits.data(), sizeof(int32_t) * pl->problem.batch);
        std::memcpy(cp.inline_row_base[i], pl->sched.row_base.data(), sizeof(int64_t) * pl->problem.batch);
    } else {
        const TableLayout lay = layout_of(pl);
        ps.nsplits = (const int32_t *)(pl->dev + lay.nsplits);
        ps.row_base = (const int64_t *)(pl->dev + lay.row_base);
    }
}

void fill_combine(const da_plan *pl, da::CombineParams &cp)
{
    cp.B = pl->problem.batch;
    cp.Hq = pl->problem.num_q_heads * (pl->problem.q_len > 0 ? pl->problem.q_len : 1);  // virtual heads
    cp.col_slices = ((int64_t)cp.B * cp.Hq < 1024) ? 4 : 1;
}

// MicroAttention into the three part_* arrays laid out in `ws`, then aggregation, on one stream.
da_status attention_into(const da_plan *pl, const void *q, const void *k_pool, const void *v_pool,
                         const int32_t *block_table, const int32_t *seq_lens, float *out, float *lse, char *ws,
                         hipStream_t stream)
{
    const size_t n = (size_t)pl->sched.num_partials;
    float *part_o = (float *)ws;
    float *part_m = (float *)(ws + align_up(n * da::kHeadDim * sizeof(float), 256));
    float *part_e = (float *)((char *)part_m + align_up(n * sizeof(float), 256));

    da::MicroParams mp = {};
    fill_micro(pl, mp);
    mp.q = q;
    mp.k_pool = k_pool;
    mp.v_pool = v_pool;
    mp.block_table = block_table;
    mp.seq_lens = seq_lens;
    mp.part_o = part_o;
    mp.part_m = part_m;
    mp.part_e = part_e;
    mp.out = out;
    mp.lse = lse;
    mp.direct_out = 1;
    da_status st = launch_micro(pl, mp, stream);
    if (st != DA_OK) return st;
    if (pl->sched.max_nsplits <= 1) return DA_OK;  // every request was normalised in the MicroAttention kernel

    da::CombineParams cp = {};
    fill_combine(pl, cp);
    fill_set(pl, part_o, part_m, part_e, cp, 0);
    cp.num_sets = 1;
    cp.out = out;
    cp.lse = lse;
    cp.skip_single = 1;
    return da::launch_combine(cp, stream) == hipSuccess ? DA_OK : DA_ERR_HIP;
}

bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace

extern "C" {

const char *da_status_string(da_status s)
{
    switch (s) {
    case DA_OK: return "ok";
    case DA_ERR_INVALID_ARG: return "invalid argument";
    case DA_ERR_UNSUPPORTED: return "unsupported configuration";
    case DA_ERR_WORKSPACE: return "workspace too small or misaligned";
    case DA_ERR_HIP: return "HIP runtime error";
    case DA_ERR_NO_SPACE: return "block pool exhausted";
    }
    return "unknown status";
}

da_status da_plan_schedule(const da_problem *problem, const int32_t *seq_lens_host, const da_tuning *tuning,
                           int32_t *nsplits_host, int64_t *num_items, int64_t *num_partials, int32_t *kernel,
                           int32_t *workgroups, int64_t *max_workgroup_tokens)
{
    if (!problem || !seq_lens_host) return DA_ERR_INVALID_ARG;
    da_tuning t = {0, 0, 0};
    if (tuning) t = *tuning;
    if (t.num_cus < 0) return DA_ERR_INVALID_ARG;
    da::Schedule s;
    da_status st = da::make_schedule(*problem, seq_lens_host, t, t.num_cus > 0 ? t.num_cus : 256, s);
    if (st != DA_OK) return st;
    if (nsplits_host) std::memcpy(nsplits_host, s.nsplits.data(), sizeof(int32_t) * problem->batch);
    if (num_items) *num_items = s.num_items;
    if (num_partials) *num_partials = s.num_partials;
    if (kernel) *kernel = s.kernel;
    if (workgroups) *workgroups = s.grid;
    if (max_workgroup_tokens) {
        int64_t worst = 0;
        for (int m = 0; m < s.ranges; ++m) {
            int64_t tok = 0;
            for (int e = s.range_start[m]; e < s.range_start[m + 1]; ++e) {
                const da::SplitEntry &en = s.entries[e];
                const int64_t L = seq_lens_host[en.r];
                tok += std::min<int64_t>(L, da::tile_first_token(en.t1, problem->block_tokens)) -
                       std::min<int64_t>(L, da::tile_first_token(en.t0, problem->block_tokens));
            }
            worst = std::max(worst, tok);
        }
        *max_workgroup_tokens = worst;
    }
    return DA_OK;
}

da_status da_plan_create(const da_problem *problem, const int32_t *seq_lens_host, const da_tuning *tuning,
                         void *stream, da_plan **plan)
{
    if (!plan) return DA_ERR_INVALID_ARG;
    *plan = nullptr;
    if (!problem || !seq_lens_host) return DA_ERR_INVALID_ARG;
    da_status st = da::validate_problem(*problem);
    if (st != DA_OK) return st;
    da_tuning t = {0, 0, 0};
    if (tuning) t = *tuning;
    if (t.num_cus < 0) return DA_ERR_INVALID_ARG;

    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return DA_ERR_HIP;
    int cus = t.num_cus;
    if (cus == 0) {
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus < 1)
            return DA_ERR_HIP;
    }

    da_plan *pl = new (std::nothrow) da_plan();
    if (!pl) return DA_ERR_HIP;
    pl->problem = *problem;
    pl->tuning = t;
    pl->num_cus = cus;
    st = da::make_schedule(pl->problem, seq_lens_host, t, cus, pl->sched);
    if (st != DA_OK) {
        delete pl;
        return st;
    }
    pl->lens.assign(seq_lens_host, seq_lens_host + problem->batch);
    bool ok = true;
    for (int i = 0; ok && i < kRing; ++i) ok = hipEventCreateWithFlags(&pl->ev[i], hipEventDisableTiming) == hipSuccess;
    if (ok) ok = publish(pl, (hipStream_t)stream) == DA_OK;
    if (!ok) {
        da_plan_destroy(pl);
        return DA_ERR_HIP;
    }
    *plan = pl;
    return DA_OK;
}

da_status da_plan_update(da_plan *pl, const int32_t *seq_lens_host, void *stream)
{
    if (!pl || !seq_lens_host) return DA_ERR_INVALID_ARG;
    da::Schedule s;
    da_status st = da::make_schedule(pl->problem, seq_lens_host, pl->tuning, pl->num_cus, s);
    if (st != DA_OK) return st;
    pl->sched = std::move(s);
    pl->lens.assign(seq_lens_host, seq_lens_host + pl->problem.batch);
    return publish(pl, (hipStream_t)stream);
}

da_status da_plan_destroy(da_plan *pl)
{
    if (!pl) return DA_OK;
    release_tables(pl);
    for (int i = 0; i < kRing; ++i)
        if (pl->ev[i]) (void)hipEventDestroy(pl->ev[i]);
    delete pl;
    return DA_OK;
}

da_status da_plan_num_partials(const da_plan *pl, int64_t *n)
{
    if (!pl || !n) return DA_ERR_INVALID_ARG;
    *n = pl->sched.num_partials;
    return DA_OK;
}

da_status da_plan_nsplits(const da_plan *pl, int32_t r, int32_t *nsplits)
{
    if (!pl || !nsplits || r < 0 || r >= pl->problem.batch) return DA_ERR_INVALID_ARG;
    *nsplits = pl->sched.nsplits[r];
    return DA_OK;
}

da_status da_plan_split(const da_plan *pl, int32_t r, int32_t j, int64_t *first_token, int64_t *end_token)
{
    if (!pl || !first_token || !end_token || r < 0 || r >= pl->problem.batch) return DA_ERR_INVALID_ARG;
    if (j < 0 || j >= pl->sched.nsplits[r]) return DA_ERR_INVALID_ARG;
    const da::SplitEntry &e = pl->sched.entries[pl->sched.first_entry[r] + j];
    const int32_t T = pl->problem.block_tokens;
    const int64_t L = pl->lens[r];
    *first_token = std::min<int64_t>(L, da::tile_first_token(e.t0, T));
    *end_token = std::min<int64_t>(L, da::tile_first_token(e.t1, T));
    return DA_OK;
}

da_status da_plan_describe(const da_plan *pl, int32_t *kernel, int32_t *head_tile, int32_t *wavefront_splits)
{
    if (!pl) return DA_ERR_INVALID_ARG;
    if (kernel) *kernel = pl->sched.kernel;
    if (head_tile) *head_tile = pl->sched.head_tile;
    if (wavefront_splits) *wavefront_splits = pl->sched.wave_items;
    return DA_OK;
}

da_status da_workspace_bytes(const da_plan *pl, size_t *bytes)
{
    if (!pl || !bytes) return DA_ERR_INVALID_ARG;
    const size_t n = (size_t)pl->sched.num_partials;
    *bytes = align_up(n * da::kHeadDim * sizeof(float), 256) + 2 * align_up(n * sizeof(float), 256);
    return DA_OK;
}

da_status da_plan_error(da_plan *pl, void *stream, int32_t *flags)
{
    if (!pl || !flags) return DA_ERR_INVALID_ARG;
    const TableLayout lay = layout_of(pl);
    hipStream_t s = (hipStream_t)stream;
    int32_t v = 0;
    if (hipMemcpyAsync(&v, pl->dev + lay.err, sizeof v, hipMemcpyDeviceToHost, s) != hipSuccess) return DA_ERR_HIP;
    if (hipMemsetAsync(pl->dev + lay.err, 0, sizeof v, s) != hipSuccess) return DA_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return DA_ERR_HIP;
    *flags = v;
    return DA_OK;
}

da_status da_partial(const da_plan *pl, const void *q, const void *k_pool, const void *v_pool,
                     const int32_t *block_table, const int32_t *seq_lens, float *part_o, float *part_m,
                     float *part_e, void *stream)
{
    if (!pl || !q || !k_pool || !v_pool || !block_table || !seq_lens || !part_o || !part_m || !part_e)
        return DA_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k_pool) || !aligned16(v_pool) || !aligned16(part_o)) return DA_ERR_INVALID_ARG;
    da::MicroParams mp = {};
    fill_micro(pl, mp);
    mp.q = q;
    mp.k_pool = k_pool;
    mp.v_pool = v_pool;
    mp.block_table = block_table;
    mp.seq_lens = seq_lens;
    mp.part_o = part_o;
    mp.part_m = part_m;
    mp.part_e = part_e;
    mp.direct_out = 0;
    return launch_micro(pl, mp, (hipStream_t)stream);
}

da_status da_combine(const da_plan *pl, const float *part_o, const float *part_m, const float *part_e, float *out,
                     float *lse, void *stream)
{
    if (!pl || !part_o || !part_m || !part_e || !out) return DA_ERR_INVALID_ARG;
    if (!aligned16(part_o) || !aligned16(out)) return DA_ERR_INVALID_ARG;
    da::CombineParams cp = {};
    fill_combine(pl, cp);
    fill_set(pl, part_o, part_m, part_e, cp, 0);
    cp.num_sets = 1;
    cp.out = out;
    cp.lse = lse;
    cp.skip_single = 0;
    return da::launch_combine(cp, (hipStream_t)stream) == hipSuccess ? DA_OK : DA_ERR_HIP;
}

da_status da_combine_multi(const da_partial_set *sets, int32_t num_sets, float *out, float *lse, void *stream)
{
    if (!sets || num_sets < 1 || !out || !aligned16(out)) return DA_ERR_INVALID_ARG;
    if (num_sets > da::kMaxPartialSets) return DA_ERR_UNSUPPORTED;
    da::CombineParams cp = {};
    for (int i = 0; i < num_sets; ++i) {
        const da_partial_set &s = sets[i];
        if (!s.plan || !s.part_o || !s.part_m || !s.part_e || !aligned16(s.part_o)) return DA_ERR_INVALID_ARG;
        const da_problem &a = s.plan->problem, &b = sets[0].plan->problem;
        // every share describes the same queries: same batch, heads and query tokens
        if (a.batch != b.batch || a.num_q_heads != b.num_q_heads || (a.q_len > 0 ? a.q_len : 1) != (b.q_len > 0 ? b.q_len : 1))
            return DA_ERR_INVALID_ARG;
        fill_set(s.plan, s.part_o, s.part_m, s.part_e, cp, i);
    }
    fill_combine(sets[0].plan, cp);
    cp.num_sets = num_sets;
    cp.out = out;
    cp.lse = lse;
    cp.skip_single = 0;
    return da::launch_combine(cp, (hipStream_t)stream) == hipSuccess ? DA_OK : DA_ERR_HIP;
}

da_status da_attention(const da_plan *pl, const void *q, const void *k_pool, const void *v_pool,
                       const int32_t *block_table, const int32_t *seq_lens, float *out, float *lse, void *workspace,
                       size_t workspace_bytes, void *stream)
{
    if (!pl || !q || !k_pool || !v_pool || !block_table || !seq_lens || !out) return DA_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k_pool) || !aligned16(v_pool) || !aligned16(out)) return DA_ERR_INVALID_ARG;
    size_t need = 0;
    da_workspace_bytes(pl, &need);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255)) return DA_ERR_WORKSPACE;
    return attention_into(pl, q, k_pool, v_pool, block_table, seq_lens, out, lse, (char *)workspace, (hipStream_t)stream);
}

da_status da_attention_noalloc(const da_plan *pl, const void *q, const void *k_pool, const void *v_pool,
                               const int32_t *block_table, const int32_t *seq_lens, float *out, float *lse,
                               void *stream)
{
    if (!pl || !q || !k_pool || !v_pool || !block_table || !seq_lens || !out) return DA_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k_pool) || !aligned16(v_pool) || !aligned16(out)) return DA_ERR_INVALID_ARG;
    size_t need = 0;
    da_workspace_bytes(pl, &need);
    if (need > kScratchBytes) return DA_ERR_WORKSPACE;  // more partial rows than the fixed array holds
    void *ws = nullptr;
    da_status st = scratch_of_current_device(&ws);
    if (st != DA_OK) return st;
    // Nothing in the array has to start at zero: the MicroAttention launch writes every partial row the
    // aggregation reads (empty splits included) before the aggregation launch, in stream order.
    return attention_into(pl, q, k_pool, v_pool, block_table, seq_lens, out, lse, (char *)ws, (hipStream_t)stream);
}

}  // extern "C"
