// Device-side walk over work items and their KV chunks, shared by the MicroAttention kernels.
//
// An item covers the tiles [t0, t1) of one request (tile = 32 tokens inside a block; a block holds
// ceil(T / 32) tiles) for one kv-head and head tile.  A kernel reads it in chunks of CH tokens (CH divides 32); wavefront w of W
// takes chunks w, w + W, ... of the item.  Everything here is uniform across a wavefront.
#pragma once
#include <hip/hip_runtime.h>

#include <cstddef>

#include "kernel_params.h"

namespace da {

// Read of a small read-only table (plan tables, block table, lengths) at a wavefront-uniform index.
// Going through the constant address space lets the compiler use scalar loads even after the kernel
// has stored to global memory; nothing in these kernels writes the tables.
template <typename T>
__device__ __forceinline__ T table_load(const T *p, int64_t i)
{
    typedef const T __attribute__((address_space(4))) * cptr;
    return ((cptr)(uintptr_t)p)[i];
}

// Column c of a kv-head's group (c < cols = q_len * G) is query token c / G and q-head c % G of the group.
struct Column {
    int live;     // c < cols
    int t, g;     // query token, head inside the group
    int vh;       // virtual head t * Hq + kvh * G + g: row of q / out inside the request, partial-row group
    int visible;  // tokens this query may see: L - (q_len - 1 - t), clamped at 0 (causal)
};
__device__ __forceinline__ Column column_of(const MicroParams &p, int c, int kvh, int L)
{
    Column col;
    col.live = c < p.cols;
    const int cc = col.live ? c : 0;
    col.t = cc / p.G;
    col.g = cc - col.t * p.G;
    col.vh = col.t * p.Hq + kvh * p.G + col.g;
    const int vis = L - (p.q_len - 1 - col.t);
    col.visible = vis > 0 ? vis : 0;
    return col;
}

struct ItemInfo {
    int valid;       // 0: past the end of the item list
    int r, j, kvh, ht, ns;
    int L;           // tokens of the request (device value, clamped to what the table can address)
    int c0, c1;      // chunk range of the item, in block-major chunk numbering
    int64_t row_base;
};

struct Chunk {
    int valid;   // 0: past the end of the item
    int c;       // chunk number
    int blk;     // logical block
    int cib;     // chunk inside the block
    int lim;     // valid tokens from the chunk's first row on (<= 0: none)
    int tok0;    // logical token index of the chunk's first row
    int64_t off; // element offset of the chunk's first row (this item's kv-head) inside a pool;
                 // 0 (always readable) when the chunk holds no valid token
};

// What a wavefront fetches for a chunk.  The kernels issue the same number of load instructions in
// every step, whatever the chunk (so that the compiler can count outstanding loads exactly and
// overlap them with arithmetic): rows past the valid ones re-read the last valid row, and a chunk
// with nothing valid re-reads row 0 of the pool; such rows are masked out of the softmax.
struct Fetch {
    int64_t off;  // element offset of the first row
    int last;     // index of the last row that may be read (>= 0)
};
__device__ __forceinline__ Fetch fetch_of(const Chunk &c)
{
    Fetch f;
    const bool any = c.valid && c.lim > 0;
    f.off = any ? c.off : 0;
    f.last = any ? c.lim - 1 : 0;
    return f;
}

// Split number `e` of the workgroup's run (valid while e < e_end), for kv-head kvh and head tile ht.
template <int CH>
__device__ __forceinline__ ItemInfo decode_item(const MicroParams &p, int e, int e_end, int kvh, int ht)
{
    constexpr int SUB = kTile / CH;  // chunks per tile
    ItemInfo it;
    it.valid = e < e_end;
    it.r = it.j = 0;
    it.kvh = kvh;
    it.ht = ht;
    it.ns = 1;
    it.L = 0;
    it.c0 = it.c1 = 0;
    it.row_base = 0;
    if (!it.valid) return it;
    typedef const SplitEntry __attribute__((address_space(4))) * entry_ptr;
    // inline tables are read where the launch put them, in the kernel-argument segment (MicroParams is
    // the kernels' only argument), never through `p` itself, which would drag the whole struct onto the stack
    typedef const char __attribute__((address_space(4))) * kernarg_ptr;
    const kernarg_ptr ka = (kernarg_ptr)__builtin_amdgcn_kernarg_segment_ptr();
    const entry_ptr ent = p.entries ? (entry_ptr)(uintptr_t)(p.entries + e)
                                    : (entry_ptr)(ka + offsetof(MicroParams, inline_entries) + (size_t)e * sizeof(SplitEntry));
    it.r = ent->r;
    it.j = ent->j;
    it.ns = ent->ns;
    it.row_base = ent->row_base;
    int L = table_load(p.seq_lens, it.r);
    L = L < 0 ? 0 : L;
    const int64_t cap = (int64_t)p.max_blocks * p.T;
    if ((int64_t)L > cap) L = (int)cap;
    it.L = L;
    // The device length decides where the request ends: the split table was cut from host lengths
    // that may be stale, and its last split of a request is open-ended.
    const int tpb = (p.T + kTile - 1) / kTile;
    int nt = 0;
    if (L > 0) {
        const int nb = (L + p.T - 1) / p.T;
        nt = (nb - 1) * tpb + (L - (nb - 1) * p.T + kTile - 1) / kTile;
    }
    const int t0 = ent->t0 < nt ? ent->t0 : nt;
    const int t1 = (it.j + 1 == it.ns || ent->t1 > nt) ? nt : ent->t1;
    it.c0 = t0 * SUB;
    it.c1 = t1 * SUB;
    return it;
}

// Fills lim and off of a chunk whose (c, blk, cib) are set.  Reads one block-table entry; a block id
// outside the pool is reported through err_flag and the chunk is treated as empty.
template <int CH>
__device__ __forceinline__ void locate_chunk(const MicroParams &p, const ItemInfo &it, Chunk &ch, int lane)
{
    ch.lim = 0;
    ch.off = 0;
    ch.tok0 = 0;
    if (!ch.valid) return;
    const int pb = table_load(p.block_table, (int64_t)it.r * p.max_blocks + ch.blk);
    const int first = ch.cib * CH;
    int valid = it.L - ch.blk * p.T;
    valid = (valid > p.T ? p.T : valid) - first;
    if ((unsigned)pb >= (unsigned)p.num_phys) {
        if (lane == 0) atomicOr(p.err_flag, 1);
        valid = 0;
    }
    ch.lim = valid;
    ch.tok0 = ch.blk * p.T + first;
    if (valid > 0)
        ch.off = (int64_t)pb * p.stride_block + (int64_t)it.kvh * p.stride_head + (int64_t)first * p.stride_token;
}

template <int CH>
__device__ __forceinline__ Chunk first_chunk(const MicroParams &p, const ItemInfo &it, int wave, int lane)
{
    constexpr int SUB = kTile / CH;
    const int cpb = ((p.T + kTile - 1) / kTile) * SUB;  // chunk slots per block
    Chunk ch;
    ch.c = it.c0 + wave;
    ch.valid = it.valid && ch.c < it.c1;
    ch.blk = ch.c / cpb;
    ch.cib = ch.c - ch.blk * cpb;
    locate_chunk<CH>(p, it, ch, lane);
    return ch;
}

template <int CH, int W>
__device__ __forceinline__ Chunk next_chunk(const MicroParams &p, const ItemInfo &it, Chunk ch, int lane)
{
    constexpr int SUB = kTile / CH;
    const int cpb = ((p.T + kTile - 1) / kTile) * SUB;
    ch.c += W;
    ch.cib += W;
    while (ch.cib >= cpb) {
        ch.cib -= cpb;
        ch.blk += 1;
    }
    ch.valid = ch.c < it.c1;
    locate_chunk<CH>(p, it, ch, lane);
    return ch;
}

}  // namespace da


namespace da {
// First and one-past-last split of run `run`.
__device__ __forceinline__ void run_bounds(const MicroParams &p, int run, int &e_begin, int &e_end)
{
    if (p.range_start) {
        e_begin = table_load(p.range_start, run);
        e_end = table_load(p.range_start, run + 1);
    } else {
        typedef const int32_t __attribute__((address_space(4))) * int_ptr;
        typedef const char __attribute__((address_space(4))) * kernarg_ptr;
        const int_ptr rs = (int_ptr)((kernarg_ptr)__builtin_amdgcn_kernarg_segment_ptr() + offsetof(MicroParams, inline_range_start));
        e_begin = rs[run];
        e_end = rs[run + 1];
    }
}
}  // namespace da
