/*
 * distattn.h - C ABI of the DistAttention decode hot path for AMD MI355X (gfx950).
 *
 * DistAttention (Infinite-LLM, Section 4) cuts the KV cache of every request
 * along the sequence into fixed-size blocks.  A run of blocks is attended to by
 * an independent MicroAttention that returns an un-normalised partial output
 * MA_j with its local score maximum m_j and exp-sum e_j (Section 4, Eq. 2 and
 * the m_j / e_j equation above it); an aggregation step (Section 4, Eq. 3 and
 * the m_g / e_g equation above it) turns the partials of one query into exactly
 * softmax(scale * q K^T) V (Section 4, Eq. 1).
 *
 * Scope: decode (one query token per request), MHA / MQA / GQA (Section 3),
 * one GPU.  Everything runs in hand-written HIP kernels; there is no CPU
 * fallback.  All entry points return a da_status; none aborts, throws or prints.
 *
 * Memory: every tensor pointer below is DEVICE memory owned by the caller
 * unless its name ends in _host.  The library allocates device memory only
 * inside da_plan_create (a few small tables) and frees it in da_plan_destroy.
 * All kernels are enqueued on `stream` (a hipStream_t passed as void*, NULL =
 * the default stream); no entry point except da_plan_error synchronises.
 *
 * Element types (da_dtype): fp32, bf16 and IEEE half for q and for the pools; the
 * matrix-core kernel needs q and the pools in the same 16-bit type.
 *
 * Layouts (element = one kv_dtype / q_dtype value; strides in elements):
 *   q            [batch][num_q_heads][head_dim], contiguous
 *   k_pool,v_pool element (pb, g, s, c) at pb*kv_block_stride + g*kv_head_stride
 *                + s*kv_token_stride + c;  pb < num_phys_blocks is a physical
 *                block, g a kv-head, s < block_tokens a slot, c < head_dim.
 *                A (token, head) row of head_dim elements is contiguous and must
 *                start on a 16-byte boundary.
 *   block_table  int32 [batch][max_blocks_per_seq]; logical token i of request r
 *                lives in physical block block_table[r][i / block_tokens] at slot
 *                i % block_tokens.  Entries past ceil(seq_len / block_tokens) are
 *                never read.
 *   seq_lens     int32 [batch]; tokens i >= seq_lens[r] never influence a result
 *                (their slots may hold anything, NaN included).
 *   out          fp32 [batch][num_q_heads][head_dim]
 *   lse          fp32 [batch][num_q_heads], m_g + ln(e_g)  (optional)
 *   part_o       fp32 [num_partials][head_dim]   MA_j, un-normalised (Eq. 2)
 *   part_m       fp32 [num_partials]             m_j (natural-log units of scale*q.k)
 *   part_e       fp32 [num_partials]             e_j
 *     A partial row belongs to one (request r, q-head h, split j):
 *       row(r, h, j) = num_q_heads * sum_{r' < r} nsplits[r'] + h * nsplits[r] + j
 *     so the rows of one (r, h) are contiguous and can be aggregated in any
 *     order or grouping.
 *
 * Semantics: q-head h reads kv-head h / (num_q_heads / num_kv_heads).  The
 * query attends to all seq_lens[r] cached tokens (no causal mask: decode).  An
 * empty request yields out = 0 and lse = -inf; an empty split yields m = -inf,
 * e = 0, MA = 0 and has weight 0 in the aggregation.
 *
 * Multi-query form (da_problem.q_len = n > 1: several new tokens per request,
 * as in speculative decoding or chunked prefill; Section 2.1, Section 3): q is
 * [batch][n][num_q_heads][head_dim], the cache already holds the n new tokens,
 * and query token t attends causally to the tokens i < seq_lens[r] - (n-1-t).
 * Every (t, h) pair behaves like a q-head of its own, "virtual head"
 * vh = t * num_q_heads + h: out is [batch][n][num_q_heads][head_dim], lse
 * [batch][n][num_q_heads], and partial rows are
 *   row(r, vh, j) = n * num_q_heads * sum_{r' < r} nsplits[r'] + vh * nsplits[r] + j.
 * A query token that precedes the start of the cache sees nothing (out = 0,
 * lse = -inf).
 */
#ifndef DISTATTN_H
#define DISTATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DA_OK = 0,
    DA_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, Hq % Hkv != 0, misaligned stride ... */
    DA_ERR_UNSUPPORTED = 2, /* head_dim != 128, block_tokens % 16 != 0, unknown dtype, group > 64 */
    DA_ERR_WORKSPACE = 3,   /* workspace smaller than da_workspace_bytes() */
    DA_ERR_HIP = 4,         /* a HIP runtime call failed (no device, launch failure, out of memory) */
    DA_ERR_NO_SPACE = 5     /* the block pool has too few free blocks */
} da_status;

typedef enum { DA_F32 = 0, DA_BF16 = 1, DA_F16 = 2 /* IEEE binary16 */ } da_dtype;

/* MicroAttention kernel families (da_tuning.kernel). */
typedef enum {
    DA_KERNEL_AUTO = 0, /* MFMA when q, K and V share a 16-bit type, or share fp32 with a query group > 1;
                           VALU otherwise */
    DA_KERNEL_VALU = 1, /* fp32 vector ALU dot products, wavefront (DPP) reductions */
    DA_KERNEL_MFMA = 2  /* matrix-core products for the (q-head group) x (KV tile) contractions; q and the pools
                           must have the same type */
} da_kernel;

typedef struct {
    int32_t batch;              /* B  >= 1 */
    int32_t num_q_heads;        /* Hq >= 1 */
    int32_t num_kv_heads;       /* Hkv >= 1, divides Hq */
    int32_t head_dim;           /* 128 */
    int32_t block_tokens;       /* T: tokens per KV block, a positive multiple of 16 */
    int32_t max_blocks_per_seq; /* row length of block_table, >= 1 */
    int32_t num_phys_blocks;    /* blocks in each pool; table entries outside [0, n) are rejected in-kernel */
    int32_t kv_dtype;           /* da_dtype of k_pool and v_pool */
    int32_t q_dtype;            /* da_dtype of q */
    float scale;                /* score scale, e.g. 1/sqrt(head_dim); finite */
    int64_t kv_block_stride;    /* elements between physical blocks */
    int64_t kv_head_stride;     /* elements between kv-heads inside a block */
    int64_t kv_token_stride;    /* elements between slots; >= head_dim */
    int32_t q_len;              /* query tokens per request: 1 (or 0) = decode; up to 128 for the multi-query form */
} da_problem;

/* Scheduling knobs; a NULL da_tuning* or a zero field means "choose". */
typedef struct {
    int32_t blocks_per_split; /* KV blocks per MicroAttention; 1 = one partial per block as in Section 4; 0 = balanced */
    int32_t num_cus;          /* compute units to fill; 0 = ask the device (256 on MI355X) */
    int32_t kernel;           /* da_kernel */
} da_tuning;

typedef struct da_plan da_plan; /* opaque: split schedule of one batch + its small device tables */

/*
 * Work scheduling (host).  Section 5.3, Eq. 5 prices attention by total KV
 * length, not batch size; Section 3 allows partitions of any length.  The
 * plan lays the 32-token tiles of all requests end to end (longest request
 * first) and cuts that stream into runs of equal cost, one run per persistent
 * workgroup and kv-head; a cut that falls inside a request splits it there.
 * Every workgroup of the MicroAttention launch therefore reads the same number
 * of bytes, from one short request to one 2M-token request, and no request is
 * split more than that balance needs (nsplits[r] >= 1).  With
 * da_tuning.blocks_per_split > 0 every split is exactly that many blocks
 * instead, and whole splits are dealt to the workgroups.
 *
 * da_plan_schedule: pure host arithmetic, no HIP call.  Writes nsplits[r] into
 *   nsplits_host[batch] (may be NULL).  *num_items = (split, kv-head) work
 *   items, *num_partials = rows of part_*, *kernel = the da_kernel chosen,
 *   *workgroups = size of the MicroAttention launch, *max_workgroup_tokens =
 *   the most tokens any one workgroup reads (any may be NULL).
 * da_plan_create: the same schedule, plus its device tables.  seq_lens_host is
 *   read during the call and not retained.  Destroy with da_plan_destroy.
 * da_plan_update: re-plan the same problem for new lengths in place.  Ordered
 *   on `stream` after earlier launches that used the plan; allocates (and
 *   waits for `stream`) only if the split table outgrew its capacity.
 * The lengths given here decide only how the work is cut; which tokens are
 * read follows the device seq_lens passed to the launch calls (the last split
 * of a request runs to that request's device length, every other split stops
 * there at the latest).  A plan made for slightly different lengths, as in a
 * decode loop that re-plans every few steps, therefore still gives exact
 * results, only a less even balance; da_plan_split reports the planned cut.
 *
 * Threads and lifetime.  da_plan_create and da_plan_update leave everything a
 * launch needs in place (device tables uploaded, or a small schedule kept for
 * the kernel arguments), and da_partial, da_combine, da_combine_multi,
 * da_attention and the da_plan_* queries only read the plan: any number of
 * host threads may call them on one plan at the same time, on any streams,
 * as long as their outputs and workspaces are distinct.  da_plan_update,
 * da_plan_error and da_plan_destroy change the plan and need it to themselves:
 * no other call on the same plan may run beside them.  A launch enqueued
 * before da_plan_update keeps the schedule it was given if the update is
 * enqueued on the same stream (or on one ordered after it).  da_plan_destroy
 * does not wait for the GPU: every launch that used the plan must have
 * completed, and no captured graph that holds such a launch may be replayed
 * afterwards (large schedules are read from device tables the plan owns).
 * Errors: DA_ERR_INVALID_ARG / DA_ERR_UNSUPPORTED from validation (before any
 * HIP call), DA_ERR_HIP if the device tables cannot be made.
 */
da_status da_plan_schedule(const da_problem *problem, const int32_t *seq_lens_host, const da_tuning *tuning,
                           int32_t *nsplits_host, int64_t *num_items, int64_t *num_partials, int32_t *kernel,
                           int32_t *workgroups, int64_t *max_workgroup_tokens);
da_status da_plan_create(const da_problem *problem, const int32_t *seq_lens_host, const da_tuning *tuning,
                         void *stream, da_plan **plan);
da_status da_plan_update(da_plan *plan, const int32_t *seq_lens_host, void *stream);
da_status da_plan_destroy(da_plan *plan);

/* Rows of part_o / part_m / part_e for this plan. */
da_status da_plan_num_partials(const da_plan *plan, int64_t *num_partials);
/* Split j of request r covers the logical tokens [*first_token, *end_token) (possibly none). */
da_status da_plan_split(const da_plan *plan, int32_t r, int32_t j, int64_t *first_token, int64_t *end_token);
/* nsplits[r]. */
da_status da_plan_nsplits(const da_plan *plan, int32_t r, int32_t *nsplits);
/*
 * What the plan's current schedule launches: the MicroAttention kernel family (da_kernel), the columns served per
 * work item, and whether each wavefront takes whole splits (1; chosen for runs of many short splits) or the four
 * wavefronts of a workgroup share every split (0).  Any pointer may be NULL.
 */
da_status da_plan_describe(const da_plan *plan, int32_t *kernel, int32_t *head_tile, int32_t *wavefront_splits);
/* Bytes of device workspace da_attention needs (the three part_* arrays, 256-byte aligned each). */
da_status da_workspace_bytes(const da_plan *plan, size_t *bytes);
/*
 * Blocking: waits for `stream`, then reports in *flags whether any kernel that
 * used this plan met a block_table entry outside [0, num_phys_blocks) (bit 0).
 * Such a block is skipped (its tokens contribute nothing) instead of being
 * read.  Clears the flag.
 */
da_status da_plan_error(da_plan *plan, void *stream, int32_t *flags);

/*
 * MicroAttention (Section 4, m_j / e_j equation and Eq. 2): for every split j
 * of every (request, kv-head) and each q-head h of that kv-head's group, over
 * the split's valid tokens i:
 *   s_i = scale * q_h . k_i,  m_j = max_i s_i,  e_j = sum_i exp(s_i - m_j),
 *   MA_j = sum_i exp(s_i - m_j) v_i
 * written to row(r, h, j) of part_o / part_m / part_e.  K and V are read once
 * per kv-head; all q-heads of a group share that read.
 */
da_status da_partial(const da_plan *plan, const void *q, const void *k_pool, const void *v_pool,
                     const int32_t *block_table, const int32_t *seq_lens,
                     float *part_o, float *part_m, float *part_e, void *stream);

/*
 * Aggregation (Section 4, m_g / e_g equation and Eq. 3): per (request, q-head)
 *   m_g = max_j m_j,  e_g = sum_j e_j exp(m_j - m_g),
 *   out = sum_j MA_j exp(m_j - m_g) / e_g,   lse = m_g + ln e_g  (lse may be NULL).
 * The partials may come from da_partial or from anywhere else that follows the
 * row convention (e.g. another device's MicroAttention).
 */
da_status da_combine(const da_plan *plan, const float *part_o, const float *part_m, const float *part_e,
                     float *out, float *lse, void *stream);

/*
 * Aggregation over several partial sets.  Section 4: the intermediate results
 * of the instances that hold parts of a request's KV cache are brought to the
 * request's home instance and aggregated there (Eq. 3); Section 5.2: the local
 * MicroAttention overlaps the remote ones.  Each set is the output of one
 * da_partial over one share of the batch's KV cache (its own pools, block
 * table, lengths and plan; all shares have the same batch, heads and q_len and
 * were given the same queries).  A request's tokens may be divided among the
 * shares in any way, a share may hold none of them (length 0).  At most 4 sets.
 * In the multi-query form every share applies the causal rule to its own
 * length, so only the share holding the newest tokens may have q_len > 1
 * tokens of them; the tests use q_len = 1.
 * Launches nothing on the shares' streams: the caller orders `stream` after
 * the da_partial launches (events) before calling.
 */
typedef struct {
    const da_plan *plan;
    const float *part_o;
    const float *part_m;
    const float *part_e;
} da_partial_set;
da_status da_combine_multi(const da_partial_set *sets, int32_t num_sets, float *out, float *lse, void *stream);

/*
 * Fused convenience call: MicroAttention into `workspace`, then aggregation,
 * on one stream = Section 4, Eq. 1.  A request with a single split is
 * normalised inside the MicroAttention kernel and skips the aggregation.
 * workspace_bytes must be >= da_workspace_bytes(); workspace 256-byte aligned.
 */
da_status da_attention(const da_plan *plan, const void *q, const void *k_pool, const void *v_pool,
                       const int32_t *block_table, const int32_t *seq_lens, float *out, float *lse,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * da_attention for callers that cannot allocate device memory or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments and result as da_attention, minus the
 * workspace: the partial results go to a fixed array of DA_NOALLOC_SCRATCH_BYTES inside the library's device
 * image (every GPU the library runs on holds one until the process ends).  The call allocates and frees nothing
 * and launches the same kernels as da_attention.  A plan whose da_workspace_bytes() exceeds
 * DA_NOALLOC_SCRATCH_BYTES is rejected with DA_ERR_WORKSPACE before anything is launched.
 * All calls on one GPU share that GPU's array, which keeps the last call's contents (nothing in it needs clearing:
 * every row that is read was written by the same call first): calls that overlap on one GPU, on different
 * streams or from different threads, race; order them on one stream or by events.
 */
#define DA_NOALLOC_SCRATCH_BYTES ((size_t)8 << 20)
da_status da_attention_noalloc(const da_plan *plan, const void *q, const void *k_pool, const void *v_pool,
                               const int32_t *block_table, const int32_t *seq_lens, float *out, float *lse,
                               void *stream);

/*
 * KV append, the step before attention in every decode iteration (Section 4:
 * the cache is sliced along the sequence dimension so that newly generated
 * tokens join the sub-block layout as they are produced).  k_new / v_new hold
 * one new token per request, [batch][num_kv_heads][head_dim] in kv_dtype
 * (16-byte aligned).  For every request r with L = seq_lens[r] >= 0 the rows
 * are written to slot L % block_tokens of block block_table[r][L / block_tokens]
 * of both pools, for all kv-heads, and seq_lens[r] becomes L + 1 (device side,
 * in stream order: an attention launch that follows on the same stream sees
 * the new token).  L < 0 marks an inactive batch slot and is left alone.  The
 * block must already be in the table (da_block_pool_grow); a request whose
 * position has no valid block (bit 0) or whose table row is full (bit 1) is
 * skipped and the bit is OR-ed into *err_flags (device int32, may be NULL).
 * Uses of `problem`: batch, num_kv_heads, head_dim, block_tokens,
 * max_blocks_per_seq, num_phys_blocks, kv_dtype and the three strides.
 */
da_status da_append(const da_problem *problem, const void *k_new, const void *v_new, void *k_pool, void *v_pool,
                    const int32_t *block_table, int32_t *seq_lens, int32_t *err_flags, void *stream);

/*
 * KV block movement (Section 5.3, move_kvcache of Algorithm 1; Section 5.2: a
 * debtor places part of a request's KV cache in a creditor's memory): block
 * src_ids[i] of (k_src, v_src) is copied to block dst_ids[i] of (k_dst, v_dst),
 * all kv-heads and all block_tokens slots, bytes unchanged, for i <
 * num_blocks.  src_ids / dst_ids are DEVICE int32 arrays.  The two layouts
 * must agree in num_kv_heads, head_dim, block_tokens and kv_dtype; their
 * strides and pool sizes may differ (fields used: those, num_phys_blocks and
 * the three strides).  The destination ids must be distinct, and when source
 * and destination are the same pools no destination block may also be a
 * source.  A pair with an id outside its pool is skipped and bit 0 is OR-ed
 * into *err_flags (device int32, may be NULL).  The caller rewrites the block
 * tables; enqueue on a second stream to run the copy beside attention.
 */
da_status da_move_blocks(const da_problem *src_layout, const da_problem *dst_layout, const void *k_src,
                         const void *v_src, void *k_dst, void *v_dst, const int32_t *src_ids, const int32_t *dst_ids,
                         int32_t num_blocks, int32_t *err_flags, void *stream);

/*
 * Host-side free list of physical KV blocks (Section 4: sub-blocks are the
 * unit in which the growing cache is managed; Section 5.1: they are pooled).
 * No GPU call.  da_block_pool_grow appends fresh block ids to a request's HOST
 * block-table row so that it can hold new_len tokens (it held cur_len); the
 * caller copies the changed entries to the device table.  If the pool has too
 * few free blocks nothing is taken and DA_ERR_NO_SPACE is returned.
 * da_block_pool_release returns the ceil(len / block_tokens) blocks of a row
 * and sets the entries to -1; an id that the pool did not hand out, or a
 * duplicate, is DA_ERR_INVALID_ARG and nothing is returned.
 */
typedef struct da_block_pool da_block_pool;
da_status da_block_pool_create(int32_t num_phys_blocks, da_block_pool **pool);
da_status da_block_pool_destroy(da_block_pool *pool);
da_status da_block_pool_free_count(const da_block_pool *pool, int32_t *count);
da_status da_block_pool_grow(da_block_pool *pool, int32_t block_tokens, int32_t max_blocks_per_seq,
                             int32_t *block_table_row_host, int32_t cur_len, int32_t new_len);
da_status da_block_pool_release(da_block_pool *pool, int32_t block_tokens, int32_t *block_table_row_host, int32_t len);

const char *da_status_string(da_status status);

#ifdef __cplusplus
}
#endif
#endif /* DISTATTN_H */
