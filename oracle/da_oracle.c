/*
 * CPU oracle for DistAttention decode attention.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, obviously-correct reference that the HIP library is
 * judged against.  It shares no code, header, table or helper with the HIP
 * path, and nothing in the product path may call it: only the tests, the smoke
 * check and the benchmark's cpu_baseline leg do.
 *
 * Everything is computed in fp64.  Stored inputs (fp32, IEEE half, or bf16 held as
 * uint16) are widened exactly; nothing is blocked, fused or reordered beyond
 * what the cited formula states.
 *
 *   oracle_attention        Section 4, Eq. 1: plain attention with the global
 *                           maximum m_g, written out as the definition.
 *   oracle_micro_attention  Section 4, the unnumbered m_j / e_j equation and
 *                           Eq. 2: MicroAttention over one partition.
 *   oracle_aggregate        Section 4, the unnumbered m_g / e_g equation and
 *                           Eq. 3: aggregation of b partial results.
 *
 * Multi-query form (several new tokens per request, e.g. speculative decoding
 * or chunked prefill; Section 2.1 describes prefill and decode, Section 3 says
 * the partition may be of arbitrary length): q is [B][q_len][Hq][d], the cache
 * already holds all q_len new tokens, and query t of a request of length L
 * attends to the tokens i < L - (q_len - 1 - t), i.e. causally.  A "virtual
 * head" index vh = t * Hq + h addresses the (query token, q-head) pairs, so
 * outputs are [B][q_len * Hq][d]; q_len = 1 is plain decode.
 *
 * Readings of the paper adopted here (it is silent on each):
 *   - scores are scale * (q . k_i); the equations print a bare QK_i^T;
 *   - one query per request (decode); it attends to every cached token
 *     i < seq_len, so there is no causal mask;
 *   - grouped-query attention: q-head h reads kv-head h / (Hq / Hkv);
 *   - logical token i of request r lives in physical block
 *     block_table[r][i / T] at slot i % T; slots at or past seq_len, and
 *     blocks the table does not name, never influence the result;
 *   - an empty request gives out = 0 and lse = -inf; an empty partition gives
 *     m = -inf, e = 0, MA = 0, and aggregation gives it weight 0.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py
 * (brute force in exact rational arithmetic, closed forms, invariances, the
 * textbook softmax(QK^T)V via a library, and the partition invariant).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2 };

/* Exact widening of one stored element to fp64. */
static double widen(const void *base, int dtype, int64_t idx)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    if (dtype == ORACLE_F16) {
        /* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits */
        uint16_t h = ((const uint16_t *)base)[idx];
        int sign = h >> 15, expo = (h >> 10) & 31, frac = h & 1023;
        double v;
        if (expo == 0)
            v = ldexp((double)frac, -24);                 /* zero and subnormals: frac * 2^-24 */
        else if (expo == 31)
            v = frac ? NAN : INFINITY;
        else
            v = ldexp(1.0 + (double)frac / 1024.0, expo - 15);
        return sign ? -v : v;
    }
    /* bf16 is the upper half of an IEEE fp32 */
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

typedef struct {
    const void *q;           /* [B][Hq][d] */
    const void *k_pool;      /* physical block pb, kv-head g, slot s, dim c at */
    const void *v_pool;      /*   pb*stride_block + g*stride_head + s*stride_token + c */
    const int32_t *block_table; /* [B][max_blocks] */
    const int32_t *seq_lens; /* [B] */
    int q_dtype, kv_dtype;
    int B, Hq, Hkv, d, T, max_blocks;
    int64_t stride_block, stride_head, stride_token;
    double scale;
    int q_len;               /* query tokens per request, >= 1 */
} oracle_problem;

/* Tokens that virtual head vh = t * Hq + h of request r may see. */
static int64_t visible_tokens(const oracle_problem *p, int r, int vh)
{
    int t = vh / p->Hq;
    int64_t n = (int64_t)p->seq_lens[r] - (p->q_len - 1 - t);
    return n > 0 ? n : 0;
}

/* Element offset of logical token i of request r, kv-head g, in a pool. */
static int64_t token_offset(const oracle_problem *p, int r, int g, int64_t i)
{
    int64_t logical_block = i / p->T;
    int64_t slot = i % p->T;
    int64_t pb = p->block_table[(int64_t)r * p->max_blocks + logical_block];
    return pb * p->stride_block + (int64_t)g * p->stride_head + slot * p->stride_token;
}

/* s_i = scale * sum_c q[r][t][h][c] * K_i[c], with vh = t * Hq + h */
static double score(const oracle_problem *p, int r, int vh, int64_t i)
{
    int g = (vh % p->Hq) / (p->Hq / p->Hkv);
    int64_t koff = token_offset(p, r, g, i);
    int64_t qoff = ((int64_t)r * p->q_len * p->Hq + vh) * p->d;
    double acc = 0.0;
    for (int c = 0; c < p->d; ++c)
        acc += widen(p->q, p->q_dtype, qoff + c) * widen(p->k_pool, p->kv_dtype, koff + c);
    return p->scale * acc;
}

/*
 * Section 4, Eq. 1.  For each listed (request, q-head) pair:
 *   m_g = max_i s_i
 *   out = sum_i exp(s_i - m_g) V_i / sum_j exp(s_j - m_g)
 *   lse = m_g + log(sum_j exp(s_j - m_g))
 * pairs: n_pairs x 2 int32 (r, h); NULL means every pair in (r, h) order.
 * out: [n_pairs][d] fp64, lse: [n_pairs] fp64 (may be NULL).
 */
int oracle_attention(const oracle_problem *p, const int32_t *pairs, int64_t n_pairs,
                     double *out, double *lse, int n_threads)
{
    if (!p || !out || p->Hkv <= 0 || p->Hq % p->Hkv != 0 || p->T <= 0 || p->q_len < 1)
        return 1;
    const int VH = p->q_len * p->Hq; /* virtual heads per request */
    if (!pairs)
        n_pairs = (int64_t)p->B * VH;
    if (n_threads < 1)
        n_threads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
    for (int64_t w = 0; w < n_pairs; ++w) {
        int r = pairs ? pairs[2 * w] : (int)(w / VH);
        int h = pairs ? pairs[2 * w + 1] : (int)(w % VH);
        int g = (h % p->Hq) / (p->Hq / p->Hkv);
        int64_t L = visible_tokens(p, r, h);
        double *o = out + w * p->d;
        for (int c = 0; c < p->d; ++c)
            o[c] = 0.0;
        if (L <= 0) {
            if (lse)
                lse[w] = -INFINITY;
            continue;
        }
        /* pass 1: the global maximum */
        double m_g = -INFINITY;
        for (int64_t i = 0; i < L; ++i) {
            double s = score(p, r, h, i);
            if (s > m_g)
                m_g = s;
        }
        /* pass 2: numerator and denominator */
        double denom = 0.0;
        for (int64_t i = 0; i < L; ++i) {
            double w_i = exp(score(p, r, h, i) - m_g);
            int64_t voff = token_offset(p, r, g, i);
            denom += w_i;
            for (int c = 0; c < p->d; ++c)
                o[c] += w_i * widen(p->v_pool, p->kv_dtype, voff + c);
        }
        for (int c = 0; c < p->d; ++c)
            o[c] /= denom;
        if (lse)
            lse[w] = m_g + log(denom);
    }
    return 0;
}

/*
 * Section 4, m_j / e_j equation and Eq. 2.  The tokens of every request are
 * cut at the caller's boundaries: partition j of request r covers tokens
 * [bounds[boff[r] + j], bounds[boff[r] + j + 1]), for j < nparts[r], where
 * boff[r] = sum_{r' < r} (nparts[r'] + 1).  Boundaries need not be multiples
 * of the block size.  Results land in row
 *   row(r, h, j) = Hq * sum_{r' < r} nparts[r']  +  h * nparts[r]  +  j
 * (Hq counts virtual heads, q_len * Hq, in the multi-query form) of MA [rows][d], m [rows], e [rows]:
 *   m_j = max_i s_i,  e_j = sum_i exp(s_i - m_j),  MA_j = sum_i exp(s_i - m_j) V_i
 * (un-normalised, as printed).
 */
int oracle_micro_attention(const oracle_problem *p, const int32_t *nparts, const int64_t *bounds,
                           double *MA, double *m, double *e, int n_threads)
{
    if (!p || !nparts || !bounds || !MA || !m || !e || p->Hkv <= 0 || p->Hq % p->Hkv != 0 || p->q_len < 1)
        return 1;
    if (n_threads < 1)
        n_threads = 1;
    const int VH = p->q_len * p->Hq;
    int64_t n_pairs = (int64_t)p->B * VH;
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
    for (int64_t w = 0; w < n_pairs; ++w) {
        int r = (int)(w / VH), h = (int)(w % VH);
        int g = (h % p->Hq) / (p->Hq / p->Hkv);
        int64_t vis = visible_tokens(p, r, h);
        int64_t row0 = 0, boff = 0;
        for (int rr = 0; rr < r; ++rr) {
            row0 += (int64_t)VH * nparts[rr];
            boff += nparts[rr] + 1;
        }
        row0 += (int64_t)h * nparts[r];
        for (int j = 0; j < nparts[r]; ++j) {
            int64_t lo = bounds[boff + j], hi = bounds[boff + j + 1];
            if (hi > vis)
                hi = vis; /* causal limit of this query token */
            double *o = MA + (row0 + j) * p->d;
            for (int c = 0; c < p->d; ++c)
                o[c] = 0.0;
            double m_j = -INFINITY;
            for (int64_t i = lo; i < hi; ++i) {
                double s = score(p, r, h, i);
                if (s > m_j)
                    m_j = s;
            }
            double e_j = 0.0;
            for (int64_t i = lo; i < hi; ++i) {
                double w_i = exp(score(p, r, h, i) - m_j);
                int64_t voff = token_offset(p, r, g, i);
                e_j += w_i;
                for (int c = 0; c < p->d; ++c)
                    o[c] += w_i * widen(p->v_pool, p->kv_dtype, voff + c);
            }
            m[row0 + j] = m_j;
            e[row0 + j] = e_j;
        }
    }
    return 0;
}

/*
 * Section 4, m_g / e_g equation and Eq. 3.  Same row convention as above:
 *   m_g = max_j m_j,  e_g = sum_j e_j exp(m_j - m_g),
 *   out = sum_j MA_j exp(m_j - m_g) / e_g,   lse = m_g + log(e_g).
 * A partition with m_j = -inf has weight 0; if every partition is empty the
 * output is 0 and lse is -inf.  out: [B][Hq][d], lse: [B][Hq] (may be NULL).
 */
int oracle_aggregate(int B, int Hq, int d, const int32_t *nparts,
                     const double *MA, const double *m, const double *e,
                     double *out, double *lse)
{
    if (!nparts || !MA || !m || !e || !out)
        return 1;
    int64_t row0 = 0;
    for (int r = 0; r < B; ++r) {
        for (int h = 0; h < Hq; ++h) {
            int b = nparts[r];
            const double *mj = m + row0, *ej = e + row0;
            double *o = out + ((int64_t)r * Hq + h) * d;
            for (int c = 0; c < d; ++c)
                o[c] = 0.0;
            double m_g = -INFINITY;
            for (int j = 0; j < b; ++j)
                if (mj[j] > m_g)
                    m_g = mj[j];
            double e_g = 0.0;
            for (int j = 0; j < b; ++j) {
                double w_j = (mj[j] == -INFINITY) ? 0.0 : exp(mj[j] - m_g);
                e_g += ej[j] * w_j;
                for (int c = 0; c < d; ++c)
                    o[c] += MA[(row0 + j) * d + c] * w_j;
            }
            if (e_g > 0.0) {
                for (int c = 0; c < d; ++c)
                    o[c] /= e_g;
                if (lse)
                    lse[(int64_t)r * Hq + h] = m_g + log(e_g);
            } else {
                for (int c = 0; c < d; ++c)
                    o[c] = 0.0;
                if (lse)
                    lse[(int64_t)r * Hq + h] = -INFINITY;
            }
            row0 += b;
        }
    }
    return 0;
}

/*
 * KV append, written out as its definition (Section 4: new tokens join the
 * sub-block layout along the sequence dimension).  For every request r with
 * L = seq_lens[r] >= 0: the K and V rows of the new token (k_new / v_new,
 * [B][Hkv][d] in the stored dtype, raw bytes) go to slot L % T of physical
 * block block_table[r][L / T] of both pools, for every kv-head, and
 * seq_lens[r] becomes L + 1.  A request whose position has no valid block, or
 * whose table row is full, is left untouched.  elem_size is 2 (bf16) or 4.
 */
int oracle_append(const void *k_new, const void *v_new, void *k_pool, void *v_pool,
                  const int32_t *block_table, int32_t *seq_lens,
                  int B, int Hkv, int d, int T, int max_blocks, int num_phys, int elem_size,
                  int64_t stride_block, int64_t stride_head, int64_t stride_token)
{
    if (!k_new || !v_new || !k_pool || !v_pool || !block_table || !seq_lens)
        return 1;
    for (int r = 0; r < B; ++r) {
        int64_t L = seq_lens[r];
        if (L < 0)
            continue;
        int64_t logical_block = L / T, slot = L % T;
        if (logical_block >= max_blocks)
            continue;
        int64_t pb = block_table[(int64_t)r * max_blocks + logical_block];
        if (pb < 0 || pb >= num_phys)
            continue;
        for (int g = 0; g < Hkv; ++g) {
            int64_t dst = (pb * stride_block + g * stride_head + slot * stride_token) * elem_size;
            int64_t src = (((int64_t)r * Hkv + g) * d) * elem_size;
            memcpy((char *)k_pool + dst, (const char *)k_new + src, (size_t)d * elem_size);
            memcpy((char *)v_pool + dst, (const char *)v_new + src, (size_t)d * elem_size);
        }
        seq_lens[r] = (int32_t)(L + 1);
    }
    return 0;
}

/*
 * KV block movement (Section 5.3, move_kvcache of Algorithm 1; Section 5.2: part
 * of a debtor's KV cache is placed in a creditor's memory).  Block src_ids[i] of
 * the source pools is copied to block dst_ids[i] of the destination pools, all
 * kv-heads, all T slots, K and V, bytes unchanged.  A pair with an id outside
 * its pool is skipped.  Pairs are taken in order (a later pair may overwrite an
 * earlier destination).  Pools are [P][Hkv][T][d] with the given element strides.
 */
int oracle_move_blocks(const void *k_src, const void *v_src, void *k_dst, void *v_dst,
                       const int32_t *src_ids, const int32_t *dst_ids, int n,
                       int Hkv, int d, int T, int elem_size, int num_src, int num_dst,
                       int64_t src_stride_block, int64_t src_stride_head, int64_t src_stride_token,
                       int64_t dst_stride_block, int64_t dst_stride_head, int64_t dst_stride_token)
{
    if (!k_src || !v_src || !k_dst || !v_dst || (n > 0 && (!src_ids || !dst_ids)))
        return 1;
    for (int i = 0; i < n; ++i) {
        int64_t a = src_ids[i], b = dst_ids[i];
        if (a < 0 || a >= num_src || b < 0 || b >= num_dst)
            continue;
        for (int g = 0; g < Hkv; ++g) {
            for (int s = 0; s < T; ++s) {
                int64_t from = (a * src_stride_block + g * src_stride_head + s * src_stride_token) * elem_size;
                int64_t to = (b * dst_stride_block + g * dst_stride_head + s * dst_stride_token) * elem_size;
                memcpy((char *)k_dst + to, (const char *)k_src + from, (size_t)d * elem_size);
                memcpy((char *)v_dst + to, (const char *)v_src + from, (size_t)d * elem_size);
            }
        }
    }
    return 0;
}
