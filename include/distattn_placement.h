/*
 * distattn_placement.h - C ABI of the cluster-level KV placement step of
 * Infinite-LLM (Section 5.3): the per-layer performance model (Eq. 5, Eq. 6),
 * the throughput of an instance and of the cluster (TPS = beta / (n T), Eq. 7)
 * and the greedy debtor / creditor scheduler (Algorithm 1).
 *
 * Pure host code: every pointer is HOST memory owned by the caller, nothing is
 * allocated that outlives a call, no GPU call is made.  All arithmetic is fp64.
 * Entry points return a da_status (distattn.h); none aborts, throws or prints.
 *
 * Model (Section 5.3).  One layer of an instance with batch size beta and
 * request lengths S^r takes T^lyr = T^natn(beta) + sum_r S^r / g  (Eq. 5),
 * T^natn(beta) = W(beta) / f(beta) being the measured non-attention time at
 * that batch size (a table) and g the attention rate in tokens per second (a
 * constant: it is the token rate of the MicroAttention kernel).  A debtor that
 * keeps K^d tokens of its KV cache on creditors saves K^d / g; a creditor that
 * holds K^c tokens for debtors pays K^c / g (Eq. 6).  TPS = beta / (n T^lyr).
 * Remote blocks are full blocks of block_tokens tokens, except that a request
 * whose every block is remote counts its S^r tokens (its last block may be
 * partly filled).
 *
 * Where the paper leaves the method open this library takes these readings:
 *  - beta' of Eq. 6: an instance states how many requests wait in its queue
 *    (`waiting`) and how many blocks one of them needs (`admit_blocks`); the
 *    blocks it frees admit as many of them as fit (and as the T^natn table
 *    covers), each adding admit_blocks * block_tokens tokens of attention work.
 *  - roles (Section 5.2: never debtor and creditor at once): an instance whose
 *    utilisation used / capacity is <= u_thres and that has lent nothing out
 *    is a creditor; a debtor has batch size <= beta_thres, is no creditor,
 *    holds at least one request and hosts nothing.
 *  - the candidate block counts are k = 0 .. Block_max - 1 (the request's last
 *    block, where new tokens are appended, stays with the debtor), bounded by
 *    the creditor's free blocks; among equal estimates the smallest k wins, so
 *    "no gain" is k = 0 and ends the debtor's turn.
 *  - a debtor tries each creditor at most once, always the untried creditor
 *    with the lowest utilisation at that moment; ties in every ordering go to
 *    the lower instance index; one request (the longest) per debtor per call.
 */
#ifndef DISTATTN_PLACEMENT_H
#define DISTATTN_PLACEMENT_H

#include <stdint.h>

#include "distattn.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t num_layers;        /* n >= 1 */
    int32_t block_tokens;      /* tokens per KV block, >= 1 */
    double attn_tokens_per_s;  /* g > 0 (may be +inf) */
    const double *t_natn;      /* [t_natn_len] seconds per layer of non-attention work at batch size b; finite, >= 0 */
    int32_t t_natn_len;        /* >= 1; batch sizes above t_natn_len - 1 are not admitted */
} da_perf_model;

typedef struct {
    int32_t num_requests;             /* beta >= 0, <= t_natn_len - 1 */
    const int64_t *req_tokens;        /* [num_requests] S^r >= 1 */
    const int32_t *req_remote_blocks; /* [num_requests] blocks of r already held by creditors, or NULL for none;
                                         0 <= value <= ceil(S^r / block_tokens) */
    int32_t hosted_blocks;            /* blocks held for other instances, >= 0 */
    int32_t capacity_blocks;          /* >= 1 */
    int32_t waiting;                  /* queued requests, >= 0 */
    int32_t admit_blocks;             /* blocks a queued request needs; 0 = nothing is admitted */
} da_instance;

typedef struct {
    int32_t debtor;   /* instance index */
    int32_t request;  /* index into the debtor's req_tokens */
    int32_t creditor; /* instance index */
    int32_t blocks;   /* >= 1 */
} da_move;

/* TPS of one instance in its present state (Eq. 5 with both shifts of Eq. 6). */
da_status da_model_instance_tps(const da_perf_model *model, const da_instance *instance, double *tps);

/* Eq. 7 over `num_instances` instances. */
da_status da_model_cluster_tps(const da_perf_model *model, const da_instance *instances, int32_t num_instances,
                               double *tps);

/*
 * perf_model_throughput_esti(k, D, C) of Algorithm 1: summed TPS of the pair
 * after k more blocks of the debtor went to the creditor (the debtor admitting
 * what then fits).  k >= 0; k is not checked against the creditor's free space.
 */
da_status da_model_pair_estimate(const da_perf_model *model, const da_instance *debtor, const da_instance *creditor,
                                 int32_t k, double *tps);

/*
 * Algorithm 1.  Writes the moves in the order they are decided to
 * moves[0 .. *num_moves); later decisions see the effect of earlier ones.  The
 * input instances are not modified.  tps_before / tps_after (optional) receive
 * the modelled cluster throughput of the given state and of the state after
 * all moves.  At most (number of debtors) x (number of creditors) moves can result; if
 * max_moves is too small DA_ERR_WORKSPACE is returned, *num_moves holds the
 * number needed and moves holds the first max_moves of them.
 * DA_ERR_INVALID_ARG: null pointer, a field outside the ranges stated above.
 */
da_status da_placement_schedule(const da_perf_model *model, const da_instance *instances, int32_t num_instances,
                                int32_t beta_thres, double u_thres, da_move *moves, int32_t max_moves,
                                int32_t *num_moves, double *tps_before, double *tps_after);

#ifdef __cplusplus
}
#endif
#endif /* DISTATTN_PLACEMENT_H */
