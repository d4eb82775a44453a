/*
 * Rounds-scheduled speculative execution on one GPU (paper Section 3.3 "Rounds-Scheduled Strategy" and
 * Section 3.4, Algorithm 1): n draft branches and one target model; a branch drafts k tokens, waits in a
 * first-come-first-served queue until the target has verified them, and drafts again from what was
 * validated ("rounds"), until it holds max_new validated tokens.
 *
 * How Algorithm 1 is mapped onto one GPU: the draft model of all branches is ONE context whose branches are
 * decoded as a batch (seed_draft_step over a subset of cache slots), the target is another context
 * (seed_verify_step over a subset of slots).  The unit of scheduling is a group of at most `unit_branches`
 * branches that were ready together: it drafts its k tokens on the draft context's stream, is queued, and is
 * verified as one batch on the target context's stream, in arrival order; its branches then become ready
 * again.  With unit_branches = n this is plain (serial) batched speculative decoding; with smaller units
 * drafting of one unit overlaps verification of another, which is the paper's point: the target stays busy.
 * The paper's per-sequence verification is unit_branches = 1.
 *
 * Randomness is an input, consumed by POSITION and never "next from a stream", so the tokens of a branch do
 * not depend on how the units were formed: the uniform of draft token j of a round that starts with L
 * validated tokens is u_draft[b][L + j], of its accept test u_acc[b][L + j], of the round's replacement
 * token u_res[b][L].
 *
 * All pointers marked device are device memory owned by the caller; the call returns when every branch is
 * finished (it synchronises with both streams).  Errors: negative SEED_E_* codes (seed_last_error()).
 */
#ifndef SEED_SCHED_H
#define SEED_SCHED_H

#include "seed_verify.h"

#ifdef __cplusplus
extern "C" {
#endif

#define SEED_SCHED_MAX_BRANCHES 32

typedef struct {
    int32_t units;        /* scheduling units verified (= verify steps)                     */
    int32_t draft_steps;  /* seed_draft_step calls                                          */
    int32_t drafted;      /* draft tokens proposed                                          */
    int32_t accepted;     /* draft tokens accepted                                          */
    int32_t emitted;      /* validated tokens produced (before truncation to max_new)       */
    double wall_ms;       /* host wall-clock time of the run                                */
} seed_sched_stats;

typedef struct {
    int32_t n_branches;    /* n <= SEED_SCHED_MAX_BRANCHES, <= max_branches of both contexts             */
    int32_t gamma;         /* k: draft tokens per round (<= max_rows_per_branch of the target context)   */
    int32_t max_new;       /* l: validated tokens to produce per branch                                  */
    int32_t unit_branches; /* branches per scheduling unit; <= 0 or >= n: all ready branches together    */
    int32_t shared_len_target, shared_len_draft; /* prefix already in the shared caches of the contexts  */
    float temperature;     /* of both models                                                             */
    const int32_t *first_tok; /* host [n]: each branch's pending token (validated, KV not cached)        */
    const float *u_draft;     /* device [n][u_stride]                                                     */
    const float *u_acc;       /* device [n][u_stride]                                                     */
    const float *u_res;       /* device [n][u_stride]                                                     */
    int32_t u_stride;         /* >= max_new + gamma                                                       */
    int32_t *target_private_len; /* device [max_branches of target]: in/out, branch b is slot b          */
    int32_t *draft_private_len;  /* device [max_branches of draft]:  in/out                               */
    void *workspace;          /* device, 256-byte aligned, seed_sched_workspace_bytes(...) bytes         */
    size_t workspace_bytes;
    int32_t *out_tok;         /* host [n][max_new] out                                                    */
    int32_t *out_len;         /* host [n] out (= max_new unless the run failed)                          */
    seed_sched_stats *stats;  /* host out, may be NULL                                                    */
} seed_sched_args;

/* Device scratch the scheduler needs: draft distributions q of the units in flight, token and uniform
 * staging, accept outputs. */
size_t seed_sched_workspace_bytes(int32_t n_branches, int32_t gamma, int32_t vocab);

/* Runs Algorithm 1 to completion.  Both contexts must be bf16 contexts of models with the same vocabulary;
 * they should have been created on two different HIP streams (on one stream the run is still correct,
 * without overlap).  Each context needs max_private >= (its private_len on entry) + max_new + gamma. */
int seed_sched_run(seed_ctx *target, seed_ctx *draft, const seed_sched_args *args);

#ifdef __cplusplus
}
#endif
#endif
