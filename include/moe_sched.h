/* moe_sched.h -- C ABI of the frontend's scheduling round (host-only; no GPU call is made).
 *
 * One round assigns queued prefill requests to the N data-parallel GPU workers (App. A,
 * Alg. 1).  For every request, in arrival order, the scheduler looks only at workers whose
 * FLOPs load L_i is still below the saturation threshold T (Sec. 7.4), picks the one whose
 * block table shares the longest run of leading prefix blocks with the request (Sec. 7.2;
 * blocks of B tokens, identified by chained hashes), breaks ties by the smaller load and then
 * by the lower worker index, charges the worker the true cost of the request after prefix
 * reuse (Eq. 2, Sec. 7.3) and retires it once L_i >= T.  The round ends when every worker is
 * saturated or the queue is empty; every saturated worker's load then lies in
 * [T, T + Delta_last] (Sec. 7.4).
 *
 * Block tables follow App. B.2: each worker has a committed set (blocks the engine reported
 * as materialised) and a pending set (blocks promised by requests already routed); the match
 * rule reads their union, and routing a request adds its not-yet-committed prefix blocks to
 * the worker's pending set at once, which is what lets same-prefix requests of one burst
 * follow each other.
 *
 * Cost model (Eq. 2; the paper names the terms and leaves their formulas to the model):
 *   Delta = C_pfx(P - M) + C_sfx(S, P)
 *   C_pfx(n)   = f_tok*n + f_attn*n(n+1)/2
 *   C_sfx(S,P) = f_tok*S + f_attn*S(S+1)/2 + f_attn*S*P
 * P, S: prefix and suffix length in tokens, M: matched tokens (a multiple of B).  f_attn = 0
 * gives Delta = (uncached tokens) * f_tok, the single-constant form of App. B.2.
 * Arithmetic: the token counts and pair counts are formed in int64, converted to double, and
 * Delta = f_tok*(double)(P - M + S) + f_attn*(double)pairs, two products and one sum in IEEE
 * double without contraction; loads are running double sums in assignment order.
 *
 * All pointers are HOST memory owned by the caller.  Functions return MOE_OK (0) or a
 * negative moe_status (moe_prefill.h); on an error nothing has been changed.  A scheduler
 * object must not be used from two threads at once.
 */
#ifndef MOE_SCHED_H
#define MOE_SCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moe_sched moe_sched_t;

typedef struct moe_cost_model {
    double f_tok;  /* FLOPs per token of all linear layers (>= 0) */
    double f_attn; /* FLOPs per (query token, key token) pair of attention, all layers (>= 0) */
} moe_cost_model_t;

/* n_workers in [1, 4096], block_tokens in [1, 65536]. */
int32_t moe_sched_create(int32_t n_workers, int32_t block_tokens, moe_sched_t **out);
void moe_sched_destroy(moe_sched_t *s);

/* Chained block hashes of a token sequence: hashes[j] identifies tokens [0, (j+1)*B), so two
 * sequences have equal hashes[j] exactly when they agree on all of their first (j+1)*B tokens
 * (up to 64-bit collisions).  Writes n_tokens / block_tokens values (the trailing partial
 * block has none).  The function is pure; every table entry must come from it. */
int32_t moe_sched_hash_blocks(const int32_t *tokens, int64_t n_tokens, int32_t block_tokens,
                              uint64_t *hashes);

/* One round (Alg. 1, step 1).
 *   block_hashes, hash_offsets[n_requests+1]: request r's prefix blocks are
 *       block_hashes[hash_offsets[r] .. hash_offsets[r+1]); their number must be
 *       prefix_tokens[r] / block_tokens.
 *   prefix_tokens[r] = |p_r|, suffix_tokens[r] = |s_r| (>= 0).
 *   loads[n_workers]: in = L_i at the start of the round (zeros for Alg. 1 as printed; a
 *       caller that decays the counters between rounds as in App. B.3 passes them back in),
 *       out = L_i after the round.
 *   assigned[r]: worker of request r, or -1 for every request from the first one that found
 *       no unsaturated worker (they stay queued; *n_assigned requests were consumed).
 *   matched_tokens[r] (M_r) and delta[r] (Delta_r): optional (NULL to skip); 0 for unassigned
 *       requests. */
int32_t moe_sched_round(moe_sched_t *s, const moe_cost_model_t *cost, double threshold,
                        int64_t n_requests, const uint64_t *block_hashes,
                        const int64_t *hash_offsets, const int64_t *prefix_tokens,
                        const int64_t *suffix_tokens, double *loads, int32_t *assigned,
                        int64_t *matched_tokens, double *delta, int64_t *n_assigned);

/* Engine life-cycle events (App. B.2, B.3; Alg. 1, step 2): blocks now materialised on a worker
 * move from pending to committed (unknown ones are added as committed); evicted blocks leave
 * the committed set. */
int32_t moe_sched_blocks_stored(moe_sched_t *s, int32_t worker, const uint64_t *hashes, int64_t n);
int32_t moe_sched_blocks_evicted(moe_sched_t *s, int32_t worker, const uint64_t *hashes, int64_t n);

/* Progress report of an engine (App. B.3): `tokens` prompt tokens were executed on `worker`, so its
 * counter decays by tokens * f_tok, never below zero: loads[worker] = max(0, loads[worker] -
 * tokens * f_tok).  Enqueue (moe_sched_round with f_attn = 0) and decay use the same f_tok, which
 * keeps the counter free of drift. */
int32_t moe_sched_tokens_executed(const moe_sched_t *s, double *loads, int32_t worker, int64_t tokens,
                                  double f_tok);

/* Entries of one worker's table. */
int32_t moe_sched_table_size(const moe_sched_t *s, int32_t worker, int64_t *committed,
                             int64_t *pending);

#ifdef __cplusplus
}
#endif
#endif /* MOE_SCHED_H */
