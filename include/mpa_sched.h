/*
 * mpa_sched — the batch scheduler that feeds mpa_kv_append / mpa_mixed_paged_attention.
 * Host-only part of libmpa.so: no HIP call, usable without a GPU.
 *
 * After every iteration it forms the batch of the next one (paper Sec. 4):
 *   - the token budget S_b = S_pf * SLO_min / T_pf (Sec. 4.2, token budget determination);
 *   - requests ordered by remaining time T_r = SLO - T_w - N_ck * T_max, urgent when
 *     T_r <= T_max (Sec. 4.3); requests of offline applications carry a JCT SLO instead, spread
 *     over their iterations as an allowed waiting time whose unused or overdrawn part moves on
 *     to the next iteration (Sec. 4.3, SLOs of offline applications);
 *   - prompts cut dynamically where the budget or the KV cache ends, one long prompt at a time
 *     (Sec. 4.2, dynamic chunking; limiting running long-prompt requests);
 *   - KV-cache demand per request in whole blocks, later chunks first filling the free slots of
 *     their last block (Sec. 4.4);
 *   - the batching algorithm: urgent requests first, the request with the largest T_r gives way
 *     while tokens or blocks are over-committed, the rest of both resources filled by repeatedly
 *     taking, among the requests within gamma of the first non-urgent one, the one whose demand
 *     (tokens, KV) is nearest to what is available (Sec. 4.4, Algorithms 1 and 2);
 * and hands out the arrays the attention path takes: chunk_starts, context_lens, slot_map and the
 * block table, over a block pool it manages itself.
 *
 * A request runs as prompt chunks until all its prompt tokens are cached; the last chunk yields
 * its first token.  From then on it is a generation task that feeds one token per iteration.  A
 * generation task preempted because blocks ran out gives its blocks back and re-enters as a
 * prompt over all its tokens (recomputation) -- or, with a swap pool configured and room in it, has
 * its blocks copied there and copied back into fresh blocks when it is scheduled again (the pairs
 * to copy come with the batch; mpa_copy_blocks does the copying); one preempted for the token
 * budget keeps its blocks.
 *
 * All pointers are host memory.  Functions return MPA_OK or a negative MPA_ERR_* of mpa.h; no C++
 * exception leaves them.  After MPA_ERR_NO_MEMORY (the host ran out of memory half way through a
 * decision) the scheduler's state is unspecified: destroy it.
 * One scheduler must not be used from two threads at once.
 */
#ifndef MPA_SCHED_H
#define MPA_SCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mpa_sched mpa_sched; /* opaque */

typedef struct {
    int32_t block_size;         /* b, tokens per KV block (any positive value)                  */
    int32_t num_blocks;         /* blocks of the pool                                           */
    int32_t pivot_forward_size; /* S_pf: forward size that saturates the GPU (Sec. 4.2)         */
    int32_t max_batch_tokens;   /* upper limit of the token budget (sizes the caller's buffers) */
    double pivot_time;          /* T_pf: batch execution time at S_pf, seconds                  */
    double max_batch_time;      /* T_max: longest batch execution time, seconds (Sec. 4.3)      */
    double gamma;               /* window of remaining times considered together (Sec. 4.4)     */
    double preempt_max_time;    /* P_max: longest preemption, seconds; offline requests only    */
    double preempt_probability; /* P: chance of a preemption after a generated token (Sec. 4.3) */
    int32_t num_swap_blocks;    /* blocks of the swap pool; 0 = preempted tasks are recomputed    */
} mpa_sched_config;

typedef struct {
    int32_t num_seqs;           /* S: sequences in the batch                                    */
    int32_t num_tokens;         /* T: forward size S_f                                          */
    int32_t token_budget;       /* S_b of this iteration                                        */
    int32_t num_prompt_chunks;  /* sequences with a prompt chunk                                */
    int32_t num_generation;     /* sequences with one generation token                          */
    int32_t num_preempted;      /* requests taken out of the batch by this decision             */
    int32_t max_blocks_per_seq; /* widest block-table row of the batch                          */
    int32_t free_blocks;        /* blocks left in the pool after this batch's allocations       */
    int32_t num_swap_out;       /* blocks to copy from the cache pool to the swap pool ...      */
    int32_t num_swap_in;        /* ... and from the swap pool into the cache pool, see below    */
} mpa_sched_batch;

/* block_order: [num_blocks], a permutation of 0..num_blocks-1 giving the order in which fresh
 * blocks are handed out (NULL = ascending).  Errors: INVALID_ARG. */
int mpa_sched_create(mpa_sched **out, const mpa_sched_config *cfg, const int32_t *block_order);
int mpa_sched_destroy(mpa_sched *s);

/* A request enters the waiting queue at time `now` (seconds).  It will produce max_new_tokens
 * tokens (the prompt's own included), with slo_first seconds allowed for the first and slo_token
 * for each later one.  Errors: INVALID_ARG (duplicate id, lengths < 1, or prompt_len +
 * max_new_tokens - 1 tokens do not fit the pool). */
int mpa_sched_add_request(mpa_sched *s, int64_t id, int32_t prompt_len, int32_t max_new_tokens,
                          double slo_first, double slo_token, double now);

/* A request of an offline application: slo_jct seconds for the whole job, predicted_new_tokens =
 * S_g, the caller's estimate of how many tokens it will generate (it still stops after
 * max_new_tokens).  Its execution time is estimated as N_ck * T_max + S_g * (T_max + P_max * P) with
 * N_ck = ceil(prompt_len / L_c); the rest of the SLO, divided by N_ck + S_g, is the waiting time it is
 * allowed per iteration.  Errors: as mpa_sched_add_request, and predicted_new_tokens < 1. */
int mpa_sched_add_offline_request(mpa_sched *s, int64_t id, int32_t prompt_len, int32_t max_new_tokens,
                                  int32_t predicted_new_tokens, double slo_jct, double now);

/* Forms the batch of the next iteration at time `now` and allocates its blocks.  An empty batch
 * (num_seqs == 0) is a valid outcome. */
int mpa_sched_next_batch(mpa_sched *s, double now, mpa_sched_batch *info);

/* Copies out the arrays of the batch formed last (any pointer may be NULL to skip it):
 *   request_ids [S]; chunk_starts [S+1]; context_lens [S] (KV length after this iteration's
 *   append); slot_map [T] (block * b + offset of every batch token); block_table
 *   [S, block_table_stride] padded with -1, block_table_stride >= max_blocks_per_seq. */
int mpa_sched_batch_arrays(const mpa_sched *s, int64_t *request_ids, int32_t *chunk_starts,
                           int32_t *context_lens, int64_t *slot_map, int32_t *block_table,
                           int32_t block_table_stride);

/* Block copies the batch formed last asks for, as {source block, destination block} pairs in the
 * layout mpa_copy_blocks takes: out_pairs [num_swap_out, 2] from the cache pool into the swap pool,
 * in_pairs [num_swap_in, 2] from the swap pool into the cache pool.  Both come before the
 * iteration's append, the copies out before the copies in (a block given up may be handed to a
 * returning request by the same decision).  Either pointer may be NULL. */
int mpa_sched_batch_swaps(const mpa_sched *s, int64_t *out_pairs, int64_t *in_pairs);

/* The iteration has run and ended at `now`: prompts advance, finished prompts become generation
 * tasks, requests that produced their last token leave and free their blocks.  Up to `cap` ids
 * of those are written to finished_ids; *num_finished receives their number. */
int mpa_sched_complete(mpa_sched *s, double now, int64_t *finished_ids, int32_t cap, int32_t *num_finished);

int32_t mpa_sched_live_requests(const mpa_sched *s);

#ifdef __cplusplus
}
#endif
#endif /* MPA_SCHED_H */
