/*
 * alora_planner.h -- base-aligned block cache and suffix planner: the step immediately before
 * alora_qkv_forward.  HOST code only (plain C ABI, host pointers everywhere); it produces the
 * per-token metadata the projection consumes: token_positions, token_seg_ids,
 * token_adapter_ids and slot_mapping of exactly the rows that still have to be projected.
 *
 * What it implements (Sec. 3, "KV-cache block hashing", and the caption of Fig. 1):
 *   - the paged KV cache is cut into blocks of block_size token slots; a FULL block is identified
 *     by a chained hash over (1) the token ids in the block, (2) the hash of the block before it in
 *     the sequence, (3) an extra identifier: the adapter id, or nothing for the base model;
 *     partially filled blocks are never cached;
 *   - for a request that invokes an aLoRA the adapter id enters the hash only of blocks that hold
 *     a token at or after the activation point; every earlier block hashes exactly as a base-model
 *     request would hash it, so base and aLoRA requests reuse each other's blocks in both
 *     directions;
 *   - blocks of a finished request return to the free pool and stay reusable through their hash
 *     until the pool hands them out again.
 * Readings where the paper is silent:
 *   - block b (positions [b*bs, (b+1)*bs)) carries the adapter id iff adapter_id >= 0 and
 *     (b+1)*bs > activation_start.  Base request: adapter_id = -1.  Standard LoRA:
 *     activation_start = 0.  An aLoRA that is never activated: activation_start >= n_tokens.
 *   - at least one token of an admitted request is always projected: at most
 *     floor((n_tokens-1)/bs) leading blocks are taken from the cache;
 *   - a block becomes reusable at alora_planner_commit (its K/V have been computed), not when it
 *     is allocated;
 *   - free blocks are handed out from the front of the free list (ids 0,1,2,... at the start); a
 *     finished request returns its blocks last-block-first; handing out a block drops its hash.
 * The hash function itself is the library's choice (64-bit); equal hashes are taken as equal blocks.
 *
 * Thread safety: one planner object must not be used from two threads at once.
 * Statuses are those of alora_qkv.h plus ALORA_ENOBLOCKS; on any error the planner is unchanged
 * and no output array element has been written (one exception: alora_planner_commit that runs out
 * of host memory, ALORA_ENOMEM, may have registered part of the request's blocks; the call can be
 * repeated).
 */
#ifndef ALORA_PLANNER_H
#define ALORA_PLANNER_H

#include <stddef.h>
#include <stdint.h>
#include "alora_qkv.h"

#ifdef __cplusplus
extern "C" {
#endif

#define ALORA_ENOBLOCKS (-7) /* not enough free cache blocks for this request */

typedef struct alora_planner alora_planner;

/* The batch under construction: host arrays owned by the caller, n_rows rows filled so far. */
typedef struct alora_plan_batch {
    int32_t *token_positions;   /* [row_cap] absolute position of each row in its request        */
    int32_t *token_seg_ids;     /* [row_cap] index of the row's request in this batch             */
    int32_t *token_adapter_ids; /* [row_cap] the request's adapter id on every one of its rows    */
    int64_t *slot_mapping;      /* [row_cap] block_table[pos / bs] * bs + pos % bs                */
    int32_t *activation_start;  /* [seg_cap] per request of the batch                             */
    int32_t row_cap, seg_cap;
    int32_t n_rows, n_segs;     /* filled so far; advanced by admit / append                      */
} alora_plan_batch;

/* A planner over n_blocks physical blocks of block_size slots each; all blocks free. */
int alora_planner_create(int32_t block_size, int64_t n_blocks, alora_planner **out);
int alora_planner_destroy(alora_planner *p);

/*
 * Prefill of a new request (req_id chosen by the caller, unused so far): finds the longest cached
 * prefix, takes references on those blocks, allocates blocks for the rest of the tokens, and
 * appends one segment (rows for positions cached_tokens .. n_tokens-1) to the batch.
 *   token_ids [n_tokens] host; n_tokens >= 1.   *cached_tokens (optional) = reused prefix length.
 */
int alora_planner_admit(alora_planner *p, int64_t req_id, const int32_t *token_ids, int32_t n_tokens,
                        int32_t adapter_id, int32_t activation_start, alora_plan_batch *batch,
                        int32_t *cached_tokens);

/*
 * Decode / continuation: request req_id grows by n_new tokens (blocks are allocated as needed);
 * appends one segment with rows for exactly those tokens.
 */
int alora_planner_append(alora_planner *p, int64_t req_id, const int32_t *new_token_ids, int32_t n_new,
                         alora_plan_batch *batch);

/* The rows planned so far for req_id have been computed: its full blocks become reusable. */
int alora_planner_commit(alora_planner *p, int64_t req_id);

/* The request is over: its blocks return to the free pool (still reusable through their hash). */
int alora_planner_finish(alora_planner *p, int64_t req_id);

/* Physical blocks of the request's logical blocks 0,1,...: writes min(*n, cap) ids, sets *n. */
int alora_planner_block_table(const alora_planner *p, int64_t req_id, int32_t *out, int32_t cap, int32_t *n);

/* Blocks in the free pool right now, or a negative status. */
int64_t alora_planner_free_blocks(const alora_planner *p);

#ifdef __cplusplus
}
#endif
#endif /* ALORA_PLANNER_H */
