/*
 * alora_attention.h -- reader of the paged K/V cache: causal softmax attention of query rows over
 * the cached keys and values of their sequences (C ABI of libalora_qkv.so, gfx950).
 *
 * What it computes (Sec. 2.1: causal softmax attention over per-token query, key and value
 * vectors, with K and V of earlier tokens taken from the cache; the paper gives no formula, the
 * textbook one is used).  For query row t at position p = token_positions[t] of sequence
 * s = token_seq_ids[t], and query head h:
 *
 *     o[t, h, :] = sum_{j=0..p} softmax_j( scale * <q[t, h, :], K_j[g(h), :]> ) * V_j[g(h), :]
 *     K_j = k_cache[slot(j)],  V_j = v_cache[slot(j)],
 *     slot(j) = block_tables[s][j / block_size] * block_size + j % block_size,
 *     g(h) = h / (n_q_heads / n_kv_heads)            (grouped-query attention)
 *
 * This is the step after alora_qkv_forward: that call wrote K and V of the step's own rows into
 * the cache, so position p itself is part of the context.  It is what turns the claim of Sec. 2.3
 * -- blocks written before the activation point are the base model's and can be read by any
 * request -- into numbers: a request that reads blocks written by another request's projection
 * gets the result of a from-scratch computation of its whole sequence.
 *
 * Layout: q and out row-major [n_tokens, n_q_heads * head_dim]; caches row-major
 * [n_slots, n_kv_heads * head_dim] (the layout alora_qkv_forward writes); block_tables row-major
 * int32 [n_seqs, max_blocks], entries past a sequence's length are never read.  All pointers are
 * DEVICE pointers, owned by the caller, 16-byte aligned; q/k_cache/v_cache/out have the dtype of
 * dims->dtype (bf16 or fp32); scores, softmax and the weighted sum are fp32, the output is rounded
 * once; scaled scores below -1e30 (in units of log2) weigh nothing.  out may not alias q.
 *
 * Limits: head_dim in {64, 128}; n_q_heads / n_kv_heads in {1, 2, 4, 8}; block_size >= 1;
 * n_tokens * n_kv_heads <= 2^31 - 1; n_slots <= 2^31 - 1.  One workgroup per (row, K/V head): meant for decode-sized
 * batches and short suffixes (rows of one sequence each read the context again).
 *
 * Errors: ALORA_EINVAL (null pointer, negative size, unknown dtype, misaligned pointer),
 * ALORA_ESHAPE (a limit above), ALORA_EHIP (launch failed).  The kernel never dereferences an
 * address derived from an out-of-range index: a row whose sequence id or position is out of range
 * gets an all-zero output, a context position whose table entry is outside [0, n_slots /
 * block_size) is left out of the softmax.  alora_paged_attention_validate reports such data
 * (ALORA_EDATA) before a call; it copies the index arrays to the host and synchronises.
 *
 * The call is enqueued on `hip_stream` (a hipStream_t, NULL = default stream) and returns without
 * synchronising; it allocates nothing and uses no workspace.
 */
#ifndef ALORA_ATTENTION_H
#define ALORA_ATTENTION_H

#include <stddef.h>
#include <stdint.h>
#include "alora_qkv.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct alora_attn_dims {
    int32_t dtype;        /* ALORA_F32 or ALORA_BF16                                         */
    int32_t n_tokens;     /* query rows                                                      */
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t n_seqs;       /* rows of block_tables                                            */
    int32_t max_blocks;   /* columns of block_tables                                         */
    int32_t block_size;   /* slots per cache block                                           */
    int64_t n_slots;      /* rows of k_cache and of v_cache                                  */
    float scale;          /* multiplies the scores; 0 selects 1 / sqrt(head_dim)             */
} alora_attn_dims;

/* Sec. 2.1 (causal softmax attention over the cached K and V); see the top of this file. */
int alora_paged_attention(const void *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
                          const int32_t *token_seq_ids, const int32_t *token_positions, void *out,
                          const alora_attn_dims *dims, void *hip_stream);

/*
 * The same computation for batches too small to fill the chip with one workgroup per (row, K/V head)
 * -- a few sequences with long contexts, the shape of an adapter evaluated on one long conversation
 * (Sec. 4.2): every row's context is cut into parts, one workgroup each (about 1024 workgroups, at
 * most 32 parts), the parts leave (running maximum, sum of weights, unnormalised output) in the
 * workspace and a second kernel combines them in part order.  Results equal those of
 * alora_paged_attention up to fp32 summation order and do not depend on timing.
 *   workspace  device, 16-byte aligned, >= alora_paged_attention_workspace_bytes() bytes (0 when the
 *              batch is large enough for one part: then this IS alora_paged_attention and the
 *              workspace may be NULL); contents on entry irrelevant; calls that share it must be
 *              stream-ordered.  Too small or misaligned: ALORA_EWORKSPACE.
 */
int alora_paged_attention_workspace_bytes(const alora_attn_dims *dims, size_t *out_bytes);
int alora_paged_attention_split(const void *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
                                const int32_t *token_seq_ids, const int32_t *token_positions, void *out,
                                const alora_attn_dims *dims, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The same computation for the rows of a projected suffix (Sec. 2.3 / 4.2: the tokens of an aLoRA
 * request that are not served from the cache, attending over the cached prefix and over each other):
 * batch rows that follow each other with the same sequence id and consecutive positions are handled
 * in blocks of 128 / (n_q_heads / n_kv_heads) rows that load every cached row once, on bf16 matrix
 * instructions (the softmax weights are rounded to bf16 for the weighted sum of V; scores, maxima
 * and sums stay fp32).  Any batch is accepted -- rows that do not continue a run form blocks of
 * their own -- and results equal those of alora_paged_attention within the bf16 tolerance; they do
 * not depend on timing (repeated calls give the same bits).
 * bf16 and head_dim 128 only (ALORA_ESHAPE otherwise); no workspace.  Block sizes that are not a
 * multiple of 4 are served by the kernel of alora_paged_attention.
 */
int alora_paged_attention_suffix(const void *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
                                 const int32_t *token_seq_ids, const int32_t *token_positions, void *out,
                                 const alora_attn_dims *dims, void *hip_stream);

/*
 * alora_paged_attention_suffix for batches with few row blocks -- the common aLoRA request: a short invocation
 * suffix over a long cached context (Sec. 4.2) -- where one workgroup per (row block, K/V head) would leave
 * most of the chip idle: every row block's context is cut into parts, one workgroup each (about 512
 * workgroups, at most 32 parts; one part when the batch has 512 or more (row block, K/V head) pairs: then
 * this IS alora_paged_attention_suffix and the workspace may be NULL), the parts leave (running maximum,
 * sum of weights, unnormalised output) in the workspace and a second kernel combines them in part order.
 * Results equal those of alora_paged_attention_suffix up to fp32 summation order and do not depend on timing.
 *   workspace  device, 16-byte aligned, >= alora_paged_attention_suffix_workspace_bytes() bytes; contents on
 *              entry irrelevant; calls that share it must be stream-ordered.  ALORA_EWORKSPACE otherwise.
 */
int alora_paged_attention_suffix_workspace_bytes(const alora_attn_dims *dims, size_t *out_bytes);
int alora_paged_attention_suffix_split(const void *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
                                       const int32_t *token_seq_ids, const int32_t *token_positions, void *out,
                                       const alora_attn_dims *dims, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Host-side check of the index data of a call (synchronous; device pointers): every sequence id in
 * [0, n_seqs), every position in [0, max_blocks * block_size), every table entry a row's context
 * reaches in [0, n_slots / block_size).  ALORA_OK, ALORA_EDATA, or an argument error. */
int alora_paged_attention_validate(const int32_t *block_tables, const int32_t *token_seq_ids,
                                   const int32_t *token_positions, const alora_attn_dims *dims);

#ifdef __cplusplus
}
#endif
#endif
