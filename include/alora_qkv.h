/*
 * alora_qkv.h - C ABI of the MI355X (gfx950) library for the activation-aware masked
 * multi-adapter QKV projection with paged K/V write used when serving Activated LoRA
 * (aLoRA) adapters beside their base model.
 *
 * What one call computes (paper Sec. 2.3 block equations; Algorithm 1; App. B mask):
 *
 *   active(t) = token_adapter_ids[t] >= 0  and
 *               token_positions[t] >= activation_start[token_seg_ids[t]]
 *   y[t,:]    = x[t,:] . W_qkv                          every row (Algorithm 1, base output)
 *   y[t,:]   += (x[t,:] . A[a]) . B[a],  a = adapter    rows with active(t) only
 *   q_out[t,:]            = y[t, 0:Nq]
 *   k_cache[slot[t], :]   = y[t, Nq:Nq+Nkv]             if slot_mapping[t] >= 0
 *   v_cache[slot[t], :]   = y[t, Nq+Nkv:N]              if slot_mapping[t] >= 0
 *
 * with Nq = n_q_heads*head_dim, Nkv = n_kv_heads*head_dim, N = Nq + 2*Nkv.  The paper's
 * mask (1 = position before the activation start, keep the base output) is the negation
 * of active() for rows that have an adapter; rows are selected, not blended, so adapter
 * data never reaches a pre-activation or base-model row.  Those rows come out bit-identical
 * to a call in which every adapter id is -1, which is what lets base-model cache blocks be
 * reused by aLoRA requests and vice versa (Sec. 2.3, Sec. 3).
 *
 * Conventions
 *   - All data pointers are DEVICE pointers unless marked (host).  The caller owns every
 *     buffer; the library allocates nothing and keeps no state between calls.
 *   - All matrices are dense row-major.  dtype applies to x, W_qkv, A[i], B[i], q_out and
 *     both caches alike.  Accumulation is fp32; the fp32 sum base+delta is rounded once
 *     (nearest-even) to the storage type.
 *   - The paged caches are [num_blocks, block_size, n_kv_heads, head_dim] = [n_slots, Nkv];
 *     slot s is offset s % block_size of physical block s / block_size (Sec. 2.4).
 *   - Work is enqueued on `hip_stream` (a hipStream_t, NULL = default stream); calls return
 *     without synchronising.  Calls that share a workspace must be stream-ordered.
 *   - Return value: ALORA_OK or a negative status.  On ALORA_EINVAL, ALORA_ESHAPE, ALORA_EWORKSPACE and
 *     ALORA_ETOOBIG nothing has been enqueued and no device memory has been written (all argument
 *     checks come before the first launch).  After ALORA_EHIP (a launch failed part-way through the
 *     call's kernel sequence) the outputs and the workspace are undefined.
 *
 * Shape limits (ALORA_ESHAPE otherwise)
 *   bf16: hidden % 64 == 0; Nq % 8 == 0; Nkv % 8 == 0; rank in {8,16,24,...,64};
 *   f32 : hidden % 4 == 0;  Nq % 4 == 0; Nkv % 4 == 0; 1 <= rank <= 64;
 *   both: 0 <= n_adapters <= ALORA_MAX_ADAPTERS; n_slots % block_size == 0; T >= 0 (T == 0
 *   is a successful no-op).  Adapters of lower rank are zero-padded by the caller; any
 *   LoRA scaling factor is folded into B by the caller.
 *
 * Preconditions on device data (not checked on the fast path; alora_qkv_validate checks them)
 *   -1 <= token_adapter_ids[t] < n_adapters; 0 <= token_seg_ids[t] < n_segments for rows that
 *   have an adapter (segment and position of base-model rows are never read);
 *   slot_mapping[t] == -1 or in [0, n_slots), the non-negative ones pairwise distinct;
 *   factors of adapters that some active row uses hold finite values.
 */
#ifndef ALORA_QKV_H
#define ALORA_QKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ALORA_F32 0
#define ALORA_BF16 1

#define ALORA_MAX_ADAPTERS 128
#define ALORA_MAX_RANK 64

#define ALORA_OK 0
#define ALORA_EINVAL (-1)      /* null pointer, negative size, unknown dtype              */
#define ALORA_ESHAPE (-2)      /* a shape limit above is violated                         */
#define ALORA_EWORKSPACE (-3)  /* workspace null, misaligned (256 B) or too small          */
#define ALORA_EHIP (-4)        /* a HIP call failed; see alora_last_hip_error()            */
#define ALORA_EDATA (-5)       /* alora_qkv_validate found a violated data precondition    */
#define ALORA_ENOMEM (-6)      /* a host-side allocation failed (validate calls, planner)   */
/* (-7 is ALORA_ENOBLOCKS of alora_planner.h) */
#define ALORA_ETOOBIG (-8)     /* alora_qkv_forward_static: the call needs more scratch than the static array holds */

/* Sizes of one call plus the two per-token index arrays of App. B. */
typedef struct alora_dims {
    int32_t dtype;                  /* ALORA_F32 or ALORA_BF16                                   */
    int32_t T;                      /* scheduled tokens in the flattened batch                   */
    int32_t hidden;
    int32_t n_q_heads, n_kv_heads, head_dim;
    int32_t n_adapters, rank;
    int32_t n_segments;             /* G: number of requests / activation segments               */
    int64_t n_slots;                /* slots in k_cache and in v_cache                           */
    const int32_t *token_seg_ids;   /* [T] App. B req_indices                        (device)    */
    const int32_t *token_positions; /* [T] App. B position_within_req, absolute      (device)    */
} alora_dims;

/* Where the integer results of the classification / grouping step sit inside the workspace
 * after alora_qkv_classify_group or alora_qkv_forward (byte offsets from its start). */
typedef struct alora_ws_layout {
    size_t active_off;      /* uint8  [T]    1 = row receives its adapter's delta              */
    size_t perm_off;        /* int32  [T]    a permutation of the rows; first offsets[L] entries: active
                                             rows grouped by adapter, increasing t inside a group  */
    size_t offsets_off;     /* int32  [L+2]  group a is perm[offsets[a] .. offsets[a+1]); the rows that
                                             keep the base output follow as one last group,
                                             perm[offsets[L] .. offsets[L+1] = T), increasing t */
    size_t total_bytes;     /* same value alora_qkv_workspace_bytes reports                    */
} alora_ws_layout;

/* Bytes of workspace alora_qkv_forward needs for these sizes.  Host only, touches no device. */
int alora_qkv_workspace_bytes(const alora_dims *dims, size_t *out_bytes);

/* Layout of the integer results inside the workspace.  Host only. */
int alora_qkv_workspace_layout(const alora_dims *dims, alora_ws_layout *out);

/*
 * Row classification and grouping only (App. B mask; grouping of adapted rows by adapter id
 * for the multi-adapter shrink): fills the workspace regions named by alora_ws_layout.
 *   token_adapter_ids [T] device, -1 = base-model row;  activation_start [G] device.
 */
int alora_qkv_classify_group(const int32_t *token_adapter_ids, const int32_t *activation_start,
                             const alora_dims *dims, void *workspace, size_t workspace_bytes,
                             void *hip_stream);

/*
 * The whole path: classification, grouping, LoRA shrink on active rows, base projection with
 * the low-rank expand added to active rows, q_out store and paged K/V store.
 *
 *   x                 [T, hidden]                              read
 *   token_adapter_ids [T]  int32, -1 = base-model row          read
 *   activation_start  [G]  int32, App. B inv_start             read
 *   W_qkv             [hidden, N]  (y = x . W)                 read
 *   A, B              (host) arrays of n_adapters device pointers, A[i] [hidden, rank],
 *                     B[i] [rank, N]; the arrays are read before the call returns.  Factors
 *                     of adapters that no active row uses are never dereferenced.
 *   q_out             [T, Nq]            every row written
 *   k_cache, v_cache  [n_slots, Nkv]     only the slots named by slot_mapping are written
 *   slot_mapping      [T]  int64, -1 = no K/V write for this row (q_out is still produced)
 *   block_size        tokens per cache block (> 0, divides n_slots)
 *   workspace         device, 256-byte aligned, >= alora_qkv_workspace_bytes() bytes; contents
 *                     on entry are irrelevant
 */
int alora_qkv_forward(const void *x, const int32_t *token_adapter_ids, const int32_t *activation_start,
                      const void *W_qkv, const void *const *A, const void *const *B,
                      void *q_out, void *k_cache, void *v_cache,
                      const int64_t *slot_mapping, int32_t block_size,
                      const alora_dims *dims, void *workspace, size_t workspace_bytes,
                      void *hip_stream);

/*
 * Adapter-layout variants the paper names, on top of alora_qkv_forward (which is this call with
 * extras = NULL):
 *   bias           Algorithm 1 computes the base output as l.apply(x, b): a bias row b [N] (device,
 *                  dtype of x, 16-byte aligned) is added to the base output of EVERY row, adapted or
 *                  not, in fp32 before the single rounding.  NULL = no bias.
 *   adapter_ranks  Sec. 4.1 serves LoRAs of rank 8 beside aLoRAs of rank 32: HOST array
 *                  [n_adapters]; adapter i has A[i] of shape [hidden, adapter_ranks[i]] and B[i] of
 *                  shape [adapter_ranks[i], N], 1 <= adapter_ranks[i] <= dims->rank (bf16: multiples
 *                  of 8), else ALORA_ESHAPE.  NULL = every adapter has rank dims->rank.  Read during
 *                  the call only.
 *   reuse_grouping App. B builds the activation mask once per forward pass of the model and every
 *                  layer reads it.  Nonzero: skip classification and grouping and use the results a
 *                  previous call (alora_qkv_classify_group, alora_qkv_forward[_ex], a graph launch)
 *                  left in THIS workspace for the same dims, token_adapter_ids, token_seg_ids,
 *                  token_positions and activation_start -- the per-layer call of a model whose
 *                  layers share one token batch.  The calls must be stream-ordered.  A workspace
 *                  that holds no such results gives wrong outputs (indices read from it are range-
 *                  checked, so nothing outside the buffers is touched).  Decode-sized bf16 batches
 *                  regroup inside the projection kernel anyway; the flag changes nothing there.
 *   rope_cos/_sin  the step between the projection and the cache write in a served Llama-family layer, fused
 *                  into the store (the paper is silent on positions; Sec. 2.1): within every q and k head,
 *                  features i and i + head_dim/2 of row t are turned by the angle whose cosine and sine
 *                  the tables hold at [token_positions[t], i]:
 *                      out[i] = y[i] cos - y[i + head_dim/2] sin,  out[i + head_dim/2] = y[i + head_dim/2] cos + y[i] sin
 *                  in fp32 on the unrounded projection output (adapter term and bias included), rounded
 *                  once; v is not rotated.  Rows before the activation point stay bit-identical to those
 *                  of a base-only call with the same tables.  token_positions must lie in
 *                  [0, rope_positions) (a position outside reads the nearest table row; alora_qkv_validate
 *                  does not know the tables).  bf16 path: head_dim 128 only (ALORA_ESHAPE otherwise);
 *                  fp32 path: any even head_dim.
 * Per-module factors (separate A^Q, A^K, A^V with B^Q, B^K, B^V; Sec. 2.3) are the block-structured
 * special case: A = [A^Q | A^K | A^V] of rank 3r and B with B^Q, B^K, B^V on its block diagonal (zeros
 * elsewhere).  The combined rank 3r obeys the limits above, so the rank per module is at most
 * ALORA_MAX_RANK / 3 = 21 (bf16: 8 or 16, since 3r must be a multiple of 8), and the expand spends
 * three times the flops of a native per-module layout on the zero blocks.
 */
typedef struct alora_extras {
    const void *bias;
    const int32_t *adapter_ranks;
    int32_t reuse_grouping;
    const float *rope_cos;    /* DEVICE fp32 [rope_positions, head_dim / 2], 16-byte aligned, or NULL: no rotation */
    const float *rope_sin;    /* the same shape; both or neither                                                  */
    int32_t rope_positions;   /* rows of the two tables                                                           */
} alora_extras;
int alora_qkv_forward_ex(const void *x, const int32_t *token_adapter_ids, const int32_t *activation_start,
                         const void *W_qkv, const void *const *A, const void *const *B,
                         void *q_out, void *k_cache, void *v_cache,
                         const int64_t *slot_mapping, int32_t block_size,
                         const alora_dims *dims, const alora_extras *extras,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The call for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  alora_qkv_forward_ex without the workspace arguments: the
 * workspace is a device array of ALORA_STATIC_SCRATCH_BYTES that is part of the library's code
 * object (every GPU the library is used on holds one copy until the process ends).  The call
 * itself calls no hipMalloc / hipFree and no allocating library routine; the caller still passes
 * every input and output.
 *   - Arguments, results, layouts and preconditions are those of alora_qkv_forward_ex (extras may
 *     be NULL), except extras->reuse_grouping, which is refused (ALORA_EINVAL): the array is
 *     shared by every call on the device, so "the grouping an earlier call left" is not the
 *     caller's to rely on.  Results are bit-identical to alora_qkv_forward_ex.
 *   - Limit: calls whose alora_qkv_workspace_bytes() exceeds ALORA_STATIC_SCRATCH_BYTES return
 *     ALORA_ETOOBIG before anything is enqueued.
 *   - All calls on one GPU share that GPU's array, which keeps the previous call's contents (no
 *     kernel relies on them: whatever must start at zero is cleared by the call itself).  Calls on
 *     one GPU must therefore be stream-ordered; calls that overlap on one GPU race.
 *   - The device address of the array is looked up on the first call on each device (with that
 *     device current), under a lock; later calls only read it.
 */
#define ALORA_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
size_t alora_qkv_static_scratch_bytes(void);
int alora_qkv_forward_static(const void *x, const int32_t *token_adapter_ids, const int32_t *activation_start,
                             const void *W_qkv, const void *const *A, const void *const *B,
                             void *q_out, void *k_cache, void *v_cache,
                             const int64_t *slot_mapping, int32_t block_size,
                             const alora_dims *dims, const alora_extras *extras, void *hip_stream);

/*
 * Graph-captured call.  Sec. 3 keeps the activation mask in a tensor of fixed address so that the
 * model's forward pass stays one captured device graph, and App. A's dummy run builds placeholder
 * aLoRA metadata only so that the mask is part of that graph.  Here: alora_qkv_graph_create records
 * ONE alora_qkv_forward with exactly these pointers and sizes into a HIP graph (on a stream of its
 * own; nothing runs) and hands back the instantiated graph; every alora_qkv_graph_launch replays
 * the whole call (classification/grouping, shrink, projection, stores) on `hip_stream`.
 *   - Arguments, layouts and preconditions are those of alora_qkv_forward_ex (extras may be NULL;
 *     the rank array is read at creation, the bias and rotary-table pointers are baked in); T must be > 0.
 *   - All addresses are baked in: before a launch the caller rewrites the CONTENTS of x,
 *     token_adapter_ids, dims->token_seg_ids, dims->token_positions, activation_start and
 *     slot_mapping in place.  A batch with fewer than T rows is padded with rows that have
 *     token_adapter_ids = -1 and slot_mapping = -1 (any x, any valid segment id): they cost a q_out
 *     row and touch no cache slot.  The A / B pointer tables are read at creation only.
 *   - Sizes (dims), block_size, the workspace and the tuning in force at creation are baked in too.
 *   - Ownership: the caller keeps every buffer alive until the graph is destroyed; the library owns
 *     the alora_graph object.  Launches of one graph must not overlap (they share the workspace).
 *   - Errors: statuses of alora_qkv_forward; on error *out is NULL and nothing was enqueued.
 */
typedef struct alora_graph alora_graph;
int alora_qkv_graph_create(const void *x, const int32_t *token_adapter_ids, const int32_t *activation_start,
                           const void *W_qkv, const void *const *A, const void *const *B,
                           void *q_out, void *k_cache, void *v_cache,
                           const int64_t *slot_mapping, int32_t block_size,
                           const alora_dims *dims, const alora_extras *extras,
                           void *workspace, size_t workspace_bytes, alora_graph **out);
int alora_qkv_graph_launch(alora_graph *graph, void *hip_stream);
int alora_qkv_graph_destroy(alora_graph *graph);

/*
 * Slow, synchronous check of the data preconditions listed at the top (copies the index
 * arrays to the host).  Returns ALORA_OK, ALORA_EDATA, or another status for bad arguments.
 * Writes no device memory.
 */
int alora_qkv_validate(const int32_t *token_adapter_ids, const int32_t *activation_start,
                       const int64_t *slot_mapping, int32_t block_size, const alora_dims *dims);

/*
 * Tuning override for tests and benchmarks of the bf16 path (process-wide: one atomic word, so a call on
 * another thread sees the old or the new setting, never a mix; set it before querying the workspace size).  By default the library picks, from (T, hidden, N) alone,
 * the width of the projection kernel's feature tile and, for batches too small to fill the chip,
 * into how many splits of the hidden dimension the base product is cut (the small-batch path:
 * split projection + a finishing kernel over the grouped rows).
 *   feature_tiles  0 = automatic, else 2, 3 or 4: tile width 128, 192 or 256 features
 *   splits         0 = automatic, 1 = never split, 2..8 = that many splits where the sizes allow
 * Any setting computes the same result up to fp32 summation order.
 */
int alora_qkv_set_tuning(int feature_tiles, int splits);

/*
 * Benchmark aid (not for serving loops: it creates HIP events).  Between _begin and _end, every
 * alora_qkv_forward records a HIP event pair on its stream around its dominant kernel, the
 * projection GEMM (Algorithm 1's base output with the adapter term fused in), for at most
 * max_calls calls.  _end waits for the recorded events and reports the average duration of
 * that kernel in milliseconds and how many calls were measured.
 */
int alora_qkv_profile_begin(int max_calls);
int alora_qkv_profile_end(double *avg_ms, int *n_calls);
/* The same, measuring only every `every`-th call (>= 1): an event pair costs a few microseconds
 * of stream time, which shows in the step time of decode-sized calls. */
int alora_qkv_profile_begin_every(int max_calls, int every);

/* Static description of a status code. */
const char *alora_status_string(int status);

/* hipError_t value of the most recent failing HIP call on this thread (0 if none). */
int alora_last_hip_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int alora_qkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ALORA_QKV_H */
