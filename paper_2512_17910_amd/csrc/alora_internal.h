// Internal declarations shared by the HIP translation units of libalora_qkv (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "alora_qkv.h"

namespace alora {

typedef uint16_t bf16_t;  // raw bf16 bit pattern

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// Device pointers of the adapters' factors, passed to kernels by value.
struct PtrTable {
    const void *p[ALORA_MAX_ADAPTERS];
};

// Rank of every adapter (A_i is [hidden, r_i], B_i is [r_i, N]), passed to kernels by value.
struct RankTable {
    uint8_t r[ALORA_MAX_ADAPTERS];
};

// Everything one forward call needs, resolved on the host.
struct Fwd {
    int dtype, T, H, Nq, Nkv, N, L, r, G;
    long long n_slots;
    int block_size;
    const void *x, *W;
    const void *bias;    // [N] or null: added to the base output of every row (Algorithm 1, l.apply(x, b))
    RankTable ranks;     // per adapter, <= r
    const float *rope_cos, *rope_sin;   // [rope_positions][D / 2] or null: rotary embedding fused into the store
    int rope_positions, D;              // D = head_dim
    const int32_t *aid, *seg, *pos, *start;
    const int64_t *slot;
    void *q, *kc, *vc;
    // workspace regions
    uint8_t *active;
    int8_t *aeff;        // [T] adapter id of adapted rows, -1 for rows that keep the base output
    int32_t *perm, *offsets;
    void *S;          // shrink result.  f32 path: [T][r] fp32.  bf16 path: [T][2r] bf16 (hi | lo halves of the fp32
                      // result), or with several shrink ranges (see plan_shrink) fp32 partials [ranges][T][r]
    float *partial;      // small-batch path: fp32 partial products [splits][T][N]
    int32_t *hist;       // large batches: rows per (2048-row slice, group), see the grouping kernels
    int4 *blocktab;      // shrink: (adapter, first perm index, rows, 0) per 32-row block; adapter -1 = unused
    int n_blocks;        // entries in blocktab (upper bound on 32-row blocks)
    // prefill-sized bf16 batches: the shrink's work list, one item per (32-row block of an adapter, range
    // of the hidden dimension), written by the grouping step from the number of adapted blocks it finds;
    // null when the shrink walks blocktab instead
    int4 *items;         // (adapter, first perm index, rows | range width/64 << 8, range | ranges << 4 | block << 8)
    int32_t *counters;   // per block: ranges that have stored their partial (zeroed by the grouping step)
    int n_items;
    int32_t *block_rows;  // decode-sized bf16 batches: the row ids of every block-table entry, 32 per entry, -1 padded
                          // (the finishing kernel then needs no look-up through perm)
    hipStream_t stream;
};

// fp32 -> bf16 bits, round to nearest even; NaN stays NaN.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// App. B mask negated and combined with "row has an adapter": -1 when the row keeps the base
// output, else its adapter id.  seg/pos/start are only read for rows that have an adapter.
__device__ __forceinline__ int effective_adapter(const int32_t *aid, const int32_t *seg, const int32_t *pos,
                                                 const int32_t *start, int t)
{
    int a = aid[t];
    if (a < 0) return -1;
    return (pos[t] >= start[seg[t]]) ? a : -1;
}

// remember a failed HIP call for alora_last_hip_error() (per host thread)
void note_hip_error(int hip_error);

// launches (each returns the hipError_t of its launch as int)
int launch_classify_group(const Fwd &f);
int launch_shrink_f32(const Fwd &f, const PtrTable &A);
int launch_gemm_f32(const Fwd &f, const PtrTable &B);
int launch_shrink_bf16(const Fwd &f, const PtrTable &A);
int launch_gemm_bf16(const Fwd &f, const PtrTable &B, const PtrTable &A, hipEvent_t after_projection);
bool prep_in_projection(const Fwd &f);   // grouping and shrink run inside the split projection kernel
int launch_finish_bf16(const Fwd &f, const PtrTable &B, int splits, int s_splits, const int32_t *block_rows);
struct GemmPlan {
    int ntw;     // 32-wide feature tiles per wavefront (tile width 64 * ntw)
    int splits;  // 1: fused kernel; > 1: split hidden dimension + finishing kernel
    int kps;     // 64-wide K-slices per split
};
GemmPlan plan_gemm(int T, int H, int N);
size_t gemm_partial_bytes(int T, int H, int N);
void set_gemm_tuning(int ntw, int splits);
int group_blocks(int T, int L);
size_t group_hist_bytes(int T);
constexpr int ALORA_SHRINK_MAX_SPLITS = 8;
constexpr int ALORA_SHRINK_TARGET_WGS = 256;   // workgroups the prefill-sized shrink aims for (one per compute unit)
struct ShrinkPlan {
    int splits;  // ranges of the hidden dimension; the shrink result is the fixed-order sum of their partials
    int kper;    // width of one range (multiple of 64)
    // Prefill-sized batches: the number of ranges is chosen on the device, per call, from the number of
    // adapted 32-row blocks (at most `splits`); the last range of a block to finish adds the partials in
    // fixed order and stores the (hi, lo) form.  The shrink then walks Fwd::items.
    bool combine;
};
// what the grouping kernels need to write the shrink's work list
struct ShrinkWork {
    int4 *items;
    int32_t *counters;
    int n_items, k64, rmax;
};
int shrink_items(int T, int L);   // entries of the work list
ShrinkPlan plan_shrink(int T, int H, int N, int L, int r);
int launch_rope_f32(const Fwd &f);   // fp32 path: rotation of the stored q and k rows in place

}  // namespace alora
