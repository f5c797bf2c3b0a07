// Reader of the paged K/V cache: causal softmax attention of query rows over the cached keys and
// values of their sequences (Sec. 2.1; formula and layout in alora_attention.h).
//
// One workgroup (4 wavefronts) per (query row, K/V head); the G = n_q_heads / n_kv_heads query heads
// that share the K/V head are processed together, so every cached byte is loaded once per row.
// The work is a stream of K and V rows (2 * head_dim elements per context position and K/V head)
// against 4 * G * head_dim flops: memory-bound, so plain fp32 vector arithmetic, no LDS staging and
// no matrix instructions.
//
// Lane layout: head_dim / 8 lanes share one context position, 8 consecutive elements (16 bytes of
// bf16) each, so a wavefront's load instruction covers 64 / (head_dim / 8) positions with whole
// contiguous head rows.  The partial dot products are summed over those lanes with DPP adds
// (quad swaps, then half-row and row mirrors: every lane ends with the same bits).  Each lane
// group keeps its own running (max, sum, weighted V) -- 16 or 32 independent streams per
// workgroup -- rescaled once per U positions; the streams are merged in a fixed order at the end
// (lane groups by shuffles, wavefronts through LDS), so the result does not depend on timing.
#include "alora_internal.h"
#include "alora_attention.h"
#include "alora_attention_internal.h"
#include <new>
#include <algorithm>
#include <vector>

namespace alora {


template <int CTRL>
__device__ __forceinline__ float dpp_add(float v)
{
    const int o = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true);
    return v + __int_as_float(o);
}

// sum over the LPP lanes that share a position; all of them receive it
template <int LPP>
__device__ __forceinline__ float group_sum(float v)
{
    v = dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);   // row_half_mirror: the other quad of the 8 lanes
    if (LPP == 16) v = dpp_add<0x140>(v);   // row_mirror: the other half of the 16 lanes
    return v;
}

// 8 consecutive elements of a cache or query row, as loaded
template <bool BF16> struct Raw8;
template <> struct Raw8<true> {
    u32x4 v;
    __device__ __forceinline__ void zero() { v = u32x4{0u, 0u, 0u, 0u}; }
    __device__ __forceinline__ void load(const void *base, size_t elem) { v = *(const u32x4 *)((const bf16_t *)base + elem); }
    __device__ __forceinline__ void widen(float f[8]) const
    {
        f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
        f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
        f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
        f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
    }
};
template <> struct Raw8<false> {
    f32x4 a, b;
    __device__ __forceinline__ void zero() { a = f32x4{0.f, 0.f, 0.f, 0.f}; b = a; }
    __device__ __forceinline__ void load(const void *base, size_t elem)
    {
        a = *(const f32x4 *)((const float *)base + elem);
        b = *(const f32x4 *)((const float *)base + elem + 4);
    }
    __device__ __forceinline__ void widen(float f[8]) const
    {
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
        f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
    }
};

constexpr float NEG_INF = -__builtin_inff();

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// <q chunk, k chunk> over 8 elements.  bf16: four packed two-element dot products on the stored bits
// (fp32 accumulate); fp32: eight FMAs.  The pairs are taken with shufflevector on the 8-element vector:
// bit casts of the single 32-bit words were compiled into four uses of the first word by this toolchain.
__device__ __forceinline__ float dot8(const Raw8<true> &q, const Raw8<true> &k)
{
    const bf16x8 qv = __builtin_bit_cast(bf16x8, q.v), kv = __builtin_bit_cast(bf16x8, k.v);
    float d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(qv, qv, 0, 1), __builtin_shufflevector(kv, kv, 0, 1), 0.f, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(qv, qv, 2, 3), __builtin_shufflevector(kv, kv, 2, 3), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(qv, qv, 4, 5), __builtin_shufflevector(kv, kv, 4, 5), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(qv, qv, 6, 7), __builtin_shufflevector(kv, kv, 6, 7), d, false);
    return d;
}
__device__ __forceinline__ float dot8(const Raw8<false> &q, const Raw8<false> &k)
{
    float d = q.a.x * k.a.x;
    d = fmaf(q.a.y, k.a.y, d); d = fmaf(q.a.z, k.a.z, d); d = fmaf(q.a.w, k.a.w, d);
    d = fmaf(q.b.x, k.b.x, d); d = fmaf(q.b.y, k.b.y, d); d = fmaf(q.b.z, k.b.z, d); d = fmaf(q.b.w, k.b.w, d);
    return d;
}

// The running maximum starts at a large negative FINITE number: differences with it stay finite, so the
// softmax needs no "nothing seen yet" cases (a position that is left out scores -inf and weighs
// exp2(-inf) = 0).  Scores below it are treated like -inf.
constexpr float M_FLOOR = -1.0e30f;

template <int D, int G, bool BF16, bool POW2>
__global__ __launch_bounds__(256) void paged_attention_kernel(AttnArgs a)
{
    constexpr int LPP = D / 8;         // lanes per context position
    constexpr int PPW = 64 / LPP;      // positions per wavefront and step
    constexpr int PPI = 4 * PPW;       // positions per workgroup and step
    constexpr int U = BF16 ? 4 : 2;    // steps per block: loaded together, one rescale of the running sums
    constexpr int BLK = PPI * U;       // positions per workgroup and block

    __shared__ float sm[4][G], sl[4][G];
    __shared__ float sacc[4][G][D];

    // workgroup -> (row, K/V head, part of the context)
    const int rh = (int)blockIdx.x / a.splits, sp = (int)blockIdx.x - rh * a.splits;
    const int t = rh / a.Hkv, hk = rh % a.Hkv;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int grp = lane / LPP, c = lane % LPP;

    const int sq = a.seq[t], p = a.pos[t];
    const long long cap = (long long)a.max_blocks * a.bs;
    int n_ctx = 0;
    if (sq >= 0 && sq < a.n_seqs && p >= 0) n_ctx = (int)(p + 1ll < cap ? p + 1ll : cap);
    const int32_t *bt = a.bt + (size_t)(n_ctx ? sq : 0) * a.max_blocks;
    // this workgroup's part of the context: whole blocks of BLK positions, the same number for every part
    int jbeg = 0;
    if (a.splits > 1) {
        const int per = ((n_ctx + a.splits * BLK - 1) / (a.splits * BLK)) * BLK;
        jbeg = min(n_ctx, sp * per);
        n_ctx = min(n_ctx, jbeg + per);
    }
    const int Nkv = a.Hkv * D;
    const int col = hk * D + 8 * c;
    const int jl = wave * PPW + grp;   // this lane group's position inside a step
    const long long n_blocks = a.n_slots / a.bs;

    Raw8<BF16> qr[G];
#pragma unroll
    for (int g = 0; g < G; ++g) qr[g].load(a.q, ((size_t)t * a.Hq + (size_t)hk * G + g) * D + 8 * c);

    float m[G], l[G], acc[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = M_FLOOR;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
    }

    // block-table entries of the block starting at j0 (-1 past the context).  Only the loads are issued
    // here: the entries are first looked at one block later, in fetch, so their latency is covered.
    auto lookup = [&](int j0, int (&blk)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + u * PPI + jl;
            blk[u] = -1;
            if (j < n_ctx) blk[u] = bt[POW2 ? (j >> a.bs_shift) : (j / a.bs)];
        }
    };
    // K and V chunks of the block starting at j0, through table entries looked up earlier; a position past
    // the context or with a table entry outside the cache is left out (zero chunks, validity bit clear).
    // Returns the validity of this lane's positions, one bit per step.
    auto fetch = [&](int j0, const int (&blk)[U], Raw8<BF16> (&kr)[U], Raw8<BF16> (&vr)[U]) {
        unsigned ok = 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int j = j0 + u * PPI + jl;
            const bool have = blk[u] >= 0 && blk[u] < n_blocks;   // blk is -1 past the context
            ok |= (unsigned)have << u;
            kr[u].zero();
            vr[u].zero();
            if (have) {
                const int off = POW2 ? (j & (a.bs - 1)) : (j % a.bs);
                const size_t at = ((size_t)blk[u] * a.bs + off) * Nkv + col;
                kr[u].load(a.kc, at);
                vr[u].load(a.vc, at);
            }
        }
        return ok;
    };
    // scores, running softmax (rescaled once per block) and weighted sum of V for one block
    auto consume = [&](const Raw8<BF16> (&kr)[U], const Raw8<BF16> (&vr)[U], unsigned ok) {
        float s[U][G];   // in units of log2
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int g = 0; g < G; ++g) s[u][g] = dot8(qr[g], kr[u]);
        // the sums over the lanes of a position, one reduction step at a time over all scores: consecutive
        // DPP instructions then work on different registers
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int g = 0; g < G; ++g) s[u][g] = dpp_add<0xB1>(s[u][g]);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int g = 0; g < G; ++g) s[u][g] = dpp_add<0x4E>(s[u][g]);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int g = 0; g < G; ++g) s[u][g] = dpp_add<0x141>(s[u][g]);
        if (LPP == 16) {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int g = 0; g < G; ++g) s[u][g] = dpp_add<0x140>(s[u][g]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int g = 0; g < G; ++g) s[u][g] = ((ok >> u) & 1u) ? s[u][g] * a.scale_log2e : NEG_INF;
        float pw[U][G];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float mx = s[0][g];
#pragma unroll
            for (int u = 1; u < U; ++u) mx = fmaxf(mx, s[u][g]);
            const float mn = fmaxf(m[g], mx);
            const float corr = __builtin_amdgcn_exp2f(m[g] - mn);
            m[g] = mn;
            float ls = l[g] * corr;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                pw[u][g] = __builtin_amdgcn_exp2f(s[u][g] - mn);
                ls += pw[u][g];
            }
            l[g] = ls;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[g][e] *= corr;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float vf[8];
            vr[u].widen(vf);
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[g][e] = fmaf(pw[u][g], vf[e], acc[g][e]);
        }
    };

    // Two register sets: while one block is consumed the next block's K/V loads and the table entries of
    // the block after it are in flight.
    int blkA[U], blkB[U];
    Raw8<BF16> krA[U], vrA[U], krB[U], vrB[U];
    lookup(jbeg, blkA);
    unsigned okA = fetch(jbeg, blkA, krA, vrA), okB;
    lookup(jbeg + BLK, blkB);
    for (int j0 = jbeg; j0 < n_ctx; j0 += 2 * BLK) {
        okB = fetch(j0 + BLK, blkB, krB, vrB);
        lookup(j0 + 2 * BLK, blkA);
        consume(krA, vrA, okA);
        if (j0 + BLK < n_ctx) {
            okA = fetch(j0 + 2 * BLK, blkA, krA, vrA);
            lookup(j0 + 3 * BLK, blkB);
            consume(krB, vrB, okB);
        }
    }

    // merge the lane groups of a wavefront (same chunk c, different positions)
#pragma unroll
    for (int off = LPP; off < 64; off <<= 1) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float mo = __shfl_xor(m[g], off), lo = __shfl_xor(l[g], off);
            const float mn = fmaxf(m[g], mo);
            const float ca = __builtin_amdgcn_exp2f(m[g] - mn), cb = __builtin_amdgcn_exp2f(mo - mn);
            l[g] = l[g] * ca + lo * cb;
            m[g] = mn;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float ao = __shfl_xor(acc[g][e], off);
                acc[g][e] = acc[g][e] * ca + ao * cb;
            }
        }
    }
    if (grp == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (c == 0) { sm[wave][g] = m[g]; sl[wave][g] = l[g]; }
#pragma unroll
            for (int e = 0; e < 8; ++e) sacc[wave][g][8 * c + e] = acc[g][e];
        }
    }
    __syncthreads();

    // merge the four wavefronts in fixed order and store
    for (int idx = tid; idx < G * D; idx += 256) {
        const int g = idx / D, dd = idx % D;
        float M = sm[0][g];
#pragma unroll
        for (int w = 1; w < 4; ++w) M = fmaxf(M, sm[w][g]);
        float L = 0.f, o = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float f = __builtin_amdgcn_exp2f(sm[w][g] - M);
            L += sl[w][g] * f;
            o += sacc[w][g][dd] * f;
        }
        if (a.splits > 1) {   // this part's (maximum, sum, unnormalised output); the merge kernel finishes
            float *pp = a.part + (((size_t)t * a.Hq + (size_t)hk * G + g) * a.splits + sp) * (D + 2);
            if (dd == 0) { pp[0] = M; pp[1] = L; }
            pp[2 + dd] = o;
            continue;
        }
        const float y = L > 0.f ? o / L : 0.f;
        const size_t at = ((size_t)t * a.Hq + (size_t)hk * G + g) * D + dd;
        if (BF16) ((bf16_t *)a.out)[at] = (bf16_t)f32_to_bf16_bits(y);
        else ((float *)a.out)[at] = y;
    }
}

// Second pass of a split call: the parts of a (row, query head) are combined in part order.
template <int D, bool BF16>
__global__ __launch_bounds__(D) void paged_attention_merge_kernel(const float *__restrict__ part, void *__restrict__ out, int splits)
{
    const size_t rh = blockIdx.x;   // row * Hq + query head
    const int dd = threadIdx.x;
    const float *pp = part + rh * splits * (D + 2);
    float M = M_FLOOR;
    for (int s2 = 0; s2 < splits; ++s2) M = fmaxf(M, pp[(size_t)s2 * (D + 2)]);
    float L = 0.f, o = 0.f;
    for (int s2 = 0; s2 < splits; ++s2) {
        const float *q2 = pp + (size_t)s2 * (D + 2);
        const float f = __builtin_amdgcn_exp2f(q2[0] - M);
        L += q2[1] * f;
        o += q2[2 + dd] * f;
    }
    const float y = L > 0.f ? o / L : 0.f;
    if (BF16) ((bf16_t *)out)[rh * D + dd] = (bf16_t)f32_to_bf16_bits(y);
    else ((float *)out)[rh * D + dd] = y;
}

template <int D, int G>
static void launch_dg(const AttnArgs &a, bool bf16, hipStream_t st)
{
    const dim3 grid((unsigned)a.T * (unsigned)a.Hkv * (unsigned)a.splits);
    const bool pow2 = a.bs_shift >= 0;
    if (bf16 && pow2) hipLaunchKernelGGL((paged_attention_kernel<D, G, true, true>), grid, dim3(256), 0, st, a);
    else if (bf16) hipLaunchKernelGGL((paged_attention_kernel<D, G, true, false>), grid, dim3(256), 0, st, a);
    else if (pow2) hipLaunchKernelGGL((paged_attention_kernel<D, G, false, true>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((paged_attention_kernel<D, G, false, false>), grid, dim3(256), 0, st, a);
    if (a.splits > 1) {
        const dim3 mgrid((unsigned)a.T * (unsigned)a.Hq);
        if (bf16) hipLaunchKernelGGL((paged_attention_merge_kernel<D, true>), mgrid, dim3(D), 0, st, a.part, a.out, a.splits);
        else hipLaunchKernelGGL((paged_attention_merge_kernel<D, false>), mgrid, dim3(D), 0, st, a.part, a.out, a.splits);
    }
}

template <int D>
static bool launch_d(const AttnArgs &a, int G, bool bf16, hipStream_t st)
{
    switch (G) {
    case 1: launch_dg<D, 1>(a, bf16, st); return true;
    case 2: launch_dg<D, 2>(a, bf16, st); return true;
    case 4: launch_dg<D, 4>(a, bf16, st); return true;
    case 8: launch_dg<D, 8>(a, bf16, st); return true;
    }
    return false;
}

static int check_dims(const alora_attn_dims *d)
{
    if (!d) return ALORA_EINVAL;
    if (d->dtype != ALORA_F32 && d->dtype != ALORA_BF16) return ALORA_EINVAL;
    if (d->n_tokens < 0 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->n_seqs < 0 || d->max_blocks < 0 ||
        d->block_size < 1 || d->n_slots < 0 || !(d->scale >= 0.f))
        return ALORA_EINVAL;
    if (d->head_dim != 64 && d->head_dim != 128) return ALORA_ESHAPE;
    if (d->n_q_heads % d->n_kv_heads) return ALORA_ESHAPE;
    const int G = d->n_q_heads / d->n_kv_heads;
    if (G != 1 && G != 2 && G != 4 && G != 8) return ALORA_ESHAPE;
    if ((long long)d->n_tokens * d->n_kv_heads > 0x7fffffffll || d->n_slots > 0x7fffffffll) return ALORA_ESHAPE;
    return ALORA_OK;
}

// Parts a row's context is cut into so that a small batch still fills the chip: about 1024 workgroups,
// at most 32 parts, one part when (rows x K/V heads) already gives that many.
static int plan_splits(const alora_attn_dims *d)
{
    const long long wgs = (long long)d->n_tokens * d->n_kv_heads;
    if (wgs <= 0 || wgs >= 1024) return 1;
    return (int)std::min<long long>(32, (1024 + wgs - 1) / wgs);
}

// The same for the row-block kernel, whose unit of work is a block of 128 / G rows: parts when the batch
// has fewer than 512 (row block, K/V head) pairs.
static int plan_block_splits(const alora_attn_dims *d)
{
    const int G = d->n_q_heads / d->n_kv_heads, rbg = 128 / G;
    const long long wgs = (long long)((d->n_tokens + rbg - 1) / rbg) * d->n_kv_heads;
    if (wgs <= 0 || wgs >= 512) return 1;
    return (int)std::min<long long>(32, (512 + wgs - 1) / wgs);
}

static size_t block_split_bytes(const alora_attn_dims *d)
{
    const int sp = plan_block_splits(d);
    if (sp <= 1) return 0;
    return (size_t)d->n_tokens * d->n_q_heads * sp * (d->head_dim + 2) * sizeof(float);
}

static size_t split_bytes(const alora_attn_dims *d)
{
    const int sp = plan_splits(d);
    if (sp <= 1) return 0;
    return (size_t)d->n_tokens * d->n_q_heads * sp * (d->head_dim + 2) * sizeof(float);
}

// which kernel an entry point asks for
enum Reader { PER_ROW, PER_ROW_SPLIT, ROW_BLOCKS, ROW_BLOCKS_SPLIT };

static int run(const void *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
               const int32_t *token_seq_ids, const int32_t *token_positions, void *out, const alora_attn_dims *dims,
               void *workspace, size_t workspace_bytes, Reader mode, void *hip_stream);

}  // namespace alora

extern "C" {

int alora_paged_attention_workspace_bytes(const alora_attn_dims *dims, size_t *out_bytes)
{
    using namespace alora;
    if (!out_bytes) return ALORA_EINVAL;
    const int st = check_dims(dims);
    if (st) return st;
    *out_bytes = split_bytes(dims);
    return ALORA_OK;
}

int alora_paged_attention_split(const void *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
                                const int32_t *token_seq_ids, const int32_t *token_positions, void *out,
                                const alora_attn_dims *dims, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return alora::run(q, k_cache, v_cache, block_tables, token_seq_ids, token_positions, out, dims, workspace,
                      workspace_bytes, alora::PER_ROW_SPLIT, hip_stream);
}

int alora_paged_attention_suffix(const void *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
                                 const int32_t *token_seq_ids, const int32_t *token_positions, void *out,
                                 const alora_attn_dims *dims, void *hip_stream)
{
    return alora::run(q, k_cache, v_cache, block_tables, token_seq_ids, token_positions, out, dims, nullptr, 0,
                      alora::ROW_BLOCKS, hip_stream);
}

int alora_paged_attention_suffix_workspace_bytes(const alora_attn_dims *dims, size_t *out_bytes)
{
    using namespace alora;
    if (!out_bytes) return ALORA_EINVAL;
    const int st = check_dims(dims);
    if (st) return st;
    if (dims->dtype != ALORA_BF16 || dims->head_dim != 128) return ALORA_ESHAPE;
    *out_bytes = block_split_bytes(dims);
    return ALORA_OK;
}

int alora_paged_attention_suffix_split(const void *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
                                       const int32_t *token_seq_ids, const int32_t *token_positions, void *out,
                                       const alora_attn_dims *dims, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return alora::run(q, k_cache, v_cache, block_tables, token_seq_ids, token_positions, out, dims, workspace,
                      workspace_bytes, alora::ROW_BLOCKS_SPLIT, hip_stream);
}

int alora_paged_attention(const void *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
                          const int32_t *token_seq_ids, const int32_t *token_positions, void *out,
                          const alora_attn_dims *dims, void *hip_stream)
{
    return alora::run(q, k_cache, v_cache, block_tables, token_seq_ids, token_positions, out, dims, nullptr, 0,
                      alora::PER_ROW, hip_stream);
}

}  // extern "C"

namespace alora {

static int run(const void *q, const void *k_cache, const void *v_cache, const int32_t *block_tables,
               const int32_t *token_seq_ids, const int32_t *token_positions, void *out, const alora_attn_dims *dims,
               void *workspace, size_t workspace_bytes, Reader mode, void *hip_stream)
{
    const int st = check_dims(dims);
    if (st) return st;
    const bool blocks_asked = mode == ROW_BLOCKS || mode == ROW_BLOCKS_SPLIT;
    if (blocks_asked && (dims->dtype != ALORA_BF16 || dims->head_dim != 128)) return ALORA_ESHAPE;
    // (the row-block kernel reads one table entry per four aligned positions; other block sizes, and a call
    // without table or cache, take the per-row kernel)
    const bool row_blocks = blocks_asked && dims->block_size % 4 == 0 && dims->n_seqs >= 1 && dims->max_blocks >= 1 &&
                            dims->n_slots >= dims->block_size;
    const int splits = mode == PER_ROW_SPLIT ? plan_splits(dims) : (mode == ROW_BLOCKS_SPLIT && row_blocks) ? plan_block_splits(dims) : 1;
    const size_t need = mode == PER_ROW_SPLIT ? split_bytes(dims) : mode == ROW_BLOCKS_SPLIT ? block_split_bytes(dims) : 0;
    if (splits > 1 && (!workspace || ((uintptr_t)workspace & 15) || workspace_bytes < need)) return ALORA_EWORKSPACE;
    if (dims->n_tokens == 0) return ALORA_OK;
    if (!q || !k_cache || !v_cache || !block_tables || !token_seq_ids || !token_positions || !out) return ALORA_EINVAL;
    if (((uintptr_t)q | (uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)out) & 15) return ALORA_EINVAL;
    if (((uintptr_t)block_tables | (uintptr_t)token_seq_ids | (uintptr_t)token_positions) & 3) return ALORA_EINVAL;
    AttnArgs a;
    a.q = q; a.kc = k_cache; a.vc = v_cache;
    a.bt = block_tables; a.seq = token_seq_ids; a.pos = token_positions;
    a.out = out;
    a.T = dims->n_tokens; a.Hq = dims->n_q_heads; a.Hkv = dims->n_kv_heads;
    a.n_seqs = dims->n_seqs; a.max_blocks = dims->max_blocks; a.bs = dims->block_size;
    a.bs_shift = -1;
    for (int sft = 0; sft < 31; ++sft)
        if ((1 << sft) == dims->block_size) a.bs_shift = sft;
    a.n_slots = dims->n_slots;
    a.splits = splits;
    a.part = (float *)workspace;
    const float scale = dims->scale > 0.f ? dims->scale : 1.0f / sqrtf((float)dims->head_dim);
    a.scale_log2e = scale * 1.4426950408889634f;
    const bool bf16 = dims->dtype == ALORA_BF16;
    const int G = dims->n_q_heads / dims->n_kv_heads;
    if (row_blocks) {
        const int e2 = launch_attention_blocks(a, G, (hipStream_t)hip_stream);
        if (e2) { note_hip_error(e2); return ALORA_EHIP; }
        if (splits > 1) {
            hipLaunchKernelGGL((paged_attention_merge_kernel<128, true>), dim3((unsigned)a.T * (unsigned)a.Hq), dim3(128), 0,
                               (hipStream_t)hip_stream, a.part, a.out, a.splits);
            const hipError_t e3 = hipGetLastError();
            if (e3) { note_hip_error((int)e3); return ALORA_EHIP; }
        }
        return ALORA_OK;
    }
    const bool launched = dims->head_dim == 128 ? launch_d<128>(a, G, bf16, (hipStream_t)hip_stream)
                                                : launch_d<64>(a, G, bf16, (hipStream_t)hip_stream);
    if (!launched) return ALORA_ESHAPE;
    const hipError_t e = hipGetLastError();
    if (e) { note_hip_error((int)e); return ALORA_EHIP; }
    return ALORA_OK;
}

}  // namespace alora

extern "C" {

int alora_paged_attention_validate(const int32_t *block_tables, const int32_t *token_seq_ids,
                                   const int32_t *token_positions, const alora_attn_dims *dims)
{
    using namespace alora;
    const int st = check_dims(dims);
    if (st) return st;
    if (dims->n_tokens == 0) return ALORA_OK;
    if (!block_tables || !token_seq_ids || !token_positions) return ALORA_EINVAL;
    const size_t T = (size_t)dims->n_tokens, nt = (size_t)dims->n_seqs * (size_t)dims->max_blocks;
    try {
    std::vector<int32_t> seq(T), pos(T), bt(nt);
    hipError_t e = hipDeviceSynchronize();
    if (!e) e = hipMemcpy(seq.data(), token_seq_ids, T * sizeof(int32_t), hipMemcpyDeviceToHost);
    if (!e) e = hipMemcpy(pos.data(), token_positions, T * sizeof(int32_t), hipMemcpyDeviceToHost);
    if (!e && nt) e = hipMemcpy(bt.data(), block_tables, nt * sizeof(int32_t), hipMemcpyDeviceToHost);
    if (e) { note_hip_error((int)e); return ALORA_EHIP; }
    const long long cap = (long long)dims->max_blocks * dims->block_size;
    const long long n_blocks = dims->n_slots / dims->block_size;
    std::vector<long long> reach((size_t)dims->n_seqs, -1);   // furthest position any row of the sequence reads
    for (size_t t = 0; t < T; ++t) {
        if (seq[t] < 0 || seq[t] >= dims->n_seqs) return ALORA_EDATA;
        if (pos[t] < 0 || pos[t] >= cap) return ALORA_EDATA;
        if (pos[t] > reach[(size_t)seq[t]]) reach[(size_t)seq[t]] = pos[t];
    }
    for (int s = 0; s < dims->n_seqs; ++s) {
        if (reach[(size_t)s] < 0) continue;
        const long long last = reach[(size_t)s] / dims->block_size;
        for (long long b = 0; b <= last; ++b) {
            const int32_t blk = bt[(size_t)s * dims->max_blocks + (size_t)b];
            if (blk < 0 || blk >= n_blocks) return ALORA_EDATA;
        }
    }
    return ALORA_OK;
    } catch (const std::bad_alloc &) {
        return ALORA_ENOMEM;
    }
}

}  // extern "C"
