// Reader of the paged K/V cache for query rows that share a context: consecutive rows of one sequence
// (a projected suffix attending over a cached prefix, Sec. 2.3 / 4.2) are handled by ONE workgroup per
// K/V head, which loads every cached row once for all of them.  bf16, head_dim 128, on bf16 MFMA.
//
// A workgroup owns up to 32 columns (query row, query head of the K/V head's group): 32 / G rows.  Row
// blocks are cut at multiples of 32 / G of the POSITION, so whether a batch row leads a block is decided
// from the row before it alone; the workgroups of the other rows exit at once.  A decode batch (every
// row its own sequence) degenerates to one row per workgroup.
//
// Per 32 context positions a wavefront runs two sets of 32x32x16 MFMAs that keep every column in one
// lane pair from the scores to the output:
//   scores^T [position x column] = K [position x d] . Q^T [d x column]   K rows loaded straight from the
//       cache into the A operand (a lane holds 8 consecutive d of one position), Q held in registers;
//   online softmax down each column: 16 accumulator registers per lane, one exchange between the two
//       lanes of a column;
//   out^T [d x column] += V^T [d x position] . P [position x column]   V goes through LDS and comes back
//       with the transposing LDS load; P is the score accumulator itself, rounded to bf16 -- the B operand
//       wants, per lane, the positions the accumulator registers of that lane already hold, up to an
//       exchange of two position bits that is applied to the V rows when they are written to LDS.
// The four wavefronts take every fourth block of 32 positions and are merged in fixed order at the end.
#include "alora_attention_internal.h"

namespace alora {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((address_space(3))) unsigned char lds_byte;

constexpr float AB_NEG_INF = -__builtin_inff();
constexpr float AB_M_FLOOR = -1.0e30f;   // finite floor of the running maximum (scores below it weigh nothing)

// k..k+3 of this lane's column, then k+4..k+7 (four rows further on)
__device__ __forceinline__ bf16x8 read_tr_frag(const lds_byte *p, int pitch)
{
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p + 4 * pitch));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

template <int G>
__global__ __launch_bounds__(256) void paged_attention_blocks_kernel(AttnArgs a)
{
    constexpr int D = 128, RB = 32 / G;   // query rows per workgroup
    constexpr int VPITCH = 256;           // bytes per position row of the V tile in LDS
    __shared__ __attribute__((aligned(16))) unsigned char vt[4][32 * VPITCH];   // one V tile per wavefront
    __shared__ float mrg[3][64][2 + 64];                                        // wavefronts 1..3 hand over to 0

    const int t0 = (int)blockIdx.x / a.Hkv, hk = (int)blockIdx.x % a.Hkv;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, li = lane & 31, lh = lane >> 5;
    const int sq = a.seq[t0], p0 = a.pos[t0];
    const bool row_ok = sq >= 0 && sq < a.n_seqs && p0 >= 0;
    // does this row lead a block?  (the row before it is the same sequence's previous position, and the
    // position is not a multiple of the block: then an earlier row leads)
    if (row_ok && t0 > 0 && (p0 % RB) != 0 && a.seq[t0 - 1] == sq && a.pos[t0 - 1] == p0 - 1) return;
    // rows of the block: up to the next multiple of RB, as long as the run continues
    int nrows = 1;
    if (row_ok) {
        const int limit = RB - (p0 % RB);
        bool cont = false;
        if (lane > 0 && lane < limit && t0 + lane < a.T) cont = a.seq[t0 + lane] == sq && a.pos[t0 + lane] == p0 + lane;
        const unsigned long long mask = __builtin_amdgcn_ballot_w64(cont) | 1ull;
        nrows = __builtin_ctzll(~mask);
    }
    const long long cap = (long long)a.max_blocks * a.bs;
    int n_ctx = 0;
    if (row_ok) n_ctx = (int)((long long)p0 + nrows < cap ? (long long)p0 + nrows : cap);
    const int32_t *bt = a.bt + (size_t)(row_ok ? sq : 0) * a.max_blocks;
    const int Nkv = a.Hkv * D;
    const long long n_blocks = a.n_slots / a.bs;

    // this lane's column: query row r_j of the block, query head g_j of the group
    const int r_j = li / G, g_j = li % G;
    const bool col_ok = row_ok && r_j < nrows;
    const int lim_j = col_ok ? p0 + r_j : -1;   // last position the column attends to
    const size_t q_at = ((size_t)(t0 + (col_ok ? r_j : 0)) * a.Hq + (size_t)hk * G + g_j) * D;
    bf16x8 qf[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (col_ok) v = *(const u32x4 *)((const bf16_t *)a.q + q_at + 16 * s + 8 * lh);
        qf[s] = __builtin_bit_cast(bf16x8, v);
    }

    f32x16 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
    float m = AB_M_FLOOR, l = 0.f;

    // V tile addressing.  Write: the row of position i (this lane's) with position bits 2 and 3 exchanged;
    // 16-byte chunks XOR-swizzled by 4 * (row % 4).  Read: fragment of d tile `t`, k step `ks`.
    lds_byte *const tile = (lds_byte *)vt[w];
    const int vrow = (li & ~12) | ((li & 4) << 1) | ((li & 8) >> 1);
    uint32_t vaddr[4];
    {
        const int s16 = lane & 15, j = s16 >> 2, blk = (lane >> 4) & 1;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int chunk = 4 * t + 2 * blk + ((s16 & 3) >> 1);
            vaddr[t] = (uint32_t)(8 * lh + j) * VPITCH + (uint32_t)((chunk ^ (j << 2)) << 4) + (uint32_t)((s16 & 1) << 3);
        }
    }

    for (int cb = 32 * w; cb < n_ctx; cb += 128) {
        // ---- this lane's position: its K row into the A operand, its V row into LDS -------------
        const int pi = cb + li;
        bool have = pi < n_ctx;
        long long slot = 0;
        if (have) {
            const int bi = a.bs_shift >= 0 ? (pi >> a.bs_shift) : (pi / a.bs);
            const int blk = bt[bi];
            have = blk >= 0 && blk < n_blocks;
            slot = (long long)blk * a.bs + (pi - bi * a.bs);
        }
        const unsigned okmask = (unsigned)__builtin_amdgcn_ballot_w64(have);   // bits 0..31: positions of the block
        const size_t at = (size_t)slot * Nkv + (size_t)hk * D + 8 * lh;
        u32x4 kf[8], vf[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            kf[s] = u32x4{0u, 0u, 0u, 0u};
            vf[s] = kf[s];
            if (have) {
                kf[s] = *(const u32x4 *)((const bf16_t *)a.kc + at + 16 * s);
                vf[s] = *(const u32x4 *)((const bf16_t *)a.vc + at + 16 * s);
            }
        }
        // ---- scores^T = K . Q^T ------------------------------------------------------------------
        f32x16 sc;
#pragma unroll
        for (int e = 0; e < 16; ++e) sc[e] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s)
            sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[s]), qf[s], sc, 0, 0, 0);
#pragma unroll
        for (int s = 0; s < 8; ++s)
            *(__attribute__((address_space(3))) u32x4 *)(tile + vrow * VPITCH + (((2 * s + lh) ^ ((vrow & 3) << 2)) << 4)) = vf[s];
        // ---- softmax down this lane's column -----------------------------------------------------
        float mx = AB_NEG_INF;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int idx = 8 * (v >> 2) + 4 * lh + (v & 3);
            const bool on = ((okmask >> idx) & 1u) && cb + idx <= lim_j;
            sc[v] = on ? sc[v] * a.scale_log2e : AB_NEG_INF;
            mx = fmaxf(mx, sc[v]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float mn = fmaxf(m, mx);
        const float corr = __builtin_amdgcn_exp2f(m - mn);
        m = mn;
        float ps = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            sc[v] = __builtin_amdgcn_exp2f(sc[v] - mn);
            ps += sc[v];
        }
        l = l * corr + ps;
        if (__builtin_amdgcn_ballot_w64(corr != 1.f)) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[t][e] *= corr;
        }
        // ---- out^T += V^T . P : P straight from the score registers --------------------------------
        bf16x8 pf[2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const u32x4 pv = {pack_bf16(sc[8 * ks + 0], sc[8 * ks + 1]), pack_bf16(sc[8 * ks + 2], sc[8 * ks + 3]),
                              pack_bf16(sc[8 * ks + 4], sc[8 * ks + 5]), pack_bf16(sc[8 * ks + 6], sc[8 * ks + 7])};
            pf[ks] = __builtin_bit_cast(bf16x8, pv);
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int t = 0; t < 4; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_tr_frag(tile + vaddr[t] + ks * 16 * VPITCH, VPITCH), pf[ks],
                                                                 acc[t], 0, 0, 0);
    }

    // ---- the two lanes of a column add their weight sums; wavefronts 1..3 hand over to wavefront 0 ---
    l += __shfl_xor(l, 32);
    if (w > 0) {
        float *dst = mrg[w - 1][lane];
        dst[0] = m;
        dst[1] = l;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) dst[2 + 16 * t + e] = acc[t][e];
    }
    __syncthreads();
    if (w > 0) return;
    float M = m;
#pragma unroll
    for (int ww = 0; ww < 3; ++ww) M = fmaxf(M, mrg[ww][lane][0]);
    float f0 = __builtin_amdgcn_exp2f(m - M);
    float L = l * f0;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] *= f0;
#pragma unroll
    for (int ww = 0; ww < 3; ++ww) {
        const float *src = mrg[ww][lane];
        const float f = __builtin_amdgcn_exp2f(src[0] - M);
        L += src[1] * f;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[t][e] += src[2 + 16 * t + e] * f;
    }
    // a row that is not valid leads a block of its own and gets zeros
    if (!(col_ok || (!row_ok && r_j == 0))) return;
    const float inv = L > 0.f ? 1.f / L : 0.f;
    bf16_t *orow = (bf16_t *)a.out + ((size_t)(t0 + r_j) * a.Hq + (size_t)hk * G + g_j) * D;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const u32x2 o = {pack_bf16(acc[t][4 * b + 0] * inv, acc[t][4 * b + 1] * inv),
                             pack_bf16(acc[t][4 * b + 2] * inv, acc[t][4 * b + 3] * inv)};
            *(u32x2 *)(orow + 32 * t + 8 * b + 4 * lh) = o;
        }
}

int launch_attention_blocks(const AttnArgs &a, int G, hipStream_t stream)
{
    const dim3 grid((unsigned)a.T * (unsigned)a.Hkv), block(256);
    switch (G) {
    case 1: hipLaunchKernelGGL(paged_attention_blocks_kernel<1>, grid, block, 0, stream, a); break;
    case 2: hipLaunchKernelGGL(paged_attention_blocks_kernel<2>, grid, block, 0, stream, a); break;
    case 4: hipLaunchKernelGGL(paged_attention_blocks_kernel<4>, grid, block, 0, stream, a); break;
    case 8: hipLaunchKernelGGL(paged_attention_blocks_kernel<8>, grid, block, 0, stream, a); break;
    default: return (int)hipErrorInvalidValue;
    }
    return (int)hipGetLastError();
}

}  // namespace alora
