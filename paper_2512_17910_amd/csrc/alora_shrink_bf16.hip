// LoRA shrink for bf16 batches: S[t,:] = x[t,:] . A[a] for adapted rows only, on bf16 MFMA with
// fp32 accumulation.  Rows come from the grouped list (adapter-major, stable): a workgroup takes
// 32 rows of ONE adapter and one slice of the hidden dimension.
//
// The kernel is latency-bound work (a few MB), so it is built around as few memory round trips as
// possible: a workgroup issues ALL loads of a 128 KB chunk up front as direct-to-LDS copies (the
// gathered token rows, 16-byte chunks XOR-swizzled by row; the adapter's A slice copied verbatim,
// it is already k-major), waits once, then runs the MFMAs out of LDS (ds_read_b128 for tokens,
// the transposing ds_read_b64_tr_b16 for A).  The hidden dimension is cut into up to four slices
// handled by different workgroups so that more CUs pull data at once.
//
// Slices are NOT summed here (that would need a grid-wide exchange).  Each slice's fp32 result is
// stored as two bf16 numbers per element, P_s = hi_s + lo_s with hi = bf16(P), lo = bf16(P - hi),
// and the projection kernel treats [hi_0 | lo_0 | hi_1 | lo_1 | ...] as one long K dimension
// against B stacked the same number of times: the expand runs on the same bf16 MFMA pipe as the
// base GEMM, keeps ~16 mantissa bits of every slice, and the sum over slices happens inside the
// fp32 MFMA accumulator in a fixed order.
#include "alora_internal.h"

namespace alora {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((address_space(3))) unsigned char lds_byte;

__device__ __attribute__((aligned(256))) uint32_t g_zero_page[64];  // zero-initialised

constexpr int SHRINK_ROWS = 32;
constexpr int SHRINK_MAX_SLICES = 4;

// chunk of the hidden dimension that fits LDS at once (tokens 32 x chunk, A chunk x rank)
static inline int shrink_chunk_len(int r) { return r <= 32 ? 1024 : 512; }

int shrink_slices(int H, int r)
{
    const int chunks = (H + shrink_chunk_len(r) - 1) / shrink_chunk_len(r);
    return chunks < SHRINK_MAX_SLICES ? chunks : SHRINK_MAX_SLICES;
}
// hidden-dimension extent of one slice: a whole number of chunks
static inline int shrink_slice_len(int H, int r)
{
    const int c = shrink_chunk_len(r);
    const int chunks = (H + c - 1) / c, ks = shrink_slices(H, r);
    return ((chunks + ks - 1) / ks) * c;
}

// KSL: chunk length; NT: 32-wide rank tiles (1 for rank <= 32, else 2)
template <int KSL, int NT>
__global__ __launch_bounds__(256) void shrink_bf16_kernel(const bf16_t *__restrict__ x, PtrTable A,
                                                          const int32_t *__restrict__ perm,
                                                          const int4 *__restrict__ blocktab, int L, int H, int r,
                                                          int slice_len, bf16_t *__restrict__ S_hl)
{
    constexpr int XROW_BYTES = KSL * 2;
    constexpr int CPR = KSL / 8;                 // 16-byte chunks per token row
    constexpr int X_BYTES = SHRINK_ROWS * XROW_BYTES;
    constexpr int A_BYTES = 65536;               // KSL * rank * 2 <= 64 KB for both instantiations
    __shared__ __attribute__((aligned(16))) unsigned char xs[X_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char as[A_BYTES + 256];
    __shared__ float red[4][NT][32][33];
    __shared__ int rows_t[SHRINK_ROWS];

    // which (adapter, 32-row block) is this workgroup?  (table written by the grouping kernel)
    const int4 entry = blocktab[blockIdx.y];
    const int a = entry.x, j0 = entry.y, cnt = entry.z;
    if (a < 0 || a >= L) return;  // unused entry or the base group; uniform across the workgroup

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int KS = gridDim.x, slice = blockIdx.x;
    const int k_begin = slice * slice_len, k_end = min(H, k_begin + slice_len);
    const bf16_t *Aa = (const bf16_t *)A.p[a];

    if (tid < SHRINK_ROWS) rows_t[tid] = tid < cnt ? perm[j0 + tid] : -1;
    __syncthreads();

    const int li = lane & 31, lh = lane >> 5;
    const int s16 = lane & 15, blk = (lane >> 4) & 1;
    const int row_bytes = 2 * r;
    f32x16 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[nt][e] = 0.f;

    for (int ks0 = k_begin; ks0 < k_end; ks0 += KSL) {
        const int klen = min(KSL, k_end - ks0);  // multiple of 64
        // ---- all loads of the chunk, up front -----------------------------------------------
        // A chunk: rows ks0 .. ks0+klen of [H, r], contiguous in memory, copied verbatim
        {
            const size_t a_bytes = (size_t)klen * r * 2;
            const unsigned char *abase = (const unsigned char *)(Aa + (size_t)ks0 * r);
#pragma unroll
            for (int qq = 0; qq < 16; ++qq) {
                const int q = w * 16 + qq;
                const size_t off = (size_t)q * 1024 + 16 * lane;
                const void *src = off < a_bytes ? (const void *)(abase + off) : (const void *)g_zero_page;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                                 (__attribute__((address_space(3))) void *)((lds_byte *)as + q * 1024),
                                                 16, 0, 0);
            }
        }
        // tokens: instruction q copies 64 chunks of row q / (CPR/64); lane -> physical chunk, which
        // holds logical chunk (physical ^ (row % 16))
        constexpr int XI = SHRINK_ROWS * CPR / 64;
        constexpr int PARTS = CPR / 64;
#pragma unroll
        for (int qq = 0; qq < XI / 4; ++qq) {
            const int q = w * (XI / 4) + qq;
            const int row = q / PARTS, part = q % PARTS;
            const int t = rows_t[row];
            const int c = (part * 64 + lane) ^ (row & 15);
            const bool ok = t >= 0 && 8 * c < klen;
            const void *src = ok ? (const void *)(x + (size_t)t * H + ks0 + 8 * c) : (const void *)g_zero_page;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                             (__attribute__((address_space(3))) void *)((lds_byte *)xs + q * 1024), 16,
                                             0, 0);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();

        // ---- MFMA out of LDS; the four wavefronts interleave over the 16-wide k steps ---------
        for (int ks = w; ks < klen / 16; ks += 4) {
            const int c = 2 * ks + lh;
            const bf16x8 xf = *(const __attribute__((address_space(3))) bf16x8 *)((const lds_byte *)xs +
                                                                                   li * XROW_BYTES + ((c ^ (li & 15)) << 4));
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int kk = 16 * ks + 8 * lh + (s16 >> 2);
                const int col = nt * 32 + 16 * blk + 4 * (s16 & 3);
                const lds_byte *p = (const lds_byte *)as + kk * row_bytes + col * 2;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)p);
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4 *)(p + 4 * row_bytes));
                const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, __builtin_bit_cast(bf16x8, v), acc[nt], 0, 0, 0);
            }
        }
        __syncthreads();  // LDS is overwritten by the next chunk
    }

    // D[row][col]: lane holds col = lane % 32, rows 8g + 4*lh + jj in register 4g + jj
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) red[w][nt][8 * g + 4 * lh + jj][li] = acc[nt][4 * g + jj];
    __syncthreads();

    // ---- add the four wavefronts in fixed order, split, store this slice's columns --------------
    for (int idx = tid; idx < 32 * 32 * NT; idx += 256) {
        const int col = idx % (32 * NT), row = idx / (32 * NT);
        const int tt = rows_t[row];
        if (tt < 0 || col >= r) continue;
        const int nt = col >> 5, c = col & 31;
        const float s = ((red[0][nt][row][c] + red[1][nt][row][c]) + red[2][nt][row][c]) + red[3][nt][row][c];
        const uint32_t hi = f32_to_bf16_bits(s);
        const uint32_t lo = f32_to_bf16_bits(s - bf16_bits_to_f32(hi));
        bf16_t *dst = S_hl + ((size_t)tt * KS + slice) * 2 * r;
        dst[col] = (bf16_t)hi;
        dst[r + col] = (bf16_t)lo;
    }
}

int launch_shrink_bf16(const Fwd &f, const PtrTable &A)
{
    if (f.T == 0 || f.L == 0) return 0;
    const dim3 grid(shrink_slices(f.H, f.r), f.n_blocks);
    const int sl = shrink_slice_len(f.H, f.r);
    if (f.r <= 32)
        hipLaunchKernelGGL((shrink_bf16_kernel<1024, 1>), grid, dim3(256), 0, f.stream, (const bf16_t *)f.x, A, f.perm,
                           f.blocktab, f.L, f.H, f.r, sl, (bf16_t *)f.S);
    else
        hipLaunchKernelGGL((shrink_bf16_kernel<512, 2>), grid, dim3(256), 0, f.stream, (const bf16_t *)f.x, A, f.perm,
                           f.blocktab, f.L, f.H, f.r, sl, (bf16_t *)f.S);
    return (int)hipGetLastError();
}

}  // namespace alora
