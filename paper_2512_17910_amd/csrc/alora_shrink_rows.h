// The shrink of one 32-row block of one adapter over one range of the hidden dimension:
// S[t,:] = x[t, kbeg:kend] . A_a[kbeg:kend, :] for the block's rows, on bf16 MFMA with fp32 accumulation.
// Device code shared by the shrink kernel and by the small-batch projection kernel, which runs the
// shrink of a decode-sized batch on the compute units its own workgroups leave free.  The caller
// provides the LDS (two token buffers, two A buffers, the cross-wavefront reduction array) and has
// the block's row ids in rows_t (-1 = no row) before the call; 256 threads, all of them call.
#pragma once
#include "alora_internal.h"

namespace alora {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((address_space(3))) unsigned char lds_byte;

constexpr int SHRINK_ROWS = 32;

template <int KSL, int NT>
struct ShrinkLds {
    static constexpr int X_BYTES = SHRINK_ROWS * KSL * 2;
    static constexpr int A_BYTES = KSL * 32 * NT * 2 + 256;
    static constexpr int RED_BYTES = 4 * NT * 32 * 33 * 4;
};

// KSL: hidden-dimension chunk per LDS buffer; NT: 32-wide rank tiles (1 for rank <= 32, else 2).
// WORK_LIST with n_ranges > 1: the ranges of a block are combined here, by the last one to finish
// (`counter` counts the block's finished ranges, `is_last` is one int of LDS).  Otherwise several
// ranges leave fp32 partials P[range][t][:] and one range stores the (hi, lo) form.
template <int KSL, int NT, bool WORK_LIST>
__device__ __forceinline__ void shrink_rows(const bf16_t *__restrict__ x, const bf16_t *Aa, int rk, const int *rows_t, int H,
                                            int r, uint32_t x_bytes, int T, int kbeg, int kend, int range, int n_ranges,
                                            int32_t *counter, void *S_out, unsigned char *xs0, unsigned char *xs1,
                                            unsigned char *as0, unsigned char *as1, float (*red)[NT][32][33], int *is_last)
{
    constexpr int XROW_BYTES = KSL * 2;
    constexpr int CPR = KSL / 8;                 // 16-byte chunks per token row
    constexpr int X_BYTES = SHRINK_ROWS * XROW_BYTES;
    constexpr int A_BYTES = KSL * 32 * NT * 2;   // KSL rows of up to 32*NT rank columns
    constexpr int XI = X_BYTES / 1024 / 4;       // token-copy instructions per wavefront and chunk
    constexpr int AI = A_BYTES / 1024 / 4;       // A-copy instructions per wavefront and chunk
    constexpr int RPI = 64 / CPR;                // token rows per copy instruction (1 or 2)
    static_assert(CPR == 64 || CPR == 32, "chunk layout");
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, lh = lane >> 5;
    const int s16 = lane & 15, blk = (lane >> 4) & 1;
    const int row_bytes = 2 * rk;
    f32x16 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[nt][e] = 0.f;

    // all copies of the chunk starting at hidden index ks0
    // Buffer descriptors: reads past the end of A (a short last chunk) return zeros by themselves;
    // masked token lanes get an offset past the end of x.
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc((void *)Aa, 0, H * rk * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)x, 0, (int)x_bytes, 0x00020000);
    // per-lane byte offsets of the token copies at hidden index 0 (0xffffffff = masked)
    uint32_t xoff[XI];
    int xchunk[XI];
#pragma unroll
    for (int qq = 0; qq < XI; ++qq) {
        const int row = (w * XI + qq) * RPI + lane / CPR;
        const int t = rows_t[row];
        xchunk[qq] = (lane % CPR) ^ (row & 15);
        xoff[qq] = t >= 0 ? (uint32_t)t * (uint32_t)H * 2u + 16u * xchunk[qq] : 0xffffffffu;
    }
    auto issue = [&](int ks0, unsigned char *xs, unsigned char *as) {
        const int klen = min(KSL, kend - ks0);  // multiple of 64
#pragma unroll
        for (int qq = 0; qq < AI; ++qq) {
            const int q = w * AI + qq;
            const uint32_t off = (uint32_t)q * 1024u + 16u * lane;
            // rows ks0 .. ks0+klen of [H, r] are contiguous; what lies beyond them in the buffer is
            // either past the end of A (zeros) or masked here
            const uint32_t vo = off < (uint32_t)klen * rk * 2 ? off : 0xffffffffu;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (__attribute__((address_space(3))) void *)((lds_byte *)as + q * 1024),
                                                     16, vo, (uint32_t)ks0 * rk * 2, 0, 0);
        }
        // tokens: instruction q copies RPI rows; lane -> physical chunk, holding logical chunk
        // (physical ^ (row % 16))
#pragma unroll
        for (int qq = 0; qq < XI; ++qq) {
            const int q = w * XI + qq;
            const uint32_t vo = 8 * xchunk[qq] < klen ? xoff[qq] : 0xffffffffu;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (__attribute__((address_space(3))) void *)((lds_byte *)xs + q * 1024),
                                                     16, vo, (uint32_t)ks0 * 2, 0, 0);
        }
    };
    // MFMAs of one chunk out of LDS; the four wavefronts interleave over the 16-wide k steps
    // (a short last chunk is zero-filled by the copies, so every chunk runs all its k steps and the
    // loop unrolls into straight-line code)
    // The LDS reads are written as assembly with their own wait: the compiler cannot tell which of
    // the in-flight copies a read depends on and would otherwise drain all of them (including the
    // next chunk's) before the first read.  The explicit waits around compute() order them.
    auto compute = [&](const unsigned char *xs, const unsigned char *as) {
        const uint32_t xbase = (uint32_t)(uintptr_t)(const lds_byte *)xs + li * XROW_BYTES;
        const uint32_t abase = (uint32_t)(uintptr_t)(const lds_byte *)as + (8 * lh + (s16 >> 2)) * row_bytes +
                               (16 * blk + 4 * (s16 & 3)) * 2;
#pragma unroll
        for (int kq = 0; kq < KSL / 64; ++kq) {
            const int ks = 4 * kq + w;
            const int c = 2 * ks + lh;
            const uint32_t xa = xbase + ((c ^ (li & 15)) << 4);
            u32x4 xv;
            u32x2 lo[NT], hi[NT];
            uint32_t pa[NT], pb[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                pa[nt] = abase + 16 * ks * row_bytes + nt * 64;
                pb[nt] = pa[nt] + 4 * row_bytes;
            }
            if constexpr (NT == 1) {
                asm volatile("ds_read_b128 %0, %3\n\tds_read_b64_tr_b16 %1, %4\n\tds_read_b64_tr_b16 %2, %5\n\t"
                             "s_waitcnt lgkmcnt(0)"
                             : "=&v"(xv), "=&v"(lo[0]), "=&v"(hi[0])
                             : "v"(xa), "v"(pa[0]), "v"(pb[0])
                             : "memory");
            } else {
                asm volatile("ds_read_b128 %0, %5\n\tds_read_b64_tr_b16 %1, %6\n\tds_read_b64_tr_b16 %2, %7\n\t"
                             "ds_read_b64_tr_b16 %3, %8\n\tds_read_b64_tr_b16 %4, %9\n\ts_waitcnt lgkmcnt(0)"
                             : "=&v"(xv), "=&v"(lo[0]), "=&v"(hi[0]), "=&v"(lo[NT - 1]), "=&v"(hi[NT - 1])
                             : "v"(xa), "v"(pa[0]), "v"(pb[0]), "v"(pa[NT - 1]), "v"(pb[NT - 1])
                             : "memory");
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const u32x4 av = {lo[nt].x, lo[nt].y, hi[nt].x, hi[nt].y};
                acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xv),
                                                                  __builtin_bit_cast(bf16x8, av), acc[nt], 0, 0, 0);
            }
        }
    };
    // wait until only the `newer` most recent copies of this wavefront are outstanding, then meet
    // the other wavefronts (whose copies the MFMAs read as well)
#define SHRINK_WAIT_OLDER() asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(XI + AI) : "memory")
#define SHRINK_WAIT_ALL() asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory")
#define SHRINK_BARRIER() asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory")

    const int nchunks = (kend - kbeg + KSL - 1) / KSL;
    issue(kbeg, xs0, as0);
    if (nchunks > 1) issue(kbeg + KSL, xs1, as1);
    for (int i = 0; i < nchunks; i += 2) {
        if (i + 1 < nchunks) SHRINK_WAIT_OLDER(); else SHRINK_WAIT_ALL();
        compute(xs0, as0);
        SHRINK_BARRIER();  // every wavefront is done with buffer 0
        if (i + 2 < nchunks) issue(kbeg + (i + 2) * KSL, xs0, as0);
        if (i + 1 >= nchunks) break;
        if (i + 2 < nchunks) SHRINK_WAIT_OLDER(); else SHRINK_WAIT_ALL();
        compute(xs1, as1);
        SHRINK_BARRIER();
        if (i + 3 < nchunks) issue(kbeg + (i + 3) * KSL, xs1, as1);
    }
#undef SHRINK_WAIT_OLDER
#undef SHRINK_WAIT_ALL
#undef SHRINK_BARRIER

    // D[row][col]: lane holds col = lane % 32, rows 8g + 4*lh + jj in register 4g + jj
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) red[w][nt][8 * g + 4 * lh + jj][li] = acc[nt][4 * g + jj];
    __syncthreads();

    // ---- add the four wavefronts in fixed order; store (hi, lo) or this range's fp32 partial -----
    const bool ranges = n_ranges > 1, ranges_gt1 = ranges;
    // Work-list mode with several ranges: what crosses workgroups inside this kernel.
    //   payload   the partials, and the (hi, lo) rows that reuse the bytes of range 0's partials, are relaxed
    //             atomic stores / loads at agent scope: stores that write through and loads that read past the
    //             per-XCD L2's non-coherent lines, so no cache-wide write-back or invalidate is needed for them;
    //   order     every wavefront waits for its stores (vmcnt(0)), the workgroup meets at a barrier, then ONE
    //             thread increments the block's counter with acquire-release semantics at agent scope.  The
    //             release makes the workgroup's partials (ordered before it by the barrier) visible before the
    //             increment; the acquire of the increment that completes the count, followed by a barrier,
    //             orders the last workgroup's loads of ALL ranges' partials behind every other range's release.
    // (An agent-scope fence executed by every thread instead was measured 3x slower; the acquire-release on the
    // single increment costs about 1 us of a 19 us kernel.)
    const bool coherent = WORK_LIST && ranges_gt1;
    auto store_hi_lo = [&](int tt, int col, float s) {
        const uint32_t hi = f32_to_bf16_bits(s);
        const uint32_t lo = f32_to_bf16_bits(s - bf16_bits_to_f32(hi));
        bf16_t *dst = (bf16_t *)S_out + (size_t)tt * 2 * r;
        if (coherent) {
            __hip_atomic_store(dst + col, (bf16_t)hi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(dst + r + col, (bf16_t)lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            dst[col] = (bf16_t)hi;
            dst[r + col] = (bf16_t)lo;
        }
    };
    for (int idx = tid; idx < 32 * 32 * NT; idx += 256) {
        const int col = idx % (32 * NT), row = idx / (32 * NT);
        const int tt = rows_t[row];
        if (tt < 0 || col >= r) continue;
        const int nt = col >> 5, c = col & 31;
        // rank columns past this adapter's own rank are zero (the consumers walk the common rank r)
        const float s = col < rk ? ((red[0][nt][row][c] + red[1][nt][row][c]) + red[2][nt][row][c]) + red[3][nt][row][c] : 0.f;
        float *part = (float *)S_out + ((size_t)range * T + tt) * r + col;
        if (coherent) __hip_atomic_store(part, s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else if (ranges) *part = s;
        else store_hi_lo(tt, col, s);
    }
    if (!WORK_LIST || !ranges) return;

    // ---- the last range of this block to get here adds the block's partials and stores (hi, lo) ----
    // The partial of range 0 of a row and the row's (hi, lo) form occupy the same 4r bytes, so every
    // partial of the block is read before the first (hi, lo) store.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wavefront's partials have been written through
    __syncthreads();
    if (tid == 0)
        *is_last = __hip_atomic_fetch_add(counter, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT) == n_ranges - 1;
    __syncthreads();
    if (!*is_last) return;
    // the counter is ready for the next call on this workspace (one that reuses the grouping results)
    if (tid == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    constexpr int PER = 32 * 32 * NT / 256;
    // all loads first (they are round trips past the L2), then the sums in range order
    float part[PER][ALORA_SHRINK_MAX_SPLITS], sum[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int idx = tid + 256 * k, col = idx % (32 * NT), tt = rows_t[idx / (32 * NT)];
#pragma unroll
        for (int g = 0; g < ALORA_SHRINK_MAX_SPLITS; ++g) {
            part[k][g] = 0.f;
            if (tt >= 0 && col < r && g < n_ranges)
                part[k][g] = __hip_atomic_load((const float *)S_out + ((size_t)g * T + tt) * r + col, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
        }
    }
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        float sv = 0.f;
#pragma unroll
        for (int g = 0; g < ALORA_SHRINK_MAX_SPLITS; ++g) sv += part[k][g];   // ranges past n_ranges add +0
        sum[k] = sv;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int idx = tid + 256 * k, col = idx % (32 * NT), tt = rows_t[idx / (32 * NT)];
        if (tt >= 0 && col < r) store_hi_lo(tt, col, sum[k]);
    }
}

}  // namespace alora
