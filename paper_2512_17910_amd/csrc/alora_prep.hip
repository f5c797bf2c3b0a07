// Row classification (App. B mask, negated and combined with "has an adapter") and the stable
// grouping of adapted rows by adapter id that the multi-adapter LoRA shrink walks.
//
// One workgroup of 16 wavefronts.  A first sweep classifies every row with independent,
// coalesced loads and parks the row's effective adapter (-1 = keeps the base output) in LDS;
// the grouping itself then runs out of LDS.  Each wavefront owns a contiguous range of token
// rows, so "wavefront index, then row index" is the original row order and the grouping is
// stable without any sort: count per (wavefront, adapter), prefix-sum the counts adapter-major /
// wavefront-minor, then place rows with wavefront-local cursors.  Ranks inside a 64-row step
// come from ballots, so there are no data-dependent atomics and the result is deterministic.
// Batches too large for the LDS row cache re-classify from global memory in both sweeps.
#include "alora_internal.h"

namespace alora {

constexpr int PREP_WAVES = 16;
constexpr int PREP_THREADS = PREP_WAVES * 64;
constexpr int PREP_CACHE_ROWS = 96 * 1024;  // int8 per row

template <bool CACHED>
__global__ __launch_bounds__(PREP_THREADS) void classify_group_kernel(
    const int32_t *__restrict__ aid, const int32_t *__restrict__ seg, const int32_t *__restrict__ pos,
    const int32_t *__restrict__ start, int T, int L, uint8_t *__restrict__ active,
    int8_t *__restrict__ aeff_out,
    int32_t *__restrict__ perm, int32_t *__restrict__ offsets,
    int4 *__restrict__ blocktab, int n_blocks)
{
    __shared__ int cnt[PREP_WAVES][ALORA_MAX_ADAPTERS];
    __shared__ int goff[ALORA_MAX_ADAPTERS + 1], bfirst[ALORA_MAX_ADAPTERS + 1], tot[ALORA_MAX_ADAPTERS];
    __shared__ int8_t aeff[CACHED ? PREP_CACHE_ROWS : 64];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int per_wave = ((T + PREP_WAVES * 64 - 1) / (PREP_WAVES * 64)) * 64;
    const int t0 = min(T, w * per_wave);
    const int t1 = min(T, t0 + per_wave);
    volatile int *my_cnt = cnt[w];

    for (int i = threadIdx.x; i < PREP_WAVES * ALORA_MAX_ADAPTERS; i += PREP_THREADS) (&cnt[0][0])[i] = 0;
    if (CACHED) {
        // classification sweep: coalesced, four independent rows per thread and trip
        for (int tb = threadIdx.x; tb < T; tb += 4 * PREP_THREADS) {
            int a[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int t = tb + u * PREP_THREADS;
                a[u] = t < T ? aid[t] : -1;
            }
            int s[4], p[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int t = tb + u * PREP_THREADS;
                s[u] = a[u] >= 0 ? seg[t] : 0;
                p[u] = a[u] >= 0 ? pos[t] : 0;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int t = tb + u * PREP_THREADS;
                if (t < T) {
                    const int e = (a[u] >= 0 && p[u] >= start[s[u]]) ? a[u] : -1;
                    aeff[t] = (int8_t)e;
                    aeff_out[t] = (int8_t)e;
                    active[t] = (uint8_t)(e >= 0);
                }
            }
        }
    }
    __syncthreads();

    // pass 1: per-(wavefront, adapter) counts
    for (int tb = t0; tb < t1; tb += 64) {
        const int t = tb + lane;
        int a = -1;
        if (t < t1) {
            if (CACHED) {
                a = aeff[t];
            } else {
                a = effective_adapter(aid, seg, pos, start, t);
                aeff_out[t] = (int8_t)a;
                active[t] = (uint8_t)(a >= 0);
            }
        }
        unsigned long long rem = __ballot(a >= 0);
        while (rem) {
            const int lead = __ffsll((long long)rem) - 1;
            const int key = __shfl(a, lead);
            const unsigned long long m = __ballot(a == key);
            if (lane == lead) my_cnt[key] = my_cnt[key] + __popcll(m);
            rem &= ~m;
        }
    }
    __syncthreads();

    // exclusive prefix over wavefronts inside each adapter, adapter totals
    if ((int)threadIdx.x < ALORA_MAX_ADAPTERS) {
        int run = 0;
        if ((int)threadIdx.x < L) {
            for (int ww = 0; ww < PREP_WAVES; ++ww) {
                const int c = cnt[ww][threadIdx.x];
                cnt[ww][threadIdx.x] = run;
                run += c;
            }
        }
        tot[threadIdx.x] = run;
    }
    __syncthreads();
    // one wavefront scans the adapter totals (two adapters per lane): row offsets of the groups
    // and first 32-row block of every adapter in the shrink's block table
    if (w == 0) {
        const int c0 = tot[2 * lane], c1 = tot[2 * lane + 1];
        const int b0 = (c0 + 31) >> 5, b1 = (c1 + 31) >> 5;
        int rows = c0 + c1, blks = b0 + b1;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int r_up = __shfl_up(rows, d), b_up = __shfl_up(blks, d);
            if (lane >= d) { rows += r_up; blks += b_up; }
        }
        goff[2 * lane] = rows - c0 - c1;
        goff[2 * lane + 1] = rows - c1;
        bfirst[2 * lane] = blks - b0 - b1;
        bfirst[2 * lane + 1] = blks - b1;
        if (lane == 63) { goff[ALORA_MAX_ADAPTERS] = rows; bfirst[ALORA_MAX_ADAPTERS] = blks; }
    }
    __syncthreads();
    if ((int)threadIdx.x <= L) offsets[threadIdx.x] = goff[threadIdx.x];
    // block table: entry b = (adapter, first index into perm, rows in block, 0); unused entries -1
    if ((int)threadIdx.x < L) {
        const int a = threadIdx.x, n = tot[a], o = goff[a];
        for (int b = 0; b * 32 < n; ++b) {
            int4 e = make_int4(a, o + 32 * b, min(32, n - 32 * b), 0);
            blocktab[bfirst[a] + b] = e;
        }
    }
    for (int b = bfirst[ALORA_MAX_ADAPTERS] + threadIdx.x; b < n_blocks; b += PREP_THREADS)
        blocktab[b] = make_int4(-1, 0, 0, 0);

    // pass 2: placement
    for (int tb = t0; tb < t1; tb += 64) {
        const int t = tb + lane;
        int a = -1;
        if (t < t1) a = CACHED ? (int)aeff[t] : effective_adapter(aid, seg, pos, start, t);
        unsigned long long rem = __ballot(a >= 0);
        while (rem) {
            const int lead = __ffsll((long long)rem) - 1;
            const int key = __shfl(a, lead);
            const unsigned long long m = __ballot(a == key);
            const int base = goff[key] + my_cnt[key];
            if (a == key) {
                const unsigned long long below = m & ((1ull << lane) - 1ull);
                perm[base + __popcll(below)] = t;
            }
            __builtin_amdgcn_wave_barrier();
            if (lane == lead) my_cnt[key] = my_cnt[key] + __popcll(m);
            __builtin_amdgcn_wave_barrier();
            rem &= ~m;
        }
    }
}

int launch_classify_group(const Fwd &f)
{
    if (f.T == 0) return 0;
    if (f.T <= PREP_CACHE_ROWS)
        hipLaunchKernelGGL(classify_group_kernel<true>, dim3(1), dim3(PREP_THREADS), 0, f.stream, f.aid, f.seg, f.pos,
                           f.start, f.T, f.L, f.active, f.aeff, f.perm, f.offsets, f.blocktab, f.n_blocks);
    else
        hipLaunchKernelGGL(classify_group_kernel<false>, dim3(1), dim3(PREP_THREADS), 0, f.stream, f.aid, f.seg,
                           f.pos, f.start, f.T, f.L, f.active, f.aeff, f.perm, f.offsets, f.blocktab, f.n_blocks);
    return (int)hipGetLastError();
}

}  // namespace alora
