// Row classification (App. B mask, negated and combined with "has an adapter") and the stable
// grouping of token rows: adapted rows by adapter id (what the multi-adapter LoRA shrink and the
// small-batch finishing kernel walk), followed by one last group of all rows that keep the base
// output.  perm therefore is a permutation of all T rows; offsets[a] .. offsets[a+1] delimits
// adapter a, offsets[L] .. offsets[L+1] (= T) the base group.
//
// One workgroup of 16 wavefronts.  A first sweep classifies every row with independent,
// coalesced loads and parks the row's group key in LDS; the grouping itself then runs out of LDS.
// Each wavefront owns a contiguous range of token rows, so "wavefront index, then row index" is
// the original row order and the grouping is stable without any sort: count per (wavefront,
// group), prefix-sum the counts group-major / wavefront-minor, then place rows with
// wavefront-local cursors.  Ranks inside a 64-row step come from ballots, so there are no
// data-dependent atomics and the result is deterministic.  Batches of 6144 rows or more take the
// two-launch, many-workgroup form further down.
#include <algorithm>
#include "alora_internal.h"

namespace alora {

constexpr int PREP_WAVES = 16;
constexpr int PREP_THREADS = PREP_WAVES * 64;
constexpr int PREP_CACHE_ROWS = 96 * 1024;     // one byte per row
constexpr int NKEYS = ALORA_MAX_ADAPTERS + 1;  // adapters + the base group

// Work list of the prefill-sized bf16 shrink.  Adapted rows fill the first bfirst[L] entries of the
// block table; each of those blocks is cut into `eff` ranges of the hidden dimension so that about
// ALORA_SHRINK_TARGET_WGS workgroups come out (never more than rmax ranges, none empty).  Item i is
// range i % eff of block i / eff; the rest of the list is marked unused.  The per-block counters of
// finished ranges start at zero.  Entries first, first + stride, ... are written by the caller.
__device__ __forceinline__ void emit_shrink_items(const ShrinkWork &sw, int L, const int *goff, const int *bfirst,
                                                  const int *tot, int n_blocks, int first, int stride)
{
    if (!sw.items) return;
    const int nab = bfirst[L];
    int eff = 1, kper64 = sw.k64;
    if (nab > 0) {
        eff = max(1, min(sw.rmax, ALORA_SHRINK_TARGET_WGS / nab));
        kper64 = (sw.k64 + eff - 1) / eff;
        eff = (sw.k64 + kper64 - 1) / kper64;
    }
    for (int i = first; i < sw.n_items; i += stride) {
        int4 v = make_int4(-1, 0, 0, 0);
        if (i < nab * eff) {
            const int e = i / eff, rg = i - e * eff;
            int lo = 0, hi = L;  // smallest group whose blocks end after e
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (bfirst[mid + 1] > e) hi = mid; else lo = mid + 1;
            }
            const int b = e - bfirst[lo];
            v = make_int4(lo, goff[lo] + 32 * b, min(32, tot[lo] - 32 * b) | (kper64 << 8), rg | (eff << 4) | (e << 8));
        }
        sw.items[i] = v;
    }
    for (int i = first; i < n_blocks; i += stride) sw.counters[i] = 0;
}

template <bool CACHED>
__global__ __launch_bounds__(PREP_THREADS) void classify_group_kernel(
    const int32_t *__restrict__ aid, const int32_t *__restrict__ seg, const int32_t *__restrict__ pos,
    const int32_t *__restrict__ start, int T, int L, uint8_t *__restrict__ active,
    int8_t *__restrict__ aeff_out, int32_t *__restrict__ perm, int32_t *__restrict__ offsets,
    int4 *__restrict__ blocktab, int n_blocks, ShrinkWork sw)
{
    __shared__ int cnt[PREP_WAVES][NKEYS];
    __shared__ int goff[3 * 64 + 1], bfirst[3 * 64 + 1], tot[3 * 64];
    __shared__ int8_t aeff[CACHED ? PREP_CACHE_ROWS : 64];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int per_wave = ((T + PREP_WAVES * 64 - 1) / (PREP_WAVES * 64)) * 64;
    const int t0 = min(T, w * per_wave);
    const int t1 = min(T, t0 + per_wave);
    int *my_cnt = cnt[w];  // plain LDS accesses: a volatile one would wait for every outstanding global store

    for (int i = threadIdx.x; i < PREP_WAVES * NKEYS; i += PREP_THREADS) (&cnt[0][0])[i] = 0;
    if (threadIdx.x < 3 * 64) tot[threadIdx.x] = 0;
    if (CACHED) {
        // classification sweep: coalesced, sixteen independent rows per thread and trip, so that a
        // batch of 16K rows pays the three dependent load latencies (adapter id -> segment and
        // position -> activation start) once
        constexpr int U = 16;
        for (int tb = threadIdx.x; tb < T; tb += U * PREP_THREADS) {
            int a[U], s[U], p[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int t = tb + u * PREP_THREADS;
                a[u] = t < T ? aid[t] : -1;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int t = tb + u * PREP_THREADS;
                s[u] = a[u] >= 0 ? seg[t] : 0;
                p[u] = a[u] >= 0 ? pos[t] : 0;
            }
            int st[U];
#pragma unroll
            for (int u = 0; u < U; ++u) st[u] = a[u] >= 0 ? start[s[u]] : 0;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int t = tb + u * PREP_THREADS;
                if (t < T) {
                    const int e = (a[u] >= 0 && p[u] >= st[u]) ? a[u] : -1;
                    aeff[t] = (int8_t)e;
                    aeff_out[t] = (int8_t)e;
                    active[t] = (uint8_t)(e >= 0);
                }
            }
        }
    }
    __syncthreads();

    // group key of row t: its adapter if adapted, L for the base group, -1 outside the batch
    auto row_key = [&](int t, bool publish) -> int {
        if (t >= t1) return -1;
        int a;
        if (CACHED) {
            a = aeff[t];
        } else {
            a = effective_adapter(aid, seg, pos, start, t);
            if (publish) {
                aeff_out[t] = (int8_t)a;
                active[t] = (uint8_t)(a >= 0);
            }
        }
        return a >= 0 ? a : L;
    };

    const int key_bits = 32 - __clz(L | 1);  // keys are 0 .. L
    // lanes of this 64-row step that hold the same key as this lane (one ballot per key bit: the
    // cost does not grow with the number of distinct groups in the step, as in a decode batch)
    auto same_key_lanes = [&](int key_l) -> unsigned long long {
        unsigned long long same = __ballot(key_l >= 0);
        for (int bit = 0; bit < key_bits; ++bit) {
            const bool mine = (key_l >> bit) & 1;
            const unsigned long long b = __ballot(mine);
            same &= mine ? b : ~b;
        }
        return key_l >= 0 ? same : 0ull;
    };
    const unsigned long long lanes_below = (1ull << lane) - 1ull;

    // pass 1: per-(wavefront, group) counts
    for (int tb = t0; tb < t1; tb += 64) {
        const int key_l = row_key(tb + lane, true);
        const unsigned long long same = same_key_lanes(key_l);
        if (same && !(same & lanes_below)) atomicAdd(&my_cnt[key_l], __popcll(same));
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();

    // exclusive prefix over wavefronts inside each group, group totals
    if ((int)threadIdx.x <= L) {
        int run = 0;
        for (int ww = 0; ww < PREP_WAVES; ++ww) {
            const int c = cnt[ww][threadIdx.x];
            cnt[ww][threadIdx.x] = run;
            run += c;
        }
        tot[threadIdx.x] = run;
    }
    __syncthreads();
    // one wavefront scans the group totals (three groups per lane): row offsets of the groups and
    // first 32-row block of every group in the block table
    if (w == 0) {
        int c[3], b[3], rows = 0, blks = 0;
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            c[u] = tot[3 * lane + u];
            b[u] = (c[u] + 31) >> 5;
            rows += c[u];
            blks += b[u];
        }
        const int my_rows = rows, my_blks = blks;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int r_up = __shfl_up(rows, d), b_up = __shfl_up(blks, d);
            if (lane >= d) { rows += r_up; blks += b_up; }
        }
        int ro = rows - my_rows, bo = blks - my_blks;
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            goff[3 * lane + u] = ro;
            bfirst[3 * lane + u] = bo;
            ro += c[u];
            bo += b[u];
        }
        if (lane == 63) { goff[3 * 64] = rows; bfirst[3 * 64] = blks; }
    }
    __syncthreads();
    if ((int)threadIdx.x <= L + 1) offsets[threadIdx.x] = goff[threadIdx.x];
    // block table: entry = (group, first index into perm, rows in block, 0); unused entries -1
    for (int e = threadIdx.x; e < n_blocks; e += PREP_THREADS) {
        int4 v = make_int4(-1, 0, 0, 0);
        if (e < bfirst[3 * 64]) {
            int lo = 0, hi = L;  // smallest group whose blocks end after e
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (bfirst[mid + 1] > e) hi = mid; else lo = mid + 1;
            }
            const int b = e - bfirst[lo];
            v = make_int4(lo, goff[lo] + 32 * b, min(32, tot[lo] - 32 * b), 0);
        }
        blocktab[e] = v;
    }
    emit_shrink_items(sw, L, goff, bfirst, tot, n_blocks, threadIdx.x, PREP_THREADS);

    // pass 2: placement
    for (int tb = t0; tb < t1; tb += 64) {
        const int t = tb + lane;
        const int key_l = row_key(t, false);
        const unsigned long long same = same_key_lanes(key_l);
        // every lane reads its group's cursor before the group's first lane advances it
        if (same) perm[goff[key_l] + my_cnt[key_l] + __popcll(same & lanes_below)] = t;
        __builtin_amdgcn_wave_barrier();
        if (same && !(same & lanes_below)) atomicAdd(&my_cnt[key_l], __popcll(same));
        __builtin_amdgcn_wave_barrier();
    }
}

// ---- large batches: the same result from two launches of many workgroups -----------------------
// Above a few thousand rows the single workgroup is the longest pole in front of the shrink, so
// the rows are cut into slices of PREP_SLICE rows, one workgroup each.  Launch 1 classifies its
// slice (App. B mask) and leaves the slice's row count per group in hist[slice][group].  Launch 2
// turns the histogram into positions: group offsets (totals over all slices), the base of this
// slice inside every group (totals of the slices before it), then the same wavefront-local
// placement as above.  "Slice, then wavefront, then row" is the original row order: stable, no
// sort, no data-dependent atomics, bit-identical to the single-workgroup kernel.
constexpr int PREP_SLICE = 2048;                      // rows per workgroup: 128 per wavefront
constexpr int PREP_SLICE_PER_WAVE = PREP_SLICE / PREP_WAVES;

__device__ __forceinline__ unsigned long long same_key_lanes_of(int key_l, int key_bits)
{
    unsigned long long same = __ballot(key_l >= 0);
    for (int bit = 0; bit < key_bits; ++bit) {
        const bool mine = (key_l >> bit) & 1;
        const unsigned long long b = __ballot(mine);
        same &= mine ? b : ~b;
    }
    return key_l >= 0 ? same : 0ull;
}

// per-(wavefront, group) row counts of this slice out of the slice's adapter bytes in LDS
__device__ __forceinline__ void slice_counts(const int8_t *aeff_s, int rows, int L, int key_bits, int *my_cnt, int w,
                                             int lane)
{
    const unsigned long long lanes_below = (1ull << lane) - 1ull;
    for (int tb = w * PREP_SLICE_PER_WAVE; tb < min(rows, (w + 1) * PREP_SLICE_PER_WAVE); tb += 64) {
        const int i = tb + lane;
        const int key_l = i < min(rows, (w + 1) * PREP_SLICE_PER_WAVE) ? (aeff_s[i] >= 0 ? aeff_s[i] : L) : -1;
        const unsigned long long same = same_key_lanes_of(key_l, key_bits);
        if (same && !(same & lanes_below)) atomicAdd(&my_cnt[key_l], __popcll(same));
        __builtin_amdgcn_wave_barrier();
    }
}

__global__ __launch_bounds__(PREP_THREADS) void classify_slices_kernel(
    const int32_t *__restrict__ aid, const int32_t *__restrict__ seg, const int32_t *__restrict__ pos,
    const int32_t *__restrict__ start, int T, int L, uint8_t *__restrict__ active, int8_t *__restrict__ aeff_out,
    int32_t *__restrict__ hist)
{
    __shared__ int cnt[PREP_WAVES][NKEYS];
    __shared__ int8_t aeff_s[PREP_SLICE];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int r0 = (int)blockIdx.x * PREP_SLICE, rows = min(T - r0, PREP_SLICE);
    for (int i = threadIdx.x; i < PREP_WAVES * NKEYS; i += PREP_THREADS) (&cnt[0][0])[i] = 0;
    // classification: two independent rows per thread, the dependent loads paid once
    constexpr int U = PREP_SLICE / PREP_THREADS;
    int a[U], s[U], p[U], st[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = threadIdx.x + u * PREP_THREADS;
        a[u] = i < rows ? aid[r0 + i] : -1;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = threadIdx.x + u * PREP_THREADS;
        s[u] = a[u] >= 0 ? seg[r0 + i] : 0;
        p[u] = a[u] >= 0 ? pos[r0 + i] : 0;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) st[u] = a[u] >= 0 ? start[s[u]] : 0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = threadIdx.x + u * PREP_THREADS;
        if (i < rows) {
            const int e = (a[u] >= 0 && p[u] >= st[u]) ? a[u] : -1;
            aeff_s[i] = (int8_t)e;
            aeff_out[r0 + i] = (int8_t)e;
            active[r0 + i] = (uint8_t)(e >= 0);
        }
    }
    __syncthreads();
    slice_counts(aeff_s, rows, L, 32 - __clz(L | 1), cnt[w], w, lane);
    __syncthreads();
    if ((int)threadIdx.x <= L) {
        int run = 0;
        for (int ww = 0; ww < PREP_WAVES; ++ww) run += cnt[ww][threadIdx.x];
        hist[(size_t)blockIdx.x * NKEYS + threadIdx.x] = run;
    }
}

__global__ __launch_bounds__(PREP_THREADS) void place_slices_kernel(
    const int8_t *__restrict__ aeff_in, const int32_t *__restrict__ hist, int T, int L, int32_t *__restrict__ perm,
    int32_t *__restrict__ offsets, int4 *__restrict__ blocktab, int n_blocks, ShrinkWork sw)
{
    __shared__ int cnt[PREP_WAVES][NKEYS];
    __shared__ int goff[3 * 64 + 1], bfirst[3 * 64 + 1], tot[3 * 64], slice_base[NKEYS];
    __shared__ int8_t aeff_s[PREP_SLICE];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int r0 = (int)blockIdx.x * PREP_SLICE, rows = min(T - r0, PREP_SLICE);
    const int key_bits = 32 - __clz(L | 1);
    for (int i = threadIdx.x; i < PREP_WAVES * NKEYS; i += PREP_THREADS) (&cnt[0][0])[i] = 0;
    if (threadIdx.x < 3 * 64) tot[threadIdx.x] = 0;
    for (int i = threadIdx.x; i < rows; i += PREP_THREADS) aeff_s[i] = aeff_in[r0 + i];
    __syncthreads();
    slice_counts(aeff_s, rows, L, key_bits, cnt[w], w, lane);
    // group totals over all slices, and the rows of earlier slices in every group
    if ((int)threadIdx.x <= L) {
        int before = 0, all = 0;
        for (int sl = 0; sl < (int)gridDim.x; ++sl) {
            const int c = hist[(size_t)sl * NKEYS + threadIdx.x];
            if (sl < (int)blockIdx.x) before += c;
            all += c;
        }
        slice_base[threadIdx.x] = before;
        tot[threadIdx.x] = all;
    }
    __syncthreads();
    // exclusive prefix over wavefronts inside each group
    if ((int)threadIdx.x <= L) {
        int run = 0;
        for (int ww = 0; ww < PREP_WAVES; ++ww) {
            const int c = cnt[ww][threadIdx.x];
            cnt[ww][threadIdx.x] = run;
            run += c;
        }
    }
    // one wavefront scans the group totals (three groups per lane): row offsets of the groups and
    // first 32-row block of every group in the block table
    if (w == 0) {
        int c[3], b[3], nrows = 0, blks = 0;
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            c[u] = tot[3 * lane + u];
            b[u] = (c[u] + 31) >> 5;
            nrows += c[u];
            blks += b[u];
        }
        const int my_rows = nrows, my_blks = blks;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int r_up = __shfl_up(nrows, d), b_up = __shfl_up(blks, d);
            if (lane >= d) { nrows += r_up; blks += b_up; }
        }
        int ro = nrows - my_rows, bo = blks - my_blks;
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            goff[3 * lane + u] = ro;
            bfirst[3 * lane + u] = bo;
            ro += c[u];
            bo += b[u];
        }
        if (lane == 63) { goff[3 * 64] = nrows; bfirst[3 * 64] = blks; }
    }
    __syncthreads();
    if (blockIdx.x == 0) {
        if ((int)threadIdx.x <= L + 1) offsets[threadIdx.x] = goff[threadIdx.x];
    }
    // block table, its entries dealt round-robin to the workgroups
    for (int e = (int)blockIdx.x * PREP_THREADS + threadIdx.x; e < n_blocks; e += (int)gridDim.x * PREP_THREADS) {
        int4 v = make_int4(-1, 0, 0, 0);
        if (e < bfirst[3 * 64]) {
            int lo = 0, hi = L;  // smallest group whose blocks end after e
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (bfirst[mid + 1] > e) hi = mid; else lo = mid + 1;
            }
            const int b = e - bfirst[lo];
            v = make_int4(lo, goff[lo] + 32 * b, min(32, tot[lo] - 32 * b), 0);
        }
        blocktab[e] = v;
    }
    emit_shrink_items(sw, L, goff, bfirst, tot, n_blocks, (int)blockIdx.x * PREP_THREADS + threadIdx.x,
                      (int)gridDim.x * PREP_THREADS);
    // placement
    const unsigned long long lanes_below = (1ull << lane) - 1ull;
    int *my_cnt = cnt[w];
    const int w_end = min(rows, (w + 1) * PREP_SLICE_PER_WAVE);
    for (int tb = w * PREP_SLICE_PER_WAVE; tb < w_end; tb += 64) {
        const int i = tb + lane;
        const int key_l = i < w_end ? (aeff_s[i] >= 0 ? aeff_s[i] : L) : -1;
        const unsigned long long same = same_key_lanes_of(key_l, key_bits);
        // every lane reads its group's cursor before the group's first lane advances it
        if (same) perm[goff[key_l] + slice_base[key_l] + my_cnt[key_l] + __popcll(same & lanes_below)] = r0 + i;
        __builtin_amdgcn_wave_barrier();
        if (same && !(same & lanes_below)) atomicAdd(&my_cnt[key_l], __popcll(same));
        __builtin_amdgcn_wave_barrier();
    }
}

int group_blocks(int T, int L) { return (T + 31) / 32 + L + 1; }

// rows from which the two-launch grouping is used, and the bytes of its histogram
constexpr int PREP_TWO_LAUNCH_FROM = 6144;
size_t group_hist_bytes(int T) { return T >= PREP_TWO_LAUNCH_FROM ? (size_t)((T + PREP_SLICE - 1) / PREP_SLICE) * NKEYS * 4 : 0; }

int shrink_items(int T, int L) { return std::max(group_blocks(T, L), ALORA_SHRINK_TARGET_WGS); }

int launch_classify_group(const Fwd &f)
{
    if (f.T == 0) return 0;
    ShrinkWork sw = {nullptr, nullptr, 0, 0, 0};
    if (f.items) sw = ShrinkWork{f.items, f.counters, f.n_items, f.H / 64, plan_shrink(f.T, f.H, f.N, f.L, f.r).splits};
    if (f.T >= PREP_TWO_LAUNCH_FROM) {
        const int slices = (f.T + PREP_SLICE - 1) / PREP_SLICE;
        hipLaunchKernelGGL(classify_slices_kernel, dim3(slices), dim3(PREP_THREADS), 0, f.stream, f.aid, f.seg, f.pos,
                           f.start, f.T, f.L, f.active, f.aeff, f.hist);
        hipLaunchKernelGGL(place_slices_kernel, dim3(slices), dim3(PREP_THREADS), 0, f.stream, (const int8_t *)f.aeff,
                           (const int32_t *)f.hist, f.T, f.L, f.perm, f.offsets, f.blocktab, f.n_blocks, sw);
        return (int)hipGetLastError();
    }
    static_assert(PREP_TWO_LAUNCH_FROM <= PREP_CACHE_ROWS, "smaller batches fit the single workgroup's LDS row cache");
    hipLaunchKernelGGL(classify_group_kernel<true>, dim3(1), dim3(PREP_THREADS), 0, f.stream, f.aid, f.seg, f.pos,
                       f.start, f.T, f.L, f.active, f.aeff, f.perm, f.offsets, f.blocktab, f.n_blocks, sw);
    return (int)hipGetLastError();
}

}  // namespace alora
