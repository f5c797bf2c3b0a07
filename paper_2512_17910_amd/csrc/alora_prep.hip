// Row classification (App. B mask, negated and combined with "has an adapter") and the stable
// grouping of adapted rows by adapter id that the multi-adapter LoRA shrink walks.
//
// One workgroup of 16 wavefronts.  Each wavefront owns a contiguous range of token rows, so
// "wavefront index, then row index" is the original row order and the grouping is stable
// without any sort: count per (wavefront, adapter), prefix-sum the counts adapter-major /
// wavefront-minor, then place rows with wavefront-local cursors.  Ranks inside a 64-row step
// come from ballots, so there are no data-dependent atomics and the result is deterministic.
#include "alora_internal.h"

namespace alora {

constexpr int PREP_WAVES = 16;

__global__ __launch_bounds__(PREP_WAVES * 64) void classify_group_kernel(
    const int32_t *__restrict__ aid, const int32_t *__restrict__ seg, const int32_t *__restrict__ pos,
    const int32_t *__restrict__ start, int T, int L, uint8_t *__restrict__ active,
    int32_t *__restrict__ perm, int32_t *__restrict__ offsets)
{
    __shared__ int cnt[PREP_WAVES][ALORA_MAX_ADAPTERS];
    __shared__ int goff[ALORA_MAX_ADAPTERS + 1];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int per_wave = ((T + PREP_WAVES * 64 - 1) / (PREP_WAVES * 64)) * 64;
    const int t0 = min(T, w * per_wave);
    const int t1 = min(T, t0 + per_wave);
    volatile int *my_cnt = cnt[w];

    for (int i = threadIdx.x; i < PREP_WAVES * ALORA_MAX_ADAPTERS; i += PREP_WAVES * 64) (&cnt[0][0])[i] = 0;
    __syncthreads();

    // pass 1: flags + per-(wavefront, adapter) counts
    for (int tb = t0; tb < t1; tb += 64) {
        const int t = tb + lane;
        int a = -1;
        if (t < t1) {
            a = effective_adapter(aid, seg, pos, start, t);
            active[t] = (uint8_t)(a >= 0);
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
    if ((int)threadIdx.x < L) {
        int run = 0;
        for (int ww = 0; ww < PREP_WAVES; ++ww) {
            const int c = cnt[ww][threadIdx.x];
            cnt[ww][threadIdx.x] = run;
            run += c;
        }
        goff[threadIdx.x + 1] = run;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        goff[0] = 0;
        for (int a = 0; a < L; ++a) goff[a + 1] += goff[a];
    }
    __syncthreads();
    if ((int)threadIdx.x <= L) offsets[threadIdx.x] = goff[threadIdx.x];

    // pass 2: placement
    for (int tb = t0; tb < t1; tb += 64) {
        const int t = tb + lane;
        int a = -1;
        if (t < t1) a = effective_adapter(aid, seg, pos, start, t);
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
    hipLaunchKernelGGL(classify_group_kernel, dim3(1), dim3(PREP_WAVES * 64), 0, f.stream,
                       f.aid, f.seg, f.pos, f.start, f.T, f.L, f.active, f.perm, f.offsets);
    return (int)hipGetLastError();
}

}  // namespace alora
