// Finishing kernel of the small-batch (decode-sized) bf16 path.
//
// With few token rows the projection is cut along the hidden dimension so that every compute unit
// streams a share of W; the splits leave fp32 partial products P[s][t][:].  This kernel walks the
// grouped row list (32 rows of one adapter, or of the base group, per workgroup and 256 features)
// and produces the final rows:
//     y[t,:] = sum_s P[s][t,:]  (fixed split order)   [+ S[t,:] . B[a]  for rows of adapter a]
// rounds once to bf16 and stores q_out / the paged K and V slots.  Rows of the base group never
// touch S or B, and their arithmetic does not depend on which rows are adapted: they come out
// bit-identical to a call without adapters.  The low-rank term is plain fp32 FMAs (rank x 8 per
// thread and row), S rebuilt from the (hi, lo) bf16 pairs the shrink stored per hidden slice.
#include "alora_internal.h"

namespace alora {

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

constexpr int FIN_COLS = 256;  // features per workgroup: 32 threads x 8 features per row

__global__ __launch_bounds__(256) void finish_bf16_kernel(const float *__restrict__ partial, int splits,
                                                          const bf16_t *__restrict__ S_hl, int kslices, PtrTable B,
                                                          const int32_t *__restrict__ perm,
                                                          const int4 *__restrict__ blocktab,
                                                          const int64_t *__restrict__ slot, bf16_t *__restrict__ q,
                                                          bf16_t *__restrict__ kc, bf16_t *__restrict__ vc, int T, int Nq,
                                                          int Nkv, int L, int r)
{
    __shared__ float s_lds[32][ALORA_MAX_RANK + 1];
    __shared__ __attribute__((aligned(16))) bf16_t b_lds[ALORA_MAX_RANK][FIN_COLS];
    __shared__ int rows_t[32];
    __shared__ int64_t rows_slot[32];

    const int4 entry = blocktab[blockIdx.x];
    const int a = entry.x, j0 = entry.y, cnt = entry.z;
    if (a < 0) return;  // unused table entry; uniform across the workgroup
    const int N = Nq + 2 * Nkv;
    const int n0 = blockIdx.y * FIN_COLS;
    const int tid = threadIdx.x;
    const bool adapted = a < L;

    if (tid < 32) {
        const int t = tid < cnt ? perm[j0 + tid] : -1;
        rows_t[tid] = t;
        rows_slot[tid] = t >= 0 ? slot[t] : -1;
    }
    __syncthreads();
    if (adapted) {
        // S rows of the block: sum of the slices' (hi + lo), slice order
        for (int idx = tid; idx < 32 * r; idx += 256) {
            const int i = idx / r, j = idx % r;
            const int t = rows_t[i];
            float s = 0.f;
            if (t >= 0) {
                const bf16_t *row = S_hl + (size_t)t * kslices * 2 * r;
                for (int sl = 0; sl < kslices; ++sl)
                    s += bf16_bits_to_f32(row[sl * 2 * r + j]) + bf16_bits_to_f32(row[sl * 2 * r + r + j]);
            }
            s_lds[i][j] = s;
        }
        // B[a][:, n0 : n0+256]
        const bf16_t *Ba = (const bf16_t *)B.p[a];
        for (int idx = tid; idx < r * (FIN_COLS / 8); idx += 256) {
            const int j = idx / (FIN_COLS / 8), c = idx % (FIN_COLS / 8);
            u32x4 v = {0u, 0u, 0u, 0u};
            if (n0 + 8 * c < N) v = *(const u32x4 *)(Ba + (size_t)j * N + n0 + 8 * c);
            *(u32x4 *)&b_lds[j][8 * c] = v;
        }
        __syncthreads();
    }

    const int c = tid & 31, n = n0 + 8 * c;
    if (n >= N) return;
    int region, col;
    if (n < Nq) { region = 0; col = n; }
    else if (n < Nq + Nkv) { region = 1; col = n - Nq; }
    else { region = 2; col = n - Nq - Nkv; }

    for (int i = tid >> 5; i < cnt; i += 8) {
        const int t = rows_t[i];
        float y[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < splits; ++s) {
            const float *p = partial + ((size_t)s * T + t) * N + n;
            const f32x4 lo = *(const f32x4 *)p, hi = *(const f32x4 *)(p + 4);
            y[0] += lo.x; y[1] += lo.y; y[2] += lo.z; y[3] += lo.w;
            y[4] += hi.x; y[5] += hi.y; y[6] += hi.z; y[7] += hi.w;
        }
        if (adapted) {
            float d[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            for (int j = 0; j < r; ++j) {
                const float sj = s_lds[i][j];
                const u32x4 bv = *(const u32x4 *)&b_lds[j][8 * c];
                d[0] = fmaf(sj, __uint_as_float(bv.x << 16), d[0]);
                d[1] = fmaf(sj, __uint_as_float(bv.x & 0xffff0000u), d[1]);
                d[2] = fmaf(sj, __uint_as_float(bv.y << 16), d[2]);
                d[3] = fmaf(sj, __uint_as_float(bv.y & 0xffff0000u), d[3]);
                d[4] = fmaf(sj, __uint_as_float(bv.z << 16), d[4]);
                d[5] = fmaf(sj, __uint_as_float(bv.z & 0xffff0000u), d[5]);
                d[6] = fmaf(sj, __uint_as_float(bv.w << 16), d[6]);
                d[7] = fmaf(sj, __uint_as_float(bv.w & 0xffff0000u), d[7]);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] += d[e];
        }
        u32x4 out;
        {
            const f32x2 p0 = {y[0], y[1]}, p1 = {y[2], y[3]}, p2 = {y[4], y[5]}, p3 = {y[6], y[7]};
            out.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(p0, bf16x2));
            out.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(p1, bf16x2));
            out.z = __builtin_bit_cast(uint32_t, __builtin_convertvector(p2, bf16x2));
            out.w = __builtin_bit_cast(uint32_t, __builtin_convertvector(p3, bf16x2));
        }
        if (region == 0) {
            *(u32x4 *)(q + (size_t)t * Nq + col) = out;
        } else {
            const int64_t sl = rows_slot[i];
            if (sl >= 0) *(u32x4 *)((region == 1 ? kc : vc) + (size_t)sl * Nkv + col) = out;
        }
    }
}

int launch_finish_bf16(const Fwd &f, const PtrTable &B, int splits)
{
    const dim3 grid(f.n_blocks, (f.N + FIN_COLS - 1) / FIN_COLS);
    hipLaunchKernelGGL(finish_bf16_kernel, grid, dim3(256), 0, f.stream, (const float *)f.partial, splits,
                       (const bf16_t *)f.S, f.L > 0 ? shrink_slices(f.H, f.r) : 0, B, f.perm, f.blocktab, f.slot,
                       (bf16_t *)f.q, (bf16_t *)f.kc, (bf16_t *)f.vc, f.T, f.Nq, f.Nkv, f.L, f.r);
    return (int)hipGetLastError();
}

}  // namespace alora
