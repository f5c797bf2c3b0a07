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
// thread) on the fp32 shrink result: the fixed-order sum of the shrink's partials (or, when the
// shrink ran as one range, hi + lo of the bf16 pair it stored).
//
// One thread per (row, 8 features): 1024 threads.  The kernel is a chain of dependent loads
// (table entry -> row ids -> data), so everything after the row ids is issued at once: all
// splits' partials, the S row and the B slice.
#include "alora_internal.h"

namespace alora {

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

constexpr int FIN_COLS = 256;  // features per workgroup: 32 threads x 8 features per row

template <int SPLITS>
__global__ __launch_bounds__(1024) void finish_bf16_kernel(const float *__restrict__ partial,
                                                           const void *__restrict__ S_any, int s_splits, PtrTable B,
                                                           RankTable ranks, const bf16_t *__restrict__ bias,
                                                           const int32_t *__restrict__ perm,
                                                           const int32_t *__restrict__ block_rows,
                                                           const int4 *__restrict__ blocktab,
                                                           const int64_t *__restrict__ slot, bf16_t *__restrict__ q,
                                                           bf16_t *__restrict__ kc, bf16_t *__restrict__ vc, int T, int Nq,
                                                           int Nkv, int L, int r, const float *__restrict__ rope_cos,
                                                           const float *__restrict__ rope_sin, const int32_t *__restrict__ pos,
                                                           int rope_positions)
{
    const float *S_part = (const float *)S_any;
    __shared__ float s_lds[32][ALORA_MAX_RANK + 1];
    __shared__ __attribute__((aligned(16))) bf16_t b_lds[ALORA_MAX_RANK][FIN_COLS];

    const int tid0 = threadIdx.x;
    // row ids straight from the per-entry list when there is one: the load does not wait for the entry
    int t_direct = -1;
    if (block_rows) t_direct = block_rows[32 * blockIdx.x + (tid0 >> 5)];
    const int4 entry = blocktab[blockIdx.x];
    const int a = entry.x, j0 = entry.y, cnt = entry.z;
    if (a < 0) return;  // unused table entry; uniform across the workgroup
    if (a > L || j0 < 0 || cnt < 0 || cnt > 32 || j0 + cnt > T) return;   // not a table of this batch
    const int N = Nq + 2 * Nkv;
    const int n0 = blockIdx.y * FIN_COLS;
    const int tid = threadIdx.x;
    const bool adapted = a < L;
    const int ra = adapted ? ranks.r[a] : 0;   // this group's rank; S and B_a rows beyond it do not exist
    const int i = tid >> 5, c = tid & 31, n = n0 + 8 * c;
    int t = block_rows ? (i < cnt ? t_direct : -1) : (i < cnt ? perm[j0 + i] : -1);
    if (t >= T) t = -1;
    const bool live = t >= 0 && n < N;

    // everything that depends on the row id, issued together
    f32x4 plo[SPLITS], phi[SPLITS];
    int64_t sl = -1;
    if (live) {
#pragma unroll
        for (int s = 0; s < SPLITS; ++s) {
            const float *p = partial + ((size_t)s * T + t) * N + n;
            plo[s] = *(const f32x4 *)p;
            phi[s] = *(const f32x4 *)(p + 4);
        }
        if (n >= Nq) sl = slot[t];
    }
    if (adapted) {
        // S of row i, rank columns c, c+32
        if (t >= 0) {
            for (int j = c; j < ra; j += 32) {
                float sj = 0.f;
                if (s_splits > 1) {
                    // all ranges' loads first, then the sum in range order (absent ranges add +0)
                    float sp[ALORA_SHRINK_MAX_SPLITS];
#pragma unroll
                    for (int ks = 0; ks < ALORA_SHRINK_MAX_SPLITS; ++ks)
                        sp[ks] = ks < s_splits ? S_part[((size_t)ks * T + t) * r + j] : 0.f;
#pragma unroll
                    for (int ks = 0; ks < ALORA_SHRINK_MAX_SPLITS; ++ks) sj += sp[ks];
                } else {
                    const bf16_t *row = (const bf16_t *)S_part + (size_t)t * 2 * r;
                    sj = bf16_bits_to_f32(row[j]) + bf16_bits_to_f32(row[r + j]);
                }
                s_lds[i][j] = sj;
            }
        }
        // B[a][:, n0 : n0+256]: rank rows x 32 chunks of 8 features
        const bf16_t *Ba = (const bf16_t *)B.p[a];
        for (int idx = tid; idx < ra * (FIN_COLS / 8); idx += 1024) {
            const int j = idx / (FIN_COLS / 8), cc = idx % (FIN_COLS / 8);
            u32x4 v = {0u, 0u, 0u, 0u};
            if (n0 + 8 * cc < N) v = *(const u32x4 *)(Ba + (size_t)j * N + n0 + 8 * cc);
            *(u32x4 *)&b_lds[j][8 * cc] = v;
        }
        __syncthreads();
    }
    if (!live) return;

    float y[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < SPLITS; ++s) {
        y[0] += plo[s].x; y[1] += plo[s].y; y[2] += plo[s].z; y[3] += plo[s].w;
        y[4] += phi[s].x; y[5] += phi[s].y; y[6] += phi[s].z; y[7] += phi[s].w;
    }
    if (bias) {   // part of the base output of every row
        const u32x4 bv = *(const u32x4 *)(bias + n);
        y[0] += __uint_as_float(bv.x << 16); y[1] += __uint_as_float(bv.x & 0xffff0000u);
        y[2] += __uint_as_float(bv.y << 16); y[3] += __uint_as_float(bv.y & 0xffff0000u);
        y[4] += __uint_as_float(bv.z << 16); y[5] += __uint_as_float(bv.z & 0xffff0000u);
        y[6] += __uint_as_float(bv.w << 16); y[7] += __uint_as_float(bv.w & 0xffff0000u);
    }
    if (adapted) {
        float d[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int j = 0; j < ra; ++j) {
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
    if (rope_cos) {
        // Rotary embedding on the unrounded row (heads of 128): the partner features i +- 64 are held by the
        // thread 8 lanes away, which is live whenever this one is (heads never straddle N).  Every live lane
        // takes part in the exchange; lanes of the v part keep their values.
        float other[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) other[e] = __shfl_xor(y[e], 8);
        if (n < Nq + Nkv) {
            const int f0 = (n & 127), i0 = f0 & 63;
            const int p = min(max(pos[t], 0), rope_positions - 1);
            const f32x4 c0 = *(const f32x4 *)(rope_cos + (size_t)p * 64 + i0), c1 = *(const f32x4 *)(rope_cos + (size_t)p * 64 + i0 + 4);
            const f32x4 s0 = *(const f32x4 *)(rope_sin + (size_t)p * 64 + i0), s1 = *(const f32x4 *)(rope_sin + (size_t)p * 64 + i0 + 4);
            const float cc[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
            const float ss[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
            const float sign = f0 < 64 ? -1.f : 1.f;     // first half: y cos - partner sin; second half: y cos + partner sin
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = y[e] * cc[e] + sign * (other[e] * ss[e]);
        }
    }
    u32x4 out;
    {
        const f32x2 p0 = {y[0], y[1]}, p1 = {y[2], y[3]}, p2 = {y[4], y[5]}, p3 = {y[6], y[7]};
        out.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(p0, bf16x2));
        out.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(p1, bf16x2));
        out.z = __builtin_bit_cast(uint32_t, __builtin_convertvector(p2, bf16x2));
        out.w = __builtin_bit_cast(uint32_t, __builtin_convertvector(p3, bf16x2));
    }
    if (n < Nq) {
        *(u32x4 *)(q + (size_t)t * Nq + n) = out;
    } else if (sl >= 0) {
        if (n < Nq + Nkv) *(u32x4 *)(kc + (size_t)sl * Nkv + (n - Nq)) = out;
        else *(u32x4 *)(vc + (size_t)sl * Nkv + (n - Nq - Nkv)) = out;
    }
}

template <int SPLITS>
static void launch_finish(const Fwd &f, const PtrTable &B, int s_splits, const int32_t *block_rows)
{
    const dim3 grid(f.n_blocks, (f.N + FIN_COLS - 1) / FIN_COLS);
    hipLaunchKernelGGL(finish_bf16_kernel<SPLITS>, grid, dim3(1024), 0, f.stream, (const float *)f.partial,
                       f.S, s_splits, B, f.ranks, (const bf16_t *)f.bias, f.perm, block_rows, f.blocktab, f.slot, (bf16_t *)f.q, (bf16_t *)f.kc,
                       (bf16_t *)f.vc, f.T, f.Nq, f.Nkv, f.L, f.r, f.rope_cos, f.rope_sin, f.pos, f.rope_positions);
}

int launch_finish_bf16(const Fwd &f, const PtrTable &B, int splits, int s_splits, const int32_t *block_rows)
{
    switch (splits) {
    case 2: launch_finish<2>(f, B, s_splits, block_rows); break;
    case 3: launch_finish<3>(f, B, s_splits, block_rows); break;
    case 4: launch_finish<4>(f, B, s_splits, block_rows); break;
    case 5: launch_finish<5>(f, B, s_splits, block_rows); break;
    case 6: launch_finish<6>(f, B, s_splits, block_rows); break;
    case 7: launch_finish<7>(f, B, s_splits, block_rows); break;
    case 8: launch_finish<8>(f, B, s_splits, block_rows); break;
    default: return (int)hipErrorInvalidValue;
    }
    return (int)hipGetLastError();
}

}  // namespace alora
