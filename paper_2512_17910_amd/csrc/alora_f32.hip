// fp32 path (plain vector ALU, fp32 accumulate): the small-layer / reference-precision variant
// of the masked multi-adapter QKV projection.  Two kernels after the grouping step:
//   shrink_f32 : S[t,:] = x[t,:] . A[a]   for adapted rows only (walks the grouped row list)
//   gemm_f32   : y = x . W (64x64 tiles through LDS), then for adapted rows y += S[t,:] . B[a],
//                then the q_out store and the paged K/V store.
// Pre-activation and base-model rows never read S, A or B (Sec. 2.3: they are the base model's).
#include "alora_internal.h"

namespace alora {

// One workgroup per adapted row; wavefront kq sums a quarter of the hidden dimension for rank
// column j = lane, the four partial sums are added in fixed order.
__global__ __launch_bounds__(256) void shrink_f32_kernel(const float *__restrict__ x, PtrTable A, RankTable ranks,
                                                         const int32_t *__restrict__ aid,
                                                         const int32_t *__restrict__ perm,
                                                         const int32_t *__restrict__ offsets, int T, int L, int H, int r,
                                                         float *__restrict__ S)
{
    __shared__ float red[4][64];
    const int n_act = offsets[L];
    if ((int)blockIdx.x >= n_act) return;
    const int t = perm[blockIdx.x];
    if (t < 0 || t >= T) return;   // (perm may be what an earlier call left in the workspace: range-checked)
    const int a = aid[t];
    if (a < 0 || a >= L) return;
    const float *xr = x + (size_t)t * H;
    const float *Aa = (const float *)A.p[a];
    const int ra = ranks.r[a];   // this adapter's rank: A_a is [H, ra]; S keeps the common row pitch r
    const int j = threadIdx.x & 63, kq = threadIdx.x >> 6;
    const int kchunk = (H + 3) / 4;
    const int k0 = kq * kchunk, k1 = min(H, k0 + kchunk);
    float acc = 0.f;
    if (j < ra)
        for (int k = k0; k < k1; ++k) acc = fmaf(xr[k], Aa[(size_t)k * ra + j], acc);
    red[kq][j] = acc;
    __syncthreads();
    if (kq == 0 && j < r) S[(size_t)t * r + j] = ((red[0][j] + red[1][j]) + red[2][j]) + red[3][j];
}

constexpr int FBM = 64, FBN = 64, FBK = 16;

__global__ __launch_bounds__(256) void gemm_f32_kernel(
    const float *__restrict__ x, const float *__restrict__ W, const float *__restrict__ bias, PtrTable B,
    RankTable ranks, const float *__restrict__ S,
    const int32_t *__restrict__ aid, const int32_t *__restrict__ seg, const int32_t *__restrict__ pos,
    const int32_t *__restrict__ start, const int64_t *__restrict__ slot, float *__restrict__ q,
    float *__restrict__ kc, float *__restrict__ vc, int T, int H, int Nq, int Nkv, int r)
{
    __shared__ float Xs[FBK][FBM + 4];
    __shared__ float Ws[FBK][FBN + 4];
    const int N = Nq + 2 * Nkv;
    const int m0 = blockIdx.y * FBM, n0 = blockIdx.x * FBN;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4] = {};

    const int xrow = threadIdx.x >> 2, xk = (threadIdx.x & 3) * 4;   // x tile: 64 rows x 16 k
    const int wk = threadIdx.x >> 4, wn = (threadIdx.x & 15) * 4;    // W tile: 16 k x 64 n
    for (int k0 = 0; k0 < H; k0 += FBK) {
        float4 xv = make_float4(0.f, 0.f, 0.f, 0.f), wv = make_float4(0.f, 0.f, 0.f, 0.f);
        if (m0 + xrow < T && k0 + xk < H) xv = *(const float4 *)(x + (size_t)(m0 + xrow) * H + k0 + xk);
        if (k0 + wk < H && n0 + wn < N) wv = *(const float4 *)(W + (size_t)(k0 + wk) * N + n0 + wn);
        Xs[xk + 0][xrow] = xv.x; Xs[xk + 1][xrow] = xv.y; Xs[xk + 2][xrow] = xv.z; Xs[xk + 3][xrow] = xv.w;
        *(float4 *)&Ws[wk][wn] = wv;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < FBK; ++k) {
            const float4 a4 = *(const float4 *)&Xs[k][ty * 4];
            const float4 b4 = *(const float4 *)&Ws[k][tx * 4];
            const float av[4] = {a4.x, a4.y, a4.z, a4.w}, bv[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }

    const int n = n0 + tx * 4;
    if (n >= N) return;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = m0 + ty * 4 + i;
        if (t >= T) continue;
        const int a = effective_adapter(aid, seg, pos, start, t);
        float4 y = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
        if (bias) {   // part of the base output of every row
            const float4 b4 = *(const float4 *)(bias + n);
            y.x += b4.x; y.y += b4.y; y.z += b4.z; y.w += b4.w;
        }
        if (a >= 0) {
            const float *Ba = (const float *)B.p[a];
            const float *Sr = S + (size_t)t * r;
            float4 d = make_float4(0.f, 0.f, 0.f, 0.f);
            const int ra = ranks.r[a];
            for (int j = 0; j < ra; ++j) {
                const float s = Sr[j];
                const float4 b4 = *(const float4 *)(Ba + (size_t)j * N + n);
                d.x = fmaf(s, b4.x, d.x); d.y = fmaf(s, b4.y, d.y);
                d.z = fmaf(s, b4.z, d.z); d.w = fmaf(s, b4.w, d.w);
            }
            y.x += d.x; y.y += d.y; y.z += d.z; y.w += d.w;
        }
        if (n < Nq) {
            *(float4 *)(q + (size_t)t * Nq + n) = y;
        } else {
            const int64_t s = slot[t];
            if (s < 0) continue;
            if (n < Nq + Nkv) *(float4 *)(kc + (size_t)s * Nkv + (n - Nq)) = y;
            else *(float4 *)(vc + (size_t)s * Nkv + (n - Nq - Nkv)) = y;
        }
    }
}

// Rotary embedding on the fp32 path: the q_out rows and the K slots this call wrote, turned in place.  The
// stored values are the unrounded fp32 outputs, so this equals a rotation fused into the store.  One
// workgroup per token row; a thread takes the pairs (i, i + D/2) of the q heads and then of the k heads.
__global__ __launch_bounds__(256) void rope_f32_kernel(float *__restrict__ q, float *__restrict__ kc,
                                                       const int64_t *__restrict__ slot, const int32_t *__restrict__ pos,
                                                       const float *__restrict__ cs, const float *__restrict__ sn,
                                                       int n_pos, int Nq, int Nkv, int D)
{
    const int t = blockIdx.x, half = D / 2;
    const int p = min(max(pos[t], 0), n_pos - 1);
    const int64_t sl = slot[t];
    const int pairs = (Nq + Nkv) / 2;
    for (int idx = threadIdx.x; idx < pairs; idx += 256) {
        const int h = idx / half, i = idx % half;
        float *row;
        if (h * D < Nq) row = q + (size_t)t * Nq + h * D;
        else if (sl >= 0) row = kc + (size_t)sl * Nkv + (h * D - Nq);
        else continue;
        const float c = cs[(size_t)p * half + i], s = sn[(size_t)p * half + i];
        const float a = row[i], b = row[i + half];
        row[i] = a * c - b * s;
        row[i + half] = b * c + a * s;
    }
}

int launch_rope_f32(const Fwd &f)
{
    if (f.T == 0) return 0;
    hipLaunchKernelGGL(rope_f32_kernel, dim3(f.T), dim3(256), 0, f.stream, (float *)f.q, (float *)f.kc, f.slot, f.pos,
                       f.rope_cos, f.rope_sin, f.rope_positions, f.Nq, f.Nkv, f.D);
    return (int)hipGetLastError();
}

int launch_shrink_f32(const Fwd &f, const PtrTable &A)
{
    if (f.T == 0 || f.L == 0) return 0;
    hipLaunchKernelGGL(shrink_f32_kernel, dim3(f.T), dim3(256), 0, f.stream, (const float *)f.x, A, f.ranks, f.aid,
                       f.perm, f.offsets, f.T, f.L, f.H, f.r, (float *)f.S);
    return (int)hipGetLastError();
}

int launch_gemm_f32(const Fwd &f, const PtrTable &B)
{
    if (f.T == 0) return 0;
    dim3 grid((f.N + FBN - 1) / FBN, (f.T + FBM - 1) / FBM);
    hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, f.stream, (const float *)f.x, (const float *)f.W,
                       (const float *)f.bias, B, f.ranks, (const float *)f.S, f.aid, f.seg, f.pos, f.start, f.slot, (float *)f.q, (float *)f.kc,
                       (float *)f.vc, f.T, f.H, f.Nq, f.Nkv, f.r);
    return (int)hipGetLastError();
}

}  // namespace alora
