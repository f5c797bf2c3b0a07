// LoRA shrink for bf16 batches: S[t,:] = x[t,:] . A[a] for adapted rows only, on bf16 MFMA with
// fp32 accumulation.  Rows are taken from the grouped list (adapter-major, stable), 32 rows of
// one adapter per workgroup; the four wavefronts split the hidden dimension and their partial
// sums are added in fixed order, so the result does not depend on scheduling.
//
// The fp32 result is handed to the projection kernel as two bf16 numbers per element,
// S = hi + lo with hi = bf16(S), lo = bf16(S - hi): the expand then runs on the same bf16 MFMA
// pipe as the base GEMM (two K-slices against the same B) while keeping ~16 mantissa bits of S.
#include "alora_internal.h"

namespace alora {

template <int NT>  // 32-wide rank tiles: 1 for rank <= 32, 2 for rank <= 64
__global__ __launch_bounds__(256) void shrink_bf16_kernel(const bf16_t *__restrict__ x, PtrTable A,
                                                          const int32_t *__restrict__ perm,
                                                          const int32_t *__restrict__ offsets, int L, int H,
                                                          int r, bf16_t *__restrict__ S_hl)
{
    __shared__ float red[4][NT][32][33];
    __shared__ int rows_t[32];
    // which (adapter, 32-row block) is this workgroup?
    int a = 0, cum = 0, j0 = 0, cnt = 0;
    for (; a < L; ++a) {
        const int o0 = offsets[a], o1 = offsets[a + 1];
        const int nb = (o1 - o0 + 31) >> 5;
        if ((int)blockIdx.x < cum + nb) {
            j0 = o0 + ((int)blockIdx.x - cum) * 32;
            cnt = min(32, o1 - j0);
            break;
        }
        cum += nb;
    }
    if (a >= L) return;  // uniform across the workgroup

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int i = lane & 31, h = lane >> 5;
    const bool rv = i < cnt;
    const int t = rv ? perm[j0 + i] : 0;
    if (w == 0 && h == 0) rows_t[i] = rv ? t : -1;
    const bf16_t *xr = x + (size_t)t * H;
    const bf16_t *Aa = (const bf16_t *)A.p[a];

    f32x16 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[nt][e] = 0.f;

    for (int k0 = w * 16; k0 < H; k0 += 64) {
        const int kk = k0 + 8 * h;
        u32x4 xv = {0u, 0u, 0u, 0u};
        if (rv) xv = *(const u32x4 *)(xr + kk);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int j = nt * 32 + i;
            u32x4 av = {0u, 0u, 0u, 0u};
            if (j < r) {
                uint32_t e[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) e[q] = Aa[(size_t)(kk + q) * r + j];
                av.x = e[0] | (e[1] << 16);
                av.y = e[2] | (e[3] << 16);
                av.z = e[4] | (e[5] << 16);
                av.w = e[6] | (e[7] << 16);
            }
            acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xv),
                                                              __builtin_bit_cast(bf16x8, av), acc[nt], 0, 0, 0);
        }
    }
    // D[row][col]: lane holds col = lane % 32, rows 8g + 4h + jj in register 4g + jj
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) red[w][nt][8 * g + 4 * h + jj][i] = acc[nt][4 * g + jj];
    __syncthreads();
    for (int idx = threadIdx.x; idx < 32 * 32 * NT; idx += 256) {
        const int col = idx % (32 * NT), row = idx / (32 * NT);
        const int tt = rows_t[row];
        if (tt < 0 || col >= r) continue;
        const int nt = col >> 5, c = col & 31;
        const float s = ((red[0][nt][row][c] + red[1][nt][row][c]) + red[2][nt][row][c]) + red[3][nt][row][c];
        const uint32_t hi = f32_to_bf16_bits(s);
        const uint32_t lo = f32_to_bf16_bits(s - bf16_bits_to_f32(hi));
        S_hl[(size_t)tt * 2 * r + col] = (bf16_t)hi;
        S_hl[(size_t)tt * 2 * r + r + col] = (bf16_t)lo;
    }
}

int launch_shrink_bf16(const Fwd &f, const PtrTable &A)
{
    if (f.T == 0 || f.L == 0) return 0;
    // upper bound on the number of 32-row blocks: every adapter may end in a partial block
    const int blocks = (f.T + 31) / 32 + f.L;
    if (f.r <= 32)
        hipLaunchKernelGGL(shrink_bf16_kernel<1>, dim3(blocks), dim3(256), 0, f.stream, (const bf16_t *)f.x, A,
                           f.perm, f.offsets, f.L, f.H, f.r, (bf16_t *)f.S);
    else
        hipLaunchKernelGGL(shrink_bf16_kernel<2>, dim3(blocks), dim3(256), 0, f.stream, (const bf16_t *)f.x, A,
                           f.perm, f.offsets, f.L, f.H, f.r, (bf16_t *)f.S);
    return (int)hipGetLastError();
}

}  // namespace alora
