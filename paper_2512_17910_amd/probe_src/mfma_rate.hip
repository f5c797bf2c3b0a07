// Sustained bf16 MFMA rate under the chip's power limit, nothing but MFMAs in the loop: the 32x32x16 shape the
// projection kernel uses against 16x16x32, random operands held in registers, the same 128 x 128 register tile per
// wavefront (one wavefront per SIMD, every compute unit busy).  Stand-alone program, built by
// `python -m paper_2512_17910_amd.probe build`, run by `python -m paper_2512_17910_amd.probe mfma`.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
__device__ uint32_t rnd(uint32_t& s) { s = s * 1664525u + 1013904223u; return s; }
__device__ uint32_t rbf2(uint32_t& s) {
    uint32_t r = rnd(s);
    uint32_t lo = ((r & 0x80ff) | 0x3f00) ^ ((r >> 3) & 0x0080);
    uint32_t hi = (((r >> 16) & 0x80ff) | 0x3f00);
    return lo | (hi << 16);
}
__device__ bf16x8 rfrag(uint32_t& s) { u32x4 u; for (int e = 0; e < 4; ++e) u[e] = rbf2(s); return __builtin_bit_cast(bf16x8, u); }
// 128 x 128 per wavefront and k = 32 per iteration in both kernels
__global__ __launch_bounds__(256) void k32(float* out, int iters)
{
    uint32_t s = threadIdx.x * 2654435761u + blockIdx.x * 97u + 12345u;
    bf16x8 a[2][4], b[2][4];
    for (int h = 0; h < 2; ++h) for (int i = 0; i < 4; ++i) { a[h][i] = rfrag(s); b[h][i] = rfrag(s); }
    f32x16 acc[16];
    for (int i = 0; i < 16; ++i) for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[h][i >> 2], b[h][(i >> 2) & 1 ? 3 - (i & 3) : (i & 3)], acc[i], 0, 0, 0);
    }
    float t = 0.f;
    for (int i = 0; i < 16; ++i) for (int e = 0; e < 16; ++e) t += acc[i][e];
    out[blockIdx.x * blockDim.x + threadIdx.x] = t;
}
__global__ __launch_bounds__(256) void k16(float* out, int iters)
{
    uint32_t s = threadIdx.x * 2654435761u + blockIdx.x * 97u + 12345u;
    bf16x8 a[8], b[8];
    for (int i = 0; i < 8; ++i) { a[i] = rfrag(s); b[i] = rfrag(s); }
    f32x4 acc[64];
    for (int i = 0; i < 64; ++i) for (int e = 0; e < 4; ++e) acc[i][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 64; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i >> 3], b[(i >> 3) & 1 ? 7 - (i & 7) : (i & 7)], acc[i], 0, 0, 0);
    }
    float t = 0.f;
    for (int i = 0; i < 64; ++i) for (int e = 0; e < 4; ++e) t += acc[i][e];
    out[blockIdx.x * blockDim.x + threadIdx.x] = t;
}
int main()
{
    float* d; (void)hipMalloc(&d, 256 * 256 * 4);
    hipEvent_t e0, e1; (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
    for (int rep = 0; rep < 3; ++rep)
        for (int which = 0; which < 2; ++which) {
            const int iters = 100000;
            (void)hipEventRecord(e0);
            if (which == 0) k32<<<256, 256>>>(d, iters); else k16<<<256, 256>>>(d, iters);
            (void)hipEventRecord(e1); (void)hipEventSynchronize(e1);
            float ms; (void)hipEventElapsedTime(&ms, e0, e1);
            double flops = 256.0 * 4 * iters * 2.0 * 128 * 128 * 32;
            printf("%s: %.3f ms, %.1f TFLOP/s, implied clock %.3f GHz\n", which == 0 ? "32x32x16" : "16x16x32", ms, flops / ms / 1e9,
                   flops / (ms * 1e-3) / 256 / 4096.0 / 1e9);
            fflush(stdout);
        }
    return 0;
}
