// Fused bf16 projection kernel: base GEMM on bf16 MFMA (fp32 accumulate) with the low-rank
// expand, the per-row activation select, the q_out store and the paged K/V store in one pass.
//
// Per 256(token) x 256(feature) tile:
//   1. classify the tile's rows (App. B mask); list the adapters its adapted rows use
//   2. expand first: for each such adapter a, accumulate [S_hi | S_lo](rows of a, else 0) . [B_a ; B_a]
//      as extra K-slices of the same MFMA loop, then zero the accumulators of rows that are not
//      adapted (a select, not a multiply: adapter data never reaches a base row)
//   3. base GEMM over the hidden dimension: rows that are not adapted see exactly the
//      instruction sequence of a call without adapters, so they come out bit-identical to it
//   4. round once to bf16 and store: columns [0,Nq) to q_out, K and V columns to the slot the
//      row maps to (rows with slot -1 write no K/V)
//
// MFMA operand roles are swapped (weights are the "A" operand, tokens the "B" operand), so each
// lane owns one token row per 32x32 block and four consecutive features per register quad:
// the select is a per-lane condition and stores are 8-byte vectors.
// LDS tiles are [row][64 k] bf16 with a 16-byte-chunk XOR swizzle; the weight tile is
// transposed in registers (k-major global layout -> k-contiguous LDS rows) on its way in.
#include "alora_internal.h"

namespace alora {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int GEMM_THREADS = 256;

__device__ __forceinline__ int swz(int row) { return ((row >> 1) ^ (row >> 3)) & 7; }
// byte offset of 16-byte chunk c (k = 8c..8c+7) of tile row `row`
__device__ __forceinline__ int lds_off(int row, int c) { return row * (BK * 2) + ((c ^ swz(row)) << 4); }

struct GemmArgs {
    const bf16_t *x, *W, *S_hl;
    const int32_t *aid, *seg, *pos, *start;
    const int64_t *slot;
    bf16_t *q, *kc, *vc;
    int T, H, Nq, Nkv, N, L, r;
    int mtiles, ntiles;
};

// Source of a K-slice: either the base operands (x rows, W rows k0..k0+63) or one adapter's
// expand operands (S_hl rows masked to the adapter's rows, B rows (k mod r) for k < 2r).
struct Slice {
    const bf16_t *xsrc;  // row-major, leading dimension xld
    int xld;
    int xk_valid;        // columns >= xk_valid read as zero
    int row_key;         // -2: every in-range row is valid; else only rows whose adapter == row_key
    const bf16_t *wsrc;  // row-major [*, N]
    int w_rows;          // k >= w_rows read as zero
    int w_mod;           // 0: source row = k; else source row = k mod w_mod
};

__global__ __launch_bounds__(GEMM_THREADS, 1) void alora_gemm_bf16_kernel(GemmArgs g, PtrTable B)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *Xs = smem;                  // [BM][BK] bf16, swizzled  (32 KB)
    unsigned char *Ws = smem + BM * BK * 2;    // [BN][BK] bf16, swizzled  (32 KB)
    int *arow = (int *)(smem + (BM + BN) * BK * 2);  // [BM] effective adapter per tile row
    int *present = arow + BM;                        // [ALORA_MAX_ADAPTERS]

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int mt = blockIdx.x % g.mtiles, nt = blockIdx.x / g.mtiles;
    const int m0 = mt * BM, n0 = nt * BN;
    const int wt = w & 1, wn = w >> 1;         // wave owns tokens [wt*128,+128) x features [wn*128,+128)
    const int li = lane & 31, lh = lane >> 5;

    // ---- 1. classify rows, list adapters --------------------------------------------------
    {
        const int t = m0 + tid;
        int a = -1;
        if (t < g.T && g.L > 0) a = effective_adapter(g.aid, g.seg, g.pos, g.start, t);
        arow[tid] = a;
        if (tid < ALORA_MAX_ADAPTERS) present[tid] = 0;
        __syncthreads();
        if (a >= 0) present[a] = 1;
        __syncthreads();
    }

    f32x16 acc[4][4];  // [feature tile][token tile]
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

    // global -> register staging of one K-slice
    u32x4 xreg[8], wreg[8];
    const int xc = tid & 7, xr0 = tid >> 3;                        // x tile: chunk xc of rows xr0 + 32 i
    const int wnb = tid & 7, wkb = (tid >> 3) & 7, wq = tid >> 6;  // W tile: 8k x 8n block
    const int wcol = n0 + wq * 64 + wnb * 8;

    auto load_slice = [&](const Slice &s, int k0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = xr0 + 32 * i;
            const int t = m0 + row;
            bool ok = (t < g.T) && (k0 + xc * 8 < s.xk_valid);
            if (s.row_key != -2) ok = ok && (arow[row] == s.row_key);
            u32x4 v = {0u, 0u, 0u, 0u};
            if (ok) v = *(const u32x4 *)(s.xsrc + (size_t)t * s.xld + k0 + xc * 8);
            xreg[i] = v;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int k = k0 + wkb * 8 + i;
            const bool ok = (k < s.w_rows) && (wcol < g.N);
            const int srow = (s.w_mod && k >= s.w_mod) ? k - s.w_mod : k;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (ok) v = *(const u32x4 *)(s.wsrc + (size_t)srow * g.N + wcol);
            wreg[i] = v;
        }
    };

    auto store_slice = [&]() {
#pragma unroll
        for (int i = 0; i < 8; ++i) *(u32x4 *)(Xs + lds_off(xr0 + 32 * i, xc)) = xreg[i];
        // 8x8 transpose of 16-bit elements: out[j] = (row0[j], row1[j], ..., row7[j])
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
            u32x4 o;
            o.x = __builtin_amdgcn_perm(wreg[1][j >> 1], wreg[0][j >> 1], sel);
            o.y = __builtin_amdgcn_perm(wreg[3][j >> 1], wreg[2][j >> 1], sel);
            o.z = __builtin_amdgcn_perm(wreg[5][j >> 1], wreg[4][j >> 1], sel);
            o.w = __builtin_amdgcn_perm(wreg[7][j >> 1], wreg[6][j >> 1], sel);
            *(u32x4 *)(Ws + lds_off(wq * 64 + wnb * 8 + j, wkb)) = o;
        }
    };

    auto compute_slice = [&]() {
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int c = 2 * ks + lh;
            bf16x8 wf[4], xf[4];
#pragma unroll
            for (int a = 0; a < 4; ++a)
                wf[a] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(Ws + lds_off(wn * 128 + a * 32 + li, c)));
#pragma unroll
            for (int b = 0; b < 4; ++b)
                xf[b] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(Xs + lds_off(wt * 128 + b * 32 + li, c)));
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[a], xf[b], acc[a][b], 0, 0, 0);
        }
    };

    // ---- 2. expand first, then select ------------------------------------------------------
    bool any_adapter = false;
    for (int a = 0; a < g.L; ++a) {
        if (!present[a]) continue;  // uniform (LDS broadcast)
        any_adapter = true;
        Slice s;
        s.xsrc = g.S_hl; s.xld = 2 * g.r; s.xk_valid = 2 * g.r; s.row_key = a;
        s.wsrc = (const bf16_t *)B.p[a]; s.w_rows = 2 * g.r; s.w_mod = g.r;
        for (int k0 = 0; k0 < 2 * g.r; k0 += BK) {
            load_slice(s, k0);
            store_slice();
            __syncthreads();
            compute_slice();
            __syncthreads();
        }
    }
    if (any_adapter) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const bool keep = arow[wt * 128 + b * 32 + li] >= 0;
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[a][b][e] = keep ? acc[a][b][e] : 0.f;
        }
    }

    // ---- 3. base GEMM ---------------------------------------------------------------------
    {
        Slice s;
        s.xsrc = g.x; s.xld = g.H; s.xk_valid = g.H; s.row_key = -2;
        s.wsrc = g.W; s.w_rows = g.H; s.w_mod = 0;
        load_slice(s, 0);
        for (int k0 = 0; k0 < g.H; k0 += BK) {
            store_slice();
            __syncthreads();
            if (k0 + BK < g.H) load_slice(s, k0 + BK);
            compute_slice();
            __syncthreads();
        }
    }

    // ---- 4. round and store ------------------------------------------------------------------
    // D[i][j]: i = feature (8g + 4*lh + jj, register 4g + jj), j = token (li)
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int t = m0 + wt * 128 + b * 32 + li;
        if (t >= g.T) continue;
        const int64_t sl = g.slot[t];
        bf16_t *qrow = g.q + (size_t)t * g.Nq;
        bf16_t *krow = g.kc + (size_t)(sl < 0 ? 0 : sl) * g.Nkv;
        bf16_t *vrow = g.vc + (size_t)(sl < 0 ? 0 : sl) * g.Nkv;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int n = n0 + wn * 128 + a * 32 + 8 * gq + 4 * lh;
                if (n >= g.N) continue;
                u32x2 v;
                v.x = f32_to_bf16_bits(acc[a][b][4 * gq + 0]) | (f32_to_bf16_bits(acc[a][b][4 * gq + 1]) << 16);
                v.y = f32_to_bf16_bits(acc[a][b][4 * gq + 2]) | (f32_to_bf16_bits(acc[a][b][4 * gq + 3]) << 16);
                if (n < g.Nq) {
                    *(u32x2 *)(qrow + n) = v;
                } else if (sl >= 0) {
                    if (n < g.Nq + g.Nkv) *(u32x2 *)(krow + (n - g.Nq)) = v;
                    else *(u32x2 *)(vrow + (n - g.Nq - g.Nkv)) = v;
                }
            }
        }
    }
}

size_t bf16_partial_bytes(int, int, int) { return 0; }

int launch_gemm_bf16(const Fwd &f, const PtrTable &B)
{
    if (f.T == 0) return 0;
    GemmArgs g;
    g.x = (const bf16_t *)f.x; g.W = (const bf16_t *)f.W; g.S_hl = (const bf16_t *)f.S;
    g.aid = f.aid; g.seg = f.seg; g.pos = f.pos; g.start = f.start; g.slot = f.slot;
    g.q = (bf16_t *)f.q; g.kc = (bf16_t *)f.kc; g.vc = (bf16_t *)f.vc;
    g.T = f.T; g.H = f.H; g.Nq = f.Nq; g.Nkv = f.Nkv; g.N = f.N; g.L = f.L; g.r = f.r;
    g.mtiles = (f.T + BM - 1) / BM;
    g.ntiles = (f.N + BN - 1) / BN;
    const size_t smem = (size_t)(BM + BN) * BK * 2 + (BM + ALORA_MAX_ADAPTERS) * sizeof(int);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)alora_gemm_bf16_kernel,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return (int)e;
        attr_set = true;
    }
    hipLaunchKernelGGL(alora_gemm_bf16_kernel, dim3(g.mtiles * g.ntiles), dim3(GEMM_THREADS), smem, f.stream, g, B);
    return (int)hipGetLastError();
}

}  // namespace alora
