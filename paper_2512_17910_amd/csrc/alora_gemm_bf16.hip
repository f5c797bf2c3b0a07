// Fused bf16 projection kernel: base GEMM on bf16 MFMA (fp32 accumulate) with the low-rank
// expand, the per-row activation select, the q_out store and the paged K/V store in one pass.
//
// Per 256(token) x 256|192|128(feature) tile, one workgroup of four wavefronts (one per SIMD):
//   1. fetch the tile's rows' effective adapters (the grouping step's classification, App. B mask)
//      and cache slots; list the adapters its adapted rows use
//   2. expand first: for each such adapter a, accumulate [S_hi | S_lo](rows of a, else 0) . [B_a ; B_a]
//      32 k at a time through the LDS areas the base prologue leaves free, then zero the
//      accumulators of rows that are not adapted (a select, not a multiply: adapter data never
//      reaches a base row)
//   3. base GEMM over the hidden dimension: rows that are not adapted see exactly the
//      instruction sequence of a call without adapters, so they come out bit-identical to it
//   4. round once to bf16 and store: columns [0,Nq) to q_out, K and V columns to the slot the
//      row maps to (rows with slot -1 write no K/V)
// Small-batch (split) mode stops after 3 over its range of the hidden dimension and stores fp32
// partials; for batches of at most 256 rows extra workgroups behind the projection's own classify,
// group and shrink the batch (alora_group_small.h, alora_shrink_rows.h) out of the same LDS stages.
//
// Data movement (gfx950):
//   - global -> LDS with buffer loads that write LDS directly (no VGPR staging); the buffer
//     descriptor's range check returns zeros for token rows past T, masked lanes get an
//     out-of-range offset.
//   - the K dimension runs through rings of LDS areas, 32 k per slice: six 24 KB stages (token
//     slice + weight slice) for the 128-wide tile; for the 192- and 256-wide tiles six token areas
//     and four weight areas of 16 KB, where a step's token copies cover half the rows of TWO
//     slices so that both halves of a 128-byte line of x are asked for by neighbouring
//     instructions (see PAIRED in the kernel).  While slice i is multiplied, the first fragments of
//     slice i+1 are already fetched from LDS and the slices after it are in flight from memory;
//     their copies are issued one per two or three MFMAs, which keeps the demand on the vector
//     memory pipe (64 B/clk per CU) uniform.  One barrier per slice, placed where the MFMAs that
//     follow it already have their operands in registers.
//   - token tile in LDS: [row][32 k], 16-byte chunks XOR-swizzled by (row/4)%4, read with
//     ds_read_b128.  Weight tile in LDS: k-major exactly as in global memory ([k][256 n]),
//     16-byte chunks XOR-swizzled by 4*(k%4), read with the transposing LDS load
//     (ds_read_b64_tr_b16), which hands each lane four consecutive k of one feature column.
//   - MFMA operand roles are swapped (weights are "A", tokens are "B"): each lane owns one token
//     row per 32x32 block and four consecutive features per register quad, so the select is a
//     per-lane condition and stores are 8-byte vectors.
#include <algorithm>
#include <atomic>
#include <type_traits>
#include "alora_internal.h"
#include "alora_group_small.h"
#include "alora_shrink_rows.h"

namespace alora {

constexpr int BM = 256, BK = 32;
constexpr int KBLK = 64;     // granularity of the hidden dimension the host plans splits in
constexpr int GEMM_THREADS = 256;
constexpr uint32_t W_OFF = 16384;      // a stage is the token tile (256 rows x 64 B) followed by the weight tile
constexpr uint32_t OOR = 0x80000000u;  // buffer offset that is out of range for every descriptor

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((address_space(3))) unsigned char lds_byte;

struct GemmArgs {
    const bf16_t *x, *W, *S_hl;
    const int8_t *aeff;   // per token: adapter id if the row is adapted, else -1 (grouping kernel)
    const int64_t *slot;
    bf16_t *q, *kc, *vc;
    int T, H, Nq, Nkv, N, L, r;
    int kx;  // length of the expand K dimension: (hi | lo) x r
    int mtiles, ntiles;
    int kps;          // split mode: 32-wide K-slices per split
    float *partial;   // split mode: [splits][T][N] fp32
    const bf16_t *bias;   // [N] or null: added to every row before rounding (fused mode)
    RankTable ranks;      // per adapter: B_a has ranks.r[a] rows
    // split mode: the grid is one-dimensional, tiles8 workgroups per split, followed by `prep_wgs`
    // workgroups that classify, group and shrink the batch (0: separate kernels did that)
    int tiles8, splits, prep_wgs;
    int prep_ranges, prep_kper;   // ranges of the hidden dimension per block-table entry, and their width
    GroupSmallArgs prep;
    void *S_out;          // shrink result written by the prep workgroups ((hi, lo) form)
    // rotary embedding fused into the store (fused mode, 256-feature tiles, heads of 128): [rope_positions][64]
    const float *rope_cos, *rope_sin;
    const int32_t *pos;
    int rope_positions;
};

// Buffer descriptor of a raw byte buffer (stride 0, 32-bit data format): offsets at or past
// `bytes` read as zero.
typedef u32x4 rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    const uint64_t p = (uint64_t)base;
    const rsrc_t r = {(uint32_t)p, (uint32_t)(p >> 32) & 0xffffu, bytes, 0x00020000u};
    return r;
}

// 64 lanes x 16 bytes from the buffer straight into LDS at M0 + IMM + 16*lane.  Written as assembly
// statements: the kernel orders these copies against its LDS reads itself (wait counts and barriers
// in the main loop), which the compiler's own bookkeeping of such loads would override with waits
// for all of them.
// The LDS address is not set per copy: the copies of one operand tile share one M0 and differ in the
// instruction's immediate offset (two scalar instructions per slice and wavefront instead of two per
// copy).  That offset also advances the global address, which the per-copy vector offsets take back
// (lds_copy_voffset); to keep those non-negative for every shape, descriptors made by make_rsrc_copy
// start LDS_COPY_BIAS bytes early (no lane ever addresses the bytes before the buffer: every valid
// offset plus its immediate is at least LDS_COPY_BIAS).
constexpr uint32_t LDS_COPY_BIAS = 4096;
constexpr uint32_t LDS_COPY_STEP = 1024;   // LDS bytes between consecutive copies of one operand tile
__device__ __forceinline__ rsrc_t make_rsrc_copy(const void *base, uint32_t bytes)
{
    return make_rsrc((const char *)base - LDS_COPY_BIAS, bytes + LDS_COPY_BIAS);
}
// vector offset of copy j (0..3) of a tile whose element sits `bytes` into the descriptor's buffer
__device__ __forceinline__ uint32_t lds_copy_voffset(uint32_t bytes, int j) { return bytes + LDS_COPY_BIAS - LDS_COPY_STEP * j; }
__device__ __forceinline__ void set_lds_base(uint32_t lds_addr)
{
    // (one wait state between a write of M0 and an LDS-direct load)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" : : "s"(lds_addr) : "memory");
}
template <int IMM>
__device__ __forceinline__ void load_lds16_imm(rsrc_t rsrc, uint32_t voffset, uint32_t soffset)
{
    asm volatile("buffer_load_dwordx4 %0, %1, %2 offen offset:%3 lds" : : "v"(voffset), "s"(rsrc), "s"(soffset), "n"(IMM) : "memory");
}
__device__ __forceinline__ void load_lds16(int j, rsrc_t rsrc, uint32_t voffset, uint32_t soffset)
{
    switch (j) {
    case 0: load_lds16_imm<0>(rsrc, voffset, soffset); break;
    case 1: load_lds16_imm<LDS_COPY_STEP>(rsrc, voffset, soffset); break;
    case 2: load_lds16_imm<2 * LDS_COPY_STEP>(rsrc, voffset, soffset); break;
    default: load_lds16_imm<3 * LDS_COPY_STEP>(rsrc, voffset, soffset); break;
    }
}
__device__ __forceinline__ uint32_t lds_addr_of(const lds_byte *p) { return (uint32_t)(uintptr_t)p; }

__device__ __forceinline__ bf16x8 read_w_frag(const lds_byte *p, int pitch)
{
    // k..k+3 of this lane's feature column, then k+4..k+7 (four weight rows further on)
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p + 4 * pitch));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

// NTW: 32-wide feature tiles per wavefront; the workgroup tile is 256 tokens x 64*NTW features.
// SPLIT: small-batch mode.  The workgroup index selects a tile and a range of K-slices; the kernel only accumulates the
// base product over that range and stores the fp32 accumulators to g.partial[split][T][N]; adapters,
// rounding and the q_out / cache stores are left to the finishing kernel.
// Probe builds (-DALORA_PROBE=bits, a library of their own that only the package's probe script loads; the
// product library is built without and contains none of this).  Bit 1: the main loop issues no global -> LDS
// copies; bit 2: it reads no fragments from LDS (both leave the MFMA sequence as it is and the results wrong);
// bit 4: every workgroup records when it passed the kernel's phases (100 MHz counter) and every wavefront the
// shader-clock cycles of its main loop, into the buffer alora_probe_set_buffer names; bit 8: every workgroup
// fetches the operands of tile (0, 0), so that the copies hit in L2; bit 16: the weight tile is addressed as if W were
// stored tile by tile, a contiguous stream per workgroup.
#ifndef ALORA_PROBE
#define ALORA_PROBE 0
#endif
#if ALORA_PROBE
constexpr int PROBE_MAX_WGS = 4096;
__device__ unsigned long long *g_probe;   // [PROBE_MAX_WGS][8] phase stamps, then [PROBE_MAX_WGS][4] loop cycles per wavefront
#define PROBE_STAMP(i)                                                                                   \
    do {                                                                                                 \
        if (g_probe && threadIdx.x == 0 && blockIdx.x < PROBE_MAX_WGS)                                   \
            g_probe[(size_t)blockIdx.x * 8 + (i)] = __builtin_amdgcn_s_memrealtime();                     \
    } while (0)
#else
#define PROBE_STAMP(i)
#endif

template <int NTW, bool SPLIT, bool ROPE = false>
__global__ __launch_bounds__(GEMM_THREADS, 1) void alora_gemm_bf16_kernel(GemmArgs g, PtrTable B, PtrTable A)
{
    PROBE_STAMP(0);   // entry
    constexpr int BN = 64 * NTW;
    // Ring geometry.  128-feature tiles keep weight rows of 256 bytes, which makes a stage 24 KB and
    // leaves room for six stages instead of four: four slices in flight instead of two, which is
    // what the small-batch path needs to keep enough of W on its way from HBM.
    constexpr int WPITCH = NTW == 2 ? 256 : 512;       // bytes per k row of the weight tile in LDS
    constexpr int NST = NTW == 2 ? 6 : 4;              // stages
    constexpr uint32_t STAGE_BYTES = W_OFF + BK * WPITCH;
    constexpr int LPW = WPITCH / 16;                   // lanes (16-byte chunks) per weight row
    constexpr int RPW = 64 / LPW;                      // weight rows per copy instruction
    constexpr int NCW = BK / RPW / 4;                  // weight-tile copy instructions per wavefront and slice
    constexpr int NC = 4 + NCW;                        // copy instructions per wavefront and slice
    // PAIRED (the 192- and 256-wide tiles): token slices and weight slices live in rings of their own, six token
    // areas and four weight areas of 16 KB, and the token copies of a step cover HALF the tile's rows for TWO
    // consecutive slices -- the two 64-byte halves of every 128-byte line of x are requested by neighbouring
    // instructions, and the second one finds the line on its way.  Measured on the main loop: 4 % (the kernel runs
    // at the clock its power draw allows, and a line fetched once from L2 instead of twice is clock).  A token
    // area then lives one step longer than a weight area, hence the separate rings; all 160 KB are ring, and the
    // small arrays below sit in a token area that the main loop does not reach before they are done with.
    constexpr bool PAIRED = NTW != 2;
    constexpr int NXA = PAIRED ? 6 : NST, NWA = PAIRED ? 4 : NST;          // token areas, weight areas
    constexpr uint32_t X_AREA = 16384, W_AREA = BK * WPITCH;
    constexpr uint32_t RING_BYTES = PAIRED ? NXA * X_AREA + NWA * W_AREA : NST * STAGE_BYTES;
    static_assert(!PAIRED || RING_BYTES == 160 * 1024, "the paired rings fill the LDS");
    __shared__ __attribute__((aligned(16))) unsigned char ring[RING_BYTES];
    __shared__ int arow_s[PAIRED ? 1 : BM];
    __shared__ int present_s[PAIRED ? 1 : ALORA_MAX_ADAPTERS];
    __shared__ int plist_s[PAIRED ? 1 : ALORA_MAX_ADAPTERS];
    __shared__ int n_present_s;
    __shared__ int64_t slot_s[PAIRED ? 1 : BM];
    lds_byte *const ring0 = (lds_byte *)ring;
    // token area k and weight area k of the ring(s)
    auto xa = [&](int k) -> lds_byte * { return PAIRED ? ring0 + k * X_AREA : ring0 + k * STAGE_BYTES; };
    auto wa = [&](int k) -> lds_byte * { return PAIRED ? ring0 + NXA * X_AREA + k * W_AREA : ring0 + k * STAGE_BYTES + W_OFF; };
    // the areas the expand phase works in (the base prologue leaves them free)
    lds_byte *const ex_x = xa(NXA - 1), *const ex_w = wa(NWA - 1);
    // effective adapter per tile row; adapters present in this tile (flags, ascending list, count); cache slot per
    // tile row (-1: no K/V write).  PAIRED: the first three in token area 4, which the main loop's first step is
    // the first to write and which the expand and select phases, their only users, are done with by then; the
    // slots stay in registers through the main loop and are parked behind wavefront 0's strip for the stores.
    int *const arow = PAIRED ? (int *)(ring + 4 * X_AREA) : arow_s;
    int *const present = PAIRED ? (int *)(ring + 4 * X_AREA + 4 * BM) : present_s;
    int *const plist = PAIRED ? (int *)(ring + 4 * X_AREA + 4 * BM + 4 * ALORA_MAX_ADAPTERS) : plist_s;
    int64_t *const slot_lds = PAIRED ? (int64_t *)(ring + 20 * 1024) : slot_s;
    int &n_present = PAIRED ? *(int *)(ring + 4 * X_AREA + 4 * BM + 8 * ALORA_MAX_ADAPTERS) : n_present_s;

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Tile of this workgroup.  Workgroups are handed to the 8 XCDs round-robin, and each XCD has its
    // own L2: XCD k = blockIdx.x % 8 takes a contiguous range of a tile order that walks panels of
    // 4 token tiles, feature tile by feature tile, so that the ~32 tiles an XCD runs at a time form
    // a 4 x 8 patch sharing their token and weight slices in that L2.
    // split mode: blockIdx.x = split * tiles8 + tile, then the prep workgroups (dispatched last, so
    // that they take the compute units the projection leaves free)
    int bx = (int)blockIdx.x, by = 0;
    if (SPLIT) {
        by = bx / g.tiles8;
        bx -= by * g.tiles8;
        if (by >= g.splits) {
            if constexpr (SPLIT && NTW == 2) {
                // One entry of the 32-row block table: group the batch, then the shrink of the block over
                // the whole hidden dimension, out of this kernel's stages (token buffers, A buffers,
                // reduction array, scratch).
                static_assert(STAGE_BYTES >= (uint32_t)ShrinkLds<256, 1>::X_BYTES && STAGE_BYTES >= (uint32_t)ShrinkLds<256, 1>::A_BYTES &&
                              STAGE_BYTES >= (uint32_t)ShrinkLds<256, 1>::RED_BYTES && STAGE_BYTES >= (GROUP_SMALL_SCRATCH + 4) * 4u,
                              "stages hold the shrink's buffers");
                // prep_ranges workgroups per entry, one per range of the hidden dimension; each works the
                // grouping out for itself, the first of them writes the entry's share of its results
                const int p = (int)blockIdx.x - g.tiles8 * g.splits;
                const int e = p / g.prep_ranges, range = p - e * g.prep_ranges;
                unsigned char *const stage0 = ring, *const stage1 = ring + STAGE_BYTES, *const stage2 = ring + 2 * STAGE_BYTES,
                                    *const stage3 = ring + 3 * STAGE_BYTES, *const stage4 = ring + 4 * STAGE_BYTES;
                int *scr = (int *)(ring + 5 * STAGE_BYTES);
                int grp, cnt;
                const int *rows = group_small(g.prep, g.T, g.L, e, range == 0, scr, grp, cnt);
                if (grp < 0 || grp >= g.L) { PROBE_STAMP(7); return; }   // unused entry or the rows that keep the base output
                const int kbeg = range * g.prep_kper;
                shrink_rows<256, 1, false>(g.x, (const bf16_t *)A.p[grp], g.ranks.r[grp], rows, g.H, g.r,
                                           (uint32_t)((size_t)g.T * g.H * 2), g.T, kbeg, min(g.H, kbeg + g.prep_kper), range,
                                           g.prep_ranges, nullptr, g.S_out, stage0, stage1, stage2, stage3,
                                           (float (*)[1][32][33])stage4, scr + GROUP_SMALL_SCRATCH);
                PROBE_STAMP(7);   // grouping and shrink of this entry done
            }
            return;
        }
    }
    int mt, nt;
    {
        const int total = g.mtiles * g.ntiles, chunk = (total + 7) >> 3;
        const int l = (bx & 7) * chunk + (bx >> 3);
        if (l >= total) return;  // grid is padded to a multiple of 8; uniform across the workgroup
        // (token tiles per panel.  Measured, L2-miss reads and kernel time at T = 8192, 8192 -> 10240 / T = 4096,
        // 4096 -> 6144: 4: 2.79 GB, 993 us / 351 MB, 180 us; 8: 2.50 GB, 993 us / 380 MB, 180 us; 2: 3.80 GB, 1019 us /
        // 636 MB, 182 us; 16: 4.15 GB, 1016 us / 619 MB, 183 us.)
        constexpr int PANEL = 4;
        const int panel = l / (PANEL * g.ntiles), rem = l - panel * PANEL * g.ntiles;
        const int pm = min(PANEL, g.mtiles - PANEL * panel);
        nt = rem / pm;
        mt = PANEL * panel + rem - nt * pm;
    }
    const int m0 = mt * BM, n0 = nt * BN;
    const int wt = w & 1, wn = w >> 1;   // wave owns tokens [wt*128,+128) x features [wn*32*NTW,+32*NTW)
    const int li = lane & 31, lh = lane >> 5;
    const int rows_valid = min(g.T - m0, BM);

    // ---- 1. this tile's rows: effective adapter (from the grouping kernel) and cache slot ------
    // The two loads are issued here and waited for only after the ring has been filled (loads
    // complete in order, so "all but the ring's copies" means these two have arrived).  They are
    // assembly statements for the reason given at load_lds16: a wait the compiler places for them
    // would also wait for every copy issued in between.
    int a_row = -1;
    int64_t slot_row = -1;
    if (!SPLIT && m0 + tid < g.T) {
        const int64_t *ps = g.slot + (m0 + tid);
        asm volatile("global_load_dwordx2 %0, %1, off" : "=v"(slot_row) : "v"(ps) : "memory");
        if (g.L > 0) {
            const int8_t *pa = g.aeff + (m0 + tid);
            asm volatile("global_load_sbyte %0, %1, off" : "=v"(a_row) : "v"(pa) : "memory");
        }
    }

    // ---- per-lane geometry of the global -> LDS copies ----------------------------------------
    // token tile: instruction ii of wave w fills rows 64w + 16ii .. +15; lane -> row +lane/4, physical
    // chunk lane%4, which holds logical chunk (lane%4) ^ swizzle(row)
    auto x_row = [&](int ii, int ln) { return 64 * w + 16 * ii + (ln >> 2); };
    auto x_chunk = [&](int ii, int ln) { return (ln & 3) ^ ((x_row(ii, ln) >> 2) & 3); };
    // weight tile: instruction jj of wave w fills the RPW k rows from 8w + RPW*jj; lane -> row
    // +lane/LPW, physical chunk lane%LPW holding logical chunk (lane%LPW) ^ 4*(k%4)
    auto w_k = [&](int jj, int ln) { return 8 * w + RPW * jj + ln / LPW; };
    auto w_chunk = [&](int jj, int ln) { return (ln % LPW) ^ ((w_k(jj, ln) & 3) << 2); };
    auto w_col_ok = [&](int jj, int ln) { return (8 * w_chunk(jj, ln) < BN) & (n0 + 8 * w_chunk(jj, ln) < g.N); };

    // ---- per-lane LDS read addresses of the MFMA operands ----------------------------------
    uint32_t xaddr;  // token fragment: row wt*128 + li (+32 b), chunk 2ks + lh
    {
        const int row0 = wt * 128 + li;
        xaddr = (uint32_t)row0 * (BK * 2) + (uint32_t)((lh ^ ((row0 >> 2) & 3)) << 4);
    }
    uint32_t waddr[NTW];  // weight fragments via transposing read; see read_w_frag
    {
        const int s = lane & 15, j = s >> 2, blk = (lane >> 4) & 1;
#pragma unroll
        for (int a = 0; a < NTW; ++a) {
            const int chunk = wn * 4 * NTW + 4 * a + 2 * blk + ((s & 3) >> 1);
            waddr[a] = (uint32_t)(8 * lh + j) * WPITCH + (uint32_t)((chunk ^ (j << 2)) << 4) + (uint32_t)((s & 1) << 3);
        }
    }

    f32x16 acc[NTW][4];  // [feature tile a][token tile b]
#pragma unroll
    for (int a = 0; a < NTW; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

    // ---- the slice sequence -------------------------------------------------------------------
#if ALORA_PROBE & 8
    // every workgroup fetches the operands of tile (0, 0): the same instruction stream with (almost) no L2 misses
    const rsrc_t rx = make_rsrc_copy(g.x, (uint32_t)min(g.T, BM) * g.H * 2);
    const rsrc_t rw = make_rsrc_copy(g.W, (uint32_t)(g.H * g.N) * 2);
#elif ALORA_PROBE & 16
    // the weight tile addressed as if W were stored tile by tile ([N / BN][hidden][BN]): a workgroup's weight
    // stream is then one contiguous range (timing of that layout; W is not stored that way, results are wrong)
    const rsrc_t rx = make_rsrc_copy(g.x + (size_t)m0 * g.H, (uint32_t)rows_valid * g.H * 2);
    const rsrc_t rw = make_rsrc_copy(g.W + (size_t)nt * g.H * BN, (uint32_t)(g.H * BN) * 2);
#else
    const rsrc_t rx = make_rsrc_copy(g.x + (size_t)m0 * g.H, (uint32_t)rows_valid * g.H * 2);
    const rsrc_t rw = make_rsrc_copy(g.W + n0, (uint32_t)(g.H * g.N - n0) * 2);
#endif
    const int w_pitch = (ALORA_PROBE & 16) ? BN : g.N;   // elements between consecutive k rows of the weight tile
    const rsrc_t rs = make_rsrc_copy(g.S_hl + (size_t)m0 * g.kx, (uint32_t)rows_valid * g.kx * 2);
    uint32_t vxb[4], vwb[NCW];
#pragma unroll
    for (int ii = 0; ii < 4; ++ii) vxb[ii] = lds_copy_voffset((uint32_t)(x_row(ii, lane) * g.H + 8 * x_chunk(ii, lane)) * 2, ii);
#pragma unroll
    for (int jj = 0; jj < NCW; ++jj)
        vwb[jj] = w_col_ok(jj, lane) ? lds_copy_voffset((uint32_t)(w_k(jj, lane) * w_pitch + 8 * w_chunk(jj, lane)) * 2, jj) : OOR;
    const uint32_t xstep = BK * 2, wstep = (uint32_t)BK * w_pitch * 2;
    // base K-slices of this workgroup: all of them, or the range of its split
    const int kt0 = SPLIT ? by * g.kps : 0;
    const int KT = SPLIT ? min(g.H / BK, kt0 + g.kps) : g.H / BK;
    const int n_base = KT - kt0;

    // copies of one 32-wide slice: this wavefront's four token-tile (c = 0..3) and NCW weight-tile
    // (c = 4..) instructions, into the token area at LDS address sta_x and the weight area at sta_w
    auto copy = [&](int c, rsrc_t r_x, const uint32_t (&vx)[4], uint32_t sx, rsrc_t r_w, const uint32_t (&vw)[NCW],
                    uint32_t sw, uint32_t sta_x, uint32_t sta_w) {
        static_assert(16 * BK * 2 == LDS_COPY_STEP && RPW * WPITCH == LDS_COPY_STEP && NCW <= 4, "immediate offsets of the copies");
        if (c == 0) set_lds_base(sta_x + (uint32_t)(64 * w) * (BK * 2));
        if (c == 4) set_lds_base(sta_w + (uint32_t)(8 * w) * WPITCH);
        if (c < 4) load_lds16(c, r_x, vx[c], sx);
        else load_lds16(c - 4, r_w, vw[c - 4], sw);
    };
    // PAIRED: token unit u = (pair p = u / 2, row half h = u % 2) is rows 128h .. 128h+127 of slices 2p and 2p+1;
    // this wavefront's copy j of it (j = 0..3) is row group 2w + j/2 (16 rows) of slice 2p + j%2, so that the two
    // halves of a row's 128-byte line are requested by neighbouring instructions.  The vector offset does not
    // depend on the slice (vxp[j/2]); row half and slice go into the scalar offset.  Units past the end repeat the
    // last pair (into areas that are free): every step issues the same number of copies.
    uint32_t vxp[2];
#pragma unroll
    for (int q = 0; q < 2; ++q)
        vxp[q] = lds_copy_voffset((uint32_t)((16 * (2 * w + q) + (lane >> 2)) * g.H + 8 * ((lane & 3) ^ ((lane >> 4) & 3))) * 2, 0);
    const int n_pairs = n_base >> 1;   // (n_base is even: the hidden dimension is a multiple of 64, splits are cut in 64s)
    // One descriptor per row half, each ending at the tile's last valid row: the scalar offset of a buffer load is
    // not part of its range check, so the row half must not travel there (rows past T would be read, and past
    // the end of x in the last tile); the scalar offset only moves along a row.
    const int xm0 = (ALORA_PROBE & 8) ? 0 : m0, xrows = (ALORA_PROBE & 8) ? min(g.T, BM) : rows_valid;
    // (readfirstlane: the clamps would otherwise be computed by a vector instruction, and the descriptor with them)
    const int xrows0 = __builtin_amdgcn_readfirstlane(min(xrows, 128)), xrows1 = __builtin_amdgcn_readfirstlane(max(xrows - 128, 0));
    const rsrc_t rxh0 = make_rsrc_copy(g.x + (size_t)xm0 * g.H, (uint32_t)xrows0 * g.H * 2);
    const rsrc_t rxh1 = make_rsrc_copy(g.x + (size_t)(xm0 + 128) * g.H, (uint32_t)xrows1 * g.H * 2);
    auto copy_unit = [&](int j, int u, int h, uint32_t sta_xa, uint32_t sta_xb) {   // h = u % 2, a constant at every call
        const int pc = min(u >> 1, n_pairs - 1);
        const uint32_t so = (uint32_t)(kt0 + 2 * pc + (j & 1)) * xstep;
        set_lds_base(((j & 1) ? sta_xb : sta_xa) + (uint32_t)(128 * h + 16 * (2 * w + (j >> 1))) * (BK * 2));
        if (h) load_lds16(0, rxh1, vxp[j >> 1], so);
        else load_lds16(0, rxh0, vxp[j >> 1], so);
    };
    auto copy_w = [&](int c, int s, uint32_t sta_w) {   // this wavefront's weight copy c (0 .. NCW-1) of base slice s
        const int kb = kt0 + min(s, n_base - 1);
        if (c == 0) set_lds_base(sta_w + (uint32_t)(8 * w) * WPITCH);
        load_lds16(c, rw, vwb[c], kb * wstep);
    };
    // Base slice s of this workgroup.  Slices past the end repeat the last one: every step issues
    // the same number of copies, which is what the in-order wait counts assume.
    auto issue_base = [&](int s, uint32_t sta_x, uint32_t sta_w) {
        const int kb = kt0 + min(s, n_base - 1);
#pragma unroll
        for (int c = 0; c < NC; ++c) copy(c, rx, vxb, kb * xstep, rw, vwb, kb * wstep, sta_x, sta_w);
    };

    // MFMA fragments of one 16-wide k step
    auto read_x = [&](const lds_byte *base, int ks, int b) {
        return *(const __attribute__((address_space(3))) bf16x8 *)(base + ((xaddr ^ (ks << 5)) + b * 32 * BK * 2));
    };
    auto read_w = [&](const lds_byte *base, int ks, int a) { return read_w_frag(base + (waddr[a] + ks * 16 * WPITCH), WPITCH); };
    auto load_frags = [&](const lds_byte *xbase, const lds_byte *wbase, int ks, bf16x8 (&wf)[NTW], bf16x8 (&xf)[4]) {
#pragma unroll
        for (int b = 0; b < 4; ++b) xf[b] = read_x(xbase, ks, b);
#pragma unroll
        for (int a = 0; a < NTW; ++a) wf[a] = read_w(wbase, ks, a);
    };
    auto mfmas = [&](const bf16x8 (&wf)[NTW], const bf16x8 (&xf)[4]) {
#pragma unroll
        for (int a = 0; a < NTW; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[a], xf[b], acc[a][b], 0, 0, 0);
    };

    bf16x8 wf0[NTW], xf0[4], wf1[NTW], xf1[4];

    // fill the ring with the first base slices; their latency also covers the expand phase.  PAIRED: in the
    // order the steps -4 .. -1 of the main loop would have issued them (step s issues token unit s+4 and weight
    // slice s+3): units 0 and 1 (slices 0, 1), weight slice 0, unit 2, weight slice 1, unit 3, weight slice 2.
    uint32_t sax[NXA], saw[NWA];
#pragma unroll
    for (int u = 0; u < NXA; ++u) sax[u] = lds_addr_of(xa(u));
#pragma unroll
    for (int u = 0; u < NWA; ++u) saw[u] = lds_addr_of(wa(u));
    constexpr int PRO = PAIRED ? 4 * 4 + 3 * NCW : NC * (NST - 1);   // copies of the prologue per wavefront
    if constexpr (PAIRED) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int j = 0; j < 4; ++j) copy_unit(j, u, u & 1, sax[2 * (u >> 1)], sax[2 * (u >> 1) + 1]);
            if (u >= 1) {
#pragma unroll
                for (int c = 0; c < NCW; ++c) copy_w(c, u - 1, saw[u - 1]);
            }
        }
    } else {
#pragma unroll
        for (int u = 0; u < NST - 1; ++u) issue_base(u, sax[u], saw[u]);
    }

    // the tile's rows have arrived (only the ring's copies may still be in flight): adapters present
    int n_exp = 0;           // expand slices ahead of the base slices
    int epa = 0;             // expand slices per adapter
    if (!SPLIT) {
        asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a_row), "+v"(slot_row) : "n"(PRO) : "memory");
        if (a_row >= g.L) a_row = -1;   // (a workspace that holds no grouping of this batch: stay inside the tables)
        if constexpr (!PAIRED) slot_lds[tid] = slot_row;
        arow[tid] = a_row;
        if (tid < ALORA_MAX_ADAPTERS) present[tid] = 0;
        __syncthreads();
        if (a_row >= 0) present[a_row] = 1;
        __syncthreads();
        if (tid < 64) {
            const bool p0 = present[tid] != 0, p1 = present[64 + tid] != 0;
            const uint64_t b0 = __ballot(p0), b1 = __ballot(p1);
            const uint64_t below = (1ull << tid) - 1ull;
            const int c0 = __popcll(b0);
            if (p0) plist[__popcll(b0 & below)] = tid;
            if (p1) plist[c0 + __popcll(b1 & below)] = 64 + tid;
            if (tid == 0) n_present = c0 + __popcll(b1);
        }
        __syncthreads();
        epa = (g.kx + BK - 1) / BK;
        n_exp = __builtin_amdgcn_readfirstlane(n_present) * epa;
    }

    PROBE_STAMP(1);   // ring prologue issued, the tile's rows known
    // ---- 2. expand first, then select ------------------------------------------------------
    // One slice at a time through the areas the prologue leaves free (few slices, not pipelined): 32 k of
    // [S_hi | S_lo] for the rows of adapter a (zeros elsewhere) against the matching rows of [B_a ; B_a].
    if (!SPLIT && n_exp > 0) {
        for (int e = 0; e < n_exp; ++e) {
            const int j = e / epa, k0 = (e - j * epa) * BK;
            const int a = __builtin_amdgcn_readfirstlane(plist[j]);
            const int ra = __builtin_amdgcn_readfirstlane((int)g.ranks.r[a]);   // rows of B_a; S columns past it are zero, B rows past it do not exist
            const rsrc_t rb =
                make_rsrc_copy((const bf16_t *)B.p[a] + n0, (uint32_t)(ra * g.N - n0) * 2);
            uint32_t vx[4], vw[NCW];
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) {
                const int row = x_row(ii, lane), kk = k0 + 8 * x_chunk(ii, lane);
                const bool ok = (arow[row] == a) & (kk < g.kx);
                vx[ii] = ok ? lds_copy_voffset((uint32_t)(row * g.kx + kk) * 2, ii) : OOR;
            }
#pragma unroll
            for (int jj = 0; jj < NCW; ++jj) {
                const int kk = k0 + w_k(jj, lane);
                const int srow = kk >= g.r ? kk - g.r : kk;   // [B ; B]: the hi and the lo half meet the same rows
                const bool ok = (kk < g.kx) & (srow < ra) & w_col_ok(jj, lane);
                vw[jj] = ok ? lds_copy_voffset((uint32_t)(srow * g.N + 8 * w_chunk(jj, lane)) * 2, jj) : OOR;
            }
#pragma unroll
            for (int c = 0; c < NC; ++c) copy(c, rs, vx, 0, rb, vw, 0, sax[NXA - 1], saw[NWA - 1]);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            load_frags(ex_x, ex_w, 0, wf0, xf0);
            load_frags(ex_x, ex_w, 1, wf1, xf1);
            mfmas(wf0, xf0);
            mfmas(wf1, xf1);
            __syncthreads();
        }
        // The select is written as a masked store of zero into the accumulator registers themselves,
        // so that the accumulators do not travel through the vector registers the main loop needs.
        // Assembly statements get no automatic hazard padding: let the last MFMAs drain first.
        asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            if (arow[wt * 128 + b * 32 + li] < 0) {
#pragma unroll
                for (int a = 0; a < NTW; ++a)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        float t = acc[a][b][e];
                        asm volatile("v_accvgpr_write_b32 %0, 0" : "+a"(t));
                        acc[a][b][e] = t;
                    }
            }
        }
        asm volatile("s_nop 7" ::: "memory");
    }

    // ---- 3. base GEMM ---------------------------------------------------------------------
    // step s: multiplies slice s (areas cur_x, cur_w); fetches the first fragments of slice s+1 (nxt_x, nxt_w);
    // issues the copies of slice s+NST-1 into the areas that slice s-1 occupied (PAIRED: weight slice s+3 into the
    // weight area of slice s-1, and token unit s+4 -- half the rows of two slices -- into the token areas
    // tgt_xa, tgt_xb, which the slices two and one, or three and two, steps back have left)
    // Within a step the source order is the issue order: behind every MFMA one fragment read for
    // the next 16 k until they are all issued, and one copy behind every third MFMA, which keeps the
    // demand on the vector memory pipe (64 B/clk per CU) uniform.
#if ALORA_PROBE
    const unsigned long long probe_loop_begin = __builtin_readcyclecounter();
#endif
    auto step = [&](int s, int par, const lds_byte *cur_x, const lds_byte *cur_w, const lds_byte *nxt_x, const lds_byte *nxt_w,
                    uint32_t tgt_xa, uint32_t tgt_xb, uint32_t tgt_w) {   // par = s % 2, a constant at every call
        // this wavefront's copies of slices <= s+1 have landed (those of slices s+2 .. s+NST-2 may be
        // in flight); behind the barrier that holds for every wavefront, and all of them are done
        // reading tgt
        asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(NC * (NST - 3)) : "memory");
        const int kb = kt0 + min(s + NST - 1, n_base - 1);
        const uint32_t sx = kb * xstep, sw = kb * wstep;
        constexpr int NM = 4 * NTW, CI = NTW == 2 ? 2 : 3;
#pragma unroll
        for (int gm = 0; gm < 2 * NM; ++gm) {
            // token tiles in snake order (0..3, 3..0, ...): across a change of the weight fragment the token
            // fragment stays, so one of the two operands repeats from every MFMA to the next.  The kernel
            // runs at the clock the power limit allows, and less switching on the operand paths is clock:
            // measured 1 to 3 % on the main loop; each accumulator still sees its slices in the same order.
            const int half = gm / NM, m = gm % NM, a = m / 4, b = (a & 1) ? 3 - m % 4 : m % 4;
            if (half == 0) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf0[a], xf0[b], acc[a][b], 0, 0, 0);
            else acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf1[a], xf1[b], acc[a][b], 0, 0, 0);
            // unit u of the other fragment buffer, in the order the MFMAs will want them: the first
            // five behind MFMAs 0..4, the rest behind every second MFMA after that
            const int u = m < 5 ? m : ((m - 5) % 2 == 0 ? 5 + (m - 5) / 2 : -1);
            if (u >= 0 && u < 4 + NTW && !(ALORA_PROBE & 2)) {
                if (half == 0) {
                    if (u == 0) wf1[0] = read_w(cur_w, 1, 0);
                    else if (u <= 4) xf1[u - 1] = read_x(cur_x, 1, u - 1);
                    else wf1[u - 4] = read_w(cur_w, 1, u - 4);
                } else {
                    if (u == 0) wf0[0] = read_w(nxt_w, 0, 0);
                    else if (u <= 4) xf0[u - 1] = read_x(nxt_x, 0, u - 1);
                    else wf0[u - 4] = read_w(nxt_w, 0, u - 4);
                }
            }
            if (gm % CI == 1 && gm / CI < NC && !(ALORA_PROBE & 1)) {
                const int c = gm / CI;
                if constexpr (PAIRED) {
                    if (c < 4) copy_unit(c, s + 4, par, tgt_xa, tgt_xb);
                    else copy_w(c - 4, s + 3, tgt_w);
                } else {
                    copy(c, rx, vxb, sx, rw, vwb, sw, tgt_xa, tgt_w);
                }
            }
        }
        // the same order, spelled out for the instruction scheduler (MFMA, then the LDS reads of its unit)
#pragma unroll
        for (int gm = 0; gm < 2 * NM; ++gm) {
            const int m = gm % NM;
            const int u = m < 5 ? m : ((m - 5) % 2 == 0 ? 5 + (m - 5) / 2 : -1);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (u >= 0 && u < 4 + NTW) {
                if (u >= 1 && u <= 4) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                else __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            }
        }
    };
    PROBE_STAMP(2);   // expand and select done
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(NC * (NST - 2)) : "memory");
    PROBE_STAMP(3);   // first slices landed
    load_frags(xa(0), wa(0), 0, wf0, xf0);
    // unrolled over one period of the rings, so that every area is a compile-time address
    constexpr int UNR = PAIRED ? 12 : NST;
    for (int s = 0; s < n_base; s += UNR) {
#pragma unroll
        for (int u = 0; u < UNR; ++u)
            if (u == 0 || s + u < n_base) {
                if constexpr (PAIRED)
                    step(s + u, u & 1, xa(u % NXA), wa(u % NWA), xa((u + 1) % NXA), wa((u + 1) % NWA),
                         sax[(u + 4 - (u & 1)) % NXA], sax[(u + 5 - (u & 1)) % NXA], saw[(u + 3) % NWA]);
                else
                    step(s + u, 0, xa(u), wa(u), xa((u + 1) % NST), wa((u + 1) % NST), sax[(u + NST - 1) % NST], 0u,
                         saw[(u + NST - 1) % NST]);
            }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    PROBE_STAMP(4);   // main loop done
#if ALORA_PROBE
    if (g_probe && lane == 0 && blockIdx.x < PROBE_MAX_WGS)
        g_probe[(size_t)PROBE_MAX_WGS * 8 + (size_t)blockIdx.x * 4 + w] = __builtin_readcyclecounter() - probe_loop_begin;
#endif

    // ---- 4. round and store ------------------------------------------------------------------
    // D[i][j]: i = feature (8g + 4*lh + jj, register 4g + jj), j = token (li).  Each wavefront turns
    // its 128 x 32*NTW block around through a private LDS strip, 32 token rows at a time (8-byte
    // writes of four consecutive features, 16-byte reads along the row), so that global stores are
    // whole row segments: 64*NTW contiguous bytes of q_out or of one cache slot per token.
    __syncthreads();  // every wavefront has finished reading the K-slice stages
    constexpr uint32_t STRIP_STEP = PAIRED ? 32768 : STAGE_BYTES;   // a wavefront's strip starts at w * STRIP_STEP
    if constexpr (PAIRED && !SPLIT) {
        slot_lds[tid] = slot_row;   // (behind wavefront 0's strip; the barrier below precedes every use)
        __syncthreads();
    }
    if (SPLIT) {
        // fp32 accumulators of this split, turned around through LDS like below: 16-byte writes of
        // four consecutive features, 16-byte reads along the row, row segments of 128*NTW bytes out
        constexpr int EP = 128 * NTW + 16;
        constexpr int LPR = 8 * NTW;           // lanes per row (four floats each)
        constexpr int RPI = 64 / LPR;
        lds_byte *strip = ring0 + w * STRIP_STEP;
        const int er = lane / LPR, ec = lane % LPR;
        const int n = n0 + wn * 32 * NTW + ec * 4;
        float *out = g.partial + (size_t)by * g.T * g.N;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
#pragma unroll
            for (int a = 0; a < NTW; ++a)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const f32x4 v = {acc[a][b][4 * gq + 0], acc[a][b][4 * gq + 1], acc[a][b][4 * gq + 2], acc[a][b][4 * gq + 3]};
                    *(__attribute__((address_space(3))) f32x4 *)(strip + li * EP + (a * 32 + 8 * gq + 4 * lh) * 4) = v;
                }
#pragma unroll
            for (int i = 0; i < (32 + RPI - 1) / RPI; ++i) {
                const int r = i * RPI + er;
                const int t = m0 + wt * 128 + b * 32 + r;
                if (er >= RPI || r >= 32 || t >= g.T || n >= g.N) continue;
                const f32x4 v = *(const __attribute__((address_space(3))) f32x4 *)(strip + r * EP + ec * 16);
                *(f32x4 *)(out + (size_t)t * g.N + n) = v;
            }
        }
    } else if (ROPE) {
        // Rotary embedding between the accumulators and the store.  NTW == 4 and heads of 128: a wavefront's
        // 128 features are one head, so both halves of every plane (i, i + 64) pass through its strip.  The
        // strip holds the unrounded fp32 rows (bias added); a lane takes 8 planes of a row -- features
        // 8c .. 8c+7 and the 8 that lie 64 further on, which share their angles -- turns them and rounds once.
        static_assert(!ROPE || NTW == 4, "a wavefront's strip must hold whole heads");
        constexpr int EP = 128 * NTW + 16;     // strip row pitch in bytes (fp32)
        constexpr int LPR = 2 * NTW;           // lanes per row (2 x 8 features each)
        constexpr int RPI = 64 / LPR;          // rows per store instruction
        lds_byte *strip = ring0 + w * STRIP_STEP;
        const int er = lane / LPR, ec = lane % LPR;
        const int n = n0 + wn * 32 * NTW + ec * 8;         // first of the lower 8 features; the upper 8 are n + 64
        u32x2 bias4[NTW][4];
#pragma unroll
        for (int a = 0; a < NTW; ++a)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int nf = n0 + wn * 32 * NTW + a * 32 + 8 * gq + 4 * lh;
                bias4[a][gq] = (u32x2){0u, 0u};
                if (g.bias && nf < g.N) bias4[a][gq] = *(const u32x2 *)(g.bias + nf);
            }
        int region = -1, col = 0;                          // the head lies in one region (N is a multiple of 128)
        if (n < g.N) {
            if (n < g.Nq) { region = 0; col = n; }
            else if (n < g.Nq + g.Nkv) { region = 1; col = n - g.Nq; }
            else { region = 2; col = n - g.Nq - g.Nkv; }
        }
        // positions of the tile's rows (clamped into the tables), kept behind the last wavefront's strip
        int *pos_lds = (int *)(ring + 120 * 1024);
        if (tid < BM) pos_lds[tid] = m0 + tid < g.T ? min(max(g.pos[m0 + tid], 0), g.rope_positions - 1) : 0;
        __syncthreads();
        auto angles = [&](int row, f32x4 (&cs)[4]) {      // cos and sin of the lane's 8 planes at the row's position
            const size_t at = (size_t)pos_lds[row] * 64 + 8 * ec;
            cs[0] = *(const f32x4 *)(g.rope_cos + at); cs[1] = *(const f32x4 *)(g.rope_cos + at + 4);
            cs[2] = *(const f32x4 *)(g.rope_sin + at); cs[3] = *(const f32x4 *)(g.rope_sin + at + 4);
        };
        constexpr int ITERS = 32 / RPI;
        f32x4 cs[4] = {}, cs_next[4] = {};
        if (region == 0 || region == 1) angles(wt * 128 + er, cs);
#pragma unroll
        for (int b = 0; b < 4; ++b) {
#pragma unroll
            for (int a = 0; a < NTW; ++a)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    f32x4 v = {acc[a][b][4 * gq + 0], acc[a][b][4 * gq + 1], acc[a][b][4 * gq + 2], acc[a][b][4 * gq + 3]};
                    v += (f32x4){__uint_as_float(bias4[a][gq].x << 16), __uint_as_float(bias4[a][gq].x & 0xffff0000u),
                                 __uint_as_float(bias4[a][gq].y << 16), __uint_as_float(bias4[a][gq].y & 0xffff0000u)};
                    *(__attribute__((address_space(3))) f32x4 *)(strip + li * EP + (a * 32 + 8 * gq + 4 * lh) * 4) = v;
                }
#pragma unroll
            for (int i = 0; i < ITERS; ++i) {
                const int r = i * RPI + er;
                const int row = wt * 128 + b * 32 + r;
                // the angles of the next row this lane handles are requested before this row's stores go out
                const int nxt = i + 1 < ITERS ? row + RPI : (b < 3 ? wt * 128 + (b + 1) * 32 + er : -1);
                if ((region == 0 || region == 1) && nxt >= 0) angles(nxt, cs_next);
                if (region >= 0 && m0 + row < g.T) {
                    const lds_byte *sr = strip + r * EP;
                    f32x4 lo0 = *(const __attribute__((address_space(3))) f32x4 *)(sr + ec * 32);
                    f32x4 lo1 = *(const __attribute__((address_space(3))) f32x4 *)(sr + ec * 32 + 16);
                    f32x4 hi0 = *(const __attribute__((address_space(3))) f32x4 *)(sr + 256 + ec * 32);
                    f32x4 hi1 = *(const __attribute__((address_space(3))) f32x4 *)(sr + 256 + ec * 32 + 16);
                    if (region != 2) {
                        const f32x4 a0 = lo0, a1 = lo1;
                        lo0 = a0 * cs[0] - hi0 * cs[2];
                        lo1 = a1 * cs[1] - hi1 * cs[3];
                        hi0 = hi0 * cs[0] + a0 * cs[2];
                        hi1 = hi1 * cs[1] + a1 * cs[3];
                    }
                    u32x4 vl, vh;
                    vl.x = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){lo0.x, lo0.y}, bf16x2));
                    vl.y = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){lo0.z, lo0.w}, bf16x2));
                    vl.z = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){lo1.x, lo1.y}, bf16x2));
                    vl.w = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){lo1.z, lo1.w}, bf16x2));
                    vh.x = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){hi0.x, hi0.y}, bf16x2));
                    vh.y = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){hi0.z, hi0.w}, bf16x2));
                    vh.z = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){hi1.x, hi1.y}, bf16x2));
                    vh.w = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){hi1.z, hi1.w}, bf16x2));
                    bf16_t *dst = nullptr;
                    if (region == 0) dst = g.q + (size_t)(m0 + row) * g.Nq + col;
                    else {
                        const int64_t sl = slot_lds[row];
                        if (sl >= 0) dst = (region == 1 ? g.kc : g.vc) + (size_t)sl * g.Nkv + col;
                    }
                    if (dst) {
                        *(u32x4 *)dst = vl;
                        *(u32x4 *)(dst + 64) = vh;
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) cs[u] = cs_next[u];
            }
        }
    } else {
        constexpr int EP = 64 * NTW + 16;      // strip row pitch in bytes
        constexpr int LPR = 4 * NTW;           // lanes per row (16 bytes each)
        constexpr int RPI = 64 / LPR;          // rows per store instruction
        lds_byte *strip = ring0 + w * STRIP_STEP;
        const int er = lane / LPR, ec = lane % LPR;
        const int n = n0 + wn * 32 * NTW + ec * 8;
        // destination of this lane's 8 features: 0 = q_out, 1 = K cache, 2 = V cache, -1 = none
        int region = -1, col = 0;
        if (er < RPI && n < g.N) {
            if (n < g.Nq) { region = 0; col = n; }
            else if (n < g.Nq + g.Nkv) { region = 1; col = n - g.Nq; }
            else { region = 2; col = n - g.Nq - g.Nkv; }
        }
        // The epilogue is bound by the number of instructions a wavefront issues, so per stored row segment it is
        // kept to one predicate and one 64-bit multiply-add: a lane's destination is base + index * pitch, where the
        // index is the token row (q_out) or the row's cache slot (K, V; negative: no write), and the layer bias is
        // only touched by calls that have one (two copies of the loop).
        bf16_t *const dbase = (region <= 0 ? g.q : region == 1 ? g.kc : g.vc) + col;
        const int64_t dpitch = region <= 0 ? g.Nq : g.Nkv;
        auto rounds = [&](auto has_bias) {
            constexpr bool BIAS = decltype(has_bias)::value;
            // bias of the four consecutive features this lane holds per (feature tile, register quad): part of the
            // base output of every row, added in fp32 before the one rounding; kept packed until it is added
            u32x2 bias4[NTW][4];
            if constexpr (BIAS) {
#pragma unroll
                for (int a = 0; a < NTW; ++a)
#pragma unroll
                    for (int gq = 0; gq < 4; ++gq) {
                        const int nf = n0 + wn * 32 * NTW + a * 32 + 8 * gq + 4 * lh;
                        bias4[a][gq] = (u32x2){0u, 0u};
                        if (nf < g.N) bias4[a][gq] = *(const u32x2 *)(g.bias + nf);
                    }
            }
#pragma unroll
            for (int b = 0; b < 4; ++b) {
#pragma unroll
                for (int a = 0; a < NTW; ++a) {
#pragma unroll
                    for (int gq = 0; gq < 4; ++gq) {
                        f32x2 p0 = {acc[a][b][4 * gq + 0], acc[a][b][4 * gq + 1]};
                        f32x2 p1 = {acc[a][b][4 * gq + 2], acc[a][b][4 * gq + 3]};
                        if constexpr (BIAS) {
                            p0 += (f32x2){__uint_as_float(bias4[a][gq].x << 16), __uint_as_float(bias4[a][gq].x & 0xffff0000u)};
                            p1 += (f32x2){__uint_as_float(bias4[a][gq].y << 16), __uint_as_float(bias4[a][gq].y & 0xffff0000u)};
                        }
                        u32x2 v;
                        v.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(p0, bf16x2));
                        v.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(p1, bf16x2));
                        *(__attribute__((address_space(3))) u32x2 *)(strip + li * EP + (a * 32 + 8 * gq + 4 * lh) * 2) = v;
                    }
                }
#pragma unroll
                for (int i = 0; i < (32 + RPI - 1) / RPI; ++i) {
                    const int r = i * RPI + er;
                    const int row = min(wt * 128 + b * 32 + r, BM - 1);   // (r can pass 31 in the last iteration: masked below)
                    const int64_t idx = region == 0 ? (int64_t)(m0 + row) : slot_lds[row];
                    const bool ok = (region >= 0) & (r < 32) & (m0 + row < g.T) & (idx >= 0);
                    if (ok) {
                        const u32x4 v = *(const __attribute__((address_space(3))) u32x4 *)(strip + r * EP + ec * 16);
                        *(u32x4 *)(dbase + idx * dpitch) = v;
                    }
                }
            }
        };
        if (g.bias) rounds(std::true_type{});
        else rounds(std::false_type{});
    }
#if ALORA_PROBE
    PROBE_STAMP(5);   // stores issued
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    PROBE_STAMP(6);   // stores left the wavefront
#endif
}

#if ALORA_PROBE
// Device buffer of at least alora_probe_buffer_bytes() bytes (zeroed by the caller) that the probe build's
// kernels write; null switches the recording off.  Exists in probe builds only.
extern "C" __attribute__((visibility("default"))) size_t alora_probe_buffer_bytes(void) { return (size_t)PROBE_MAX_WGS * (8 + 4) * 8; }
extern "C" __attribute__((visibility("default"))) int alora_probe_set_buffer(void *device_buffer)
{
    unsigned long long *p = (unsigned long long *)device_buffer;
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_probe), &p, sizeof(p));
}
#endif

// ---- host side: how a call of given sizes is tiled ---------------------------------------------
// Everything below depends on (T, hidden, N) and on the tuning overrides only, never on adapter
// data: a call in which every adapter id is -1 is tiled exactly like the adapted call, which is
// what makes rows that keep the base output bit-identical between the two.
// Process-wide override, one word (feature tiles in the low byte, splits above it) so that a reader never
// sees half of a new setting.
static std::atomic<int> g_force_tuning{0};

void set_gemm_tuning(int ntw, int splits) { g_force_tuning.store((ntw & 0xff) | (splits << 8), std::memory_order_relaxed); }

GemmPlan plan_gemm(int T, int H, int N)
{
    const int forced = g_force_tuning.load(std::memory_order_relaxed);
    const int g_force_ntw = forced & 0xff, g_force_splits = forced >> 8;
    constexpr int CUS = 256;                       // MI355X
    const int cand[3] = {4, 3, 2};
    const double unit[3] = {1.0, 0.78, 0.56};      // time of one K-slice relative to the 256-wide tile
    const int mtiles = (T + BM - 1) / BM, KT = H / KBLK;
    GemmPlan best = {4, 1, KT};
    double best_cost = 1e300;
    for (int i = 0; i < 3; ++i) {
        if (g_force_ntw && cand[i] != g_force_ntw) continue;
        const long tiles = (long)mtiles * ((N + 64 * cand[i] - 1) / (64 * cand[i]));
        // one workgroup per compute unit and round; with too few tiles to fill the chip, cut the
        // hidden dimension into splits (each split costs an extra pass over its fp32 partials)
        int max_splits = 1;
        if (tiles * 2 <= CUS) max_splits = (int)std::min<long>(std::min(8, KT), CUS / tiles);
        // A batch of one token tile leaves a quarter of the compute units to the workgroups that group and
        // shrink it inside the projection kernel (see prep_in_projection): measured 40 us per step against
        // 48 us when the projection takes 240 of the 256 units (decode batch of 256 rows, 8B shapes).
        if (mtiles == 1 && max_splits > 1) max_splits = (int)std::max<long>(1, std::min<long>(max_splits, (CUS - CUS / 4) / tiles));
        for (int sp = 1; sp <= max_splits; ++sp) {
            if (g_force_splits && sp != std::min(g_force_splits, std::min(8, KT))) continue;
            const int kps = (KT + sp - 1) / sp;
            const int eff = (KT + kps - 1) / kps;
            if (eff != sp) continue;
            const long rounds = (tiles * sp + CUS - 1) / CUS;
            const double cost = (double)rounds * (kps * unit[i] + 3.0) + (sp > 1 ? 4.0 + 0.6 * sp : 0.0);
            if (cost < best_cost - 1e-9) { best_cost = cost; best = {cand[i], sp, kps}; }
        }
    }
    return best;
}

size_t gemm_partial_bytes(int T, int H, int N)
{
    // room for the most splits any plan (or tuning override) can choose for these sizes
    (void)H;
    const long mtiles = (T + BM - 1) / BM;
    const bool may_split = mtiles * ((N + 255) / 256) * 2 <= 256;
    return may_split ? (size_t)8 * T * N * 4 : 0;
}

template <int NTW>
static void launch_ntw(const GemmArgs &g, const PtrTable &B, const PtrTable &A, hipStream_t stream)
{
    const dim3 block(GEMM_THREADS);
    if (g.splits > 1)
        hipLaunchKernelGGL((alora_gemm_bf16_kernel<NTW, true>), dim3(g.tiles8 * g.splits + g.prep_wgs), block, 0, stream, g, B, A);
    else if (NTW == 4 && g.rope_cos)
        hipLaunchKernelGGL((alora_gemm_bf16_kernel<4, false, true>), dim3(g.tiles8), block, 0, stream, g, B, A);
    else
        hipLaunchKernelGGL((alora_gemm_bf16_kernel<NTW, false>), dim3(g.tiles8), block, 0, stream, g, B, A);
}

// Decode-sized bf16 batches: classification, grouping and shrink run inside the split projection kernel,
// on workgroups behind its own (the projection of such a batch does not fill every compute unit).
bool prep_in_projection(const Fwd &f)
{
    if (f.dtype != ALORA_BF16 || f.L <= 0 || f.T <= 0 || f.T > GROUP_SMALL_ROWS || f.r > 32 || !f.block_rows) return false;
    const GemmPlan plan = plan_gemm(f.T, f.H, f.N);
    return plan.splits > 1 && plan.ntw == 2;
}

int launch_gemm_bf16(const Fwd &f, const PtrTable &B, const PtrTable &A, hipEvent_t after_projection)
{
    if (f.T == 0) return 0;
    GemmPlan plan = plan_gemm(f.T, f.H, f.N);
    // the fused rotary embedding wants whole heads of 128 in a wavefront's strip: 256-feature tiles (the number
    // of splits, which the shrink's layout depends on, stays what the sizes alone give; with splits the
    // finishing kernel rotates)
    if (f.rope_cos && plan.splits == 1) plan.ntw = 4;
    GemmArgs g;
    g.x = (const bf16_t *)f.x; g.W = (const bf16_t *)f.W; g.S_hl = (const bf16_t *)f.S;
    g.aeff = f.aeff; g.slot = f.slot;
    g.q = (bf16_t *)f.q; g.kc = (bf16_t *)f.kc; g.vc = (bf16_t *)f.vc;
    g.T = f.T; g.H = f.H; g.Nq = f.Nq; g.Nkv = f.Nkv; g.N = f.N; g.L = f.L; g.r = f.r;
    g.kx = 2 * f.r;
    g.mtiles = (f.T + BM - 1) / BM;
    g.ntiles = (f.N + 64 * plan.ntw - 1) / (64 * plan.ntw);
    g.kps = plan.kps * (KBLK / BK);
    g.partial = f.partial;
    g.bias = (const bf16_t *)f.bias;
    g.ranks = f.ranks;
    g.tiles8 = (g.mtiles * g.ntiles + 7) / 8 * 8;   // see the tile order in the kernel
    g.splits = plan.splits;
    const bool prep = prep_in_projection(f);
    // shrink ranges of the prep workgroups: about 1024 wide, at most 4, none empty
    const int want = std::max(1, std::min(4, f.H / 1024));
    g.prep_kper = ((f.H / 64 + want - 1) / want) * 64;
    g.prep_ranges = (f.H + g.prep_kper - 1) / g.prep_kper;
    g.prep_wgs = prep ? f.n_blocks * g.prep_ranges : 0;
    g.prep = GroupSmallArgs{f.aid, f.seg, f.pos, f.start, f.active, f.aeff, f.perm, f.offsets, f.blocktab, f.n_blocks, f.block_rows};
    g.S_out = f.S;
    g.rope_cos = f.rope_cos; g.rope_sin = f.rope_sin; g.pos = f.pos; g.rope_positions = f.rope_positions;
    if (plan.ntw == 4) launch_ntw<4>(g, B, A, f.stream);
    else if (plan.ntw == 3) launch_ntw<3>(g, B, A, f.stream);
    else launch_ntw<2>(g, B, A, f.stream);
    int e = (int)hipGetLastError();
    if (!e && after_projection) e = (int)hipEventRecord(after_projection, f.stream);
    if (e || plan.splits == 1) return e;
    return launch_finish_bf16(f, B, plan.splits, prep ? g.prep_ranges : plan_shrink(f.T, f.H, f.N, f.L, f.r).splits,
                              prep ? f.block_rows : nullptr);
}

}  // namespace alora
