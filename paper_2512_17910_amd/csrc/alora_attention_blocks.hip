// Reader of the paged K/V cache for query rows that share a context: consecutive rows of one sequence
// (a projected suffix attending over a cached prefix, Sec. 2.3 / 4.2) are handled by ONE workgroup per
// K/V head, which loads every cached row once for all of them.  bf16, head_dim 128, on bf16 MFMA.
//
// A wavefront owns 16 columns (query row, query head of the K/V head's group): 16 / G rows; the eight
// wavefronts of a workgroup 128 / G consecutive rows, which share the K and V tiles of 32 context positions
// through LDS: every cached row is loaded once per 128 / G query rows.  Row blocks are cut at multiples of
// 128 / G of the POSITION, so whether a batch row leads a block is decided from the row before it alone.
// A workgroup owns a range of batch rows (chosen on the host: a whole row block for large batches, down to
// one row for a decode batch, where every row leads a block of its own) and works through the blocks that
// start in it; the range index is permuted so that the leading rows of a long run do not all fall to the
// same shader engine.
//
// For batches with few row blocks the context of every block is cut into parts, one workgroup each, which
// leave (running maximum, weight sum, unnormalised output) per column for the kernel that combines them.
//
// Per 32 context positions a wavefront runs two sets of 16x16x32 MFMAs that keep every column in the same
// four lanes (c, c+16, c+32, c+48) from the scores to the output:
//   scores^T [position x column] = K [position x d] . Q^T [d x column]   two tiles of 16 positions; K rows
//       from the LDS tile into the A operand (a lane holds 8 consecutive d of one position), Q in registers;
//   online softmax down each column: 8 accumulator registers per lane, two exchanges between the four
//       lanes of a column; no masking arithmetic on blocks that every column of the wavefront sees whole;
//   out^T [d x column] += V^T [d x position] . P [position x column]   eight tiles of 16 d; V comes back
//       from LDS with the transposing load, whose two halves are taken sixteen rows apart: that hands a
//       lane exactly the positions its score registers hold, so P is the score accumulator itself, rounded
//       to bf16.
// K and V rows go from global memory straight into LDS (no registers in between): four tile pairs, one being
// multiplied while three are on their way, one barrier per 32 positions; the block-table entries of 64 such
// steps sit in an LDS window.  An assembly statement never reads a register an MFMA writes (the compiler
// cannot place the wait states for it); the copies and their wait counts are assembly because the compiler's
// own bookkeeping would wait for all of them.
#include "alora_attention_internal.h"

namespace alora {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((address_space(3))) unsigned char lds_byte;

constexpr float AB_NEG_INF = -__builtin_inff();
constexpr float AB_M_FLOOR = -1.0e30f;   // finite floor of the running maximum (scores below it weigh nothing)

// four k of this lane's column, then the four that lie sixteen rows further on
__device__ __forceinline__ bf16x8 read_tr_frag(const lds_byte *p, int pitch)
{
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p + 16 * pitch));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// 16 bytes straight from global memory into LDS at lds_addr + 16 * lane.  An assembly statement: the
// kernel orders these copies against its LDS reads itself (wait counts and barriers in the main loop).
__device__ __forceinline__ void load_lds16(uint32_t lds_addr, const void *p)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_addr), "v"(p) : "memory");
}
// the same with a scalar base address and a 32-bit byte offset per lane
__device__ __forceinline__ void load_lds16(uint32_t lds_addr, const void *base, uint32_t voffset)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_addr), "v"(voffset), "s"(base) : "memory");
}
// Exchanges between the four lanes of a column (lanes c, c+16, c+32, c+48), as assembly statements (the
// builtin of the 32-lane swap returned its first result twice) with wait states on both sides, which the
// compiler cannot place for an instruction it does not see.  Checked with in-bounds probes:
//   v_permlane16_swap on two copies of x: ev <- x of the even 16-lane row of this lane's row pair, od <- the odd row's
//   v_permlane32_swap on two copies of x: lo <- x of the lower 32 lanes, hi <- the upper 32 lanes'
__device__ __forceinline__ void row_pair(float x, float &ev, float &od)
{
    ev = x, od = x;
    asm("s_nop 3\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 3" : "+v"(ev), "+v"(od));
}
__device__ __forceinline__ void both_halves(float x, float &lo, float &hi)
{
    lo = x, hi = x;
    asm("s_nop 3\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 3" : "+v"(lo), "+v"(hi));
}
__device__ __forceinline__ float max_over_column(float x)
{
    float a, b, c, d;
    row_pair(x, a, b);
    both_halves(fmaxf(a, b), c, d);
    return fmaxf(c, d);
}
__device__ __forceinline__ float sum_over_column(float x)
{
    float a, b, c, d;
    row_pair(x, a, b);
    both_halves(a + b, c, d);
    return c + d;
}

// what a lane loads for a position that is not part of the context (the weighted sum multiplies it by 0)
__device__ const uint32_t ab_zero_chunk[4] = {0u, 0u, 0u, 0u};

template <int G, bool POW2>   // POW2: the block size is a power of two (shifts instead of divisions)
__global__ __launch_bounds__(512, 4) void paged_attention_blocks_kernel(AttnArgs a, int R)
{
    constexpr int D = 128;
    constexpr int NW = 8;             // wavefronts per workgroup
    constexpr int RBW = 16 / G;       // query rows per wavefront (16 columns = rows x heads of the group)
    constexpr int RBG = NW * RBW;     // query rows per workgroup
    constexpr int PITCH = 256;        // bytes per position row of the K and V tiles in LDS
    constexpr int TILE = 32 * PITCH;  // one tile: 32 positions
    constexpr int NB = 4;             // (K, V) tile pairs: one is multiplied while three are on their way
    __shared__ __attribute__((aligned(1024))) unsigned char tiles[NB * 2 * TILE];
    __shared__ __attribute__((aligned(16))) unsigned char ok_bytes[NB][NW];     // byte w: validity of positions 4w .. 4w+3 of a pair
    __shared__ unsigned long long run_mask[2];
    constexpr int WIN = 64;            // blocks of 32 positions whose table entries the window below holds
    __shared__ int32_t window[WIN * 32 / 4 + 2];   // block sizes are multiples of 4

    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, c16 = lane & 15, g4 = lane >> 4;
    const int wu = __builtin_amdgcn_readfirstlane(w);
    // grid: (range of batch rows, K/V head, part of the context); a.splits parts, 1 = the whole context
    const int part = (int)blockIdx.x % a.splits, bid = (int)blockIdx.x / a.splits;
    const int hk = bid % a.Hkv;
    // ---- this workgroup's R batch rows (R a power of two <= 32, <= RBG) ------------------------------------
    // With R < RBG a long run of rows has a leading row in every (RBG / R)-th range only, and workgroups are
    // handed to the shader engines of an XCD in turn (four of them): without the exchange of the two low index
    // bits below, all the work of such a batch would land on one engine in four.
    int k = bid / a.Hkv;
    {
        const int n_ranges = (a.T + R - 1) / R, mm = RBG / R;
        if (mm > 1 && (k | 3) < n_ranges) k ^= (k / mm) & (mm >= 4 ? 3 : 1);
    }
    const int r_begin = k * R, r_end = min(a.T, r_begin + R);
    // which of them lead a block: a row does unless the row before it in the batch is the same sequence's
    // previous position and the position is not a multiple of RBG (then an earlier row leads)
    unsigned leaders;
    {
        bool lead = false;
        const int t = r_begin + lane;
        if (lane < R && t < r_end) {
            const int sq = a.seq[t], p0 = a.pos[t];
            const bool ok = sq >= 0 && sq < a.n_seqs && p0 >= 0;
            lead = !(ok && t > 0 && (p0 % RBG) != 0 && a.seq[t - 1] == sq && a.pos[t - 1] == p0 - 1);
        }
        leaders = (unsigned)__builtin_amdgcn_ballot_w64(lead);
    }
    const int Nkv = a.Hkv * D;
    const long long n_blocks = a.n_slots / a.bs;
    const long long cap = (long long)a.max_blocks * a.bs;
    const uint32_t tiles_at = (uint32_t)(uintptr_t)(lds_byte *)tiles;
    const uint32_t row_bytes = (uint32_t)Nkv * 2u, head_bytes = (uint32_t)hk * D * 2u;
    const unsigned n_blocks_u = (unsigned)(n_blocks < 0x7fffffffll ? n_blocks : 0x7fffffffll);
    // ---- copies global -> LDS: wavefront w fills positions 4w .. 4w+3 of a block of 32 with one K and one V
    // instruction (one cache block: block sizes are multiples of 4, so its table entry is a scalar); lane ->
    // position + lane / 16, physical 16-byte chunk lane % 16.
    // K tile: row = position, the physical chunk holds logical chunk XOR (row % 16) (the score product reads
    // one logical chunk of 16 rows).  V tile: row = position, XOR 4 * (row % 4) + 2 * (row / 4 % 2) (the
    // transposing read takes two chunks of four rows per 16 lanes, rows 4 apart in the next 16 lanes).
    const int row_c = 4 * wu + g4;                                   // this lane's position within a block of 32
    const uint32_t row_off = (uint32_t)g4 * (uint32_t)Nkv * 2u;
    const uint32_t k_off = row_off + (uint32_t)((c16 ^ (row_c & 15)) << 4);
    const uint32_t v_off = row_off + (uint32_t)((c16 ^ (((row_c & 3) << 2) | (((row_c >> 2) & 1) << 1))) << 4);
    // K fragment of position tile pt, k step ks: row 16pt + c16, chunk 4ks + g4 -> pt * 4096 + (k_base ^ (ks << 6))
    const uint32_t k_base = (uint32_t)c16 * PITCH + (uint32_t)((g4 ^ c16) << 4);
    // V fragment of d tile dt: rows 4g4 + j (then 16 further on), j = c16 / 4; the 8 bytes of d = 16dt + 4(c16 % 4) ..
    // -> v_base ^ (dt << 5)
    uint32_t v_base;
    {
        const int j = c16 >> 2, vrow = 4 * g4 + j;
        const int swz = (j << 2) | ((g4 & 1) << 1);
        v_base = (uint32_t)vrow * PITCH + (uint32_t)((swz ^ ((c16 & 3) >> 1)) << 4) + (uint32_t)((c16 & 1) << 3);
    }

  for (bool first = true; leaders; leaders &= leaders - 1, first = false) {
    const int t0 = r_begin + __builtin_ctz(leaders);
    if (!first) __syncthreads();      // everyone is done with the tiles and masks of the block before
    const int sq = a.seq[t0], p0 = a.pos[t0];
    const bool row_ok = sq >= 0 && sq < a.n_seqs && p0 >= 0;
    // rows of the block: up to the next multiple of RBG, as long as the run continues
    int nrows = 1;
    if (row_ok) {
        const int limit = RBG - (p0 % RBG);
        bool cont = tid == 0;
        if (tid > 0 && tid < limit && t0 + tid < a.T) cont = a.seq[t0 + tid] == sq && a.pos[t0 + tid] == p0 + tid;
        const unsigned long long mk = __builtin_amdgcn_ballot_w64(cont);
        if (lane == 0 && w < 2) run_mask[w] = mk;
        __syncthreads();
        nrows = 0;
#pragma unroll
        for (int ww = 0; ww < 2; ++ww) {
            const unsigned long long mw = run_mask[ww];
            if (nrows == 64 * ww) nrows += mw == ~0ull ? 64 : __builtin_ctzll(~mw);
        }
        nrows = __builtin_amdgcn_readfirstlane(nrows);
    }
    int n_ctx = 0;
    if (row_ok) n_ctx = (int)((long long)p0 + nrows < cap ? (long long)p0 + nrows : cap);
    // this workgroup's part of the context: blocks c_lo .. c_hi - 1 of 32 positions (all of them without parts)
    int c_lo = 0, c_hi = (n_ctx + 31) >> 5;
    if (a.splits > 1) {
        const int per = (c_hi + a.splits - 1) / a.splits;
        c_lo = min(part * per, c_hi);
        c_hi = min(c_lo + per, c_hi);
        n_ctx = min(n_ctx, 32 * c_hi);                 // positions past the part are not loaded
    }
    const int n_chunks = c_hi;
    const int32_t *bt = a.bt + (size_t)(row_ok ? sq : 0) * a.max_blocks;

    // this lane's column: query row r_j of the block (rows w*RBW .. of this wavefront), query head g_j
    const int r_j = w * RBW + c16 / G, g_j = c16 % G;
    const bool col_ok = row_ok && r_j < nrows;
    const int lim_j = col_ok ? p0 + r_j : -1;                        // last position the column attends to
    const int lim_w = (row_ok && wu * RBW < nrows) ? p0 + min((wu + 1) * RBW, nrows) - 1 : -1;   // ... and any column of this wavefront
    const int lim_first = p0 + wu * RBW;                             // ... and the wavefront's first column
    const size_t q_at = ((size_t)(t0 + (col_ok ? r_j : 0)) * a.Hq + (size_t)hk * G + g_j) * D;
    bf16x8 qf[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        u32x4 v = {0u, 0u, 0u, 0u};
        if (col_ok) v = *(const u32x4 *)((const bf16_t *)a.q + q_at + 32 * s + 8 * g4);
        qf[s] = __builtin_bit_cast(bf16x8, v);
    }
    // (a use of the query registers ahead of the loop: the compiler places its wait for these loads here and
    // not in front of the first MFMA of every step, where it would also wait for the copies in flight)
#pragma unroll
    for (int s = 0; s < 4; ++s) asm volatile("" : "+v"(qf[s]));

    f32x4 acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[t][e] = 0.f;
    float m = AB_M_FLOOR, l = 0.f;

    // Table entries come from a window in LDS that holds those of WIN blocks of 32 positions and is refilled
    // by the whole workgroup when the lookups reach its end (the index of four aligned positions is the same
    // in every lane); an entry past the context reads as -1.
    auto entry_of = [&](int pu) { return POW2 ? (pu >> a.bs_shift) : (pu / a.bs); };
    int win_first = 0, win_block = 0;        // table index of window[0]; first block the window covers
    auto refill = [&](int cw) {              // entries of blocks cw .. cw + WIN - 1; all wavefronts call it together
        win_block = cw;
        win_first = entry_of(32 * cw);
        const int last = entry_of(min(32 * (cw + WIN), n_ctx) - 1);      // n_ctx > 32 * cw whenever this is called
        __syncthreads();
        for (int i = tid; win_first + i <= last; i += 64 * NW) window[i] = bt[win_first + i];
        __syncthreads();
    };
    auto lookup = [&](int cb) {
        const int pu = cb + 4 * wu;
        return pu < n_ctx ? __builtin_amdgcn_readfirstlane(window[entry_of(pu) - win_first]) : -1;
    };
    // (the scalar unit of a CU serves all its wavefronts: what a wavefront computes per step besides the
    // matrix and vector work is kept to a few instructions)
    auto issue = [&](int c, int blk) {
        const int pu = 32 * c + 4 * wu;                          // first of the four positions
        const uint32_t k_to = tiles_at + ((uint32_t)(c & (NB - 1)) << 14) + ((uint32_t)wu << 10), v_to = k_to + TILE;
        static_assert(2 * TILE == 1 << 14 && 4 * PITCH == 1 << 10, "tile geometry");
        unsigned okb = 0xfu;
        if ((unsigned)blk < n_blocks_u && pu + 4 <= n_ctx) {   // the usual case: scalar base, the lane's constant offset
            const unsigned slot = (POW2 ? ((unsigned)blk << a.bs_shift) : (unsigned)blk * (unsigned)a.bs) + (unsigned)(POW2 ? (pu & (a.bs - 1)) : (pu % a.bs));
            const unsigned long long at = (unsigned long long)slot * row_bytes + head_bytes;   // first of the four cache rows
            load_lds16(k_to, (const char *)a.kc + at, k_off);
            load_lds16(v_to, (const char *)a.vc + at, v_off);
        } else {           // rows that are not part of the context read 16 zero bytes
            const bool blk_ok = (unsigned)blk < n_blocks_u;
            const int n_ok = blk_ok ? max(0, min(4, n_ctx - pu)) : 0;
            okb = (1u << n_ok) - 1u;
            const unsigned slot = (blk_ok ? (unsigned)blk * (unsigned)a.bs : 0u) + (unsigned)(pu % a.bs);
            const unsigned long long at = (unsigned long long)slot * row_bytes + head_bytes;
            const bool have = g4 < n_ok;
            const void *kp = have ? (const void *)((const char *)a.kc + at + k_off) : (const void *)ab_zero_chunk;
            const void *vp = have ? (const void *)((const char *)a.vc + at + v_off) : (const void *)ab_zero_chunk;
            load_lds16(k_to, kp);
            load_lds16(v_to, vp);
        }
        ok_bytes[c & (NB - 1)][wu] = (unsigned char)okb;      // (every lane writes the same byte)
    };

    auto consume = [&](int c) {
        const int cb = 32 * c;
        const lds_byte *kb = (const lds_byte *)tiles + (c & (NB - 1)) * (2 * TILE), *vb = kb + TILE;
        // ---- scores^T = K . Q^T : two tiles of 16 positions ------------------------------------------
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const bf16x8 k0 = *(const __attribute__((address_space(3))) bf16x8 *)(kb + (k_base ^ (uint32_t)(ks << 6)));
            const bf16x8 k1 = *(const __attribute__((address_space(3))) bf16x8 *)(kb + 16 * PITCH + (k_base ^ (uint32_t)(ks << 6)));
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, qf[ks], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, qf[ks], s1, 0, 0, 0);
        }
        // ---- softmax down this lane's column (its 32 positions sit in four lanes) --------------------
        __builtin_amdgcn_s_setprio(2);   // the vector arithmetic of this wavefront goes ahead of wavefronts waiting for the matrix unit
        const u32x2 ob = *(const u32x2 *)ok_bytes[c & (NB - 1)];
        const unsigned ok_lo = __builtin_amdgcn_readfirstlane(ob.x), ok_hi = __builtin_amdgcn_readfirstlane(ob.y);
        float sc[8] = {s0[0], s0[1], s0[2], s0[3], s1[0], s1[1], s1[2], s1[3]};
        if (!((ok_lo & ok_hi) == 0x0f0f0f0fu && cb + 31 <= lim_first)) {   // a block that every column of the wavefront sees whole needs no mask
            auto nibbles = [](unsigned x) { x |= x >> 4; return (x & 0xffu) | ((x >> 8) & 0xff00u); };
            const unsigned okmask = nibbles(ok_lo) | (nibbles(ok_hi) << 16);
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                const int idx = 16 * (v >> 2) + 4 * g4 + (v & 3);
                const bool on = ((okmask >> idx) & 1u) && cb + idx <= lim_j;
                sc[v] = on ? sc[v] : AB_NEG_INF;
            }
        }
        float mx = fmaxf(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3])), fmaxf(fmaxf(sc[4], sc[5]), fmaxf(sc[6], sc[7])));
        mx = max_over_column(mx);
        const float mn = fmaxf(m, mx * a.scale_log2e);
        const float corr = __builtin_amdgcn_exp2f(m - mn);
        m = mn;
        float ps = 0.f;
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            sc[v] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[v], a.scale_log2e, -mn));
            ps += sc[v];
        }
        l = l * corr + ps;
        if (__builtin_amdgcn_ballot_w64(corr != 1.f)) {
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[t][e] *= corr;
        }
        // ---- out^T += V^T . P : P straight from the score registers (positions 4g4 .. +3 and 16 + 4g4 .. +3) --
        const u32x4 pv = {pack_bf16(sc[0], sc[1]), pack_bf16(sc[2], sc[3]), pack_bf16(sc[4], sc[5]), pack_bf16(sc[6], sc[7])};
        __builtin_amdgcn_s_setprio(0);
        const bf16x8 pf = __builtin_bit_cast(bf16x8, pv);
#pragma unroll
        for (int t = 0; t < 8; ++t)
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(read_tr_frag(vb + (v_base ^ (uint32_t)(t << 5)), PITCH), pf, acc[t], 0, 0, 0);
    };

    // ---- the context, 32 positions at a time: all eight wavefronts share the tiles ------------------
    // Block c lives in tile pair c % 4.  In the step of block c every wavefront waits for its own copies of
    // block c (those of c+1 and c+2, two instructions each, stay in flight), the barrier makes that hold for
    // all of them and tells that block c-1 has been multiplied by everyone; its pair then takes the copies of
    // block c+3, whose table entry was looked up a step earlier.  Blocks past the context are copied too (all
    // zeros, from one 16-byte constant), which keeps the count of copies in flight the same in every step.
    {
        if (n_chunks > c_lo) refill(c_lo);
#pragma unroll
        for (int kk = 0; kk < NB - 1; ++kk) issue(c_lo + kk, lookup(32 * (c_lo + kk)));
        int b0 = lookup(32 * (c_lo + NB - 1));
        auto step = [&](int c) {
            asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            issue(c + NB - 1, b0);
            const int cn = c + NB;
            if (cn == win_block + WIN && 32 * cn < n_ctx) refill(cn);
            b0 = lookup(32 * cn);
        };
        // (two loops: the accumulators live in the first only)
        const int n_chunks_w = lim_w >= 0 ? min((lim_w >> 5) + 1, n_chunks) : 0;
        int c = c_lo;
        for (; c < n_chunks_w; ++c) {
            step(c);
            consume(c);
        }
        for (; c < n_chunks; ++c) step(c);
        // nothing may be on its way into LDS when the workgroup gives it back
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }

    // ---- the four lanes of a column add their weight sums; normalise and store ---------------------
    l = sum_over_column(l);
    if (a.splits > 1) {
        // this part's (running maximum, weight sum, unnormalised output) of every column, for the kernel that
        // combines the parts of a (row, query head) in part order
        if (col_ok || (!row_ok && w == 0 && c16 < G)) {
            float *pp = a.part + (((size_t)(t0 + (col_ok ? r_j : 0)) * a.Hq + (size_t)hk * G + g_j) * a.splits + part) * (D + 2);
            if (g4 == 0) *(f32x2 *)pp = (f32x2){m, l};
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                *(f32x2 *)(pp + 2 + 16 * t + 4 * g4) = (f32x2){acc[t][0], acc[t][1]};
                *(f32x2 *)(pp + 2 + 16 * t + 4 * g4 + 2) = (f32x2){acc[t][2], acc[t][3]};
            }
        }
        continue;
    }
    // a row that is not valid leads a block of its own and gets zeros
    if (col_ok || (!row_ok && w == 0 && c16 < G)) {
        const float inv = l > 0.f ? 1.f / l : 0.f;
        bf16_t *orow = (bf16_t *)a.out + ((size_t)(t0 + (col_ok ? r_j : 0)) * a.Hq + (size_t)hk * G + g_j) * D;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const u32x2 o = {pack_bf16(acc[t][0] * inv, acc[t][1] * inv), pack_bf16(acc[t][2] * inv, acc[t][3] * inv)};
            *(u32x2 *)(orow + 16 * t + 4 * g4) = o;
        }
    }
  }
}

int launch_attention_blocks(const AttnArgs &a, int G, hipStream_t stream)
{
    // batch rows per workgroup: a whole row block where that still makes a few workgroups per CU, fewer for
    // small batches (a decode batch: every row leads a block of its own)
    int R = 128 / G < 32 ? 128 / G : 32;
    // (with the context cut into parts the batch is small: whole row blocks per workgroup, the parts fill the chip)
    while (a.splits == 1 && R > 1 && (long long)((a.T + R - 1) / R) * a.Hkv < 2048) R /= 2;
    const dim3 grid((unsigned)((a.T + R - 1) / R) * (unsigned)a.Hkv * (unsigned)a.splits), block(512);
    const bool pow2 = a.bs_shift >= 0;
#define AB_LAUNCH(GG) \
    if (pow2) hipLaunchKernelGGL((paged_attention_blocks_kernel<GG, true>), grid, block, 0, stream, a, R); \
    else hipLaunchKernelGGL((paged_attention_blocks_kernel<GG, false>), grid, block, 0, stream, a, R)
    switch (G) {
    case 1: AB_LAUNCH(1); break;
    case 2: AB_LAUNCH(2); break;
    case 4: AB_LAUNCH(4); break;
    case 8: AB_LAUNCH(8); break;
    default: return (int)hipErrorInvalidValue;
    }
#undef AB_LAUNCH
    return (int)hipGetLastError();
}

}  // namespace alora
