// LoRA shrink for bf16 batches: S[t,:] = x[t,:] . A[a] for adapted rows only, on bf16 MFMA with
// fp32 accumulation.  Rows come from the grouped list (adapter-major, stable): a workgroup takes
// 32 rows of ONE adapter and one range of the hidden dimension (blockIdx.y).
//
// A workgroup pulls its 32 token rows and the whole of its adapter's A (for its range) through one
// compute unit's vector memory pipe (64 B/clk), which is what bounds it once the loads overlap; so
// it streams: its range is cut into chunks, two LDS buffers alternate, and all loads of a chunk are
// issued at once as direct-to-LDS copies (the gathered token rows, 16-byte chunks XOR-swizzled by
// row; the adapter's A rows copied verbatim, they are already k-major) while the previous chunk
// runs its MFMAs out of LDS (ds_read_b128 for tokens, the transposing ds_read_b64_tr_b16 for A).
// The four wavefronts split every chunk's k steps; their partial sums are added in fixed order at
// the end.
//
// Two forms of the result, chosen by the host with the projection's plan:
//   - prefill-sized batches (fused projection kernel): the fp32 result is handed on as two bf16
//     numbers per element, S = hi + lo with hi = bf16(S), lo = bf16(S - hi), stored as
//     [hi_0..hi_{r-1} | lo_0..lo_{r-1}] per row: the projection kernel runs the expand on the same
//     bf16 MFMA pipe as the base GEMM ([S_hi | S_lo] against [B ; B]) and still sees ~16 mantissa
//     bits of S.  The workgroups walk a work list the grouping step wrote: with few adapted blocks
//     every block is cut into ranges of the hidden dimension (one workgroup each, about one per
//     compute unit in all); a range stores its fp32 partial, and the LAST range of a block to
//     finish (a counter per block) adds the block's partials in range order and stores (hi, lo) --
//     the sum does not depend on which range came last;
//   - small batches (split projection + finishing kernel): every range leaves an fp32 partial
//     P[range][t][:], and the finishing kernel adds the ranges in fixed order.
#include <algorithm>
#include "alora_internal.h"
#include "alora_shrink_rows.h"

namespace alora {


// KSL: hidden-dimension chunk per LDS buffer; NT: 32-wide rank tiles (1 for rank <= 32, else 2)
// WORK_LIST: walk the (block, range) items of the grouping step and combine the ranges of a block
// here; otherwise walk the block table with blockIdx.y as the range.
template <int KSL, int NT, bool WORK_LIST>
__global__ __launch_bounds__(256) void shrink_bf16_kernel(const bf16_t *__restrict__ x, PtrTable A, RankTable ranks,
                                                          const int32_t *__restrict__ perm,
                                                          const int4 *__restrict__ blocktab, int32_t *counters, int L, int H,
                                                          int r, uint32_t x_bytes, int T, int kper, void *S_out)
{
    typedef ShrinkLds<KSL, NT> Lds;
    // separate LDS objects per buffer: reads of one do not wait for copies into the other
    __shared__ __attribute__((aligned(16))) unsigned char xs0[Lds::X_BYTES], xs1[Lds::X_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char as0[Lds::A_BYTES], as1[Lds::A_BYTES];
    __shared__ float red[4][NT][32][33];
    __shared__ int rows_t[SHRINK_ROWS];
    __shared__ int is_last;

    // which (adapter, 32-row block) is this workgroup?  (table written by the grouping kernel)
    const int4 entry = blocktab[blockIdx.x];
    const int a = entry.x, j0 = entry.y, cnt = WORK_LIST ? (entry.z & 0xff) : entry.z;
    if (a < 0 || a >= L) return;  // unused entry or the base group; uniform across the workgroup
    // this workgroup's range of the hidden dimension (sized so that none is empty)
    const int range = WORK_LIST ? (entry.w & 15) : (int)blockIdx.y;
    const int n_ranges = WORK_LIST ? ((entry.w >> 4) & 15) : (int)gridDim.y;
    if (WORK_LIST) kper = (entry.z >> 8) * 64;
    if (kper <= 0 || kper > H + 63 || range < 0 || range >= n_ranges || n_ranges > ALORA_SHRINK_MAX_SPLITS) return;
    const int kbeg = range * kper, kend = min(H, kbeg + kper);

    const int tid = threadIdx.x;
    // (the table and perm may be what an earlier call left in the workspace: indices are range-checked)
    if (j0 < 0 || cnt < 0 || cnt > SHRINK_ROWS || j0 + cnt > T || n_ranges < 1 || kbeg >= H) return;
    if (WORK_LIST && (uint32_t)(entry.w >> 8) >= gridDim.x) return;
    if (tid < SHRINK_ROWS) {
        const int t = tid < cnt ? perm[j0 + tid] : -1;
        rows_t[tid] = (t >= 0 && t < T) ? t : -1;
    }
    __syncthreads();
    // this adapter's rank (multiple of 8): A_a is [H, rk]; S keeps the common pitch r
    shrink_rows<KSL, NT, WORK_LIST>(x, (const bf16_t *)A.p[a], ranks.r[a], rows_t, H, r, x_bytes, T, kbeg, kend, range, n_ranges,
                                    WORK_LIST ? counters + (entry.w >> 8) : nullptr, S_out, xs0, xs1, as0, as1, red, &is_last);
}

// Ranges of the hidden dimension the shrink is cut into, never more than 8, each a multiple of 64 wide
// and none empty.  Small-batch path (split projection + finishing kernel): fixed by the host, about 512
// workgroups' worth of row blocks at most.  Prefill-sized path: one range unless a block's loads are large
// (wide hidden dimension, high rank); then `splits` is the upper limit (ranges at least 512 wide) and the
// grouping step picks the number per call from the adapted blocks it finds.
ShrinkPlan plan_shrink(int T, int H, int N, int L, int r)
{
    ShrinkPlan p = {1, H, false};
    if (T <= 0 || L <= 0) return p;
    if (plan_gemm(T, H, N).splits == 1) {
        // Cutting a block into ranges adds a chain of round trips past the L2 (partials written through,
        // counter, partials read back: about 6 us); it pays once a block's 32 token rows and its adapter's
        // A, all pulled through one compute unit, take clearly longer than that (0.5 MB is about 11 us).
        if ((size_t)(SHRINK_ROWS + r) * H * 2 >= (768u << 10)) {
            p.splits = std::max(1, std::min(ALORA_SHRINK_MAX_SPLITS, H / 512));
            p.combine = p.splits > 1;
        }
        return p;
    }
    const int want = std::max(1, std::min(ALORA_SHRINK_MAX_SPLITS, 512 / group_blocks(T, L)));
    const int k64 = H / 64;
    p.kper = ((k64 + want - 1) / want) * 64;
    p.splits = (H + p.kper - 1) / p.kper;
    return p;
}

template <int KSL, int NT>
static void launch_shrink(const Fwd &f, const PtrTable &A, const ShrinkPlan &sp)
{
    const uint32_t x_bytes = (uint32_t)((size_t)f.T * f.H * 2);
    if (sp.combine)
        hipLaunchKernelGGL((shrink_bf16_kernel<KSL, NT, true>), dim3(f.n_items), dim3(256), 0, f.stream, (const bf16_t *)f.x, A,
                           f.ranks, f.perm, (const int4 *)f.items, f.counters, f.L, f.H, f.r, x_bytes, f.T, 0, f.S);
    else
        hipLaunchKernelGGL((shrink_bf16_kernel<KSL, NT, false>), dim3(f.n_blocks, sp.splits), dim3(256), 0, f.stream,
                           (const bf16_t *)f.x, A, f.ranks, f.perm, (const int4 *)f.blocktab, (int32_t *)nullptr, f.L, f.H, f.r,
                           x_bytes, f.T, sp.kper, f.S);
}

int launch_shrink_bf16(const Fwd &f, const PtrTable &A)
{
    if (f.T == 0 || f.L == 0) return 0;
    const ShrinkPlan sp = plan_shrink(f.T, f.H, f.N, f.L, f.r);
    if (sp.combine && !f.items) return (int)hipErrorInvalidValue;
    if (f.r <= 32) launch_shrink<512, 1>(f, A, sp);
    else launch_shrink<256, 2>(f, A, sp);
    return (int)hipGetLastError();
}

}  // namespace alora
