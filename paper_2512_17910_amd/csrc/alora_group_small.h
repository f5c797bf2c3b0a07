// Row classification and grouping of a decode-sized batch (at most 256 rows) inside ONE workgroup
// of 256 threads, for one entry of the 32-row block table.
//
// The small-batch projection kernel runs the shrink of such a batch on the compute units its own
// workgroups leave free; each of those workgroups works out the whole grouping itself (one row per
// thread, a few microseconds) instead of waiting for a grouping kernel, and writes its share of the
// grouping step's results: its block-table entry, its block's slice of perm, the classification of
// 32 rows, and (entry 0) the group offsets.  The results are the same, bit for bit, as those of the
// grouping kernels: groups are the adapters in ascending order followed by the rows that keep the
// base output, rows inside a group in ascending order (App. B mask; Sec. 2.3).
#pragma once
#include "alora_internal.h"

namespace alora {

constexpr int GROUP_SMALL_ROWS = 256;
// ints of LDS scratch group_small needs: keys[256], tot/goff/bfirst[ALORA_MAX_ADAPTERS + 2] each, rows[32]
constexpr int GROUP_SMALL_SCRATCH = 256 + 3 * (ALORA_MAX_ADAPTERS + 2) + 32;

struct GroupSmallArgs {
    const int32_t *aid, *seg, *pos, *start;
    uint8_t *active;
    int8_t *aeff;
    int32_t *perm, *offsets;
    int4 *blocktab;
    int n_blocks;
    int32_t *block_rows;   // [n_blocks][32] row ids per entry, -1 padded
};

// Entry `e` of the block table of the batch: returns the group in `grp` (-1: unused entry), the
// number of rows in `cnt`, writes this entry's share of the results if `write`, and leaves the row ids in scr's last 32 ints (returned pointer; -1 = no
// row).  All 256 threads call; the caller may use the row ids after the call (it ends in a barrier).
__device__ __forceinline__ const int *group_small(const GroupSmallArgs &ga, int T, int L, int e, bool write, int *scr, int &grp,
                                                  int &cnt)
{
    int *keys = scr, *tot = scr + 256, *goff = tot + ALORA_MAX_ADAPTERS + 2, *bfirst = goff + ALORA_MAX_ADAPTERS + 2;
    int *rows = bfirst + ALORA_MAX_ADAPTERS + 2;
    const int tid = threadIdx.x;
    int key = -1;
    if (tid < T) {
        const int ae = effective_adapter(ga.aid, ga.seg, ga.pos, ga.start, tid);
        key = ae >= 0 ? ae : L;
    }
    keys[tid] = key;
    if (tid <= L) tot[tid] = 0;
    if (tid < 32) rows[tid] = -1;
    __syncthreads();
    if (key >= 0) atomicAdd(&tot[key], 1);   // counts only: their values do not depend on the order
    __syncthreads();
    // exclusive prefixes over the groups before each group: rows and 32-row blocks
    if (tid <= L + 1) {
        int rsum = 0, bsum = 0;
        for (int g2 = 0; g2 < tid; ++g2) {
            rsum += tot[g2];
            bsum += (tot[g2] + 31) >> 5;
        }
        goff[tid] = rsum;
        bfirst[tid] = bsum;
    }
    // rank of this row inside its group: rows before it with the same key
    int rank = 0;
    for (int t2 = 0; t2 < T; ++t2) rank += (t2 < tid) & (keys[t2] == key);
    __syncthreads();
    grp = -1;
    cnt = 0;
    int j0 = 0, b = 0;
    if (e < bfirst[L + 1]) {
        int lo = 0, hi = L;   // smallest group whose blocks end after e
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (bfirst[mid + 1] > e) hi = mid; else lo = mid + 1;
        }
        grp = lo;
        b = e - bfirst[lo];
        j0 = goff[lo] + 32 * b;
        cnt = min(32, tot[lo] - 32 * b);
    }
    if (grp >= 0 && key == grp && rank >= 32 * b && rank < 32 * b + 32) rows[rank - 32 * b] = tid;
    __syncthreads();
    // this workgroup's share of the grouping results (one writer per entry)
    if (!write) return rows;
    if (e < ga.n_blocks && tid == 0) ga.blocktab[e] = grp >= 0 ? make_int4(grp, j0, cnt, 0) : make_int4(-1, 0, 0, 0);
    if (tid < cnt) ga.perm[j0 + tid] = rows[tid];
    if (e < ga.n_blocks && tid < 32) ga.block_rows[32 * e + tid] = rows[tid];
    if (e == 0 && tid <= L + 1) ga.offsets[tid] = goff[tid];
    if (tid < 32) {
        const int t = 32 * e + tid;
        if (t < T) {
            const int k = keys[t];
            ga.aeff[t] = (int8_t)(k == L ? -1 : k);
            ga.active[t] = (uint8_t)(k != L);
        }
    }
    return rows;
}

}  // namespace alora
