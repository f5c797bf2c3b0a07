/*
 * CPU fp64 oracle for the activation-aware masked multi-adapter QKV projection
 * with paged K/V write (Activated LoRA serving).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU
 * library is checked against.  It shares no code with the GPU path and is never
 * called by it.  Everything is fp64, straight loops, summation in index order;
 * OpenMP only splits independent token rows across threads.
 *
 * Notation (paper Sec. 2.2-2.3, Algorithm 1, App. B):
 *   x [T,H]            layer input, one row per scheduled token of the flattened batch
 *   W [H,N]            fused base weight, N = Nq + 2*Nkv; columns [0,Nq) are Q,
 *                      [Nq,Nq+Nkv) are K, [Nq+Nkv,N) are V
 *   A_i [H,r], B_i [r,N]   low-rank factors of adapter i; Delta_i = A_i B_i
 *   aid[t]             adapter of token t, -1 = base model request
 *   seg[t], pos[t]     App. B's req_indices and position_within_req (absolute position)
 *   start[g]           App. B's inv_start: first adapted position of request g
 *
 * Every function here is pinned by the CPU tests (tests/test_oracle_*.py) against
 * hand-worked values, closed forms, merged-weight matmuls and invariants; none is
 * "parity unpinned".
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* App. B: the runner's mask is 1 where position_within_req < inv_start (keep base).
 * A row receives its adapter's delta iff it has an adapter and is NOT masked:
 * the row at the activation start itself is adapted (Sec. 2.3, "after the start of
 * the invocation sequence"). */
void oracle_classify(int64_t T, const int32_t *aid, const int32_t *seg, const int32_t *pos,
                     const int32_t *start, uint8_t *paper_mask, uint8_t *active)
{
    for (int64_t t = 0; t < T; ++t) {
        int keep_base = pos[t] < start[seg[t]];
        paper_mask[t] = (uint8_t)keep_base;
        active[t] = (uint8_t)(aid[t] >= 0 && !keep_base);
    }
}

/* Stable grouping of active rows by adapter: rows of adapter a, in increasing t,
 * occupy perm[offsets[a] .. offsets[a+1]). */
void oracle_group(int64_t T, int32_t L, const int32_t *aid, const uint8_t *active,
                  int32_t *perm, int32_t *offsets)
{
    for (int32_t a = 0; a <= L; ++a) offsets[a] = 0;
    for (int64_t t = 0; t < T; ++t)
        if (active[t]) offsets[aid[t] + 1] += 1;
    for (int32_t a = 0; a < L; ++a) offsets[a + 1] += offsets[a];
    int32_t n = 0;
    for (int32_t a = 0; a < L; ++a)
        for (int64_t t = 0; t < T; ++t)
            if (active[t] && aid[t] == a) perm[n++] = (int32_t)t;
}

/* Base projection of selected rows, y[i,:] = x[rows[i],:] W  (Algorithm 1, first step;
 * top rows of the Sec. 2.3 block equations).  Written as one dot product per output. */
void oracle_base_rows(int64_t n_rows, const int32_t *rows, int32_t H, int32_t N,
                      const double *x, const double *W, double *y)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_rows; ++i) {
        const double *xr = x + (size_t)rows[i] * H;
        for (int32_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int32_t k = 0; k < H; ++k) acc += xr[k] * W[(size_t)k * N + n];
            y[(size_t)i * N + n] = acc;
        }
    }
}

/* The aLoRA projection of selected rows (Sec. 2.3 block equations, select form):
 *   y = x W                       for every row
 *   y += (x A_a) B_a              iff active[t], a = aid[t]
 * Inactive rows never touch A or B. */
void oracle_alora_rows(int64_t n_rows, const int32_t *rows, int32_t H, int32_t N, int32_t r,
                       const double *x, const double *W,
                       const double *const *A, const double *const *B,
                       const int32_t *aid, const uint8_t *active, double *y)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_rows; ++i) {
        const int64_t t = rows[i];
        const double *xr = x + (size_t)t * H;
        double *yr = y + (size_t)i * N;
        for (int32_t n = 0; n < N; ++n) yr[n] = 0.0;
        for (int32_t k = 0; k < H; ++k) {
            const double xv = xr[k];
            const double *wr = W + (size_t)k * N;
            for (int32_t n = 0; n < N; ++n) yr[n] += xv * wr[n];
        }
        if (active[t]) {
            const double *Aa = A[aid[t]], *Ba = B[aid[t]];
            double s[256];
            for (int32_t j = 0; j < r; ++j) s[j] = 0.0;
            for (int32_t k = 0; k < H; ++k)
                for (int32_t j = 0; j < r; ++j) s[j] += xr[k] * Aa[(size_t)k * r + j];
            for (int32_t n = 0; n < N; ++n) {
                double d = 0.0;
                for (int32_t j = 0; j < r; ++j) d += s[j] * Ba[(size_t)j * N + n];
                yr[n] += d;
            }
        }
    }
}

/* The same projection with the layer's bias and one rank per adapter:
 *   y = x W + b                   for every row  (Algorithm 1: output = l.apply(x, b); b may be NULL)
 *   y += (x A_a) B_a              iff active[t], a = aid[t]; A_a is [H, ranks[a]], B_a is [ranks[a], N]
 *                                 (Sec. 4.1: adapters of different rank are served side by side) */
void oracle_alora_rows_var(int64_t n_rows, const int32_t *rows, int32_t H, int32_t N, const int32_t *ranks,
                           const double *x, const double *W, const double *bias,
                           const double *const *A, const double *const *B,
                           const int32_t *aid, const uint8_t *active, double *y)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_rows; ++i) {
        const int64_t tok = rows[i];
        const double *xt = x + (size_t)tok * H;
        double *yt = y + (size_t)i * N;
        for (int32_t n = 0; n < N; ++n) yt[n] = 0.0;
        for (int32_t k = 0; k < H; ++k) {
            const double xk = xt[k];
            const double *wk = W + (size_t)k * N;
            for (int32_t n = 0; n < N; ++n) yt[n] += xk * wk[n];
        }
        if (bias)
            for (int32_t n = 0; n < N; ++n) yt[n] += bias[n];
        if (active[tok]) {
            const int32_t ad = aid[tok], ra = ranks[ad];
            const double *Ar = A[ad], *Br = B[ad];
            double sv[256];
            for (int32_t j = 0; j < ra; ++j) sv[j] = 0.0;
            for (int32_t k = 0; k < H; ++k)
                for (int32_t j = 0; j < ra; ++j) sv[j] += xt[k] * Ar[(size_t)k * ra + j];
            for (int32_t n = 0; n < N; ++n) {
                double dl = 0.0;
                for (int32_t j = 0; j < ra; ++j) dl += sv[j] * Br[(size_t)j * N + n];
                yt[n] += dl;
            }
        }
    }
}

/* Algorithm 1 taken literally, for rows that have an adapter:
 *   base = apply(x); out = add_adapter(clone(base), x); final = base*mask + out*(1-mask)
 * with mask = 1 on pre-activation rows.  Rows of base-model requests (aid = -1) have no
 * adapter to add, so out = base there.  Agrees with the select form on finite data. */
void oracle_blend_rows(int64_t n_rows, const int32_t *rows, int32_t H, int32_t N, int32_t r,
                       const double *x, const double *W,
                       const double *const *A, const double *const *B,
                       const int32_t *aid, const uint8_t *paper_mask, double *y)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_rows; ++i) {
        const int64_t t = rows[i];
        const double *xr = x + (size_t)t * H;
        double *yr = y + (size_t)i * N;
        const double m = paper_mask[t] ? 1.0 : 0.0;
        for (int32_t n = 0; n < N; ++n) {
            double base = 0.0;
            for (int32_t k = 0; k < H; ++k) base += xr[k] * W[(size_t)k * N + n];
            double out = base;
            if (aid[t] >= 0) {
                const double *Aa = A[aid[t]], *Ba = B[aid[t]];
                double d = 0.0;
                for (int32_t j = 0; j < r; ++j) {
                    double s = 0.0;
                    for (int32_t k = 0; k < H; ++k) s += xr[k] * Aa[(size_t)k * r + j];
                    d += s * Ba[(size_t)j * N + n];
                }
                out = base + d;
            }
            yr[n] = base * m + out * (1.0 - m);
        }
    }
}

/* Paged layout: slot s lives in physical block s / block_size at offset s % block_size. */
void oracle_slot_coords(int64_t T, const int64_t *slot, int32_t block_size,
                        int64_t *block, int32_t *offset)
{
    for (int64_t t = 0; t < T; ++t) {
        if (slot[t] < 0) { block[t] = -1; offset[t] = -1; continue; }
        block[t] = slot[t] / block_size;
        offset[t] = (int32_t)(slot[t] % block_size);
    }
}

/* Split projected rows y [n_rows,N] (row i belongs to token rows[i]) into q_out and the
 * paged caches.  Caches are [num_blocks, block_size, Nkv]; a token with slot -1 writes no
 * K/V; every slot not named by a projected token keeps its contents. */
void oracle_store_rows(int64_t n_rows, const int32_t *rows, int32_t Nq, int32_t Nkv,
                       const double *y, const int64_t *slot, int32_t block_size,
                       double *q_out, double *k_cache, double *v_cache)
{
    const int32_t N = Nq + 2 * Nkv;
    for (int64_t i = 0; i < n_rows; ++i) {
        const int64_t t = rows[i];
        const double *yr = y + (size_t)i * N;
        for (int32_t c = 0; c < Nq; ++c) q_out[(size_t)t * Nq + c] = yr[c];
        if (slot[t] < 0) continue;
        const int64_t blk = slot[t] / block_size;
        const int64_t off = slot[t] % block_size;
        double *kd = k_cache + ((size_t)blk * block_size + off) * Nkv;
        double *vd = v_cache + ((size_t)blk * block_size + off) * Nkv;
        for (int32_t c = 0; c < Nkv; ++c) kd[c] = yr[Nq + c];
        for (int32_t c = 0; c < Nkv; ++c) vd[c] = yr[Nq + Nkv + c];
    }
}
