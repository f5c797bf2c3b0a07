// C ABI of libalora_qkv: argument checking, workspace carving and the launch sequence.
// Host code only; every step of the path runs in the kernels of the other translation units.
#include <new>
#include <vector>
#include <algorithm>
#include <mutex>
#include "alora_internal.h"
#include "alora_planner.h"

namespace alora {

static thread_local int g_last_hip_error = 0;
void note_hip_error(int hip_error) { g_last_hip_error = hip_error; }

// Benchmark aid: HIP events around the dominant kernel (the projection GEMM) of each forward call.
struct Profile {
    bool on = false;
    int used = 0;
    int every = 1, seen = 0;   // every `every`-th call is measured
    std::vector<hipEvent_t> ev0, ev1;
};
static Profile g_prof;
static std::mutex g_prof_mutex;   // forward calls of several host threads may meet the benchmark aid

static inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

struct Layout {
    size_t active, aeff, perm, offsets, S, blocktab, items, counters, block_rows, hist, partial, total;
    int n_blocks, n_items;
};

static int check_dims(const alora_dims *d)
{
    if (!d) return ALORA_EINVAL;
    if (d->dtype != ALORA_F32 && d->dtype != ALORA_BF16) return ALORA_EINVAL;
    if (d->T < 0 || d->hidden <= 0 || d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->head_dim <= 0 ||
        d->n_adapters < 0 || d->n_segments < 0 || d->n_slots < 0 || d->rank < 0)
        return ALORA_EINVAL;
    const long long Nq = (long long)d->n_q_heads * d->head_dim, Nkv = (long long)d->n_kv_heads * d->head_dim;
    if (Nq + 2 * Nkv > (1ll << 30) || (long long)d->T * d->hidden > (1ll << 40)) return ALORA_ESHAPE;
    if (d->n_adapters > ALORA_MAX_ADAPTERS) return ALORA_ESHAPE;
    if (d->n_adapters > 0 && (d->rank < 1 || d->rank > ALORA_MAX_RANK)) return ALORA_ESHAPE;
    if (d->dtype == ALORA_BF16) {
        if (d->hidden % 64 || Nq % 8 || Nkv % 8) return ALORA_ESHAPE;
        if (d->n_adapters > 0 && d->rank % 8) return ALORA_ESHAPE;
        // 32-bit byte offsets inside the weight matrix (buffer addressing; the projection's descriptors start
        // 4 KiB before the matrix and offsets from 2^31 on mark masked lanes)
        if ((long long)d->hidden * (Nq + 2 * Nkv) * 2 + 4096 >= (1ll << 31)) return ALORA_ESHAPE;
        // 32-bit byte offsets of the gathered token rows in the shrink
        if (d->n_adapters > 0 && (long long)d->T * d->hidden * 2 > 0xfffffff0ll) return ALORA_ESHAPE;
    } else {
        if (d->hidden % 4 || Nq % 4 || Nkv % 4) return ALORA_ESHAPE;
    }
    return ALORA_OK;
}

static Layout make_layout(const alora_dims *d)
{
    Layout l;
    const size_t T = (size_t)d->T, L = (size_t)d->n_adapters, r = (size_t)d->rank;
    size_t o = 0;
    l.active = o;  o += up256(T);
    l.aeff = o;    o += up256(T);
    l.perm = o;    o += up256(4 * T);
    l.offsets = o; o += up256(4 * (L + 2));
    // fp32 shrink result; the bf16 path keeps one partial per range of the hidden dimension
    l.S = o;       o += up256(T * r * 4 * (d->dtype == ALORA_BF16 ? (size_t)ALORA_SHRINK_MAX_SPLITS : 1));
    l.n_blocks = group_blocks(d->T, d->n_adapters);
    l.blocktab = o; o += up256(16 * (size_t)l.n_blocks);
    l.n_items = d->dtype == ALORA_BF16 ? shrink_items(d->T, d->n_adapters) : 0;
    l.items = o;    o += up256(16 * (size_t)l.n_items);
    l.counters = o; o += up256(4 * (size_t)l.n_items);   // one per block; indexed below n_items
    l.block_rows = o; o += up256(d->dtype == ALORA_BF16 && d->T <= 256 ? 4 * 32 * (size_t)l.n_blocks : 0);
    l.hist = o;     o += up256(group_hist_bytes(d->T));
    l.partial = o;
    if (d->dtype == ALORA_BF16) o += up256(gemm_partial_bytes(d->T, d->hidden, (d->n_q_heads + 2 * d->n_kv_heads) * d->head_dim));
    l.total = std::max<size_t>(o, 256);
    return l;
}

static int check_ws(const alora_dims *d, const void *ws, size_t bytes, Layout *l)
{
    *l = make_layout(d);
    if (!ws || ((uintptr_t)ws & 255) || bytes < l->total) return ALORA_EWORKSPACE;
    return ALORA_OK;
}

static bool misaligned16(const void *p) { return ((uintptr_t)p & 15) != 0; }

static void fill_common(Fwd &f, const alora_dims *d, const Layout &l, void *ws, void *stream)
{
    f.dtype = d->dtype; f.T = d->T; f.H = d->hidden;
    f.Nq = d->n_q_heads * d->head_dim; f.Nkv = d->n_kv_heads * d->head_dim; f.N = f.Nq + 2 * f.Nkv;
    f.L = d->n_adapters; f.r = d->rank; f.G = d->n_segments; f.n_slots = d->n_slots;
    f.seg = d->token_seg_ids; f.pos = d->token_positions;
    unsigned char *b = (unsigned char *)ws;
    f.active = b + l.active;
    f.aeff = (int8_t *)(b + l.aeff);
    f.perm = (int32_t *)(b + l.perm);
    f.offsets = (int32_t *)(b + l.offsets);
    f.S = b + l.S;
    f.blocktab = (int4 *)(b + l.blocktab);
    f.hist = (int32_t *)(b + l.hist);
    const int N_all = (d->n_q_heads + 2 * d->n_kv_heads) * d->head_dim;
    const bool work_list = d->dtype == ALORA_BF16 && plan_shrink(d->T, d->hidden, N_all, d->n_adapters, d->rank).combine;
    f.items = work_list ? (int4 *)(b + l.items) : nullptr;
    f.counters = work_list ? (int32_t *)(b + l.counters) : nullptr;
    f.n_items = work_list ? l.n_items : 0;
    f.block_rows = (d->dtype == ALORA_BF16 && d->T <= 256) ? (int32_t *)(b + l.block_rows) : nullptr;
    f.partial = (float *)(b + l.partial);
    f.n_blocks = l.n_blocks;
    f.stream = (hipStream_t)stream;
}

}  // namespace alora

// ---- the entry point that allocates nothing ------------------------------------------------------
// The workspace of the call is a file-scope device array: every GPU the library runs on holds its own
// copy, at its own address, until the process ends.  Host code never uses the array's name as an
// address; it asks the runtime for the device address once per device and passes that on.
// (No "used" attribute on it: the compiler gives a static device variable that host code names
// external visibility in the code object, which is how the runtime finds it by name; marked "used"
// it stays a local symbol and the look-up fails.)
static __device__ __align__(256) unsigned char scratch[ALORA_STATIC_SCRATCH_BYTES];

namespace alora {
constexpr int MAX_DEVICES = 64;
static void *g_scratch_ptr[MAX_DEVICES];
static std::mutex g_scratch_mutex;

// device address of `scratch` on the current device (looked up on the first call per device)
static int static_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e) { g_last_hip_error = (int)e; return ALORA_EHIP; }
    if (dev < 0 || dev >= MAX_DEVICES) return ALORA_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e || !p) { g_last_hip_error = (int)e; return ALORA_EHIP; }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ALORA_OK;
}
}  // namespace alora

using namespace alora;

extern "C" {

int alora_qkv_version(void) { return 100; }

int alora_last_hip_error(void) { return g_last_hip_error; }

const char *alora_status_string(int s)
{
    switch (s) {
    case ALORA_OK: return "ok";
    case ALORA_EINVAL: return "invalid argument (null or misaligned pointer, negative size, unknown dtype)";
    case ALORA_ESHAPE: return "unsupported shape (see the shape limits in alora_qkv.h)";
    case ALORA_EWORKSPACE: return "workspace missing, not 256-byte aligned, or too small";
    case ALORA_EHIP: return "a HIP call failed (see alora_last_hip_error)";
    case ALORA_EDATA: return "device data violates a documented precondition";
    case ALORA_ENOMEM: return "a host-side allocation failed";
    case ALORA_ETOOBIG: return "the call needs more scratch than the static device array holds (alora_qkv_forward_static)";
    case ALORA_ENOBLOCKS: return "not enough free cache blocks (planner)";
    default: return "unknown status";
    }
}

int alora_qkv_workspace_bytes(const alora_dims *dims, size_t *out_bytes)
{
    if (!out_bytes) return ALORA_EINVAL;
    int s = check_dims(dims);
    if (s) return s;
    *out_bytes = make_layout(dims).total;
    return ALORA_OK;
}

int alora_qkv_workspace_layout(const alora_dims *dims, alora_ws_layout *out)
{
    if (!out) return ALORA_EINVAL;
    int s = check_dims(dims);
    if (s) return s;
    const Layout l = make_layout(dims);
    out->active_off = l.active;
    out->perm_off = l.perm;
    out->offsets_off = l.offsets;
    out->total_bytes = l.total;
    return ALORA_OK;
}

int alora_qkv_classify_group(const int32_t *token_adapter_ids, const int32_t *activation_start,
                             const alora_dims *dims, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int s = check_dims(dims);
    if (s) return s;
    if (dims->T > 0 && (!token_adapter_ids || !dims->token_seg_ids || !dims->token_positions)) return ALORA_EINVAL;
    if (dims->T > 0 && dims->n_segments > 0 && !activation_start) return ALORA_EINVAL;
    Layout l;
    s = check_ws(dims, workspace, workspace_bytes, &l);
    if (s) return s;
    Fwd f = {};
    fill_common(f, dims, l, workspace, hip_stream);
    f.aid = token_adapter_ids; f.start = activation_start;
    int e = launch_classify_group(f);
    if (e) { g_last_hip_error = e; return ALORA_EHIP; }
    return ALORA_OK;
}

// Argument checks and the launch sequence of one forward call.  `allow_timing`: the benchmark's
// event pairs may be recorded (never while the stream is being captured).
static int forward_on(const void *x, const int32_t *token_adapter_ids, const int32_t *activation_start,
                      const void *W_qkv, const void *const *A, const void *const *B, void *q_out, void *k_cache,
                      void *v_cache, const int64_t *slot_mapping, int32_t block_size, const alora_dims *dims,
                      void *workspace, size_t workspace_bytes, void *hip_stream, bool allow_timing,
                      const alora_extras *extras = nullptr)
{
    int s = check_dims(dims);
    if (s) return s;
    if (block_size <= 0) return ALORA_EINVAL;
    if (dims->n_slots % block_size) return ALORA_ESHAPE;
    if (dims->T > 0) {
        if (!x || !token_adapter_ids || !W_qkv || !q_out || !slot_mapping || !dims->token_seg_ids ||
            !dims->token_positions)
            return ALORA_EINVAL;
        if (dims->n_slots > 0 && (!k_cache || !v_cache)) return ALORA_EINVAL;
        if (dims->n_segments > 0 && !activation_start) return ALORA_EINVAL;
        if (misaligned16(x) || misaligned16(W_qkv) || misaligned16(q_out) || misaligned16(k_cache) ||
            misaligned16(v_cache))
            return ALORA_EINVAL;
    }
    PtrTable ta = {}, tb = {};
    if (dims->n_adapters > 0) {
        if (!A || !B) return ALORA_EINVAL;
        for (int i = 0; i < dims->n_adapters; ++i) {
            if (!A[i] || !B[i] || misaligned16(A[i]) || misaligned16(B[i])) return ALORA_EINVAL;
            ta.p[i] = A[i];
            tb.p[i] = B[i];
        }
    }
    RankTable ranks;
    for (int i = 0; i < ALORA_MAX_ADAPTERS; ++i) ranks.r[i] = (uint8_t)dims->rank;
    const void *bias = nullptr;
    const bool reuse_grouping = extras && extras->reuse_grouping != 0;
    if (extras) {
        bias = extras->bias;
        if (bias && misaligned16(bias)) return ALORA_EINVAL;
        if ((extras->rope_cos != nullptr) != (extras->rope_sin != nullptr)) return ALORA_EINVAL;
        if (extras->rope_cos) {
            if (misaligned16(extras->rope_cos) || misaligned16(extras->rope_sin) || extras->rope_positions < 1) return ALORA_EINVAL;
            if (dims->head_dim % 2 || (dims->dtype == ALORA_BF16 && dims->head_dim != 128)) return ALORA_ESHAPE;
        }
        if (extras->adapter_ranks) {
            for (int i = 0; i < dims->n_adapters; ++i) {
                const int ri = extras->adapter_ranks[i];
                if (ri < 1 || ri > dims->rank) return ALORA_ESHAPE;
                if (dims->dtype == ALORA_BF16 && ri % 8) return ALORA_ESHAPE;
                ranks.r[i] = (uint8_t)ri;
            }
        }
    }
    Layout l;
    s = check_ws(dims, workspace, workspace_bytes, &l);
    if (s) return s;
    if (dims->T == 0) return ALORA_OK;

    Fwd f = {};
    fill_common(f, dims, l, workspace, hip_stream);
    f.bias = bias;
    f.ranks = ranks;
    f.D = dims->head_dim;
    if (extras && extras->rope_cos) { f.rope_cos = extras->rope_cos; f.rope_sin = extras->rope_sin; f.rope_positions = extras->rope_positions; }
    f.block_size = block_size;
    f.x = x; f.W = W_qkv; f.aid = token_adapter_ids; f.start = activation_start; f.slot = slot_mapping;
    f.q = q_out; f.kc = k_cache; f.vc = v_cache;

    // (the lock is held over the launches only while the benchmark aid is switched on)
    std::unique_lock<std::mutex> prof_lock(g_prof_mutex, std::defer_lock);
    bool timed = false;
    if (allow_timing) {
        prof_lock.lock();
        timed = g_prof.on && g_prof.used < (int)g_prof.ev0.size();
        if (timed) timed = (g_prof.seen++ % g_prof.every) == 0;
        if (!timed) prof_lock.unlock();
    }
    // decode-sized bf16 batches: grouping and shrink ride in the projection kernel (two launches in all)
    const bool prep_inside = prep_in_projection(f);
    int e = (prep_inside || reuse_grouping) ? 0 : launch_classify_group(f);
    if (!e) {
        if (f.dtype == ALORA_F32) {
            e = launch_shrink_f32(f, ta);
            if (!e && timed) e = (int)hipEventRecord(g_prof.ev0[g_prof.used], f.stream);
            if (!e) e = launch_gemm_f32(f, tb);
            if (!e && f.rope_cos) e = launch_rope_f32(f);
            if (!e && timed) e = (int)hipEventRecord(g_prof.ev1[g_prof.used], f.stream);
        } else {
            if (!prep_inside) e = launch_shrink_bf16(f, ta);
            if (!e && timed) e = (int)hipEventRecord(g_prof.ev0[g_prof.used], f.stream);
            // the second event is recorded right behind the projection kernel (before the finishing
            // kernel of the small-batch path)
            if (!e) e = launch_gemm_bf16(f, tb, ta, timed ? g_prof.ev1[g_prof.used] : nullptr);
        }
        if (!e && timed) g_prof.used++;
    }
    if (e) { g_last_hip_error = e; return ALORA_EHIP; }
    return ALORA_OK;
}

int alora_qkv_forward(const void *x, const int32_t *token_adapter_ids, const int32_t *activation_start,
                      const void *W_qkv, const void *const *A, const void *const *B, void *q_out, void *k_cache,
                      void *v_cache, const int64_t *slot_mapping, int32_t block_size, const alora_dims *dims,
                      void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return forward_on(x, token_adapter_ids, activation_start, W_qkv, A, B, q_out, k_cache, v_cache, slot_mapping,
                      block_size, dims, workspace, workspace_bytes, hip_stream, true);
}

int alora_qkv_forward_ex(const void *x, const int32_t *token_adapter_ids, const int32_t *activation_start,
                         const void *W_qkv, const void *const *A, const void *const *B, void *q_out, void *k_cache,
                         void *v_cache, const int64_t *slot_mapping, int32_t block_size, const alora_dims *dims,
                         const alora_extras *extras, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return forward_on(x, token_adapter_ids, activation_start, W_qkv, A, B, q_out, k_cache, v_cache, slot_mapping,
                      block_size, dims, workspace, workspace_bytes, hip_stream, true, extras);
}

struct alora_graph {
    hipGraph_t graph;
    hipGraphExec_t exec;
};

int alora_qkv_graph_create(const void *x, const int32_t *token_adapter_ids, const int32_t *activation_start,
                           const void *W_qkv, const void *const *A, const void *const *B, void *q_out,
                           void *k_cache, void *v_cache, const int64_t *slot_mapping, int32_t block_size,
                           const alora_dims *dims, const alora_extras *extras, void *workspace,
                           size_t workspace_bytes, alora_graph **out)
{
    if (!out) return ALORA_EINVAL;
    *out = nullptr;
    if (!dims || dims->T <= 0) return ALORA_EINVAL;
    hipStream_t cs = nullptr;
    hipError_t e = hipStreamCreateWithFlags(&cs, hipStreamNonBlocking);
    if (e) { g_last_hip_error = (int)e; return ALORA_EHIP; }
    e = hipStreamBeginCapture(cs, hipStreamCaptureModeThreadLocal);
    if (e) { (void)hipStreamDestroy(cs); g_last_hip_error = (int)e; return ALORA_EHIP; }
    // argument errors are found before anything is enqueued; the capture is ended either way
    const int status = forward_on(x, token_adapter_ids, activation_start, W_qkv, A, B, q_out, k_cache, v_cache,
                                  slot_mapping, block_size, dims, workspace, workspace_bytes, cs, false, extras);
    hipGraph_t graph = nullptr;
    e = hipStreamEndCapture(cs, &graph);
    (void)hipStreamDestroy(cs);
    if (status != ALORA_OK) {
        if (graph) (void)hipGraphDestroy(graph);
        return status;
    }
    if (e || !graph) { g_last_hip_error = (int)e; return ALORA_EHIP; }
    hipGraphExec_t exec = nullptr;
    e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    if (e) { (void)hipGraphDestroy(graph); g_last_hip_error = (int)e; return ALORA_EHIP; }
    alora_graph *g = new alora_graph;
    g->graph = graph;
    g->exec = exec;
    *out = g;
    return ALORA_OK;
}

int alora_qkv_graph_launch(alora_graph *graph, void *hip_stream)
{
    if (!graph || !graph->exec) return ALORA_EINVAL;
    const hipError_t e = hipGraphLaunch(graph->exec, (hipStream_t)hip_stream);
    if (e) { g_last_hip_error = (int)e; return ALORA_EHIP; }
    return ALORA_OK;
}

int alora_qkv_graph_destroy(alora_graph *graph)
{
    if (!graph) return ALORA_OK;
    hipError_t e = hipSuccess;
    if (graph->exec) e = hipGraphExecDestroy(graph->exec);
    if (graph->graph) { const hipError_t e2 = hipGraphDestroy(graph->graph); if (!e) e = e2; }
    delete graph;
    if (e) { g_last_hip_error = (int)e; return ALORA_EHIP; }
    return ALORA_OK;
}

size_t alora_qkv_static_scratch_bytes(void) { return ALORA_STATIC_SCRATCH_BYTES; }

int alora_qkv_forward_static(const void *x, const int32_t *token_adapter_ids, const int32_t *activation_start,
                             const void *W_qkv, const void *const *A, const void *const *B, void *q_out, void *k_cache,
                             void *v_cache, const int64_t *slot_mapping, int32_t block_size, const alora_dims *dims,
                             const alora_extras *extras, void *hip_stream)
{
    int s = check_dims(dims);
    if (s) return s;
    if (make_layout(dims).total > ALORA_STATIC_SCRATCH_BYTES) return ALORA_ETOOBIG;
    // a grouping left by "an earlier call" could be any caller's: every call on a device shares the array
    if (extras && extras->reuse_grouping) return ALORA_EINVAL;
    void *ws = nullptr;
    s = static_scratch(&ws);
    if (s) return s;
    return forward_on(x, token_adapter_ids, activation_start, W_qkv, A, B, q_out, k_cache, v_cache, slot_mapping,
                      block_size, dims, ws, ALORA_STATIC_SCRATCH_BYTES, hip_stream, false, extras);
}

int alora_qkv_set_tuning(int feature_tiles, int splits)
{
    if (feature_tiles != 0 && (feature_tiles < 2 || feature_tiles > 4)) return ALORA_EINVAL;
    if (splits < 0 || splits > 8) return ALORA_EINVAL;
    set_gemm_tuning(feature_tiles, splits);
    return ALORA_OK;
}

int alora_qkv_profile_begin(int max_calls) { return alora_qkv_profile_begin_every(max_calls, 1); }

int alora_qkv_profile_begin_every(int max_calls, int every)
{
    if (max_calls <= 0 || max_calls > (1 << 20) || every < 1) return ALORA_EINVAL;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (g_prof.on) return ALORA_EINVAL;
    const int pairs = (max_calls + every - 1) / every;   // calls that can be measured
    try {
        g_prof.ev0.assign((size_t)pairs, nullptr);
        g_prof.ev1.assign((size_t)pairs, nullptr);
    } catch (const std::bad_alloc &) {
        return ALORA_ENOMEM;
    }
    for (int i = 0; i < pairs; ++i) {
        hipError_t e = hipEventCreate(&g_prof.ev0[i]);
        if (!e) e = hipEventCreate(&g_prof.ev1[i]);
        if (e) { g_last_hip_error = (int)e; return ALORA_EHIP; }
    }
    g_prof.used = 0;
    g_prof.every = every;
    g_prof.seen = 0;
    g_prof.on = true;
    return ALORA_OK;
}

int alora_qkv_profile_end(double *avg_ms, int *n_calls)
{
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (!g_prof.on) return ALORA_EINVAL;
    g_prof.on = false;
    double sum = 0.0;
    int n = 0, status = ALORA_OK;
    for (int i = 0; i < g_prof.used; ++i) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(g_prof.ev1[i]);
        if (!e) e = hipEventElapsedTime(&ms, g_prof.ev0[i], g_prof.ev1[i]);
        if (e) { g_last_hip_error = (int)e; status = ALORA_EHIP; break; }
        sum += ms;
        ++n;
    }
    for (size_t i = 0; i < g_prof.ev0.size(); ++i) {
        if (g_prof.ev0[i]) (void)hipEventDestroy(g_prof.ev0[i]);
        if (g_prof.ev1[i]) (void)hipEventDestroy(g_prof.ev1[i]);
    }
    g_prof.ev0.clear();
    g_prof.ev1.clear();
    if (avg_ms) *avg_ms = n ? sum / n : 0.0;
    if (n_calls) *n_calls = n;
    return status;
}

int alora_qkv_validate(const int32_t *token_adapter_ids, const int32_t *activation_start,
                       const int64_t *slot_mapping, int32_t block_size, const alora_dims *dims)
{
    int s = check_dims(dims);
    if (s) return s;
    if (block_size <= 0) return ALORA_EINVAL;
    if (dims->n_slots % block_size) return ALORA_ESHAPE;
    const size_t T = (size_t)dims->T;
    if (T == 0) return ALORA_OK;
    if (!token_adapter_ids || !slot_mapping || !dims->token_seg_ids || !dims->token_positions) return ALORA_EINVAL;
    if (dims->n_segments > 0 && !activation_start) return ALORA_EINVAL;
    try {
    std::vector<int32_t> aid(T), seg(T), pos(T), start((size_t)dims->n_segments);
    std::vector<int64_t> slot(T);
    hipError_t e = hipMemcpy(aid.data(), token_adapter_ids, 4 * T, hipMemcpyDeviceToHost);
    if (!e) e = hipMemcpy(seg.data(), dims->token_seg_ids, 4 * T, hipMemcpyDeviceToHost);
    if (!e) e = hipMemcpy(pos.data(), dims->token_positions, 4 * T, hipMemcpyDeviceToHost);
    if (!e) e = hipMemcpy(slot.data(), slot_mapping, 8 * T, hipMemcpyDeviceToHost);
    if (!e && dims->n_segments > 0)
        e = hipMemcpy(start.data(), activation_start, 4 * (size_t)dims->n_segments, hipMemcpyDeviceToHost);
    if (e) { g_last_hip_error = (int)e; return ALORA_EHIP; }
    for (size_t t = 0; t < T; ++t) {
        if (aid[t] < -1 || aid[t] >= dims->n_adapters) return ALORA_EDATA;
        if (aid[t] >= 0 && (seg[t] < 0 || seg[t] >= dims->n_segments)) return ALORA_EDATA;
        if (slot[t] < -1 || slot[t] >= dims->n_slots) return ALORA_EDATA;
    }
    std::vector<int64_t> used;
    used.reserve(T);
    for (size_t t = 0; t < T; ++t)
        if (slot[t] >= 0) used.push_back(slot[t]);
    std::sort(used.begin(), used.end());
    if (std::adjacent_find(used.begin(), used.end()) != used.end()) return ALORA_EDATA;
    return ALORA_OK;
    } catch (const std::bad_alloc &) {
        return ALORA_ENOMEM;
    }
}

}  // extern "C"
