// Base-aligned block cache and suffix planner (host code only; no kernels in this file).
//
// Sec. 3: every full KV-cache block is identified by a chained hash over the block's token ids,
// the hash of the block before it, and an extra identifier (the adapter id, or nothing for the
// base model).  Fig. 1 caption: for a request that invokes an aLoRA the adapter id is hashed only
// into blocks holding tokens at or after the activation point, and partial blocks are not cached.
// The planner finds the longest cached prefix of a request, allocates blocks for the remainder and
// emits the rows the projection still has to compute (positions, segment ids, adapter ids, slots).
//
// Data structures: hash -> block map, per-block (hash, keyed flag, reference count), an intrusive
// doubly linked free list (front = next to hand out, so the pool is least-recently-freed first and
// a block reused through its hash is unlinked in O(1)), and the live requests.
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <new>
#include <unordered_map>
#include <vector>
#include "alora_planner.h"

namespace {

// 64-bit mixing step (the finaliser of a well-known family of multiply-xorshift hashes)
inline uint64_t mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xbf58476d1ce4e5b9ull;
    z ^= z >> 27; z *= 0x94d049bb133111ebull;
    z ^= z >> 31;
    return z;
}

constexpr uint64_t ROOT_HASH = 0x9e3779b97f4a7c15ull;   // "hash of the block before block 0"
constexpr uint64_t NO_EXTRA = 0x5851f42d4c957f2dull;    // extra identifier of a base-model block

// Sec. 3 items (1)-(3): tokens of the block, hash of the previous block, extra identifier.
uint64_t block_hash(uint64_t parent, const int32_t *tok, int bs, bool with_adapter, int32_t adapter)
{
    uint64_t h = mix64(parent ^ 0xd6e8feb86659fd93ull);
    for (int i = 0; i < bs; ++i) h = mix64(h ^ (uint64_t)(uint32_t)tok[i] ^ ((uint64_t)(i + 1) << 32));
    const uint64_t extra = with_adapter ? mix64(0xa24baed4963ee407ull + (uint64_t)(uint32_t)adapter) : NO_EXTRA;
    return mix64(h ^ extra);
}

struct Request {
    std::vector<int32_t> tokens;
    std::vector<int32_t> table;       // physical block per logical block
    std::vector<uint64_t> hashes;     // chained hashes of the full blocks computed so far
    int32_t adapter = -1, start = 0;
    int32_t keyed = 0;                // leading blocks already registered in (or taken from) the cache
};

}  // namespace

struct alora_planner {
    int32_t bs = 0;
    int64_t n_blocks = 0;
    std::vector<uint64_t> hash_of;    // per block, valid when keyed
    std::vector<uint8_t> keyed;
    std::vector<int32_t> ref;
    std::vector<int32_t> prev, next;  // free list links (-1 = none); only meaningful while ref == 0
    int32_t head = -1, tail = -1;
    int64_t n_free = 0;
    std::unordered_map<uint64_t, int32_t> block_of;
    std::unordered_map<int64_t, Request> reqs;

    void push_back_free(int32_t b)
    {
        prev[b] = tail; next[b] = -1;
        if (tail >= 0) next[tail] = b; else head = b;
        tail = b;
        ++n_free;
    }
    void unlink_free(int32_t b)
    {
        if (prev[b] >= 0) next[prev[b]] = next[b]; else head = next[b];
        if (next[b] >= 0) prev[next[b]] = prev[b]; else tail = prev[b];
        --n_free;
    }
    // front of the free list; whatever the block held is forgotten (eviction)
    int32_t take_free()
    {
        const int32_t b = head;
        unlink_free(b);
        if (keyed[b]) {
            auto it = block_of.find(hash_of[b]);
            if (it != block_of.end() && it->second == b) block_of.erase(it);
            keyed[b] = 0;
        }
        return b;
    }
    // the adapter id enters block b's hash iff the block holds a position at or after the activation point
    bool with_adapter(const Request &r, int64_t b) const { return r.adapter >= 0 && (b + 1) * (int64_t)bs > r.start; }
    // extend r.hashes to cover every full block of r.tokens
    void hash_full_blocks(Request &r) const
    {
        const int64_t nfull = (int64_t)r.tokens.size() / bs;
        for (int64_t b = (int64_t)r.hashes.size(); b < nfull; ++b) {
            const uint64_t parent = b ? r.hashes[b - 1] : ROOT_HASH;
            r.hashes.push_back(block_hash(parent, r.tokens.data() + b * bs, bs, with_adapter(r, b), r.adapter));
        }
    }
};

namespace {

bool batch_ok(const alora_plan_batch *b)
{
    return b && b->token_positions && b->token_seg_ids && b->token_adapter_ids && b->slot_mapping &&
           b->activation_start && b->row_cap >= 0 && b->seg_cap >= 0 && b->n_rows >= 0 && b->n_segs >= 0 &&
           b->n_rows <= b->row_cap && b->n_segs <= b->seg_cap;
}

// one segment: rows for positions first .. n-1 of request r
void emit_rows(const alora_planner *p, const Request &r, int64_t first, alora_plan_batch *b)
{
    const int32_t seg = b->n_segs++;
    b->activation_start[seg] = r.start;
    for (int64_t pos = first; pos < (int64_t)r.tokens.size(); ++pos) {
        const int32_t i = b->n_rows++;
        b->token_positions[i] = (int32_t)pos;
        b->token_seg_ids[i] = seg;
        b->token_adapter_ids[i] = r.adapter;
        b->slot_mapping[i] = (int64_t)r.table[pos / p->bs] * p->bs + pos % p->bs;
    }
}

}  // namespace

extern "C" {

int alora_planner_create(int32_t block_size, int64_t n_blocks, alora_planner **out)
{
    if (!out) return ALORA_EINVAL;
    *out = nullptr;
    if (block_size <= 0 || n_blocks < 0 || n_blocks > 0x7fffffff) return ALORA_EINVAL;
    alora_planner *p = new (std::nothrow) alora_planner;
    if (!p) return ALORA_ENOMEM;
    try {
        p->bs = block_size;
        p->n_blocks = n_blocks;
        p->hash_of.assign((size_t)n_blocks, 0);
        p->keyed.assign((size_t)n_blocks, 0);
        p->ref.assign((size_t)n_blocks, 0);
        p->prev.assign((size_t)n_blocks, -1);
        p->next.assign((size_t)n_blocks, -1);
    } catch (const std::bad_alloc &) {
        delete p;
        return ALORA_ENOMEM;
    }
    for (int64_t b = 0; b < n_blocks; ++b) p->push_back_free((int32_t)b);
    *out = p;
    return ALORA_OK;
}

int alora_planner_destroy(alora_planner *p)
{
    delete p;
    return ALORA_OK;
}

int alora_planner_admit(alora_planner *p, int64_t req_id, const int32_t *token_ids, int32_t n_tokens,
                        int32_t adapter_id, int32_t activation_start, alora_plan_batch *batch,
                        int32_t *cached_tokens)
{
    if (!p || !token_ids || n_tokens < 1 || adapter_id < -1 || activation_start < 0 || !batch_ok(batch))
        return ALORA_EINVAL;
    if (p->reqs.count(req_id)) return ALORA_EINVAL;
    try {   // everything that allocates happens before the pool is touched
    Request r;
    r.tokens.assign(token_ids, token_ids + n_tokens);
    r.adapter = adapter_id;
    r.start = activation_start;
    p->hash_full_blocks(r);
    const int64_t bs = p->bs, n = n_tokens;
    const int64_t limit = std::min<int64_t>((int64_t)r.hashes.size(), (n - 1) / bs);
    int64_t hit = 0;
    std::vector<int32_t> reuse;
    int64_t reuse_from_pool = 0;
    while (hit < limit) {
        auto it = p->block_of.find(r.hashes[hit]);
        if (it == p->block_of.end()) break;
        reuse.push_back(it->second);
        if (p->ref[it->second] == 0) ++reuse_from_pool;
        ++hit;
    }
    const int64_t need = (n + bs - 1) / bs - hit;
    const int64_t rows = n - hit * bs;
    if (need > p->n_free - reuse_from_pool) return ALORA_ENOBLOCKS;
    if (rows > batch->row_cap - batch->n_rows || batch->n_segs >= batch->seg_cap) return ALORA_ESHAPE;
    r.table.reserve((size_t)(hit + need));
    auto ins = p->reqs.emplace(req_id, Request());
    // nothing can fail from here on
    for (int32_t b : reuse) {
        if (p->ref[b] == 0) p->unlink_free(b);
        ++p->ref[b];
        r.table.push_back(b);
    }
    for (int64_t i = 0; i < need; ++i) {
        const int32_t b = p->take_free();
        p->ref[b] = 1;
        r.table.push_back(b);
    }
    r.keyed = (int32_t)hit;
    emit_rows(p, r, hit * bs, batch);
    if (cached_tokens) *cached_tokens = (int32_t)(hit * bs);
    ins.first->second = std::move(r);
    return ALORA_OK;
    } catch (const std::bad_alloc &) {
        return ALORA_ENOMEM;
    }
}

int alora_planner_append(alora_planner *p, int64_t req_id, const int32_t *new_token_ids, int32_t n_new,
                         alora_plan_batch *batch)
{
    if (!p || !new_token_ids || n_new < 1 || !batch_ok(batch)) return ALORA_EINVAL;
    auto it = p->reqs.find(req_id);
    if (it == p->reqs.end()) return ALORA_EINVAL;
    Request &r = it->second;
    const int64_t bs = p->bs, first = (int64_t)r.tokens.size(), total = first + n_new;
    if (total > 0x7fffffff) return ALORA_ESHAPE;
    const int64_t need = (total + bs - 1) / bs - (int64_t)r.table.size();
    if (need > p->n_free) return ALORA_ENOBLOCKS;
    if (n_new > batch->row_cap - batch->n_rows || batch->n_segs >= batch->seg_cap) return ALORA_ESHAPE;
    try {   // allocate first, then touch the pool
        r.table.reserve(r.table.size() + (size_t)std::max<int64_t>(need, 0));
        r.tokens.insert(r.tokens.end(), new_token_ids, new_token_ids + n_new);
    } catch (const std::bad_alloc &) {
        return ALORA_ENOMEM;
    }
    for (int64_t i = 0; i < need; ++i) {
        const int32_t b = p->take_free();
        p->ref[b] = 1;
        r.table.push_back(b);
    }
    emit_rows(p, r, first, batch);
    return ALORA_OK;
}

int alora_planner_commit(alora_planner *p, int64_t req_id)
{
    if (!p) return ALORA_EINVAL;
    auto it = p->reqs.find(req_id);
    if (it == p->reqs.end()) return ALORA_EINVAL;
    Request &r = it->second;
    try {   // a failed allocation leaves the blocks registered so far registered; the call can be repeated
        p->hash_full_blocks(r);
        for (int64_t b = r.keyed; b < (int64_t)r.hashes.size(); ++b) {
            const int32_t blk = r.table[b];
            // an equal block registered by another request in the meantime keeps the entry
            if (!p->keyed[blk] && !p->block_of.count(r.hashes[b])) {
                p->block_of.emplace(r.hashes[b], blk);
                p->hash_of[blk] = r.hashes[b];
                p->keyed[blk] = 1;
            }
        }
    } catch (const std::bad_alloc &) {
        return ALORA_ENOMEM;
    }
    r.keyed = (int32_t)r.hashes.size();
    return ALORA_OK;
}

int alora_planner_finish(alora_planner *p, int64_t req_id)
{
    if (!p) return ALORA_EINVAL;
    auto it = p->reqs.find(req_id);
    if (it == p->reqs.end()) return ALORA_EINVAL;
    const Request &r = it->second;
    for (size_t i = r.table.size(); i-- > 0;) {
        const int32_t b = r.table[i];
        if (--p->ref[b] == 0) p->push_back_free(b);
    }
    p->reqs.erase(it);
    return ALORA_OK;
}

int alora_planner_block_table(const alora_planner *p, int64_t req_id, int32_t *out, int32_t cap, int32_t *n)
{
    if (!p || !n || cap < 0 || (cap > 0 && !out)) return ALORA_EINVAL;
    auto it = p->reqs.find(req_id);
    if (it == p->reqs.end()) return ALORA_EINVAL;
    const std::vector<int32_t> &t = it->second.table;
    const int32_t m = (int32_t)std::min<size_t>(t.size(), (size_t)cap);
    if (m > 0) std::memcpy(out, t.data(), (size_t)m * sizeof(int32_t));
    *n = (int32_t)t.size();
    return ALORA_OK;
}

int64_t alora_planner_free_blocks(const alora_planner *p)
{
    if (!p) return ALORA_EINVAL;
    return p->n_free;
}

}  // extern "C"
