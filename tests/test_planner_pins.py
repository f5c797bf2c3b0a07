"""Pins of the block-cache / suffix-planner oracle (oracle/prefix_cache.py) against what Sec. 3 and
the caption of Fig. 1 fix, plus invariants and a brute-force cross-check; and parity of the
library's C++ planner (include/alora_planner.h) with that oracle, bit for bit, on the same traces.
Host code only: nothing here needs a GPU."""
import json
import os

import numpy as np
import pytest

from oracle.prefix_cache import OutOfBlocks, PrefixCacheOracle
from paper_2512_17910_amd import planner as pl
from paper_2512_17910_amd.binding import ALORA_EINVAL, ALORA_ESHAPE, AloraError

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "fig1_prefix_cache.json")
NEVER = 1 << 30   # activation point of a base request (irrelevant: no adapter)


# --------------------------------------------------------------------------------------------
# a thin common face over the oracle and the C++ planner, so that every scenario runs on both
# --------------------------------------------------------------------------------------------
class OracleFace:
    def __init__(self, bs, n_blocks):
        self.o = PrefixCacheOracle(bs, n_blocks)

    def admit(self, rid, tokens, adapter, start):
        try:
            p = self.o.admit(rid, tokens, adapter, start)
        except OutOfBlocks:
            return None
        return p.cached_tokens, p.positions, p.slots, p.block_table

    def append(self, rid, new):
        try:
            p = self.o.append(rid, new)
        except OutOfBlocks:
            return None
        return p.positions, p.slots, p.block_table

    def commit(self, rid):
        self.o.commit(rid)

    def finish(self, rid):
        self.o.finish(rid)

    def free(self):
        return self.o.n_free()


class LibFace:
    def __init__(self, bs, n_blocks):
        self.p = pl.Planner(bs, n_blocks)

    def admit(self, rid, tokens, adapter, start):
        b = pl.Batch(len(tokens), 1)
        try:
            cached = self.p.admit(rid, tokens, adapter, start, b)
        except AloraError as e:
            assert e.status == pl.ALORA_ENOBLOCKS
            assert b.n_rows == 0 and b.n_segs == 0
            return None
        pos, seg, aid, slot, starts = b.rows()
        assert np.all(seg == 0) and np.all(aid == adapter) and list(starts) == [start]
        return cached, list(map(int, pos)), list(map(int, slot)), list(map(int, self.p.block_table(rid)))

    def append(self, rid, new):
        b = pl.Batch(len(new), 1)
        try:
            self.p.append(rid, new, b)
        except AloraError as e:
            assert e.status == pl.ALORA_ENOBLOCKS
            return None
        pos, seg, aid, slot, _ = b.rows()
        return list(map(int, pos)), list(map(int, slot)), list(map(int, self.p.block_table(rid)))

    def commit(self, rid):
        self.p.commit(rid)

    def finish(self, rid):
        self.p.finish(rid)

    def free(self):
        return self.p.free_blocks()


FACES = [OracleFace, LibFace]
face = pytest.mark.parametrize("Face", FACES, ids=["oracle", "library"])


# --------------------------------------------------------------------------------------------
# Fig. 1 caption
# --------------------------------------------------------------------------------------------
@face
def test_fig1_caption_structure(Face):
    g = json.load(open(GOLDEN))
    e = g["expect"]
    bs = g["block_size"]
    c = Face(bs, g["n_blocks"])
    prompt, act, gen, a = g["prompt"], g["activation_tokens"], g["generated"], g["adapter"]
    # turn 1: the base model prefills the prompt
    cached, pos, slots, table = c.admit(1, prompt, -1, NEVER)
    assert cached == e["base_first_turn_cached"] and pos == list(range(len(prompt)))
    c.commit(1)
    c.finish(1)
    # turn 2: the aLoRA is invoked on the same prompt + its activation tokens
    start = len(prompt)
    cached, pos, slots, table2 = c.admit(2, prompt + act, a, start)
    assert cached == e["alora_turn_cached_tokens"] and pos == e["alora_turn_rows_positions"]
    assert table2[: cached // bs] == table[: cached // bs]          # the very blocks the base request filled
    c.commit(2)                                                       # activation tokens: no full block, nothing new
    probe = Face.__name__ == "OracleFace" and len(c.o.block_of)
    if probe is not False:
        assert probe == e["blocks_with_identity_after_alora_prefill_commit"]
    # the adapter generates; its blocks fill up and carry the adapter id
    c.append(2, gen)
    c.commit(2)
    full = prompt + act + gen
    assert c.admit(3, full, -1, NEVER)[0] == e["base_after_generation_cached_tokens"]
    assert c.admit(4, full, a, start)[0] == e["same_adapter_after_generation_cached_tokens"]
    assert c.admit(5, full, g["other_adapter"], start)[0] == e["other_adapter_after_generation_cached_tokens"]


# --------------------------------------------------------------------------------------------
# Sec. 3: reuse in both directions; standard LoRA stays isolated
# --------------------------------------------------------------------------------------------
def _toks(rng, n, vocab=50):
    return [int(t) for t in rng.integers(0, vocab, n)]


@face
def test_alora_first_then_base_reuses_the_pre_activation_blocks(Face):
    rng = np.random.default_rng(1)
    bs, t = 4, _toks(rng, 23)
    c = Face(bs, 64)
    start = 14                       # inside block 3 (positions 12..15)
    assert c.admit(1, t, 2, start)[0] == 0
    c.commit(1)
    # blocks 0,1,2 end at or before position 12 <= start: base identity.  block 3 holds 14,15: adapter id
    assert c.admit(2, t, -1, NEVER)[0] == 3 * bs
    # the same aLoRA reuses everything the cap allows: floor(22/4) = 5 full blocks
    assert c.admit(3, t, 2, start)[0] == 5 * bs
    # another aLoRA with a later activation point shares one more block with the base request than with aLoRA 2
    assert c.admit(4, t, 3, 16)[0] == 3 * bs


@face
def test_base_first_then_alora_and_activation_on_a_block_boundary(Face):
    rng = np.random.default_rng(2)
    bs, t = 4, _toks(rng, 21)
    c = Face(bs, 64)
    c.admit(1, t, -1, NEVER)
    c.commit(1)
    # activation exactly at a block boundary (16): blocks 0..3 hold only positions < 16
    assert c.admit(2, t, 0, 16)[0] == 16
    # one position earlier (15): block 3 holds position 15 >= start, so it is the adapter's own
    assert c.admit(3, t, 0, 15)[0] == 12


@face
def test_standard_lora_shares_nothing_with_the_base_model(Face):
    rng = np.random.default_rng(3)
    bs, t = 4, _toks(rng, 17)
    c = Face(bs, 64)
    c.admit(1, t, -1, NEVER)
    c.commit(1)
    assert c.admit(2, t, 5, 0)[0] == 0          # activation at 0 = standard LoRA: every block carries the id
    c.commit(2)
    assert c.admit(3, t, 5, 0)[0] == 16         # but it reuses its own
    assert c.admit(4, t, 6, 0)[0] == 0          # and another adapter does not


@face
def test_chain_one_changed_token_cuts_the_reuse_at_its_block(Face):
    rng = np.random.default_rng(4)
    bs, t = 4, _toks(rng, 41)
    c = Face(bs, 64)
    c.admit(1, t, -1, NEVER)
    c.commit(1)
    for j in (0, 3, 4, 17, 39):
        u = list(t)
        u[j] += 1000
        rid = 100 + j
        assert c.admit(rid, u, -1, NEVER)[0] == (j // bs) * bs
        c.finish(rid)


@face
def test_only_full_blocks_and_at_least_one_row(Face):
    bs = 4
    c = Face(bs, 64)
    t = list(range(100, 112))                   # exactly 3 blocks
    c.admit(1, t, -1, NEVER)
    c.commit(1)
    cached, pos, _, _ = c.admit(2, t, -1, NEVER)
    assert cached == 8 and pos == [8, 9, 10, 11]        # the last block is computed again
    cached, pos, _, _ = c.admit(3, t + [7], -1, NEVER)
    assert cached == 12 and pos == [12]
    cached, pos, _, _ = c.admit(4, t[:11], -1, NEVER)    # 2 full blocks + 3 tokens
    assert cached == 8 and pos == [8, 9, 10]
    assert c.admit(5, [1], -1, NEVER)[0] == 0


@face
def test_uncommitted_blocks_are_not_reusable(Face):
    bs, t = 4, list(range(20))
    c = Face(bs, 64)
    c.admit(1, t, -1, NEVER)
    assert c.admit(2, t, -1, NEVER)[0] == 0
    c.commit(1)
    assert c.admit(3, t, -1, NEVER)[0] == 16
    c.commit(2)                                 # duplicates of already registered blocks stay anonymous
    assert c.admit(4, t, -1, NEVER)[3][:4] == c.admit(5, t, -1, NEVER)[3][:4]


@face
def test_pool_order_eviction_and_exhaustion(Face):
    bs = 2
    c = Face(bs, 7)
    a = c.admit(1, [1, 2, 3, 4], -1, NEVER)
    assert a[3] == [0, 1] and c.free() == 5          # lowest ids first
    c.commit(1)
    c.finish(1)                                      # returns 1 then 0 to the back of the pool
    assert c.free() == 7
    b = c.admit(2, [9, 9, 9, 9, 9, 9, 9], -1, NEVER) # 4 blocks from the front: 2,3,4,5
    assert b[3] == [2, 3, 4, 5] and c.free() == 3
    # request 1's blocks are still in the pool with their identity: reusable, and then no longer free
    r = c.admit(3, [1, 2, 3, 4, 5], -1, NEVER)
    assert r[0] == 4 and r[3] == [0, 1, 6] and c.free() == 0
    # nothing left: a further request fails and changes nothing
    assert c.admit(4, [5, 5], -1, NEVER) is None
    assert c.free() == 0
    c.finish(2)                                      # 5,4,3,2 go to the back in that order
    assert c.free() == 4
    d = c.admit(5, [7, 7, 7, 7, 7, 7], -1, NEVER)
    assert d[3] == [5, 4, 3]
    # a request that would need blocks it is about to reuse out of the pool does not count them twice
    c2 = Face(bs, 3)
    c2.admit(1, [1, 2, 3, 4], -1, NEVER)
    c2.commit(1)
    c2.finish(1)                                     # pool: 2, 1, 0 (all free, two with identity)
    assert c2.admit(2, [1, 2, 3, 4, 5, 6, 7], -1, NEVER) is None   # reuses 2 + needs 2 > 3 blocks
    assert c2.free() == 3
    assert c2.admit(3, [1, 2, 3, 4, 5], -1, NEVER)[3] == [0, 1, 2]


@face
def test_append_allocates_on_block_boundaries_and_emits_the_new_rows(Face):
    bs = 4
    c = Face(bs, 16)
    c.admit(1, [1, 2, 3], 0, 1)
    pos, slots, table = c.append(1, [4])
    assert pos == [3] and len(table) == 1 and slots == [table[0] * bs + 3]
    pos, slots, table = c.append(1, [5, 6, 7, 8, 9])
    assert pos == [4, 5, 6, 7, 8] and len(table) == 3
    assert slots == [table[p // bs] * bs + p % bs for p in pos]


# --------------------------------------------------------------------------------------------
# brute force on the oracle: reuse length straight from the definition, no chaining
# --------------------------------------------------------------------------------------------
def _brute_cached(committed, tokens, adapter, start, bs):
    """committed: list of (tokens, adapter, start) of every committed-and-still-cached request.
    A block is interchangeable iff all tokens up to its end agree and the extra ids of all
    blocks up to it agree."""
    def extras(ad, st, nb):
        return [ad if (ad >= 0 and (b + 1) * bs > st) else None for b in range(nb)]
    n = len(tokens)
    best = 0
    for ct, ca, cs in committed:
        k = 0
        while (k + 1) * bs <= min(len(ct), n) and ct[: (k + 1) * bs] == tokens[: (k + 1) * bs] and \
                extras(ca, cs, k + 1) == extras(adapter, start, k + 1):
            k += 1
        best = max(best, k)
    return min(best, (n - 1) // bs) * bs


def test_oracle_reuse_length_equals_the_flat_definition():
    rng = np.random.default_rng(7)
    bs = 3
    for trial in range(60):
        o = PrefixCacheOracle(bs, 10_000)       # never evicts
        committed = []
        base = _toks(rng, 30, vocab=3)
        for rid in range(12):
            n = int(rng.integers(1, 30))
            t = list(base[:n])
            if rng.random() < 0.5:              # perturb one token
                t[int(rng.integers(0, n))] = int(rng.integers(0, 3))
            ad = int(rng.integers(-1, 3))
            st = int(rng.integers(0, 32))
            plan = o.admit(rid, t, ad, st)
            assert plan.cached_tokens == _brute_cached(committed, t, ad, st, bs), (trial, rid)
            assert plan.positions == list(range(plan.cached_tokens, n))
            o.commit(rid)
            committed.append((t, ad, st))


def _check_invariants(o: PrefixCacheOracle):
    n = len(o.ref)
    assert sorted(o.free) == [b for b in range(n) if o.ref[b] == 0]
    assert all(r >= 0 for r in o.ref)
    for k, b in o.block_of.items():
        assert o.key_of[b] == k
    assert sum(1 for k in o.key_of if k is not None) == len(o.block_of)
    counts = [0] * n
    for r in o.reqs.values():
        assert len(r.table) == -(-len(r.tokens) // o.bs)
        for b in r.table:
            counts[b] += 1
    assert counts == o.ref
    # a block shared by two live requests holds a full, identified block
    for b in range(n):
        if counts[b] > 1:
            assert o.key_of[b] is not None


# --------------------------------------------------------------------------------------------
# parity: the C++ planner against the oracle on random traces (everything is an integer: equal)
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("seed,bs,n_blocks", [(0, 4, 40), (1, 16, 64), (2, 1, 50), (3, 3, 24), (4, 8, 400)])
def test_library_planner_equals_the_oracle_on_random_traces(seed, bs, n_blocks):
    rng = np.random.default_rng(100 + seed)
    o, c = OracleFace(bs, n_blocks), LibFace(bs, n_blocks)
    stems = [_toks(rng, 12 * bs, vocab=4) for _ in range(3)]
    live, next_id = [], 0
    for step in range(400):
        op = rng.random()
        if op < 0.45 or not live:
            stem = stems[int(rng.integers(0, 3))]
            n = int(rng.integers(1, len(stem) + 1))
            t = list(stem[:n])
            if rng.random() < 0.3:
                t[int(rng.integers(0, n))] = int(rng.integers(0, 4))
            ad, st = int(rng.integers(-1, 3)), int(rng.integers(0, n + 2))
            ro, rc = o.admit(next_id, t, ad, st), c.admit(next_id, t, ad, st)
            assert ro == rc, (step, "admit")
            if ro is not None:
                live.append(next_id)
            next_id += 1
        elif op < 0.65:
            rid = live[int(rng.integers(0, len(live)))]
            new = _toks(rng, int(rng.integers(1, 2 * bs + 1)), vocab=4)
            assert o.append(rid, new) == c.append(rid, new), (step, "append")
        elif op < 0.85:
            rid = live[int(rng.integers(0, len(live)))]
            o.commit(rid)
            c.commit(rid)
        else:
            rid = live.pop(int(rng.integers(0, len(live))))
            if rng.random() < 0.7:
                o.commit(rid)
                c.commit(rid)
            o.finish(rid)
            c.finish(rid)
        assert o.free() == c.free(), step
        if step % 20 == 0:
            _check_invariants(o.o)
    _check_invariants(o.o)


def test_library_planner_argument_errors_leave_it_unchanged():
    p = pl.Planner(4, 8)
    b = pl.Batch(16, 2)
    with pytest.raises(AloraError) as e:
        p.admit(1, [], -1, 0, b)
    assert e.value.status == ALORA_EINVAL
    with pytest.raises(AloraError) as e:
        p.admit(1, [1, 2, 3], -2, 0, b)
    assert e.value.status == ALORA_EINVAL
    small = pl.Batch(2, 1)
    with pytest.raises(AloraError) as e:
        p.admit(1, [1, 2, 3], -1, 0, small)     # rows do not fit the batch arrays
    assert e.value.status == ALORA_ESHAPE and small.n_rows == 0 and p.free_blocks() == 8
    p.admit(1, [1, 2, 3], -1, 0, b)
    with pytest.raises(AloraError):
        p.admit(1, [4], -1, 0, b)               # request id in use
    with pytest.raises(AloraError):
        p.commit(99)
    with pytest.raises(AloraError):
        p.finish(99)
    assert b.n_rows == 3 and b.n_segs == 1 and p.free_blocks() == 7


def test_two_requests_planned_into_one_batch():
    p = pl.Planner(4, 32)
    b = pl.Batch(64, 4)
    p.admit(1, list(range(10)), -1, NEVER, b)
    p.admit(2, list(range(50, 57)), 3, 5, b)
    pos, seg, aid, slot, starts = b.rows()
    assert list(pos) == list(range(10)) + list(range(7))
    assert list(seg) == [0] * 10 + [1] * 7 and list(aid) == [-1] * 10 + [3] * 7
    assert list(starts) == [NEVER, 5]
    assert len(set(map(int, slot))) == 17


def test_long_conversation_chain_both_sides():
    """A chain of a thousand blocks (config-5 scale: 16384 tokens, block size 16), base turn then aLoRA turn."""
    rng = np.random.default_rng(11)
    bs, n = 16, 16384
    conv = [int(t) for t in rng.integers(0, 32000, n)]
    o, c = OracleFace(bs, 2100), LibFace(bs, 2100)
    for f in (o, c):
        assert f.admit(1, conv[: n - 96], -1, NEVER)[0] == 0
        f.commit(1)
        f.finish(1)
    ro, rc = o.admit(2, conv, 1, n - 96), c.admit(2, conv, 1, n - 96)
    assert ro == rc and ro[0] == n - 96 and ro[1] == list(range(n - 96, n))
