"""Oracle for the base-aligned block cache and suffix planner (Sec. 3, Fig. 1 caption).

TEST INFRASTRUCTURE ONLY, like the rest of this package: plain Python, slow, obviously correct;
the C++ planner of the library shares no code with it.

What the paper fixes (Sec. 3): the KV cache is cut into blocks of `block_size` token slots; a block
is identified by a chain over (1) the tokens in the block, (2) the identity of the blocks before
it in the sequence, (3) extra identifiers such as the adapter id.  Only full blocks are cached
(Fig. 1 caption).  Blocks of a finished request go back to the free pool but stay reusable through
their identity.  For a request that invokes an aLoRA, the adapter id enters the identity only of
blocks holding tokens processed with the adapter, i.e. tokens at or after the activation point
(Fig. 1 caption); every block before that carries the identity a base-model request would give
it, so base and aLoRA requests reuse each other's blocks in both directions.

This oracle uses the chain ITSELF as the identity -- the triple
(parent identity, tokens of the block, extra), with every distinct triple given a serial number so
that a parent is named by its number instead of being nested (a chain of a thousand blocks would
otherwise be a thousand tuples deep) -- so there is no hash function and no collision: two blocks
are interchangeable exactly when the paper says they are.  (The hash function of the
product is "parity unpinned": any collision-resistant hash is valid; what is pinned is which
blocks share an identity.)

Readings where the paper is silent:
  - a block "holds tokens processed with the adapter" iff it contains a position >= activation_start,
    i.e. (b+1)*block_size > activation_start; a standard LoRA is activation_start = 0, a base request
    has adapter -1 (no block ever carries an id);
  - at least one token of every admitted request is projected: the reusable prefix is capped at
    floor((n-1)/block_size) blocks;
  - blocks become reusable when the caller says their contents have been computed (commit), not
    when they are allocated;
  - free blocks are taken from the front of the free list (lowest ids first at start); a finished
    request returns its blocks last-block-first, so that the tail of a sequence is evicted before its
    head; taking a free block that still has an identity forgets that identity (eviction).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple


class OutOfBlocks(Exception):
    pass


@dataclass
class Plan:
    cached_tokens: int                 # tokens whose K/V are reused from the cache (multiple of block_size)
    positions: List[int]               # absolute positions of the rows to project
    slots: List[int]                   # cache slot of each of those rows
    block_table: List[int]             # physical block of every logical block of the request


@dataclass
class _Req:
    tokens: List[int]
    adapter: int
    start: int
    table: List[int] = field(default_factory=list)
    keyed: int = 0                     # leading blocks that already carry an identity in the cache


class PrefixCacheOracle:
    def __init__(self, block_size: int, n_blocks: int):
        assert block_size > 0 and n_blocks >= 0
        self.bs = block_size
        self.free: List[int] = list(range(n_blocks))
        self.ref = [0] * n_blocks
        self.key_of: List[Optional[tuple]] = [None] * n_blocks
        self.block_of: Dict[tuple, int] = {}
        self.serial: Dict[tuple, int] = {}      # serial number of every identity ever formed
        self.reqs: Dict[int, _Req] = {}

    # -- identities ---------------------------------------------------------------------
    def _extra(self, adapter: int, start: int, b: int):
        """Sec. 3 item (3) with the Fig. 1 rule: the adapter id only for blocks that hold a position
        at or after the activation point."""
        return adapter if (adapter >= 0 and (b + 1) * self.bs > start) else None

    def keys(self, tokens: Sequence[int], adapter: int, start: int) -> List[tuple]:
        out, parent = [], None
        for b in range(len(tokens) // self.bs):
            key = (parent, tuple(int(t) for t in tokens[b * self.bs:(b + 1) * self.bs]), self._extra(adapter, start, b))
            out.append(key)
            # the next block names this one by its serial number (equal triples get equal numbers)
            parent = self.serial.setdefault(key, len(self.serial))
        return out

    # -- block pool ---------------------------------------------------------------------
    def _take_free(self) -> int:
        if not self.free:
            raise OutOfBlocks()
        blk = self.free.pop(0)
        k = self.key_of[blk]
        if k is not None:              # eviction: the block's old contents are about to be overwritten
            del self.block_of[k]
            self.key_of[blk] = None
        return blk

    def _rows(self, r: _Req, first_pos: int) -> Tuple[List[int], List[int]]:
        pos = list(range(first_pos, len(r.tokens)))
        return pos, [r.table[p // self.bs] * self.bs + p % self.bs for p in pos]

    # -- requests -----------------------------------------------------------------------
    def admit(self, req_id: int, tokens: Sequence[int], adapter: int, start: int) -> Plan:
        assert req_id not in self.reqs and len(tokens) > 0
        n = len(tokens)
        keys = self.keys(tokens, adapter, start)
        limit = min(len(keys), (n - 1) // self.bs)
        hit = 0
        while hit < limit and keys[hit] in self.block_of:
            hit += 1
        need = -(-n // self.bs) - hit
        reuse = [self.block_of[keys[b]] for b in range(hit)]
        # blocks that are reused out of the free pool are no longer available for allocation
        available = len(self.free) - sum(1 for blk in reuse if self.ref[blk] == 0)
        if need > available:
            raise OutOfBlocks()
        r = _Req(list(int(t) for t in tokens), adapter, start)
        for blk in reuse:
            if self.ref[blk] == 0:
                self.free.remove(blk)
            self.ref[blk] += 1
            r.table.append(blk)
        for _ in range(need):
            blk = self._take_free()
            self.ref[blk] = 1
            r.table.append(blk)
        r.keyed = hit
        self.reqs[req_id] = r
        pos, slots = self._rows(r, hit * self.bs)
        return Plan(hit * self.bs, pos, slots, list(r.table))

    def append(self, req_id: int, new_tokens: Sequence[int]) -> Plan:
        """Decode: the request grows by new_tokens; rows for exactly those tokens."""
        r = self.reqs[req_id]
        first = len(r.tokens)
        total = first + len(new_tokens)
        need = -(-total // self.bs) - len(r.table)
        if need > len(self.free):
            raise OutOfBlocks()
        r.tokens.extend(int(t) for t in new_tokens)
        for _ in range(need):
            blk = self._take_free()
            self.ref[blk] = 1
            r.table.append(blk)
        pos, slots = self._rows(r, first)
        return Plan(0, pos, slots, list(r.table))

    def commit(self, req_id: int) -> None:
        """The request's rows planned so far have been computed: its full blocks become reusable."""
        r = self.reqs[req_id]
        keys = self.keys(r.tokens, r.adapter, r.start)
        for b in range(r.keyed, len(keys)):
            blk = r.table[b]
            if keys[b] not in self.block_of and self.key_of[blk] is None:
                self.block_of[keys[b]] = blk
                self.key_of[blk] = keys[b]
        r.keyed = len(keys)

    def finish(self, req_id: int) -> None:
        r = self.reqs.pop(req_id)
        for blk in reversed(r.table):
            self.ref[blk] -= 1
            if self.ref[blk] == 0:
                self.free.append(blk)

    def n_free(self) -> int:
        return len(self.free)
