"""Seeded synthetic inputs for the masked multi-adapter aLoRA QKV projection.

This module only *draws* data: token batches, weights, adapter factors, activation
points and paged-cache slot maps shaped like the paper's multi-turn, multi-adapter
pipelines (random prompts and random adapters, Sec. 4.1; long cached context with a
short activated tail, Sec. 4.2; several adapters per batch, Sec. 4.4.1).  It holds
none of the method's arithmetic: no projection, no mask, no grouping.  Both the CPU
oracle's tests and the HIP path's tests/benchmark take their inputs from here and
nothing else is shared between the two.

Values are drawn with numpy's counter-based Philox generator, keyed by
(seed, stream), so every array is reproducible independently of the others.
bf16 arrays are carried as uint16 bit patterns (round-to-nearest-even from fp32).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

SEED = 0x2512_1791_0A10_4A5D  # one fixed 64-bit constant; streams select the array

# stream ids (second half of the Philox key)
_ST_X, _ST_W, _ST_A, _ST_B, _ST_STRUCT, _ST_SLOTS, _ST_CACHE, _ST_BIAS, _ST_Q = 1, 2, 3, 4, 5, 6, 7, 8, 9


# --------------------------------------------------------------------------------------
# storage-format helpers (bit manipulation only)
# --------------------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> the exactly equal fp32 values."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def widen_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Storage array (fp32 values, or bf16 bit patterns) -> exactly equal fp64 values."""
    if dtype == "bf16":
        return bf16_bits_to_f32(a).astype(np.float64)
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def _rng(seed: int, stream: int, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & (2**64 - 1), (stream << 32) | sub]))


def _normal(seed: int, stream: int, sub: int, shape, std: float, dtype: str) -> np.ndarray:
    g = _rng(seed, stream, sub)
    a = g.standard_normal(size=shape, dtype=np.float32)
    a *= np.float32(std)
    if dtype == "bf16":
        return f32_to_bf16_bits(a)
    return a


# --------------------------------------------------------------------------------------
# the workload container
# --------------------------------------------------------------------------------------
@dataclass
class Segment:
    """One (adapter, activation point) unit: the paper's 'request' (App. B)."""
    seq: int               # which sequence's block table the tokens use
    first_pos: int         # absolute position of the segment's first projected token
    n_tokens: int
    adapter: int           # -1 = base model request
    activation_start: int  # absolute position; >= first_pos + n_tokens means never active


@dataclass
class Workload:
    name: str
    dtype: str             # "f32" | "bf16"
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_adapters: int
    rank: int
    block_size: int
    n_slots: int
    segments: List[Segment]
    x: np.ndarray = None                   # [T, hidden]
    W: np.ndarray = None                   # [hidden, N]
    A: List[np.ndarray] = field(default_factory=list)   # each [hidden, rank]
    B: List[np.ndarray] = field(default_factory=list)   # each [rank, N]
    token_adapter_ids: np.ndarray = None   # int32 [T]
    token_seg_ids: np.ndarray = None       # int32 [T]
    token_positions: np.ndarray = None     # int32 [T]
    activation_start: np.ndarray = None    # int32 [G]
    slot_mapping: np.ndarray = None        # int64 [T]
    cached_prefix_slots: Optional[np.ndarray] = None  # slots of skipped, already cached prefixes
    bias: Optional[np.ndarray] = None      # [N] layer bias (Algorithm 1's b), storage dtype; None = no bias
    adapter_ranks: Optional[List[int]] = None   # per-adapter rank r_i <= rank: A[i] is [hidden, r_i], B[i] is [r_i, N]

    @property
    def T(self) -> int:
        return int(self.token_adapter_ids.shape[0])

    @property
    def Nq(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def Nkv(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def N(self) -> int:
        return self.Nq + 2 * self.Nkv

    @property
    def n_segments(self) -> int:
        return int(self.activation_start.shape[0])

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4


def cache_fill(n_slots: int, width: int, dtype: str, which: int, seed: int = SEED) -> np.ndarray:
    """Pre-existing cache contents ("someone else's blocks"): small seeded finite values."""
    g = _rng(seed, _ST_CACHE, which)
    a = g.standard_normal(size=(n_slots, width), dtype=np.float32)
    a *= np.float32(0.25)
    return f32_to_bf16_bits(a) if dtype == "bf16" else a


def assemble(name: str, dtype: str, hidden: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
             n_adapters: int, rank: int, block_size: int, segments: Sequence[Segment],
             seq_max_len: Sequence[int], seed: int = SEED, extra_blocks: int = 0,
             weight_key: int = 0, pad_rows: Sequence[int] = (),
             x_std: float = 1.0, with_values: bool = True) -> Workload:
    """Lay segments out as one flattened token batch and draw values.

    seq_max_len[s] fixes how many cache blocks sequence s owns (ceil(len/block_size));
    physical block ids are a seeded permutation of all blocks (+extra_blocks spare ones).
    pad_rows: token rows that become padding (adapter -1, slot -1) after layout.
    """
    Nq, Nkv = n_q_heads * head_dim, n_kv_heads * head_dim
    N = Nq + 2 * Nkv
    blocks_per_seq = [(int(m) + block_size - 1) // block_size for m in seq_max_len]
    n_blocks = int(sum(blocks_per_seq)) + int(extra_blocks)
    perm = _rng(seed, _ST_SLOTS).permutation(n_blocks).astype(np.int64)
    tables, o = [], 0
    for nb in blocks_per_seq:
        tables.append(perm[o:o + nb])
        o += nb

    aid, seg, pos, slot, starts = [], [], [], [], []
    for g, s in enumerate(segments):
        p = np.arange(s.first_pos, s.first_pos + s.n_tokens, dtype=np.int64)
        aid.append(np.full(s.n_tokens, s.adapter, dtype=np.int32))
        seg.append(np.full(s.n_tokens, g, dtype=np.int32))
        pos.append(p.astype(np.int32))
        slot.append(tables[s.seq][p // block_size] * block_size + p % block_size)
        starts.append(s.activation_start)
    cat = lambda l, dt: (np.concatenate(l).astype(dt) if l else np.zeros(0, dt))
    w = Workload(name=name, dtype=dtype, hidden=hidden, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads,
                 head_dim=head_dim, n_adapters=n_adapters, rank=rank, block_size=block_size,
                 n_slots=n_blocks * block_size, segments=list(segments))
    w.token_adapter_ids = cat(aid, np.int32)
    w.token_seg_ids = cat(seg, np.int32)
    w.token_positions = cat(pos, np.int32)
    w.slot_mapping = cat(slot, np.int64)
    w.activation_start = np.asarray(starts, dtype=np.int32).reshape(-1)
    for r in pad_rows:
        w.token_adapter_ids[r] = -1
        w.slot_mapping[r] = -1
    w._tables = tables
    if with_values:
        T = w.T
        w.x = _normal(seed, _ST_X, 0, (T, hidden), x_std, dtype)
        wk = weight_key if weight_key else seed
        w.W = _normal(wk, _ST_W, 0, (hidden, N), hidden ** -0.5, dtype)
        w.A = [_normal(wk, _ST_A, i, (hidden, rank), hidden ** -0.5, dtype) for i in range(n_adapters)]
        w.B = [_normal(wk, _ST_B, i, (rank, N), rank ** -0.5, dtype) for i in range(n_adapters)]
    return w


def with_variants(w: Workload, ranks: Optional[Sequence[int]] = None, bias: bool = False, seed: int = SEED) -> Workload:
    """The same batch with adapter-layout variants: adapter i keeps only its first ranks[i] rank
    components (A[i][:, :r_i], B[i][:r_i, :]), and/or a seeded layer bias ~ N(0, 1)."""
    import copy
    v = copy.copy(w)
    v.name = w.name + "+variants"
    if ranks is not None:
        assert len(ranks) == w.n_adapters and all(1 <= r <= w.rank for r in ranks)
        v.adapter_ranks = [int(r) for r in ranks]
        v.A = [np.ascontiguousarray(a[:, :r]) for a, r in zip(w.A, ranks)]
        v.B = [np.ascontiguousarray(b[:r, :]) for b, r in zip(w.B, ranks)]
    if bias:
        v.bias = _normal(seed, _ST_BIAS, 0, (w.N,), 1.0, w.dtype)
    return v


def with_per_module_factors(w: Workload, seed: int = SEED):
    """Sec. 2.3 gives every module its own low-rank update (Delta^Q, Delta^K, Delta^V).  Draws separate
    factors A^m_i [hidden, r], B^m_i [r, N_m] with r = w.rank / 3 for m in (Q, K, V) and returns
    (v, A_mod, B_mod): v is the same batch whose fused factors are the block-structured encoding
    A_i = [A^Q_i | A^K_i | A^V_i], B_i = blockdiag(B^Q_i, B^K_i, B^V_i); A_mod[m][i], B_mod[m][i] are the
    module factors in the storage dtype.  Layout only: no arithmetic of the method."""
    import copy
    assert w.rank % 3 == 0
    r = w.rank // 3
    widths = (w.Nq, w.Nkv, w.Nkv)
    A_mod = [[_normal(seed ^ 0x3D, _ST_A, 16 * i + m, (w.hidden, r), w.hidden ** -0.5, w.dtype)
              for i in range(w.n_adapters)] for m in range(3)]
    B_mod = [[_normal(seed ^ 0x3D, _ST_B, 16 * i + m, (r, widths[m]), r ** -0.5, w.dtype)
              for i in range(w.n_adapters)] for m in range(3)]
    v = copy.copy(w)
    v.name = w.name + "+per-module"
    v.A, v.B = [], []
    for i in range(w.n_adapters):
        v.A.append(np.ascontiguousarray(np.concatenate([A_mod[m][i] for m in range(3)], axis=1)))
        Bf = np.zeros((w.rank, w.N), dtype=B_mod[0][i].dtype)     # zero bits are zero in both storage types
        col = 0
        for m in range(3):
            Bf[m * r:(m + 1) * r, col:col + widths[m]] = B_mod[m][i]
            col += widths[m]
        v.B.append(Bf)
    return v, A_mod, B_mod


def sample_rows(w: Workload, n: int) -> np.ndarray:
    """Rows the oracle is timed/checked on: every segment's activation boundary +-2, first and last
    row of every segment, then evenly spaced rows up to n."""
    must = set()
    t0 = 0
    for s in w.segments:
        t1 = t0 + s.n_tokens
        must.update((t0, t1 - 1))
        b = t0 + (s.activation_start - s.first_pos)
        for d in range(-2, 3):
            if t0 <= b + d < t1:
                must.add(b + d)
        t0 = t1
    must = sorted(must)[:n]
    rest = [int(t) for t in np.linspace(0, w.T - 1, num=max(n - len(must), 0), dtype=np.int64)]
    return np.array(sorted(set(must) | set(rest)), dtype=np.int32)



# --------------------------------------------------------------------------------------
# the five benchmark configurations
# --------------------------------------------------------------------------------------
_W8B = SEED ^ 0x8B8B8B8B      # weights shared by every 8B-shaped config
_W70B = SEED ^ 0x70707070


def config1(seed: int = SEED, with_values: bool = True) -> Workload:
    """Tiny fp32 layer: 2 sequences x 32 tokens, activation at 24 and at 32 (never)."""
    segs = [Segment(0, 0, 32, 0, 24), Segment(1, 0, 32, 1, 32)]
    return assemble("cfg1-tiny-f32", "f32", 256, 4, 2, 64, 2, 8, 16, segs, [32, 32],
                    seed=seed ^ 1, extra_blocks=4, with_values=with_values)


def config2(seed: int = SEED, with_values: bool = True) -> Workload:
    """Llama-3-8B-shaped prefill chunk: 8 sequences x 512 tokens, 8 rank-32 adapters."""
    g = _rng(seed ^ 2, _ST_STRUCT)
    segs = []
    for s in range(8):
        segs.append(Segment(s, 0, 512, int(g.integers(0, 8)), int(g.integers(256, 512))))
    return assemble("cfg2-8b-prefill", "bf16", 4096, 32, 8, 128, 8, 32, 16, segs, [512] * 8,
                    seed=seed ^ 2, weight_key=_W8B, with_values=with_values)


def config3(seed: int = SEED, with_values: bool = True) -> Workload:
    """Llama-3-8B-shaped decode: 256 sequences x 1 token, 16 adapters, 25% base-only rows."""
    g = _rng(seed ^ 3, _ST_STRUCT)
    base_rows = set(g.permutation(256)[:64].tolist())
    segs = []
    for s in range(256):
        p = int(g.integers(1, 2048))
        a = int(g.integers(0, 16))
        st = int(g.integers(0, p + 1))
        segs.append(Segment(s, p, 1, -1 if s in base_rows else a, st))
    return assemble("cfg3-8b-decode", "bf16", 4096, 32, 8, 128, 16, 32, 16, segs, [2048] * 256,
                    seed=seed ^ 3, weight_key=_W8B, with_values=with_values)


def config4(seed: int = SEED, with_values: bool = True) -> Workload:
    """Llama-3-70B-shaped prefill: 4 sequences x 2048 tokens, 4 rank-64 adapters, late activation."""
    g = _rng(seed ^ 4, _ST_STRUCT)
    segs = [Segment(s, 0, 2048, int(g.integers(0, 4)), int(g.integers(1844, 2048))) for s in range(4)]
    return assemble("cfg4-70b-prefill", "bf16", 8192, 64, 8, 128, 4, 64, 16, segs, [2048] * 4,
                    seed=seed ^ 4, weight_key=_W70B, with_values=with_values)


def config5(seed: int = SEED, with_values: bool = True) -> Workload:
    """Long-context multi-turn mix on 8B shapes: 4 x 16384-token sequences whose base-aligned
    prefix (a multiple of 16 tokens, 60-90% of the sequence) is already cached and skipped;
    each projected suffix holds 1-3 (adapter, activation point) segments."""
    g = _rng(seed ^ 5, _ST_STRUCT)
    segs, prefix = [], []
    for s in range(4):
        pre = 16 * int(g.integers(615, 922))
        prefix.append(pre)
        n_seg = int(g.integers(1, 4))
        cuts = sorted(int(c) for c in g.choice(np.arange(pre + 64, 16384 - 64), size=n_seg - 1, replace=False))
        bounds = [pre] + cuts + [16384]
        for b0, b1 in zip(bounds[:-1], bounds[1:]):
            segs.append(Segment(s, b0, b1 - b0, int(g.integers(0, 32)), int(g.integers(b0, b1))))
    w = assemble("cfg5-8b-longctx", "bf16", 4096, 32, 8, 128, 32, 16, 16, segs, [16384] * 4,
                 seed=seed ^ 5, weight_key=_W8B, with_values=with_values)
    pre_slots = []
    for s in range(4):
        p = np.arange(0, prefix[s], dtype=np.int64)
        pre_slots.append(w._tables[s][p // 16] * 16 + p % 16)
    w.cached_prefix_slots = np.concatenate(pre_slots)
    return w


def config6(seed: int = SEED, with_values: bool = True) -> Workload:
    """Adapter-layout variants in one prefill batch (not one of the five headline configurations):
    Llama-3-8B shapes, 8 sequences x 512 tokens mixing base-model requests, standard LoRAs of rank 8
    (activation at 0) and aLoRAs of rank 32 activated in the second half, plus a layer bias."""
    g = _rng(seed ^ 6, _ST_STRUCT)
    kinds = ["alora", "lora", "base", "alora", "lora", "alora", "base", "alora"]
    ranks = [32, 32, 32, 32, 8, 8, 8, 8]          # adapters 0-3: aLoRAs, 4-7: standard LoRAs
    segs = []
    for s, kind in enumerate(kinds):
        if kind == "base":
            segs.append(Segment(s, 0, 512, -1, 0))
        elif kind == "lora":
            segs.append(Segment(s, 0, 512, 4 + int(g.integers(0, 4)), 0))
        else:
            segs.append(Segment(s, 0, 512, int(g.integers(0, 4)), int(g.integers(256, 512))))
    w = assemble("cfg6-8b-mixed-variants", "bf16", 4096, 32, 8, 128, 8, 32, 16, segs, [512] * 8,
                 seed=seed ^ 6, weight_key=_W8B, with_values=with_values)
    if not with_values:
        w.adapter_ranks = ranks
        return w
    v = with_variants(w, ranks=ranks, bias=True, seed=seed ^ 6)
    v.name = w.name
    return v


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5, 6: config6}


def small_mixed(dtype: str = "bf16", hidden: int = 256, n_q_heads: int = 4, n_kv_heads: int = 2,
                head_dim: int = 64, n_adapters: int = 3, rank: int = 16, block_size: int = 16,
                seq_lens: Sequence[int] = (150, 37, 1, 90), seed: int = 7, pad_every: int = 0,
                x_std: float = 1.0) -> Workload:
    """A small heterogeneous batch for parity tests: ragged sequence lengths, every kind of
    request (base-only, standard LoRA = activation at 0, aLoRA activated mid-sequence,
    aLoRA never activated), optional padding rows, spare cache blocks."""
    g = _rng(SEED ^ seed, _ST_STRUCT)
    segs = []
    kinds = ["alora", "lora", "base", "never"]
    for s, n in enumerate(seq_lens):
        kind = kinds[s % 4]
        first = int(g.integers(0, 40))
        a = int(g.integers(0, n_adapters))
        if kind == "base":
            segs.append(Segment(s, first, n, -1, 0))
        elif kind == "lora":
            segs.append(Segment(s, first, n, a, 0))
        elif kind == "never":
            segs.append(Segment(s, first, n, a, first + n))
        else:
            segs.append(Segment(s, first, n, a, first + int(g.integers(0, max(n, 1)))))
    T = sum(seq_lens)
    pads = list(range(pad_every - 1, T, pad_every)) if pad_every else []
    return assemble(f"small-{dtype}-{seed}", dtype, hidden, n_q_heads, n_kv_heads, head_dim,
                    n_adapters, rank, block_size, segs,
                    [s.first_pos + s.n_tokens for s in segs], seed=SEED ^ seed,
                    extra_blocks=5, pad_rows=pads, x_std=x_std)


# --------------------------------------------------------------------------------------
# inputs of the cache reader (attention over the paged K/V cache)
# --------------------------------------------------------------------------------------
@dataclass
class AttentionCase:
    """Query rows, a paged K/V cache and the block tables to read it through.  Values only: no scores,
    no softmax."""
    name: str
    dtype: str
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    block_size: int
    q: np.ndarray              # [T, n_q_heads*head_dim] storage dtype
    k_cache: np.ndarray        # [n_slots, n_kv_heads*head_dim]
    v_cache: np.ndarray
    block_tables: np.ndarray   # int32 [n_seqs, max_blocks], -1 past a sequence's blocks
    token_seq_ids: np.ndarray  # int32 [T]
    token_positions: np.ndarray  # int32 [T]
    seq_lens: np.ndarray       # tokens cached per sequence (every row's position is below it)

    @property
    def T(self) -> int:
        return int(self.token_seq_ids.shape[0])

    @property
    def context_bytes(self) -> int:
        """K and V bytes the rows' contexts cover (each row reads positions 0..p of all K/V heads)."""
        eb = 2 if self.dtype == "bf16" else 4
        return int((self.token_positions.astype(np.int64) + 1).sum()) * 2 * self.n_kv_heads * self.head_dim * eb


def block_tables_of(w: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """(block_tables int32 [n_seq, max_blocks], token_seq_ids int32 [T]) of a Workload: the sequence of a
    row is the sequence of its segment."""
    tabs = w._tables
    mb = max(len(t) for t in tabs)
    bt = np.full((len(tabs), mb), -1, np.int32)
    for s, t in enumerate(tabs):
        bt[s, :len(t)] = t
    seq_of_seg = np.asarray([sg.seq for sg in w.segments], np.int32)
    return bt, seq_of_seg[w.token_seg_ids]


def attention_case(name: str, dtype: str, seq_lens: Sequence[int], rows_per_seq: Sequence[int], n_q_heads: int,
                   n_kv_heads: int, head_dim: int, block_size: int, seed: int = SEED, extra_blocks: int = 2,
                   table_slack: int = 1, kv_std: float = 1.0) -> AttentionCase:
    """Sequence s holds seq_lens[s] cached tokens; its last rows_per_seq[s] positions are query rows (a
    decode step has one, a projected suffix several).  Physical blocks are a seeded permutation; slots
    no context covers (spare blocks, tails of last blocks) hold NaN so that a read of them shows."""
    lens = np.asarray(seq_lens, np.int64)
    nb = (lens + block_size - 1) // block_size
    n_blocks = int(nb.sum()) + extra_blocks
    perm = _rng(seed, _ST_SLOTS, 1).permutation(n_blocks)
    bt = np.full((len(lens), int(nb.max()) + table_slack), -1, np.int32)
    covered = np.zeros(n_blocks * block_size, bool)
    o = 0
    for s in range(len(lens)):
        bt[s, :nb[s]] = perm[o:o + nb[s]]
        j = np.arange(lens[s])
        covered[perm[o:o + nb[s]][j // block_size] * block_size + j % block_size] = True
        o += int(nb[s])
    seq, pos = [], []
    for s in range(len(lens)):
        r = int(min(rows_per_seq[s], lens[s]))
        seq += [s] * r
        pos += list(range(int(lens[s]) - r, int(lens[s])))
    width = n_kv_heads * head_dim
    kc = _normal(seed, _ST_CACHE, 10, (n_blocks * block_size, width), kv_std, "f32")
    vc = _normal(seed, _ST_CACHE, 11, (n_blocks * block_size, width), kv_std, "f32")
    kc[~covered] = np.nan
    vc[~covered] = np.nan
    q = _normal(seed, _ST_Q, 0, (len(seq), n_q_heads * head_dim), 1.0, dtype)
    if dtype == "bf16":
        kc, vc = f32_to_bf16_bits(kc), f32_to_bf16_bits(vc)
    return AttentionCase(name, dtype, n_q_heads, n_kv_heads, head_dim, block_size, q, kc, vc, bt,
                         np.asarray(seq, np.int32), np.asarray(pos, np.int32), lens)


def rope_table(max_pos: int, head_dim: int, base: float = 10000.0) -> Tuple[np.ndarray, np.ndarray]:
    """(cos, sin) fp32 [max_pos, head_dim / 2] of the angles position * base ** (-2 i / head_dim): the table a
    serving engine keeps as a constant buffer of the model and hands to the projection as an input."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    ang = np.arange(max_pos, dtype=np.float64)[:, None] * base ** (-2.0 * i / head_dim)[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)
