"""GPU parity of the paged-cache reader (alora_paged_attention) against the fp64 oracle
(oracle/attention.py: causal softmax attention, Sec. 2.1), through the C ABI.

Slots no context covers hold NaN in every case, so a read outside a row's causal context shows up
as a NaN in the output."""
import numpy as np
import pytest
import torch

from oracle import attention as oatt
from paper_2512_17910_amd import binding as ab
from paper_2512_17910_amd import workloads as wl
from gpu_util import TOL, maxnorm_rel, raw_bits, to_dev, to_f64

pytestmark = pytest.mark.gpu


class DeviceCase:
    def __init__(self, c: wl.AttentionCase, scale: float = 0.0):
        self.c = c
        self.q = to_dev(c.q, c.dtype)
        self.kc = to_dev(c.k_cache, c.dtype)
        self.vc = to_dev(c.v_cache, c.dtype)
        self.bt = torch.from_numpy(c.block_tables).to("cuda")
        self.seq = torch.from_numpy(c.token_seq_ids).to("cuda")
        self.pos = torch.from_numpy(c.token_positions).to("cuda")
        self.out = torch.full_like(self.q, float("nan"))
        self.dims = ab.make_attn_dims(self.q, self.kc, self.bt, c.n_q_heads, c.n_kv_heads, c.head_dim, c.block_size, scale)

    def run(self):
        ab.alora_paged_attention(self.q, self.kc, self.vc, self.bt, self.seq, self.pos, self.out, self.dims)
        torch.cuda.synchronize()
        return self.out

    def oracle(self, rows=None, scale=None):
        c = self.c
        return oatt.paged_attention(wl.widen_f64(c.q, c.dtype), wl.widen_f64(c.k_cache, c.dtype),
                                    wl.widen_f64(c.v_cache, c.dtype), c.block_tables, c.token_seq_ids,
                                    c.token_positions, c.block_size, c.n_q_heads, c.n_kv_heads, c.head_dim,
                                    scale=scale, rows=rows)


def _ragged_lens(seed, n, hi):
    rng = np.random.default_rng(seed)
    lens = rng.integers(1, hi + 1, n)
    lens[0] = 1                       # a context of one position
    lens[1] = hi
    return lens


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("head_dim", [64, 128])
@pytest.mark.parametrize("group", [1, 2, 4, 8])
def test_matches_the_oracle_on_ragged_contexts(dtype, head_dim, group):
    n_kv = 2
    lens = _ragged_lens(100 + group + head_dim, 9, 333)
    rows = [1, 3, 1, 2, 1, 5, 1, 1, 4]
    for bs in (16, 5):                # a power of two and not
        c = wl.attention_case(f"ragged-{dtype}-d{head_dim}-g{group}-bs{bs}", dtype, lens, rows, n_kv * group, n_kv,
                              head_dim, bs, seed=wl.SEED ^ (head_dim * 8 + group))
        print(f"[case] {c.name} T={c.T} lens={list(lens)}", flush=True)
        d = DeviceCase(c)
        assert ab.alora_paged_attention_validate(d.bt, d.seq, d.pos, d.dims) == ab.ALORA_OK
        out = to_f64(d.run())
        assert np.isfinite(out).all()
        assert maxnorm_rel(out, d.oracle()) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_long_contexts_and_explicit_scale(dtype):
    lens = [5000, 4097, 4096, 63, 64, 65, 1023]
    c = wl.attention_case(f"long-{dtype}", dtype, lens, [2, 1, 1, 1, 1, 1, 1], 8, 2, 128, 16, seed=wl.SEED ^ 77)
    print(f"[case] {c.name}", flush=True)
    d = DeviceCase(c, scale=0.05)
    out = to_f64(d.run())
    assert np.isfinite(out).all()
    assert maxnorm_rel(out, d.oracle(scale=0.05)) <= TOL[dtype]


def test_contexts_of_sixteen_thousand_positions():
    """The long-context shape of the reader's benchmark (--long): 32 query / 8 K/V heads of 128, contexts
    of 16384 and 8193 positions, every output element against the oracle."""
    c = wl.attention_case("16k", "bf16", [16384, 8193, 12000], [1, 2, 1], 32, 8, 128, 16, seed=wl.SEED ^ 91)
    d = DeviceCase(c)
    out = to_f64(d.run())
    assert np.isfinite(out).all()
    assert maxnorm_rel(out, d.oracle()) <= TOL["bf16"]


def test_peaked_scores_do_not_overflow():
    """Large score ranges: keys scaled so that scores span hundreds; the running maximum keeps every power
    of two in range."""
    c = wl.attention_case("peaked", "bf16", [700, 300, 40], [1, 2, 3], 4, 1, 128, 16, seed=wl.SEED ^ 5, kv_std=6.0)
    d = DeviceCase(c)
    out = to_f64(d.run())
    assert np.isfinite(out).all()
    assert maxnorm_rel(out, d.oracle()) <= TOL["bf16"]


def test_rows_of_one_sequence_see_exactly_their_causal_context():
    """A projected suffix: 40 consecutive rows of one sequence.  Changing the cached K/V of position j
    changes rows at positions >= j and leaves the rows before it bit-identical."""
    c = wl.attention_case("suffix", "bf16", [200, 90], [40, 1], 8, 2, 64, 16, seed=wl.SEED ^ 9)
    d = DeviceCase(c)
    base = raw_bits(d.run()).copy()
    assert maxnorm_rel(to_f64(d.out), d.oracle()) <= TOL["bf16"]
    j = 180                                             # row index 20 of the suffix (positions 160..199)
    slot = int(c.block_tables[0][j // 16]) * 16 + j % 16
    d.vc[slot] += 1.0
    d.kc[slot] *= -1.0
    after = raw_bits(d.run())
    rows_before = np.flatnonzero((c.token_seq_ids == 0) & (c.token_positions < j))
    rows_after = np.flatnonzero((c.token_seq_ids == 0) & (c.token_positions >= j))
    assert rows_before.size == 20 and rows_after.size == 20
    assert np.array_equal(after[rows_before], base[rows_before])
    assert all((after[r] != base[r]).any() for r in rows_after)
    other = np.flatnonzero(c.token_seq_ids == 1)
    assert np.array_equal(after[other], base[other])


def test_two_calls_give_the_same_bits_and_the_stream_argument_is_honoured():
    c = wl.attention_case("repeat", "bf16", _ragged_lens(3, 40, 900), [1] * 40, 32, 8, 128, 16, seed=wl.SEED ^ 21)
    d = DeviceCase(c)
    first = raw_bits(d.run()).copy()
    d.out.fill_(float("nan"))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    ab.alora_paged_attention(d.q, d.kc, d.vc, d.bt, d.seq, d.pos, d.out, d.dims, stream=side)
    side.synchronize()
    assert np.array_equal(raw_bits(d.out), first)


def test_out_of_range_indices_are_reported_and_never_dereferenced():
    c = wl.attention_case("bad-indices", "bf16", [50, 60, 70], [1, 1, 1], 4, 2, 64, 16, seed=wl.SEED ^ 33)
    d = DeviceCase(c)
    good = to_f64(d.run()).copy()
    n_blocks = c.k_cache.shape[0] // 16
    # a sequence id outside the table, a negative position: rows of zeros
    seq = c.token_seq_ids.copy()
    seq[0] = 7
    pos = c.token_positions.copy()
    pos[1] = -3
    d.seq.copy_(torch.from_numpy(seq))
    d.pos.copy_(torch.from_numpy(pos))
    assert ab.alora_paged_attention_validate(d.bt, d.seq, d.pos, d.dims) == ab.ALORA_EDATA
    out = to_f64(d.run())
    assert (out[0] == 0).all() and (out[1] == 0).all()
    assert np.array_equal(out[2], good[2])
    # table entries outside the cache inside a context: those positions are left out of the softmax
    d.seq.copy_(torch.from_numpy(c.token_seq_ids))
    d.pos.copy_(torch.from_numpy(c.token_positions))
    bt = c.block_tables.copy()
    bt[2, 1] = n_blocks + 5          # positions 16..31 of sequence 2
    bt[2, 3] = -1                    # positions 48..63
    d.bt.copy_(torch.from_numpy(bt))
    assert ab.alora_paged_attention_validate(d.bt, d.seq, d.pos, d.dims) == ab.ALORA_EDATA
    out = to_f64(d.run())
    assert np.isfinite(out).all()
    keep = np.r_[0:16, 32:48, 64:70]
    kc, vc = wl.widen_f64(c.k_cache, "bf16"), wl.widen_f64(c.v_cache, "bf16")
    slots = oatt.context_slots(c.block_tables[2], 70, 16)[keep]
    dense_bt = np.arange((len(keep) + 15) // 16, dtype=np.int32)[None, :]
    kd = np.zeros((dense_bt.size * 16, kc.shape[1])); kd[:len(keep)] = kc[slots]
    vd = np.zeros((dense_bt.size * 16, vc.shape[1])); vd[:len(keep)] = vc[slots]
    ref = oatt.paged_attention(wl.widen_f64(c.q, "bf16")[2:3], kd, vd, dense_bt, np.zeros(1, np.int32),
                               np.asarray([len(keep) - 1], np.int32), 16, 4, 2, 64)
    assert maxnorm_rel(out[2:3], ref) <= TOL["bf16"]
    assert np.array_equal(out[:2], good[:2])


def test_empty_batch_is_a_no_op():
    c = wl.attention_case("empty", "bf16", [20], [1], 4, 2, 64, 16, seed=wl.SEED ^ 41)
    d = DeviceCase(c)
    dims = ab.make_attn_dims(d.q[:0], d.kc, d.bt, 4, 2, 64, 16)
    ab.alora_paged_attention(d.q[:0], d.kc, d.vc, d.bt, d.seq[:0], d.pos[:0], d.out[:0], dims)
    torch.cuda.synchronize()
    assert torch.isnan(d.out).all()


def test_decode_batch_at_benchmark_size_on_sampled_rows():
    """The reader's benchmark configuration (256 decode rows, 32 query / 8 K/V heads of 128, contexts up
    to 2048): every row finite, 24 sampled rows against the oracle."""
    rng = np.random.default_rng(8)
    lens = rng.integers(2, 2049, 256)
    c = wl.attention_case("decode-256", "bf16", lens, [1] * 256, 32, 8, 128, 16, seed=wl.SEED ^ 55)
    d = DeviceCase(c)
    out = to_f64(d.run())
    assert np.isfinite(out).all()
    rows = np.r_[np.argmax(lens), np.argmin(lens), rng.choice(256, 22, replace=False)]
    assert maxnorm_rel(out[rows], d.oracle(rows=rows)) <= TOL["bf16"]


@pytest.mark.parametrize("dtype,head_dim,group", [("bf16", 128, 4), ("f32", 64, 2), ("bf16", 64, 8), ("bf16", 128, 1)])
def test_split_contexts_match_the_oracle_and_the_single_pass(dtype, head_dim, group):
    """Few rows: every context is cut into up to 32 parts that a second kernel combines.  Ragged contexts
    (shorter than one part, exactly on part boundaries, thousands of positions), against the oracle and,
    to summation order, against the one-workgroup-per-row call; two calls give the same bits."""
    lens = [1, 3, 64, 65, 4096, 4097, 1000, 2048 * 3 + 17]
    c = wl.attention_case(f"split-{dtype}-{head_dim}-{group}", dtype, lens, [1, 2, 1, 1, 1, 3, 1, 1], 2 * group, 2, head_dim,
                          16, seed=wl.SEED ^ (77 + group))
    d = DeviceCase(c)
    nbytes = ab.alora_paged_attention_workspace_bytes(d.dims)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    ab.alora_paged_attention_split(d.q, d.kc, d.vc, d.bt, d.seq, d.pos, d.out, d.dims, ws)
    torch.cuda.synchronize()
    got = to_f64(d.out)
    bits = raw_bits(d.out).copy()
    assert np.isfinite(got).all()
    assert maxnorm_rel(got, d.oracle()) <= TOL[dtype]
    single = to_f64(d.run())
    assert maxnorm_rel(got, single) <= TOL[dtype]
    ws.fill_(0xFF)                                  # leftovers in the workspace do not matter
    d.out.fill_(float("nan"))
    ab.alora_paged_attention_split(d.q, d.kc, d.vc, d.bt, d.seq, d.pos, d.out, d.dims, ws)
    torch.cuda.synchronize()
    assert np.array_equal(raw_bits(d.out), bits)
    with pytest.raises(ab.AloraError):
        ab.alora_paged_attention_split(d.q, d.kc, d.vc, d.bt, d.seq, d.pos, d.out, d.dims, ws[: nbytes - 16])


def test_split_call_on_a_large_batch_is_the_single_pass():
    c = wl.attention_case("split-large", "bf16", _ragged_lens(4, 140, 300), [1] * 140, 32, 8, 128, 16, seed=wl.SEED ^ 23)
    d = DeviceCase(c)
    assert ab.alora_paged_attention_workspace_bytes(d.dims) == 0          # 140 rows x 8 K/V heads fill the chip
    first = raw_bits(d.run()).copy()
    d.out.fill_(float("nan"))
    ab.alora_paged_attention_split(d.q, d.kc, d.vc, d.bt, d.seq, d.pos, d.out, d.dims, None)
    torch.cuda.synchronize()
    assert np.array_equal(raw_bits(d.out), first)


def _run_suffix(d):
    d.out.fill_(float("nan"))
    ab.alora_paged_attention_suffix(d.q, d.kc, d.vc, d.bt, d.seq, d.pos, d.out, d.dims)
    torch.cuda.synchronize()
    return d.out


@pytest.mark.parametrize("group", [1, 2, 4, 8])
def test_suffix_rows_share_their_context_and_match_the_oracle(group):
    """Runs of consecutive rows (projected suffixes of 1..70 rows starting at arbitrary positions), single
    decode rows in between, contexts from 1 to thousands of positions, block sizes 16 and 5: every row
    against the oracle; uncovered slots hold NaN."""
    lens = [1, 40, 333, 64, 2500, 97, 1031]
    rows = [1, 40, 70, 1, 33, 5, 8]
    for bs in (16, 5):
        c = wl.attention_case(f"suffix-g{group}-bs{bs}", "bf16", lens, rows, 2 * group, 2, 128, bs, seed=wl.SEED ^ (300 + group))
        print(f"[case] {c.name} T={c.T}", flush=True)
        d = DeviceCase(c)
        out = to_f64(_run_suffix(d))
        assert np.isfinite(out).all()
        assert maxnorm_rel(out, d.oracle()) <= TOL["bf16"]


def test_suffix_call_on_a_decode_batch_and_on_interleaved_rows():
    """No two batch rows continue each other: every row is a block of its own."""
    rng = np.random.default_rng(5)
    lens = rng.integers(1, 700, 60)
    c = wl.attention_case("suffix-decode", "bf16", lens, [1] * 60, 32, 8, 128, 16, seed=wl.SEED ^ 61)
    d = DeviceCase(c)
    out = to_f64(_run_suffix(d))
    assert maxnorm_rel(out, d.oracle()) <= TOL["bf16"]
    # rows of two sequences interleaved (positions consecutive per sequence, but not in the batch)
    c2 = wl.attention_case("suffix-interleaved", "bf16", [300, 300], [16, 16], 8, 2, 128, 16, seed=wl.SEED ^ 62)
    order = np.arange(32).reshape(2, 16).T.reshape(-1)
    c2.q, c2.token_seq_ids, c2.token_positions = c2.q[order], c2.token_seq_ids[order], c2.token_positions[order]
    d2 = DeviceCase(c2)
    out2 = to_f64(_run_suffix(d2))
    assert maxnorm_rel(out2, d2.oracle()) <= TOL["bf16"]


def _mixed_batch(seed, n_q, n_kv, min_rows):
    """Decode rows and projected suffixes of 2..70 rows side by side, short contexts: at least min_rows rows."""
    rng = np.random.default_rng(seed)
    rows, lens = [], []
    while sum(rows) < min_rows:
        r = 1 if rng.random() < 0.6 else int(rng.integers(2, 71))
        rows.append(r)
        lens.append(r + int(rng.integers(0, 150)))
    return wl.attention_case(f"suffix-mixed-{n_q}-{n_kv}", "bf16", lens, rows, n_q, n_kv, 128, 16, seed=wl.SEED ^ seed)


@pytest.mark.parametrize("heads", [(8, 8), (32, 8)])
def test_suffix_call_on_a_batch_large_enough_for_whole_row_blocks_per_workgroup(heads):
    """More than 8192 rows x 8 K/V heads: a workgroup then owns 32 batch rows and works through every block
    that starts among them (decode rows: up to 32 blocks, runs: one or two), with the permuted range index
    where a block spans several ranges (group size 1: 128 rows).  Sampled rows against the oracle, all rows
    finite, and all rows equal to the per-row kernel's within the tolerance."""
    c = _mixed_batch(77 + heads[0], heads[0], heads[1], 8300)
    print(f"[case] {c.name} T={c.T}", flush=True)
    d = DeviceCase(c)
    out = to_f64(_run_suffix(d)).copy()
    assert np.isfinite(out).all()
    per_row = to_f64(d.run())
    assert maxnorm_rel(out, per_row) <= TOL["bf16"]
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([rng.integers(0, c.T, 400), np.arange(64), np.arange(c.T - 64, c.T)]))
    assert maxnorm_rel(out[rows], d.oracle(rows=rows)) <= TOL["bf16"]


def test_suffix_call_at_benchmark_size_on_sampled_rows():
    """The row-block reader's benchmark shape (4 sequences of 16384 positions, the last 2048 of each are query
    rows, 32 query / 8 K/V heads of 128, block size 16): every row finite, 40 sampled rows (first and last
    rows of runs and of row blocks among them) against the oracle; the window of table entries is refilled
    seven times per row block at this length."""
    c = wl.attention_case("suffix-4x16384", "bf16", [16384] * 4, [2048] * 4, 32, 8, 128, 16, seed=wl.SEED ^ 91)
    d = DeviceCase(c)
    out = to_f64(_run_suffix(d))
    assert np.isfinite(out).all()
    rng = np.random.default_rng(9)
    rows = np.unique(np.r_[0, 31, 32, 2047, 2048, 4095 + 33, c.T - 1, rng.choice(c.T, 33, replace=False)])
    assert maxnorm_rel(out[rows], d.oracle(rows=rows)) <= TOL["bf16"]


@pytest.mark.parametrize("group", [1, 4, 8])
def test_suffix_split_cuts_the_context_of_few_row_blocks_into_parts(group):
    """Short suffixes over long contexts (the shape of an aLoRA request): few row blocks, so every block's
    context is cut into parts that a second kernel combines.  Contexts shorter than one part, on part
    boundaries, across several table windows (more than 2048 positions per part); against the oracle, against
    the unsplit call (to summation order), and two calls give the same bits."""
    lens = [5000, 37, 2048 * 3 + 17, 64, 9000, 1]
    rows = [16, 5, 33, 1, 40, 1]
    c = wl.attention_case(f"suffix-split-g{group}", "bf16", lens, rows, 2 * group, 2, 128, 16, seed=wl.SEED ^ (500 + group))
    d = DeviceCase(c)
    nbytes = ab.alora_paged_attention_suffix_workspace_bytes(d.dims)
    assert nbytes > 0
    ws = torch.full((nbytes,), 0xff, dtype=torch.uint8, device="cuda")      # NaN patterns: every entry read is written first
    d.out.fill_(float("nan"))
    ab.alora_paged_attention_suffix_split(d.q, d.kc, d.vc, d.bt, d.seq, d.pos, d.out, d.dims, ws)
    torch.cuda.synchronize()
    got = to_f64(d.out)
    bits = raw_bits(d.out).copy()
    assert np.isfinite(got).all()
    assert maxnorm_rel(got, d.oracle()) <= TOL["bf16"]
    assert maxnorm_rel(got, to_f64(_run_suffix(d))) <= 2.0 ** -7
    d.out.fill_(float("nan"))
    ab.alora_paged_attention_suffix_split(d.q, d.kc, d.vc, d.bt, d.seq, d.pos, d.out, d.dims, ws)
    torch.cuda.synchronize()
    assert np.array_equal(raw_bits(d.out), bits)
    # too small a workspace is refused
    with pytest.raises(ab.AloraError) as e:
        ab.alora_paged_attention_suffix_split(d.q, d.kc, d.vc, d.bt, d.seq, d.pos, d.out, d.dims, ws[:nbytes // 2])
    assert e.value.status == ab.ALORA_EWORKSPACE


def test_suffix_split_on_a_large_batch_is_the_unsplit_call():
    c = _mixed_batch(91, 8, 8, 8300)
    d = DeviceCase(c)
    assert ab.alora_paged_attention_suffix_workspace_bytes(d.dims) == 0
    first = raw_bits(_run_suffix(d)).copy()
    d.out.fill_(float("nan"))
    ab.alora_paged_attention_suffix_split(d.q, d.kc, d.vc, d.bt, d.seq, d.pos, d.out, d.dims, None)
    torch.cuda.synchronize()
    assert np.array_equal(raw_bits(d.out), first)


@pytest.mark.parametrize("seed", range(10))
def test_suffix_calls_on_random_batches_agree_with_the_oracle_and_the_per_row_kernel(seed):
    """Random mixes of decode rows and runs, group sizes 1..8, block sizes that are powers of two, multiples of
    four that are not (12, 20, 24: divisions instead of shifts) and neither (6: served by the per-row kernel),
    contexts up to a few thousand positions; the unsplit and the split call."""
    rng = np.random.default_rng(1000 + seed)
    group = int(rng.choice([1, 2, 4, 8]))
    bs = [4, 12, 16, 20, 64, 24, 8, 6, 32, 128][seed]
    n_seq = int(rng.integers(1, 9))
    rows = [int(rng.choice([1, 1, int(rng.integers(2, 150))])) for _ in range(n_seq)]
    lens = [r + int(rng.integers(0, 2600)) for r in rows]
    c = wl.attention_case(f"suffix-random-{seed}", "bf16", lens, rows, 2 * group, 2, 128, bs, seed=wl.SEED ^ (900 + seed))
    print(f"[case] {c.name} G={group} bs={bs} rows={rows} lens={lens}", flush=True)
    d = DeviceCase(c)
    want = d.oracle()
    per_row = to_f64(d.run()).copy()
    assert maxnorm_rel(per_row, want) <= TOL["bf16"]
    got = to_f64(_run_suffix(d))
    assert np.isfinite(got).all() and maxnorm_rel(got, want) <= TOL["bf16"]
    ws = torch.full((max(ab.alora_paged_attention_suffix_workspace_bytes(d.dims), 16),), 0xff, dtype=torch.uint8, device="cuda")
    d.out.fill_(float("nan"))
    ab.alora_paged_attention_suffix_split(d.q, d.kc, d.vc, d.bt, d.seq, d.pos, d.out, d.dims, ws)
    torch.cuda.synchronize()
    got = to_f64(d.out)
    assert np.isfinite(got).all() and maxnorm_rel(got, want) <= TOL["bf16"]


def test_suffix_call_gives_the_same_bits_on_every_call():
    """The row-block kernel takes no timing-dependent decision: 200 calls on one batch (blocks that need no
    mask, diagonal blocks, single rows), every one bit-identical to the first."""
    c = wl.attention_case("suffix-repeat", "bf16", [200, 90, 700], [40, 1, 65], 8, 2, 128, 16, seed=wl.SEED ^ 9)
    d = DeviceCase(c)
    first = raw_bits(_run_suffix(d)).copy()
    assert maxnorm_rel(to_f64(d.out), d.oracle()) <= TOL["bf16"]
    for it in range(200):
        assert np.array_equal(raw_bits(_run_suffix(d)), first), it


def test_suffix_call_causal_boundaries_bad_indices_and_shapes():
    c = wl.attention_case("suffix-causal", "bf16", [200, 90], [40, 1], 8, 2, 128, 16, seed=wl.SEED ^ 9)
    d = DeviceCase(c)
    base = raw_bits(_run_suffix(d)).copy()
    assert maxnorm_rel(to_f64(d.out), d.oracle()) <= TOL["bf16"]
    j = 180
    slot = int(c.block_tables[0][j // 16]) * 16 + j % 16
    d.vc[slot] += 1.0
    d.kc[slot] *= -1.0
    after = raw_bits(_run_suffix(d))
    before_rows = np.flatnonzero((c.token_seq_ids == 0) & (c.token_positions < j))
    after_rows = np.flatnonzero((c.token_seq_ids == 0) & (c.token_positions >= j))
    assert np.array_equal(after[before_rows], base[before_rows])
    assert all((after[r] != base[r]).any() for r in after_rows)
    # a row with a bad sequence id gets zeros, its neighbours are unaffected
    seq = c.token_seq_ids.copy()
    seq[10] = 99
    d.seq.copy_(torch.from_numpy(seq))
    out = to_f64(_run_suffix(d))
    assert (out[10] == 0).all() and np.isfinite(out).all()
    # fp32 and head_dim 64 are not served by this entry point
    c3 = wl.attention_case("suffix-f32", "f32", [20], [2], 4, 2, 128, 16, seed=wl.SEED ^ 1)
    d3 = DeviceCase(c3)
    with pytest.raises(ab.AloraError):
        ab.alora_paged_attention_suffix(d3.q, d3.kc, d3.vc, d3.bt, d3.seq, d3.pos, d3.out, d3.dims)
