"""GPU parity: the HIP path, called through the C ABI, against the CPU fp64 oracle on the same
seeded inputs.  Integer/index results bit-exact; floating point within the stated max-norm
relative error (1e-5 fp32, 2e-2 bf16); pre-activation rows bit-identical to a base-only GPU run."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_17910_amd import binding as ab
from paper_2512_17910_amd import workloads as wl
from gpu_util import DeviceBatch, TOL, check_grouping, host_operands, maxnorm_rel, raw_bits, to_dev, to_f64

pytestmark = pytest.mark.gpu


def _oracle_full(w):
    x, W, A, B = host_operands(w)
    k0 = wl.widen_f64(wl.cache_fill(w.n_slots, w.Nkv, w.dtype, 0), w.dtype)
    v0 = wl.widen_f64(wl.cache_fill(w.n_slots, w.Nkv, w.dtype, 1), w.dtype)
    bias = wl.widen_f64(w.bias, w.dtype) if w.bias is not None else None
    return oracle.alora_qkv_forward(x, w.token_adapter_ids, w.token_seg_ids, w.token_positions,
                                    w.activation_start, W, A, B, w.slot_mapping, w.block_size, w.Nq, w.Nkv, k0, v0,
                                    bias=bias)


def _check_full(w, db=None, elementwise=True):
    """Every element of q_out and of both caches against the oracle."""
    print(f"[case] {w.name} T={w.T} H={w.hidden} N={w.N} L={w.n_adapters} r={w.rank}", flush=True)
    db = db or DeviceBatch(w)
    assert db.validate() == ab.ALORA_OK
    db.forward()
    ref = _oracle_full(w)
    tol = TOL[w.dtype]
    q, kc, vc = to_f64(db.q), to_f64(db.kc), to_f64(db.vc)
    wr = ref.written_slots
    assert maxnorm_rel(q, ref.q_out) <= tol
    assert maxnorm_rel(kc[wr], ref.k_cache[wr]) <= tol
    assert maxnorm_rel(vc[wr], ref.v_cache[wr]) <= tol
    if elementwise:
        # tighter, per element: one rounding to storage precision plus fp32 accumulation noise
        u, floor = (2.0 ** -8, 2.0 ** -12) if w.dtype == "bf16" else (2.0 ** -20, 4e-6)
        scale = np.max(np.abs(ref.q_out)) if ref.q_out.size else 1.0
        for got, want in ((q, ref.q_out), (kc[wr], ref.k_cache[wr]), (vc[wr], ref.v_cache[wr])):
            assert np.all(np.abs(got - want) <= u * np.abs(want) + floor * scale)
    # slots that no token names keep their bytes
    un = np.setdiff1d(np.arange(w.n_slots), wr)
    assert np.array_equal(raw_bits(db.kc)[un], raw_bits(db.k0)[un])
    assert np.array_equal(raw_bits(db.vc)[un], raw_bits(db.v0)[un])
    # integer results left in the workspace
    check_grouping(*ab.workspace_int_views(db.dims, db.ws), ref.active, ref.perm, ref.offsets)
    return db, ref


def test_config1_fp32():
    db, ref = _check_full(wl.config1())
    assert int(ref.active.sum()) == 8


SMALL = [
    dict(dtype="bf16", seed=1),
    dict(dtype="bf16", seed=2, seq_lens=(300, 41, 1, 77, 256, 3), pad_every=17),
    dict(dtype="bf16", seed=3, n_q_heads=5, n_kv_heads=2, head_dim=40, hidden=192, rank=8, seq_lens=(70, 9)),
    dict(dtype="bf16", seed=4, rank=64, n_adapters=2, hidden=128, seq_lens=(33, 64, 31)),
    dict(dtype="bf16", seed=5, rank=24, n_adapters=5, hidden=320, n_q_heads=9, head_dim=32, seq_lens=(513, 5)),
    dict(dtype="f32", seed=6, hidden=100, n_q_heads=3, n_kv_heads=1, head_dim=20, rank=5, seq_lens=(70, 9, 130)),
    dict(dtype="f32", seed=7, rank=64, pad_every=5),
]


@pytest.mark.parametrize("kw", SMALL, ids=[f"{k['dtype']}-{k['seed']}" for k in SMALL])
def test_small_mixed(kw):
    _check_full(wl.small_mixed(**kw))


@pytest.fixture
def tuning():
    """Force a tiling of the bf16 path for one test, restore the automatic choice afterwards."""
    yield ab.alora_qkv_set_tuning
    ab.alora_qkv_set_tuning(0, 0)


# (feature tiles, splits): every kernel variant, fused and split, on multi-tile ragged batches
TILINGS = [(4, 1), (3, 1), (2, 1), (4, 2), (3, 4), (2, 3), (0, 0)]


@pytest.mark.parametrize("ft,sp", TILINGS, ids=[f"tiles{a}-splits{b}" for a, b in TILINGS])
def test_every_tiling_matches_the_oracle(tuning, ft, sp):
    tuning(ft, sp)
    _check_full(wl.small_mixed("bf16", seed=2, seq_lens=(300, 41, 1, 77, 256, 3), pad_every=17))
    _check_full(wl.small_mixed("bf16", seed=5, rank=24, n_adapters=5, hidden=320, n_q_heads=9, head_dim=32,
                               seq_lens=(513, 5)))
    _check_full(wl.small_mixed("bf16", seed=4, rank=64, n_adapters=2, hidden=128, seq_lens=(33, 64, 31)))
    # fewer 32-wide K-slices than the LDS ring has stages (hidden 64), and a slice count that is no
    # multiple of the ring depth (hidden 448: 14 slices)
    _check_full(wl.small_mixed("bf16", seed=11, rank=8, n_adapters=2, hidden=64, seq_lens=(70, 200, 9)))
    _check_full(wl.small_mixed("bf16", seed=12, rank=32, n_adapters=4, hidden=448, n_q_heads=3, head_dim=64,
                               seq_lens=(260, 31)))
    # the narrowest matrices the bf16 path takes: 24 output features (a weight row is shorter than the step
    # between two copies of a tile), rank 8 (so is a row of the shrink result)
    _check_full(wl.small_mixed("bf16", seed=13, rank=8, n_adapters=3, hidden=64, n_q_heads=1, n_kv_heads=1, head_dim=8,
                               seq_lens=(40, 7, 300)))


@pytest.mark.parametrize("ft,sp", [(4, 1), (2, 4)], ids=["fused", "split"])
def test_pre_activation_bit_identity_in_both_paths(tuning, ft, sp):
    tuning(ft, sp)
    test_pre_activation_rows_bit_identical_to_base_run("bf16")


def test_decode_like_many_adapters():
    """One token per sequence, many adapters inside one tile, some base-only rows."""
    segs = []
    rng = np.random.default_rng(9)
    for s in range(200):
        p = int(rng.integers(1, 100))
        a = -1 if s % 5 == 0 else int(rng.integers(0, 16))
        segs.append(wl.Segment(s, p, 1, a, int(rng.integers(0, p + 1))))
    w = wl.assemble("decode-like", "bf16", 256, 4, 2, 64, 16, 32, 16, segs, [100] * 200, seed=99, extra_blocks=3)
    _check_full(w)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_pre_activation_rows_bit_identical_to_base_run(dtype):
    w = wl.small_mixed(dtype, seed=2, seq_lens=(300, 41, 1, 77, 256, 3))
    db = DeviceBatch(w)
    db.forward()
    q1, k1, v1 = raw_bits(db.q), raw_bits(db.kc), raw_bits(db.vc)
    db.reset()
    base_ids = torch.full_like(db.aid, -1)
    db.forward(aid=base_ids)
    q0, k0, v0 = raw_bits(db.q), raw_bits(db.kc), raw_bits(db.vc)
    _, act = oracle.classify(w.token_adapter_ids, w.token_seg_ids, w.token_positions, w.activation_start)
    pre = act == 0
    assert pre.any() and (~pre).any()
    assert np.array_equal(q1[pre], q0[pre])
    sl = w.slot_mapping
    pre_slots = sl[pre & (sl >= 0)]
    assert np.array_equal(k1[pre_slots], k0[pre_slots]) and np.array_equal(v1[pre_slots], v0[pre_slots])
    act_rows = ~pre
    assert not np.array_equal(q1[act_rows], q0[act_rows])
    # run-to-run determinism of the adapted call
    db.reset()
    db.forward()
    assert np.array_equal(raw_bits(db.q), q1) and np.array_equal(raw_bits(db.kc), k1)
    assert np.array_equal(raw_bits(db.vc), v1)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_base_rows_never_see_adapter_data(dtype):
    """All rows base-only while A and B hold NaN: the result is the base projection (select, not blend)."""
    w = wl.small_mixed(dtype, seed=1)
    db = DeviceBatch(w)
    base_ids = torch.full_like(db.aid, -1)
    db.forward(aid=base_ids)
    q0 = raw_bits(db.q)
    nanA = [torch.full_like(a, float("nan")) for a in db.A]
    nanB = [torch.full_like(b, float("nan")) for b in db.B]
    db.reset()
    db.forward(aid=base_ids, A=nanA, B=nanB)
    assert np.array_equal(raw_bits(db.q), q0)
    x, W, _, _ = host_operands(w)
    ref = oracle.base_rows(x, W, np.arange(w.T, dtype=np.int32))
    assert maxnorm_rel(to_f64(db.q), ref[:, : w.Nq]) <= TOL[dtype]
    # mixed batch, NaN only in an adapter no active row uses
    db.reset()
    used = set(int(a) for a in w.token_adapter_ids[w.token_adapter_ids >= 0])
    unused = [i for i in range(w.n_adapters) if i not in used]
    if unused:
        A2 = list(db.A); B2 = list(db.B)
        A2[unused[0]] = nanA[unused[0]]; B2[unused[0]] = nanB[unused[0]]
        db.forward(A=A2, B=B2)
        assert np.isfinite(to_f64(db.q)).all()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_degenerate_batches(dtype):
    # no adapters at all
    w = wl.small_mixed(dtype, seed=8, n_adapters=1, seq_lens=(5, 9))
    w.token_adapter_ids[:] = -1
    w.n_adapters = 0; w.A = []; w.B = []
    _check_full(w)
    # every row adapted from position 0 (standard LoRA)
    segs = [wl.Segment(0, 0, 70, 1, 0), wl.Segment(1, 3, 9, 0, 0)]
    _check_full(wl.assemble("all-active", dtype, 128, 2, 1, 64, 2, 16, 8, segs, [70, 12], seed=5))
    # never activated, and no K/V written anywhere (all slots -1)
    segs = [wl.Segment(0, 0, 40, 0, 40)]
    w = wl.assemble("none-active", dtype, 128, 2, 1, 64, 1, 8, 16, segs, [40], seed=6, pad_rows=range(40))
    w.token_adapter_ids[:] = 0
    _check_full(w)
    # a single token
    _check_full(wl.assemble("one-token", dtype, 64, 1, 1, 32, 1, 8, 4, [wl.Segment(0, 6, 1, 0, 6)], [7], seed=7))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_empty_batch_is_a_noop(dtype):
    w = wl.assemble("empty", dtype, 64, 1, 1, 32, 1, 8, 4, [], [], seed=3, extra_blocks=2)
    db = DeviceBatch(w)
    db.forward()
    assert np.array_equal(raw_bits(db.kc), raw_bits(db.k0))


def test_classify_group_large_random():
    """Grouping alone on batches far larger than one tile, up to the adapter limit."""
    rng = np.random.default_rng(4)
    # 6144 rows is where the grouping switches from one workgroup to 2048-row slices over two launches
    for T, L, G in ((1, 1, 1), (63, 2, 3), (5000, 128, 40), (6143, 7, 5), (6144, 7, 5), (6145, 1, 2), (8193, 128, 9),
                    (26176, 32, 12), (100001, 3, 50)):
        aid = rng.integers(-1, L, size=T).astype(np.int32)
        seg = rng.integers(0, G, size=T).astype(np.int32)
        pos = rng.integers(0, 50, size=T).astype(np.int32)
        start = rng.integers(0, 50, size=G).astype(np.int32)
        mask, act = oracle.classify(aid, seg, pos, start)
        perm, off = oracle.group(aid, act, L)
        d = [torch.from_numpy(a).to("cuda") for a in (aid, seg, pos, start)]
        dims = ab.make_dims(ab.ALORA_BF16, T, 64, 1, 1, 8, L, 8, G, 16, d[1], d[2])
        ws = ab.alloc_workspace(dims)
        a_g, p_g, o_g = ab.alora_qkv_classify_group(d[0], d[3], dims, ws)
        torch.cuda.synchronize()
        check_grouping(a_g, p_g, o_g, act, perm, off)


def test_validate_reports_bad_data():
    w = wl.small_mixed("bf16", seed=1)
    db = DeviceBatch(w)
    assert db.validate() == ab.ALORA_OK
    db.slot[1] = db.slot[0]
    assert db.validate() == ab.ALORA_EDATA
    db.slot[1] = w.n_slots
    assert db.validate() == ab.ALORA_EDATA
    db.slot[1] = -1
    assert db.validate() == ab.ALORA_OK
    db.aid[0] = w.n_adapters
    assert db.validate() == ab.ALORA_EDATA


def _random_shape(rng, dtype):
    """A seeded random small batch: odd head counts and dims, ragged lengths, padding rows."""
    if dtype == "bf16":
        hidden = 64 * int(rng.integers(1, 9))
        head_dim = 8 * int(rng.integers(1, 17))
        rank = 8 * int(rng.integers(1, 9))
    else:
        hidden = 4 * int(rng.integers(4, 80))
        head_dim = 4 * int(rng.integers(1, 20))
        rank = int(rng.integers(1, 65))
    n_seq = int(rng.integers(1, 7))
    return dict(dtype=dtype, hidden=hidden, head_dim=head_dim, n_q_heads=int(rng.integers(1, 8)),
                n_kv_heads=int(rng.integers(1, 4)), n_adapters=int(rng.integers(1, 12)), rank=rank,
                seq_lens=tuple(int(rng.integers(1, 400)) for _ in range(n_seq)),
                pad_every=int(rng.choice([0, 3, 11])), seed=int(rng.integers(1, 1 << 20)))


@pytest.mark.parametrize("dtype,n_cases", [("bf16", 14), ("f32", 6)])
def test_random_shapes_match_the_oracle(dtype, n_cases):
    rng = np.random.default_rng(20250 + len(dtype))
    for _ in range(n_cases):
        kw = _random_shape(rng, dtype)
        print(f"[shape] {kw}", flush=True)
        _check_full(wl.small_mixed(**kw))


# ---- adapter-layout variants: layer bias (Algorithm 1) and one rank per adapter (Sec. 4.1) ----------
VARIANTS = [
    dict(base=dict(dtype="bf16", seed=21, rank=32, n_adapters=4, seq_lens=(300, 41, 77, 256)), ranks=(8, 32, 16, 24), bias=True),
    dict(base=dict(dtype="bf16", seed=22, rank=64, n_adapters=3, hidden=192, seq_lens=(130, 9, 64)), ranks=(64, 8, 40), bias=False),
    dict(base=dict(dtype="bf16", seed=23, rank=16, n_adapters=2), ranks=None, bias=True),
    dict(base=dict(dtype="f32", seed=24, rank=12, n_adapters=3, hidden=100, n_q_heads=3, n_kv_heads=1, head_dim=20,
                   seq_lens=(70, 9, 130)), ranks=(1, 12, 5), bias=True),
]


@pytest.mark.parametrize("v", VARIANTS, ids=[f"{v['base']['dtype']}-{v['base']['seed']}" for v in VARIANTS])
def test_bias_and_per_adapter_ranks_match_the_oracle(v):
    _check_full(wl.with_variants(wl.small_mixed(**v["base"]), ranks=v["ranks"], bias=v["bias"]))


@pytest.mark.parametrize("ft,sp", [(4, 1), (3, 1), (2, 1), (2, 4), (3, 2)], ids=lambda t: str(t))
def test_variants_under_every_tiling(tuning, ft, sp):
    tuning(ft, sp)
    v = VARIANTS[0]
    _check_full(wl.with_variants(wl.small_mixed(**v["base"]), ranks=v["ranks"], bias=v["bias"]))


def test_zero_padded_adapters_equal_native_ranks_on_base_rows_and_within_tolerance_elsewhere():
    """The caller-side alternative (pad every adapter with zero rank components up to the common rank)
    and the native per-adapter ranks describe the same function."""
    base = wl.small_mixed("bf16", seed=25, rank=32, n_adapters=3, seq_lens=(200, 90))
    ranks = (8, 32, 16)
    native = wl.with_variants(base, ranks=ranks)
    import copy
    padded = copy.copy(base)
    padded.A = [np.where(np.arange(32)[None, :] < r, a, 0).astype(a.dtype) for a, r in zip(base.A, ranks)]
    padded.B = [np.where(np.arange(32)[:, None] < r, b, 0).astype(b.dtype) for b, r in zip(base.B, ranks)]
    d1, d2 = DeviceBatch(native), DeviceBatch(padded)
    d1.forward()
    d2.forward()
    assert np.array_equal(raw_bits(d1.q), raw_bits(d2.q))
    assert np.array_equal(raw_bits(d1.kc), raw_bits(d2.kc)) and np.array_equal(raw_bits(d1.vc), raw_bits(d2.vc))


def test_forward_ex_rejects_bad_ranks():
    w = wl.small_mixed("bf16", seed=1)
    db = DeviceBatch(w)
    for bad in ([w.rank + 8] * w.n_adapters, [0] * w.n_adapters, [4] * w.n_adapters):
        with pytest.raises(ab.AloraError) as e:
            ab.alora_qkv_forward_ex(db.x, db.aid, db.start, db.W, db.A, db.B, db.q, db.kc, db.vc, db.slot,
                                    w.block_size, db.dims, db.ws, adapter_ranks=bad)
        assert e.value.status == ab.ALORA_ESHAPE
    assert np.array_equal(raw_bits(db.kc), raw_bits(db.k0))


@pytest.mark.parametrize("variant", ["common-rank", "per-adapter-ranks"])
def test_wide_hidden_high_rank_shrink_cuts_blocks_into_ranges_and_combines_them_in_the_kernel(tuning, variant):
    """hidden 8192 with rank 64: a 32-row block's loads are large enough that the prefill-sized shrink cuts
    it into ranges of the hidden dimension, the last range of a block to finish adding the partials.
    The fused projection is forced (the batch is small), the result matches the oracle, and two calls
    give the same bits whichever range finishes last."""
    w = wl.small_mixed("bf16", seed=21, hidden=8192, rank=64, n_adapters=3, seq_lens=(300, 41, 1, 77, 130, 64),
                       pad_every=23)
    if variant == "per-adapter-ranks":
        w = wl.with_variants(w, ranks=(64, 8, 40), bias=True)
    for ft in (2, 4):
        tuning(ft, 1)
        if variant == "common-rank":
            db, _ = _check_full(w)
        else:
            db = DeviceBatch(w)
            db.forward()
            x, W, A, B = host_operands(w)
            _, act = oracle.classify(w.token_adapter_ids, w.token_seg_ids, w.token_positions, w.activation_start)
            y = oracle.alora_rows_var(x, W, A, B, w.token_adapter_ids, act, np.arange(w.T, dtype=np.int32),
                                      wl.widen_f64(w.bias, w.dtype))
            assert maxnorm_rel(to_f64(db.q), y[:, : w.Nq]) <= TOL["bf16"]
        first = (raw_bits(db.q).copy(), raw_bits(db.kc).copy(), raw_bits(db.vc).copy())
        for _ in range(3):
            db.reset()
            db.forward()
            assert all(np.array_equal(a, b) for a, b in zip(first, (raw_bits(db.q), raw_bits(db.kc), raw_bits(db.vc))))


def _decode_batch(n_rows, n_adapters, rank, kind, seed, hidden=256):
    """n_rows one-token sequences: 'mixed' = base rows, never-activated and activated rows of random
    adapters; 'one' = every row adapted by the last adapter; 'base' = no row adapted."""
    rng = np.random.default_rng(seed)
    segs = []
    for s in range(n_rows):
        p = int(rng.integers(1, 60))
        if kind == "base":
            a, st = -1, 0
        elif kind == "one":
            a, st = n_adapters - 1, 0
        else:
            a = -1 if rng.random() < 0.2 else int(rng.integers(0, n_adapters))
            st = int(rng.integers(0, p + 2))          # p + 1: not activated yet
        segs.append(wl.Segment(s, p, 1, a, st))
    return wl.assemble(f"decode-{kind}-{n_rows}x{n_adapters}r{rank}", "bf16", hidden, 4, 2, 64, n_adapters, rank, 16, segs,
                       [64] * n_rows, seed=500 + seed, extra_blocks=2)


@pytest.mark.parametrize("forced", [(0, 0), (2, 2), (2, 4)], ids=["auto", "128-wide-2-splits", "128-wide-4-splits"])
@pytest.mark.parametrize("n_rows", [1, 31, 32, 33, 64, 255, 256, 257])
def test_batches_of_at_most_256_rows_are_grouped_and_shrunk_inside_the_projection_kernel(tuning, n_rows, forced):
    """Up to 256 rows the split projection kernel classifies, groups and shrinks the batch on workgroups of
    its own (257 rows take the separate kernels): integer results bit-exact against the oracle's stable
    grouping, outputs within tolerance, for many small groups (128 adapters), one full group, no group.
    The forced tilings are the ones that path needs (128-wide tiles, hidden dimension split)."""
    tuning(*forced)
    _check_full(_decode_batch(n_rows, 128, 8, "mixed", n_rows))
    _check_full(_decode_batch(n_rows, 5, 32, "mixed", 1000 + n_rows, hidden=1024))
    _check_full(_decode_batch(n_rows, 3, 16, "one", 2000 + n_rows))
    _check_full(_decode_batch(n_rows, 3, 16, "base", 3000 + n_rows))


def test_in_kernel_grouping_with_bias_and_per_adapter_ranks(tuning):
    tuning(2, 4)
    w = wl.with_variants(_decode_batch(200, 4, 32, "mixed", 77, hidden=2048), ranks=(8, 32, 16, 24), bias=True)
    db = DeviceBatch(w)
    db.forward()
    x, W, A, B = host_operands(w)
    ref_active, act = oracle.classify(w.token_adapter_ids, w.token_seg_ids, w.token_positions, w.activation_start)
    y = oracle.alora_rows_var(x, W, A, B, w.token_adapter_ids, act, np.arange(w.T, dtype=np.int32), wl.widen_f64(w.bias, w.dtype))
    assert maxnorm_rel(to_f64(db.q), y[:, : w.Nq]) <= TOL["bf16"]
    wr = w.slot_mapping[w.slot_mapping >= 0]
    assert maxnorm_rel(to_f64(db.kc)[wr], y[w.slot_mapping >= 0][:, w.Nq: w.Nq + w.Nkv]) <= TOL["bf16"]


def _as_next_layer(w, seed):
    """The same token batch entering another layer: same metadata, new x, W, A, B (and bias)."""
    v = wl.assemble(w.name + "-next", w.dtype, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_adapters, w.rank,
                    w.block_size, w.segments, [s.first_pos + s.n_tokens for s in w.segments], seed=seed, extra_blocks=5)
    for name in ("token_adapter_ids", "token_seg_ids", "token_positions", "activation_start", "slot_mapping"):
        setattr(v, name, getattr(w, name))
    v.n_slots = w.n_slots
    return v


@pytest.mark.parametrize("kw", [dict(dtype="bf16", seed=2, seq_lens=(300, 41, 1, 77, 256, 3), pad_every=17),
                                dict(dtype="bf16", seed=21, hidden=8192, rank=64, n_adapters=3, seq_lens=(300, 41, 1, 77, 130)),
                                dict(dtype="f32", seed=7, rank=64, pad_every=5),
                                dict(dtype="bf16", seed=9, seq_lens=(100, 60))],
                         ids=["bf16-prefill", "bf16-wide-ranged-shrink", "f32", "bf16-decode-sized"])
def test_a_later_layer_reuses_the_grouping_left_in_the_workspace(kw):
    """App. B builds the mask once per forward pass.  Layer 1 runs the whole call; layers 2 and 3 (same token
    batch, other activations and weights) run with reuse_grouping on the same workspace and must give
    exactly the bits of a complete call on those inputs."""
    w1 = wl.small_mixed(**kw)
    db = DeviceBatch(w1)
    db.forward()
    for layer in (2, 3):
        wn = _as_next_layer(w1, 7000 + layer)
        assert np.array_equal(wn.slot_mapping, w1.slot_mapping)
        fresh = DeviceBatch(wn)
        fresh.forward()
        x, W = to_dev(wn.x, wn.dtype), to_dev(wn.W, wn.dtype)
        A, B = [to_dev(a, wn.dtype) for a in wn.A], [to_dev(b, wn.dtype) for b in wn.B]
        db.reset()
        ab.alora_qkv_forward_ex(x, db.aid, db.start, W, A, B, db.q, db.kc, db.vc, db.slot, wn.block_size, db.dims, db.ws,
                                reuse_grouping=True)
        torch.cuda.synchronize()
        assert np.array_equal(raw_bits(db.q), raw_bits(fresh.q))
        assert np.array_equal(raw_bits(db.kc), raw_bits(fresh.kc)) and np.array_equal(raw_bits(db.vc), raw_bits(fresh.vc))
        ref = _oracle_full(wn)
        assert maxnorm_rel(to_f64(db.q), ref.q_out) <= TOL[wn.dtype]


@pytest.mark.parametrize("dtype,rank,seq_lens", [("bf16", 48, (300, 41, 1, 77, 190)), ("bf16", 24, (33, 1, 7, 120)),
                                                 ("f32", 15, (60, 9, 31))])
def test_per_module_factors_as_block_structured_adapters(dtype, rank, seq_lens):
    """Sec. 2.3 writes one low-rank update per module (Delta^Q, Delta^K, Delta^V).  Separate module factors of
    rank r are handed to the library as A = [A^Q | A^K | A^V] of rank 3r with B^Q, B^K, B^V on B's block
    diagonal; the result must match three separately projected modules (the oracle's per-module routine)."""
    w0 = wl.small_mixed(dtype, seed=31, seq_lens=seq_lens, rank=rank)
    w, A_mod, B_mod = wl.with_per_module_factors(w0)
    print(f"[case] per-module factors {dtype} rank 3x{rank // 3} T={w.T}", flush=True)
    db = DeviceBatch(w)
    assert db.validate() == ab.ALORA_OK
    db.forward()
    x = wl.widen_f64(w.x, w.dtype)
    Wf = wl.widen_f64(w.W, w.dtype)
    W_mod = [Wf[:, : w.Nq], Wf[:, w.Nq: w.Nq + w.Nkv], Wf[:, w.Nq + w.Nkv:]]
    A64 = [[wl.widen_f64(a, w.dtype) for a in A_mod[m]] for m in range(3)]
    B64 = [[wl.widen_f64(b, w.dtype) for b in B_mod[m]] for m in range(3)]
    _, act = oracle.classify(w.token_adapter_ids, w.token_seg_ids, w.token_positions, w.activation_start)
    rows = np.arange(w.T, dtype=np.int32)
    y = oracle.alora_rows_per_module(x, [np.ascontiguousarray(m) for m in W_mod], A64, B64, w.token_adapter_ids, act, rows)
    tol = TOL[w.dtype]
    assert maxnorm_rel(to_f64(db.q), y[:, : w.Nq]) <= tol
    has = w.slot_mapping >= 0
    sidx = torch.from_numpy(w.slot_mapping[has]).to("cuda")
    assert maxnorm_rel(to_f64(db.kc[sidx]), y[has][:, w.Nq: w.Nq + w.Nkv]) <= tol
    assert maxnorm_rel(to_f64(db.vc[sidx]), y[has][:, w.Nq + w.Nkv:]) <= tol
    # the adapter term is there: adapted rows differ from the base projection
    yb = oracle.base_rows(x, Wf, rows[act == 1][:8])
    assert maxnorm_rel(y[act == 1][:8], yb) > 0.05
