"""GPU parity of the rotary embedding fused into the store of the projection (alora_extras.rope_cos / rope_sin):
the three places it is computed -- the epilogue of the fused bf16 projection kernel, the finishing kernel of the
small-batch bf16 path, the in-place pass of the fp32 path -- against the CPU fp64 oracle (projection rows,
then oracle/rope.py, then the paged store) on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
from oracle import rope as orope
from paper_2512_17910_amd import binding as ab
from paper_2512_17910_amd import workloads as wl
from gpu_util import DeviceBatch, TOL, host_operands, maxnorm_rel, raw_bits, to_f64

pytestmark = pytest.mark.gpu


def _tables(w, slack=3):
    cos, sin = wl.rope_table(int(w.token_positions.max()) + 1 + slack, w.head_dim)
    dev = (torch.from_numpy(cos).to("cuda"), torch.from_numpy(sin).to("cuda"))
    return cos, sin, dev


def _run(db, rope, aid=None):
    db.reset()
    ab.alora_qkv_forward_ex(db.x, db.aid if aid is None else aid, db.start, db.W, db.A, db.B, db.q, db.kc, db.vc, db.slot,
                            db.w.block_size, db.dims, db.ws, bias=db.bias, adapter_ranks=db.w.adapter_ranks, rope=rope)
    torch.cuda.synchronize()


def _oracle(w, cos, sin):
    x, W, A, B = host_operands(w)
    _, act = oracle.classify(w.token_adapter_ids, w.token_seg_ids, w.token_positions, w.activation_start)
    rows = np.arange(w.T, dtype=np.int32)
    bias = wl.widen_f64(w.bias, w.dtype) if w.bias is not None else None
    y = oracle.alora_rows_var(x, W, A, B, w.token_adapter_ids, act, rows, bias)
    y = orope.rope_rows(y, w.token_positions, cos, sin, w.n_q_heads, w.n_kv_heads, w.head_dim)
    q = np.zeros((w.T, w.Nq))
    kc = wl.widen_f64(wl.cache_fill(w.n_slots, w.Nkv, w.dtype, 0), w.dtype)
    vc = wl.widen_f64(wl.cache_fill(w.n_slots, w.Nkv, w.dtype, 1), w.dtype)
    oracle.store_rows(y, rows, w.Nq, w.Nkv, w.slot_mapping, w.block_size, q, kc, vc)
    sm = np.asarray(w.slot_mapping, np.int64)
    return q, kc, vc, np.sort(sm[sm >= 0]), act


def _check(w, tuning=(0, 0)):
    print(f"[case] {w.name} T={w.T} head_dim={w.head_dim} tuning={tuning}", flush=True)
    cos, sin, dev = _tables(w)
    db = DeviceBatch(w)
    ab.alora_qkv_set_tuning(*tuning)
    try:
        db2 = DeviceBatch(w) if tuning != (0, 0) else db      # the workspace is sized for the tuning in force
        _run(db2, dev)
        q, kc, vc = to_f64(db2.q), to_f64(db2.kc), to_f64(db2.vc)
        rq, rk, rv, wr, act = _oracle(w, cos, sin)
        tol = TOL[w.dtype]
        assert maxnorm_rel(q, rq) <= tol
        assert maxnorm_rel(kc[wr], rk[wr]) <= tol
        assert maxnorm_rel(vc[wr], rv[wr]) <= tol
        un = np.setdiff1d(np.arange(w.n_slots), wr)
        assert np.array_equal(raw_bits(db2.kc)[un], raw_bits(db2.k0)[un])
        # rows that keep the base output: bit-identical to a base-only call with the same tables
        mine = (raw_bits(db2.q).copy(), raw_bits(db2.kc).copy(), raw_bits(db2.vc).copy())
        _run(db2, dev, aid=torch.full_like(db2.aid, -1))
        keep = np.flatnonzero(act == 0)
        assert np.array_equal(raw_bits(db2.q)[keep], mine[0][keep])
        sl = np.asarray(w.slot_mapping, np.int64)[keep]
        sl = sl[sl >= 0]
        assert np.array_equal(raw_bits(db2.kc)[sl], mine[1][sl]) and np.array_equal(raw_bits(db2.vc)[sl], mine[2][sl])
        # and the rotation is really applied: without the tables q differs from the reference by far more than the gate
        _run(db2, None)
        assert maxnorm_rel(to_f64(db2.q), rq) > 10 * tol
    finally:
        ab.alora_qkv_set_tuning(0, 0)


@pytest.mark.parametrize("tuning", [(0, 1), (2, 1), (3, 1)])
def test_fused_projection_kernel_rotates_q_and_k(tuning):
    """Unsplit bf16 projection (forced: these batches are small): the rotation happens in the kernel's epilogue,
    whatever tile width the sizes or the override ask for; ragged T, padding rows, every kind of request."""
    _check(wl.small_mixed("bf16", head_dim=128, seq_lens=(150, 37, 1, 90, 300), seed=21, pad_every=7), tuning)


def test_fused_projection_kernel_with_bias_and_mixed_ranks():
    w = wl.with_variants(wl.small_mixed("bf16", head_dim=128, rank=32, seed=22), ranks=[8, 32, 16], bias=True)
    _check(w, (0, 1))
    _check(w, (0, 2))


@pytest.mark.parametrize("splits", [0, 2, 4])
def test_finishing_kernel_of_decode_sized_batches_rotates(splits):
    """Split projection + finishing kernel (decode-sized batches; the split count automatic or forced)."""
    _check(wl.small_mixed("bf16", hidden=1024, head_dim=128, seq_lens=(100, 31, 1, 64), seed=23), (0, splits))


@pytest.mark.parametrize("head_dim", [64, 128, 32])
def test_fp32_path_rotates_in_place(head_dim):
    _check(wl.small_mixed("f32", head_dim=head_dim, seq_lens=(70, 37, 1, 40), seed=24 + head_dim))


def test_argument_checks():
    w = wl.small_mixed("bf16", head_dim=64, seed=3)
    cos, sin, dev = _tables(w)
    db = DeviceBatch(w)
    with pytest.raises(ab.AloraError) as e:
        _run(db, dev)                                   # bf16 path: heads of 128 only
    assert e.value.status == ab.ALORA_ESHAPE
    w = wl.small_mixed("bf16", head_dim=128, seed=3)
    cos, sin, dev = _tables(w)
    db = DeviceBatch(w)
    with pytest.raises(ab.AloraError) as e:
        _run(db, (dev[0], None))                        # one table without the other
    assert e.value.status == ab.ALORA_EINVAL


def test_graph_replays_carry_the_rotation():
    """A captured call with the tables baked in: three replays (eager work and synchronisations in between)
    give the bits of the eager call."""
    w = wl.small_mixed("bf16", hidden=1024, head_dim=128, seq_lens=(100, 31, 1, 64), seed=29)
    cos, sin, dev = _tables(w)
    db = DeviceBatch(w)
    _run(db, dev)
    want = (raw_bits(db.q).copy(), raw_bits(db.kc).copy(), raw_bits(db.vc).copy())
    st = DeviceBatch(w)
    g = ab.alora_qkv_graph_create(st.x, st.aid, st.start, st.W, st.A, st.B, st.q, st.kc, st.vc, st.slot, w.block_size,
                                  st.dims, st.ws, rope=dev)
    try:
        for _ in range(3):
            st.reset()
            torch.cuda.synchronize()
            ab.alora_qkv_graph_launch(g)
            torch.cuda.synchronize()
            assert np.array_equal(raw_bits(st.q), want[0])
            assert np.array_equal(raw_bits(st.kc), want[1]) and np.array_equal(raw_bits(st.vc), want[2])
    finally:
        ab.alora_qkv_graph_destroy(g)


@pytest.mark.parametrize("cfg,n_sample", [(2, 64), (3, 128)])
def test_rotation_at_benchmark_size_on_sampled_rows(cfg, n_sample):
    """Configurations 2 (fused projection kernel) and 3 (split projection + finishing kernel) with the tables,
    in the launch configuration bench.py --rope times: sampled rows (activation boundaries +-2, segment ends,
    spread rows) against the oracle, and the pre-activation rows against a base-only call."""
    w = wl.CONFIGS[cfg]()
    print(f"[case] config {cfg} with rotation: T={w.T}", flush=True)
    cos, sin, dev = _tables(w, slack=0)
    db = DeviceBatch(w, cache_fill=False)
    _run(db, dev)
    _, act = oracle.classify(w.token_adapter_ids, w.token_seg_ids, w.token_positions, w.activation_start)
    rows = wl.sample_rows(w, n_sample)
    x, W, A, B = host_operands(w)
    y = oracle.alora_rows(x, W, A, B, w.token_adapter_ids, act, rows)
    del x, W
    y = orope.rope_rows(y, w.token_positions[rows], cos, sin, w.n_q_heads, w.n_kv_heads, w.head_dim)
    ridx = torch.from_numpy(rows.astype(np.int64)).to("cuda")
    tol = TOL[w.dtype]
    assert maxnorm_rel(to_f64(db.q[ridx]), y[:, : w.Nq]) <= tol
    sl = w.slot_mapping[rows]
    has = sl >= 0
    sidx = torch.from_numpy(sl[has]).to("cuda")
    assert maxnorm_rel(to_f64(db.kc[sidx]), y[has][:, w.Nq: w.Nq + w.Nkv]) <= tol
    assert maxnorm_rel(to_f64(db.vc[sidx]), y[has][:, w.Nq + w.Nkv:]) <= tol
    q1, k1 = db.q.clone(), db.kc.clone()
    _run(db, dev, aid=torch.full_like(db.aid, -1))
    pre_rows = torch.from_numpy(np.nonzero(act == 0)[0]).to("cuda")
    assert torch.equal(db.q[pre_rows].view(torch.int16), q1[pre_rows].view(torch.int16))
    pre_slots = torch.from_numpy(w.slot_mapping[(act == 0) & (w.slot_mapping >= 0)]).to("cuda")
    assert torch.equal(db.kc[pre_slots].view(torch.int16), k1[pre_slots].view(torch.int16))


@pytest.mark.parametrize("tuning", [(0, 1), (0, 2)])
def test_repeated_calls_give_the_same_bits(tuning):
    """Fifty calls of the fused kernel (and of the split path with its finishing kernel): no timing-dependent bit."""
    w = wl.small_mixed("bf16", hidden=1024, head_dim=128, seq_lens=(150, 37, 1, 90, 300), seed=31)
    cos, sin, dev = _tables(w)
    ab.alora_qkv_set_tuning(*tuning)
    try:
        db = DeviceBatch(w)
        _run(db, dev)
        first = (raw_bits(db.q).copy(), raw_bits(db.kc).copy(), raw_bits(db.vc).copy())
        for it in range(50):
            _run(db, dev)
            assert np.array_equal(raw_bits(db.q), first[0]), it
            assert np.array_equal(raw_bits(db.kc), first[1]) and np.array_equal(raw_bits(db.vc), first[2]), it
    finally:
        ab.alora_qkv_set_tuning(0, 0)
