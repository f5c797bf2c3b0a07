"""Graph-captured call (alora_qkv_graph_*): one forward recorded into a HIP graph over buffers of
fixed address, then replayed with the batch rewritten in place; smaller batches are padded with
rows of adapter -1 / slot -1.  Every replay must equal the eager call bit for bit and match the
fp64 oracle; eager work and synchronisations sit between the replays on purpose."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_17910_amd import binding as ab
from paper_2512_17910_amd import workloads as wl
from gpu_util import DeviceBatch, TOL, check_grouping, host_operands, maxnorm_rel, raw_bits, to_dev, to_f64

pytestmark = pytest.mark.gpu

T_CAP = 256


def _decode_step(step: int, n_real: int, hidden=256, n_adapters=16, rank=32, dtype="bf16"):
    """T_CAP single-token sequences (decode), the last T_CAP - n_real of them padding rows."""
    rng = np.random.default_rng(4242 + step)
    segs = []
    for s in range(T_CAP):
        p = int(rng.integers(1, 100))
        a = -1 if s % 5 == 0 else int(rng.integers(0, n_adapters))
        segs.append(wl.Segment(s, p, 1, a, int(rng.integers(0, p + 1))))
    return wl.assemble(f"graph-decode-step{step}", dtype, hidden, 4, 2, 64, n_adapters, rank, 16, segs,
                       [100] * T_CAP, seed=9000 + step, weight_key=777, extra_blocks=3,
                       pad_rows=list(range(n_real, T_CAP)))


def _load_into(db: DeviceBatch, w) -> None:
    """Rewrite the batch inside db's buffers (addresses unchanged)."""
    db.x.copy_(to_dev(w.x, w.dtype))
    db.aid.copy_(torch.from_numpy(w.token_adapter_ids))
    db.seg.copy_(torch.from_numpy(w.token_seg_ids))
    db.pos.copy_(torch.from_numpy(w.token_positions))
    db.start.copy_(torch.from_numpy(w.activation_start))
    db.slot.copy_(torch.from_numpy(w.slot_mapping))
    db.reset()


def _oracle_full(w):
    x, W, A, B = host_operands(w)
    k0 = wl.widen_f64(wl.cache_fill(w.n_slots, w.Nkv, w.dtype, 0), w.dtype)
    v0 = wl.widen_f64(wl.cache_fill(w.n_slots, w.Nkv, w.dtype, 1), w.dtype)
    return oracle.alora_qkv_forward(x, w.token_adapter_ids, w.token_seg_ids, w.token_positions,
                                    w.activation_start, W, A, B, w.slot_mapping, w.block_size, w.Nq, w.Nkv, k0, v0)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_replays_equal_eager_calls_and_the_oracle(dtype):
    kw = dict(dtype=dtype) if dtype == "bf16" else dict(dtype=dtype, hidden=128, n_adapters=4, rank=8)
    w0 = _decode_step(0, T_CAP, **kw)
    static = DeviceBatch(w0)
    g = ab.alora_qkv_graph_create(static.x, static.aid, static.start, static.W, static.A, static.B, static.q,
                                  static.kc, static.vc, static.slot, w0.block_size, static.dims, static.ws)
    try:
        # nothing ran at creation
        assert np.array_equal(raw_bits(static.kc), raw_bits(static.k0))
        for step, n_real in enumerate((T_CAP, 200, 17, 1, T_CAP, 129)):
            w = _decode_step(step, n_real, **kw)
            print(f"[case] {w.name} real rows {n_real}", flush=True)
            assert (w.n_slots, w.n_segments, w.T) == (w0.n_slots, w0.n_segments, w0.T)
            _load_into(static, w)
            torch.cuda.synchronize()
            ab.alora_qkv_graph_launch(g)
            torch.cuda.synchronize()
            q, kc, vc = raw_bits(static.q), raw_bits(static.kc), raw_bits(static.vc)
            grouping = [t.clone() for t in ab.workspace_int_views(static.dims, static.ws)]
            # the same batch through the eager entry point, in buffers of its own
            eager = DeviceBatch(w)
            assert eager.validate() == ab.ALORA_OK
            eager.forward()
            assert np.array_equal(q, raw_bits(eager.q))
            assert np.array_equal(kc, raw_bits(eager.kc)) and np.array_equal(vc, raw_bits(eager.vc))
            # and against the oracle
            ref = _oracle_full(w)
            wr = ref.written_slots
            assert wr.size == min(n_real, T_CAP)
            tol = TOL[w.dtype]
            assert maxnorm_rel(to_f64(static.q)[:n_real], ref.q_out[:n_real]) <= tol
            assert maxnorm_rel(to_f64(static.kc)[wr], ref.k_cache[wr]) <= tol
            assert maxnorm_rel(to_f64(static.vc)[wr], ref.v_cache[wr]) <= tol
            un = np.setdiff1d(np.arange(w.n_slots), wr)
            assert np.array_equal(kc[un], raw_bits(static.k0)[un]) and np.array_equal(vc[un], raw_bits(static.v0)[un])
            check_grouping(*grouping, ref.active, ref.perm, ref.offsets)
            # padding rows are base rows: never active
            assert not ref.active[n_real:].any()
    finally:
        ab.alora_qkv_graph_destroy(g)


def test_replay_twice_without_rewriting_is_idempotent():
    w = _decode_step(3, 180)
    static = DeviceBatch(w)
    g = ab.alora_qkv_graph_create(static.x, static.aid, static.start, static.W, static.A, static.B, static.q,
                                  static.kc, static.vc, static.slot, w.block_size, static.dims, static.ws)
    try:
        ab.alora_qkv_graph_launch(g)
        torch.cuda.synchronize()
        first = (raw_bits(static.q), raw_bits(static.kc), raw_bits(static.vc))
        scratch = torch.randn(1 << 20, device="cuda").sum().item()   # unrelated eager work in between
        assert np.isfinite(scratch)
        ab.alora_qkv_graph_launch(g)
        ab.alora_qkv_graph_launch(g)
        torch.cuda.synchronize()
        again = (raw_bits(static.q), raw_bits(static.kc), raw_bits(static.vc))
        assert all(np.array_equal(a, b) for a, b in zip(first, again))
    finally:
        ab.alora_qkv_graph_destroy(g)


def test_create_rejects_bad_arguments_without_leaving_a_capture_open():
    w = _decode_step(1, 64)
    static = DeviceBatch(w)
    with pytest.raises(ab.AloraError):
        ab.alora_qkv_graph_create(static.x, static.aid, static.start, static.W, static.A, static.B, static.q,
                                  static.kc, static.vc, static.slot, 0, static.dims, static.ws)   # block_size 0
    # the library is still usable: eager call and a proper capture both work
    static.forward()
    g = ab.alora_qkv_graph_create(static.x, static.aid, static.start, static.W, static.A, static.B, static.q,
                                  static.kc, static.vc, static.slot, w.block_size, static.dims, static.ws)
    ab.alora_qkv_graph_launch(g)
    torch.cuda.synchronize()
    ab.alora_qkv_graph_destroy(g)


def test_graph_with_bias_and_per_adapter_ranks():
    w = wl.with_variants(_decode_step(7, 220, n_adapters=4, rank=32), ranks=(8, 32, 16, 24), bias=True)
    static = DeviceBatch(w)
    g = ab.alora_qkv_graph_create(static.x, static.aid, static.start, static.W, static.A, static.B, static.q,
                                  static.kc, static.vc, static.slot, w.block_size, static.dims, static.ws,
                                  bias=static.bias, adapter_ranks=w.adapter_ranks)
    try:
        ab.alora_qkv_graph_launch(g)
        torch.cuda.synchronize()
        eager = DeviceBatch(w)
        eager.forward()
        assert np.array_equal(raw_bits(static.q), raw_bits(eager.q))
        assert np.array_equal(raw_bits(static.kc), raw_bits(eager.kc)) and np.array_equal(raw_bits(static.vc), raw_bits(eager.vc))
        x, W, A, B = host_operands(w)
        _, act = oracle.classify(w.token_adapter_ids, w.token_seg_ids, w.token_positions, w.activation_start)
        rows = np.arange(w.T, dtype=np.int32)
        y = oracle.alora_rows_var(x, W, A, B, w.token_adapter_ids, act, rows, wl.widen_f64(w.bias, w.dtype))
        assert maxnorm_rel(to_f64(static.q), y[:, : w.Nq]) <= TOL[w.dtype]
    finally:
        ab.alora_qkv_graph_destroy(g)
