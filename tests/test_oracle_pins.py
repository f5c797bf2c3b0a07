"""Pins for the CPU oracle: hand-worked values, closed forms, library routines on special
cases, invariants and exact brute force.  Nothing here touches the GPU library.

Each check is a function `pin_*()` so that tests/test_oracle_mutants.py can re-run the same
suite against deliberately broken copies of the oracle and see it fail.
"""
import itertools
import json
import os

import numpy as np
import pytest

import oracle
from paper_2512_17910_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden", "worked_example.json")


# ----------------------------------------------------------------------------------------
# helpers
# ----------------------------------------------------------------------------------------
def _rand_ints(rng, shape, lo=-3, hi=4):
    return rng.integers(lo, hi, size=shape).astype(np.float64)


def _tiny(rng, T=5, H=3, Nq=2, Nkv=2, r=2, L=2):
    N = Nq + 2 * Nkv
    x = _rand_ints(rng, (T, H))
    W = _rand_ints(rng, (H, N))
    A = [_rand_ints(rng, (H, r)) for _ in range(L)]
    B = [_rand_ints(rng, (r, N)) for _ in range(L)]
    return x, W, A, B


def _forward_small(w: wl.Workload, A=None, B=None, W=None, start=None, aid=None, order=None):
    """Full oracle forward on a Workload (values widened exactly to fp64)."""
    x = wl.widen_f64(w.x, w.dtype)
    Wm = wl.widen_f64(w.W, w.dtype) if W is None else W
    Am = [wl.widen_f64(a, w.dtype) for a in w.A] if A is None else A
    Bm = [wl.widen_f64(b, w.dtype) for b in w.B] if B is None else B
    aid = w.token_adapter_ids if aid is None else aid
    seg, pos, slot = w.token_seg_ids, w.token_positions, w.slot_mapping
    if order is not None:
        x, aid, seg, pos, slot = x[order], aid[order], seg[order], pos[order], slot[order]
    st = w.activation_start if start is None else start
    kc = wl.widen_f64(wl.cache_fill(w.n_slots, w.Nkv, w.dtype, 0), w.dtype)
    vc = wl.widen_f64(wl.cache_fill(w.n_slots, w.Nkv, w.dtype, 1), w.dtype)
    res = oracle.alora_qkv_forward(x, aid, seg, pos, st, Wm, Am, Bm, slot, w.block_size, w.Nq, w.Nkv, kc, vc)
    return res, kc, vc


# ----------------------------------------------------------------------------------------
# pins
# ----------------------------------------------------------------------------------------
def pin_worked_example():
    """Every stage against the hand-worked fixture."""
    g = json.load(open(GOLD))
    e = g["expect"]
    x, W = np.array(g["x"], float), np.array(g["W"], float)
    A = [np.array(a, float) for a in g["A"]]
    B = [np.array(b, float) for b in g["B"]]
    aid, seg, pos = g["token_adapter_ids"], g["token_seg_ids"], g["token_positions"]
    mask, act = oracle.classify(aid, seg, pos, g["activation_start"])
    assert mask.tolist() == e["paper_mask"] and act.tolist() == e["active"]
    perm, off = oracle.group(aid, act, 2)
    assert perm.tolist() == e["perm"] and off.tolist() == e["offsets"]
    rows = np.arange(4, dtype=np.int32)
    assert oracle.base_rows(x, W, rows).tolist() == e["base_y"]
    assert oracle.alora_rows(x, W, A, B, aid, act, rows).tolist() == e["y"]
    assert oracle.blend_rows(x, W, A, B, aid, mask, rows).tolist() == e["y"]
    blk, offs = oracle.slot_coords(g["slot_mapping"], g["block_size"])
    assert blk.tolist() == e["block"] and offs.tolist() == e["offset"]
    kc = np.array(g["k_cache_before"], float).reshape(-1, 1)
    vc = np.array(g["v_cache_before"], float).reshape(-1, 1)
    res = oracle.alora_qkv_forward(x, aid, seg, pos, g["activation_start"], W, A, B, g["slot_mapping"],
                                   g["block_size"], g["Nq"], g["Nkv"], kc, vc)
    assert res.q_out.tolist() == e["q_out"]
    assert res.k_cache.ravel().tolist() == e["k_cache_after"]
    assert res.v_cache.ravel().tolist() == e["v_cache_after"]
    assert res.written_slots.tolist() == [0, 2, 5]
    # reversed row subset: output row i belongs to token rows[i]
    rev = np.array([3, 1], dtype=np.int32)
    assert oracle.alora_rows(x, W, A, B, aid, act, rev).tolist() == [e["y"][3], e["y"][1]]
    assert oracle.base_rows(x, W, rev).tolist() == [e["base_y"][3], e["base_y"][1]]


def pin_one_hot_closed_form():
    """x = e_k picks row k of W (+ row k of A times B): catches transposed or mis-indexed operands."""
    rng = np.random.default_rng(11)
    H, Nq, Nkv, r, L = 5, 3, 2, 3, 2
    N = Nq + 2 * Nkv
    W = rng.standard_normal((H, N))
    A = [rng.standard_normal((H, r)) for _ in range(L)]
    B = [rng.standard_normal((r, N)) for _ in range(L)]
    x = np.eye(H)
    aid = np.array([0, 1, 0, 1, -1], dtype=np.int32)
    act = np.array([1, 1, 0, 1, 0], dtype=np.uint8)
    y = oracle.alora_rows(x, W, A, B, aid, act, np.arange(H, dtype=np.int32))
    for k in range(H):
        want = W[k].copy()
        if act[k]:
            a = aid[k]
            want = want + sum(A[a][k, j] * B[a][j] for j in range(r))
        np.testing.assert_allclose(y[k], want, rtol=0, atol=1e-14)
    np.testing.assert_array_equal(oracle.base_rows(x, W, np.arange(H, dtype=np.int32)), W)


def pin_activation_zero_is_lora():
    """Activation at position 0 == standard LoRA == x (W + A B) with the weight merged first
    (Sec. 2.2 equations), computed with numpy's matmul."""
    w = wl.small_mixed("f32", seq_lens=(9, 6, 4), n_adapters=3, rank=8, hidden=64, head_dim=16)
    x = wl.widen_f64(w.x, "f32"); W = wl.widen_f64(w.W, "f32")
    A = [wl.widen_f64(a, "f32") for a in w.A]; B = [wl.widen_f64(b, "f32") for b in w.B]
    aid = np.array([t % 3 for t in range(w.T)], dtype=np.int32)
    seg = np.zeros(w.T, dtype=np.int32)
    mask, act = oracle.classify(aid, seg, w.token_positions, [0])
    assert act.all() and not mask.any()
    y = oracle.alora_rows(x, W, A, B, aid, act, np.arange(w.T, dtype=np.int32))
    for t in range(w.T):
        merged = W + A[aid[t]] @ B[aid[t]]
        want = x[t] @ merged
        assert np.max(np.abs(y[t] - want)) <= 1e-12 * np.max(np.abs(want))


def pin_pre_activation_rows_are_base_exactly():
    """Inactive rows equal the separately written base-only routine bit for bit (Sec. 2.3:
    K and V before the invocation are the base model's)."""
    w = wl.small_mixed("bf16", seq_lens=(20, 7, 1, 12), hidden=64, head_dim=16)
    res, _, _ = _forward_small(w)
    x = wl.widen_f64(w.x, w.dtype); W = wl.widen_f64(w.W, w.dtype)
    base = oracle.base_rows(x, W, np.arange(w.T, dtype=np.int32))
    y = np.concatenate([res.q_out], axis=1)
    inact = res.active == 0
    assert inact.any() and (~inact).any()
    assert np.array_equal(y[inact], base[inact][:, : w.Nq])
    assert not np.array_equal(y[~inact], base[~inact][:, : w.Nq])
    # K/V of inactive rows with a slot
    for t in np.nonzero(inact)[0]:
        s = w.slot_mapping[t]
        if s >= 0:
            assert np.array_equal(res.k_cache[s], base[t, w.Nq: w.Nq + w.Nkv])
            assert np.array_equal(res.v_cache[s], base[t, w.Nq + w.Nkv:])


def pin_zero_B_and_never_activated():
    w = wl.small_mixed("bf16", seq_lens=(20, 7, 1, 12), hidden=64, head_dim=16)
    x = wl.widen_f64(w.x, w.dtype); W = wl.widen_f64(w.W, w.dtype)
    rows = np.arange(w.T, dtype=np.int32)
    base = oracle.base_rows(x, W, rows)
    zB = [np.zeros((w.rank, w.N)) for _ in w.B]
    res, _, _ = _forward_small(w, B=zB)
    assert np.array_equal(res.q_out, base[:, : w.Nq])
    # activation point one past each segment's last position -> nothing is active
    never = np.array([s.first_pos + s.n_tokens for s in w.segments], dtype=np.int32)
    res2, _, _ = _forward_small(w, start=never)
    assert res2.active.sum() == 0 and res2.perm.size == 0
    assert np.array_equal(res2.q_out, base[:, : w.Nq])
    # one position earlier -> exactly the last row of every adapter segment is active
    res3, _, _ = _forward_small(w, start=never - 1)
    want = sum(1 for s in w.segments if s.adapter >= 0)
    assert int(res3.active.sum()) == want


def pin_blend_equals_select():
    """Algorithm 1's base*mask + out*(1-mask) equals the select form on finite data."""
    w = wl.small_mixed("bf16", seq_lens=(20, 7, 1, 12), hidden=64, head_dim=16)
    x = wl.widen_f64(w.x, w.dtype); W = wl.widen_f64(w.W, w.dtype)
    A = [wl.widen_f64(a, w.dtype) for a in w.A]; B = [wl.widen_f64(b, w.dtype) for b in w.B]
    mask, act = oracle.classify(w.token_adapter_ids, w.token_seg_ids, w.token_positions, w.activation_start)
    rows = np.arange(w.T, dtype=np.int32)
    ys = oracle.alora_rows(x, W, A, B, w.token_adapter_ids, act, rows)
    yb = oracle.blend_rows(x, W, A, B, w.token_adapter_ids, mask, rows)
    assert np.max(np.abs(ys - yb)) <= 1e-13 * np.max(np.abs(ys))
    assert np.array_equal(ys[act == 0], yb[act == 0])


def pin_mask_closed_form_counts():
    """Active-row counts of the benchmark structures have closed forms (App. B mask)."""
    w1 = wl.config1(with_values=False)
    m, a = oracle.classify(w1.token_adapter_ids, w1.token_seg_ids, w1.token_positions, w1.activation_start)
    assert np.nonzero(a)[0].tolist() == list(range(24, 32))
    assert m.tolist() == [1] * 24 + [0] * 8 + [1] * 32
    perm, off = oracle.group(w1.token_adapter_ids, a, 2)
    assert perm.tolist() == list(range(24, 32)) and off.tolist() == [0, 8, 8]
    w2 = wl.config2(with_values=False)
    _, a2 = oracle.classify(w2.token_adapter_ids, w2.token_seg_ids, w2.token_positions, w2.activation_start)
    assert int(a2.sum()) == sum(512 - s.activation_start for s in w2.segments)
    w3 = wl.config3(with_values=False)
    _, a3 = oracle.classify(w3.token_adapter_ids, w3.token_seg_ids, w3.token_positions, w3.activation_start)
    assert int(a3.sum()) == 192 and int((w3.token_adapter_ids < 0).sum()) == 64
    w5 = wl.config5(with_values=False)
    _, a5 = oracle.classify(w5.token_adapter_ids, w5.token_seg_ids, w5.token_positions, w5.activation_start)
    assert int(a5.sum()) == sum(s.first_pos + s.n_tokens - s.activation_start for s in w5.segments)
    # boundary: the row AT the activation start is adapted, the one before is not
    for s_idx, s in enumerate(w5.segments):
        t_rows = np.nonzero(w5.token_seg_ids == s_idx)[0]
        t_at = t_rows[0] + (s.activation_start - s.first_pos)
        assert a5[t_at] == 1 and (t_at == t_rows[0] or a5[t_at - 1] == 0)


def pin_group_matches_stable_sort():
    rng = np.random.default_rng(5)
    for T, L in ((1, 1), (17, 3), (300, 16), (1000, 33)):
        aid = rng.integers(-1, L, size=T).astype(np.int32)
        act = (rng.random(T) < 0.6).astype(np.uint8) & (aid >= 0).astype(np.uint8)
        perm, off = oracle.group(aid, act, L)
        idx = np.nonzero(act)[0]
        want = idx[np.argsort(aid[idx], kind="stable")]
        assert np.array_equal(perm, want.astype(np.int32))
        cnt = np.bincount(aid[idx], minlength=L)
        assert np.array_equal(off, np.concatenate([[0], np.cumsum(cnt)]).astype(np.int32))


def pin_brute_force_exact():
    """Small integers: every product and sum is exact, so Python integer arithmetic gives the
    one right answer; all 2^T activation patterns x adapter assignments on a tiny shape."""
    rng = np.random.default_rng(3)
    T, H, Nq, Nkv, r, L = 4, 3, 2, 1, 2, 2
    N = Nq + 2 * Nkv
    x, W, A, B = _tiny(rng, T, H, Nq, Nkv, r, L)
    xi, Wi = x.astype(int).tolist(), W.astype(int).tolist()
    Ai = [a.astype(int).tolist() for a in A]; Bi = [b.astype(int).tolist() for b in B]
    rows = np.arange(T, dtype=np.int32)
    for act_bits in itertools.product([0, 1], repeat=T):
        for aids in itertools.product([-1, 0, 1], repeat=T):
            # realise the pattern through positions/starts: pos = 1, start = 1 (active) or 2 (not)
            pos = np.ones(T, dtype=np.int32)
            start = np.array([1 if b else 2 for b in act_bits], dtype=np.int32)
            seg = np.arange(T, dtype=np.int32)
            aid = np.array(aids, dtype=np.int32)
            mask, act = oracle.classify(aid, seg, pos, start)
            want_act = [int(b and a >= 0) for b, a in zip(act_bits, aids)]
            assert act.tolist() == want_act and mask.tolist() == [1 - b for b in act_bits]
            y = oracle.alora_rows(x, W, A, B, aid, act, rows)
            for t in range(T):
                for n in range(N):
                    v = sum(xi[t][k] * Wi[k][n] for k in range(H))
                    if want_act[t]:
                        a = aids[t]
                        v += sum(sum(xi[t][k] * Ai[a][k][j] for k in range(H)) * Bi[a][j][n] for j in range(r))
                    assert y[t, n] == v


def pin_linearity():
    """delta scales exactly with B (power-of-two factor); adapters on disjoint rows add."""
    rng = np.random.default_rng(8)
    T, H, Nq, Nkv, r, L = 6, 4, 2, 2, 2, 2
    x, W, A, B = _tiny(rng, T, H, Nq, Nkv, r, L)
    rows = np.arange(T, dtype=np.int32)
    aid = np.array([0, 1, 0, 1, 0, 1], dtype=np.int32)
    act = np.ones(T, dtype=np.uint8)
    base = oracle.base_rows(x, W, rows)
    d1 = oracle.alora_rows(x, W, A, B, aid, act, rows) - base
    d4 = oracle.alora_rows(x, W, A, [4 * b for b in B], aid, act, rows) - base
    assert np.array_equal(d4, 4 * d1)
    only0 = oracle.alora_rows(x, W, A, [B[0], 0 * B[1]], aid, act, rows) - base
    only1 = oracle.alora_rows(x, W, A, [0 * B[0], B[1]], aid, act, rows) - base
    assert np.array_equal(only0 + only1, d1)
    assert not only0[1::2].any() and not only1[0::2].any() and d1.any()


def pin_row_permutation():
    """Token rows are independent: permuting the batch permutes q_out and leaves the caches alike."""
    w = wl.small_mixed("bf16", seq_lens=(20, 7, 1, 12), hidden=64, head_dim=16, pad_every=9)
    res, _, _ = _forward_small(w)
    order = np.random.default_rng(2).permutation(w.T)
    res_p, _, _ = _forward_small(w, order=order)
    assert np.array_equal(res_p.q_out, res.q_out[order])
    assert np.array_equal(res_p.k_cache, res.k_cache) and np.array_equal(res_p.v_cache, res.v_cache)
    assert np.array_equal(res_p.active, res.active[order])


def pin_paged_store():
    """Exactly the mapped slots change; everything else keeps its bytes; -1 rows write nothing
    but still produce q_out; slot = block * block_size + offset."""
    w = wl.small_mixed("bf16", seq_lens=(20, 7, 1, 12), hidden=64, head_dim=16, pad_every=9)
    res, k0, v0 = _forward_small(w)
    changed_k = np.nonzero((res.k_cache != k0).any(axis=1))[0]
    changed_v = np.nonzero((res.v_cache != v0).any(axis=1))[0]
    want = np.sort(w.slot_mapping[w.slot_mapping >= 0])
    assert np.array_equal(changed_k, want) and np.array_equal(changed_v, want)
    assert (w.slot_mapping < 0).any() and len(want) < w.n_slots
    x = wl.widen_f64(w.x, w.dtype); W = wl.widen_f64(w.W, w.dtype)
    pad = np.nonzero(w.slot_mapping < 0)[0]
    base = oracle.base_rows(x, W, pad.astype(np.int32))
    assert np.array_equal(res.q_out[pad], base[:, : w.Nq])
    blk, off = oracle.slot_coords(w.slot_mapping, w.block_size)
    ok = w.slot_mapping >= 0
    d, m = np.divmod(w.slot_mapping[ok], w.block_size)
    assert np.array_equal(blk[ok], d) and np.array_equal(off[ok], m)
    assert (blk[~ok] == -1).all() and (off[~ok] == -1).all()
    # K and V land in different tensors from different column ranges
    t = int(np.nonzero(ok)[0][0])
    y = oracle.base_rows(x, W, np.array([t], dtype=np.int32))[0] if not res.active[t] else None
    if y is not None:
        s = w.slot_mapping[t]
        assert np.array_equal(res.k_cache[s], y[w.Nq: w.Nq + w.Nkv])
        assert np.array_equal(res.v_cache[s], y[w.Nq + w.Nkv:])


def pin_cached_prefix_untouched():
    """The skipped, block-aligned prefix of the long-context workload owns slots the call never names."""
    w5 = wl.config5(with_values=False)
    pre = w5.cached_prefix_slots
    assert pre.size % 16 == 0 and pre.size >= 4 * 16 * 615
    assert np.intersect1d(pre, w5.slot_mapping).size == 0
    assert np.unique(w5.slot_mapping).size == w5.T
    first_rows = [int(np.nonzero(w5.token_seg_ids == g)[0][0]) for g in range(w5.n_segments)]
    assert all(w5.token_positions[r] == w5.segments[g].first_pos for g, r in enumerate(first_rows))


def pin_column_split():
    """Changing only the K columns of W changes only K outputs (three separate equations)."""
    w = wl.small_mixed("bf16", seq_lens=(10, 5), hidden=64, head_dim=16)
    W = wl.widen_f64(w.W, w.dtype)
    res, _, _ = _forward_small(w)
    W2 = W.copy()
    W2[:, w.Nq: w.Nq + w.Nkv] += 1.0
    res2, _, _ = _forward_small(w, W=W2)
    assert np.array_equal(res.q_out, res2.q_out) and np.array_equal(res.v_cache, res2.v_cache)
    wr = res.written_slots
    assert (res.k_cache[wr] != res2.k_cache[wr]).any(axis=1).all()
    W3 = W.copy()
    W3[:, w.Nq + w.Nkv:] += 1.0
    res3, _, _ = _forward_small(w, W=W3)
    assert np.array_equal(res.q_out, res3.q_out) and np.array_equal(res.k_cache, res3.k_cache)
    assert (res.v_cache[wr] != res3.v_cache[wr]).any(axis=1).all()


def pin_variants_small_integers_exact():
    """Bias (Algorithm 1: base output = l.apply(x, b)) and one rank per adapter (Sec. 4.1): with
    small-integer data every product and sum is exact in fp64, so the result must EQUAL the
    definition written with numpy, whatever the summation order."""
    rng = np.random.default_rng(77)
    T, H, N = 9, 5, 7
    ranks = [1, 3, 2]
    x, W = _rand_ints(rng, (T, H)), _rand_ints(rng, (H, N))
    A = [_rand_ints(rng, (H, r)) for r in ranks]
    B = [_rand_ints(rng, (r, N)) for r in ranks]
    b = _rand_ints(rng, (N,))
    aid = np.array([0, 1, 2, -1, 2, 1, 0, -1, 1], np.int32)
    act = np.array([1, 0, 1, 0, 1, 1, 0, 0, 1], np.uint8)
    rows = np.arange(T, dtype=np.int32)
    for bias in (None, b):
        y = oracle.alora_rows_var(x, W, A, B, aid, act, rows, bias)
        for t in range(T):
            want = x[t] @ W + (bias if bias is not None else 0)
            if act[t]:
                want = want + (x[t] @ A[aid[t]]) @ B[aid[t]]
            assert np.array_equal(y[t], want), (t, bias is not None)


def pin_variants_reduce_to_the_plain_form():
    """Equal ranks and no bias: the variant routine IS the plain one; zero-padding an adapter's missing
    rank components changes nothing (adding exact zeros); W = 0 with no adapter leaves the bias."""
    rng = np.random.default_rng(78)
    T, H, N, r = 11, 16, 12, 4
    x, W = rng.standard_normal((T, H)), rng.standard_normal((H, N))
    A = [rng.standard_normal((H, r)) for _ in range(3)]
    B = [rng.standard_normal((r, N)) for _ in range(3)]
    aid = rng.integers(-1, 3, T).astype(np.int32)
    act = ((aid >= 0) & (rng.random(T) < 0.6)).astype(np.uint8)
    rows = np.arange(T, dtype=np.int32)
    assert np.array_equal(oracle.alora_rows_var(x, W, A, B, aid, act, rows), oracle.alora_rows(x, W, A, B, aid, act, rows))
    ranks = [1, 4, 2]
    At = [a[:, :k].copy() for a, k in zip(A, ranks)]
    Bt = [b[:k, :].copy() for b, k in zip(B, ranks)]
    Ap = [np.where(np.arange(r)[None, :] < k, a, 0.0) for a, k in zip(A, ranks)]
    Bp = [np.where(np.arange(r)[:, None] < k, b, 0.0) for b, k in zip(B, ranks)]
    assert np.array_equal(oracle.alora_rows_var(x, W, At, Bt, aid, act, rows), oracle.alora_rows(x, W, Ap, Bp, aid, act, rows))
    bias = rng.standard_normal(N)
    y = oracle.alora_rows_var(x, np.zeros_like(W), At, Bt, aid, np.zeros(T, np.uint8), rows, bias)
    assert np.array_equal(y, np.tile(bias, (T, 1)))


def _module_factors(rng, H, Nq, Nkv, r, L, ints=True):
    """Separate (A^m_i, B^m_i) per module m in (Q, K, V) and the block-structured fused encoding of them:
    A_i = [A^Q_i | A^K_i | A^V_i] of rank 3r, B_i with B^Q_i, B^K_i, B^V_i on its block diagonal."""
    widths = (Nq, Nkv, Nkv)
    draw = (lambda shape: _rand_ints(rng, shape)) if ints else (lambda shape: rng.standard_normal(shape))
    A_mod = [[draw((H, r)) for _ in range(L)] for _ in range(3)]
    B_mod = [[draw((r, widths[m])) for _ in range(L)] for m in range(3)]
    A_fused, B_fused = [], []
    N = Nq + 2 * Nkv
    for i in range(L):
        A_fused.append(np.concatenate([A_mod[m][i] for m in range(3)], axis=1))
        Bf = np.zeros((3 * r, N))
        col = 0
        for m in range(3):
            Bf[m * r:(m + 1) * r, col:col + widths[m]] = B_mod[m][i]
            col += widths[m]
        B_fused.append(Bf)
    return A_mod, B_mod, A_fused, B_fused


def pin_per_module_factors_exact():
    """Sec. 2.3 writes one equation per module with its own Delta^Q, Delta^K, Delta^V.  On small integers
    (every product and sum exact) the per-module routine must EQUAL the three equations written out with
    Python integers, and the fused routine fed the block-structured encoding must EQUAL it too."""
    rng = np.random.default_rng(91)
    T, H, Nq, Nkv, r, L = 7, 4, 3, 2, 2, 2
    x = _rand_ints(rng, (T, H))
    W_mod = [_rand_ints(rng, (H, n)) for n in (Nq, Nkv, Nkv)]
    A_mod, B_mod, A_f, B_f = _module_factors(rng, H, Nq, Nkv, r, L)
    aid = np.array([0, 1, -1, 1, 0, 0, 1], np.int32)
    act = np.array([1, 0, 0, 1, 0, 1, 1], np.uint8)
    rows = np.arange(T, dtype=np.int32)
    y = oracle.alora_rows_per_module(x, W_mod, A_mod, B_mod, aid, act, rows)
    for t in range(T):
        want = []
        for m in range(3):
            n_m = W_mod[m].shape[1]
            for n in range(n_m):
                v = sum(int(x[t, k]) * int(W_mod[m][k, n]) for k in range(H))
                if act[t]:
                    a = int(aid[t])
                    for j in range(r):
                        sj = sum(int(x[t, k]) * int(A_mod[m][a][k, j]) for k in range(H))
                        v += sj * int(B_mod[m][a][j, n])
                want.append(v)
        assert [int(v) for v in y[t]] == want, t
    fused = oracle.alora_rows(x, np.concatenate(W_mod, axis=1), A_f, B_f, aid, act, rows)
    assert np.array_equal(fused, y)
    # the modules really are separate: changing only the K module's factors changes only K columns
    B_mod2 = [B_mod[0], [b + 1.0 for b in B_mod[1]], B_mod[2]]
    y2 = oracle.alora_rows_per_module(x, W_mod, A_mod, B_mod2, aid, act, rows)
    assert np.array_equal(y2[:, :Nq], y[:, :Nq]) and np.array_equal(y2[:, Nq + Nkv:], y[:, Nq + Nkv:])
    assert not np.array_equal(y2[act == 1][:, Nq:Nq + Nkv], y[act == 1][:, Nq:Nq + Nkv])


PINS = [pin_per_module_factors_exact, pin_variants_small_integers_exact, pin_variants_reduce_to_the_plain_form, pin_worked_example, pin_one_hot_closed_form, pin_activation_zero_is_lora,
        pin_pre_activation_rows_are_base_exactly, pin_zero_B_and_never_activated,
        pin_blend_equals_select, pin_mask_closed_form_counts, pin_group_matches_stable_sort,
        pin_brute_force_exact, pin_linearity, pin_row_permutation, pin_paged_store,
        pin_cached_prefix_untouched, pin_column_split]


@pytest.mark.parametrize("pin", PINS, ids=[p.__name__ for p in PINS])
def test_pin(pin):
    pin()


def test_config1_full_forward_runs_fast():
    w = wl.config1()
    res, _, _ = _forward_small(w)
    assert res.q_out.shape == (64, 256) and int(res.active.sum()) == 8
