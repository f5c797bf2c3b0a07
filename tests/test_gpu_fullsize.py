"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: EVERY token row
against the fp64 oracle, element by element, for q_out and the written K and V slots (at the 70B shape:
16 rows of every token tile plus the activation boundaries), plus properties that hold at any size (exact
integer results, untouched cache slots, bit-identity of pre-activation rows with a base-only run,
determinism).  Includes the mixed base / rank-8 LoRA / rank-32 aLoRA / bias batch (Sec. 3, Sec. 4.1)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_17910_amd import binding as ab
from paper_2512_17910_amd import workloads as wl
from gpu_util import DeviceBatch, TOL, check_grouping, host_operands, maxnorm_rel, to_f64

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.view(torch.int16)


def _rows_to_check(w, cfg):
    """Every row where the oracle over all rows takes seconds; at the 70B shape 16 rows of every 256-row
    token tile (all features of a row are checked, so every token tile x feature tile pair is hit) plus the
    activation boundaries and segment ends."""
    if cfg != 4:
        return np.arange(w.T, dtype=np.int32)
    spread = np.concatenate([t0 + np.linspace(0, 255, 16).astype(np.int64) for t0 in range(0, w.T, 256)])
    return np.unique(np.concatenate([spread[spread < w.T], wl.sample_rows(w, 64).astype(np.int64)])).astype(np.int32)


@pytest.mark.parametrize("cfg", [2, 3, 4, 5, 6])
def test_full_size_config(cfg):
    w = wl.CONFIGS[cfg]()
    print(f"[case] config {cfg}: {w.name} T={w.T} H={w.hidden} N={w.N} L={w.n_adapters} r={w.rank}", flush=True)
    db = DeviceBatch(w, cache_fill=False)
    assert db.validate() == ab.ALORA_OK
    db.forward()

    # integer results, exact
    mask, act = oracle.classify(w.token_adapter_ids, w.token_seg_ids, w.token_positions, w.activation_start)
    perm, off = oracle.group(w.token_adapter_ids, act, w.n_adapters)
    check_grouping(*ab.workspace_int_views(db.dims, db.ws), act, perm, off)

    # rows against the oracle, element by element: q_out and the written K and V slots
    rows = _rows_to_check(w, cfg)
    assert cfg != 4 or len(rows) >= 512
    x, W, A, B = host_operands(w)
    bias64 = wl.widen_f64(w.bias, w.dtype) if w.bias is not None else None
    y = oracle.alora_rows_var(x, W, A, B, w.token_adapter_ids, act, rows, bias64)
    print(f"[case] config {cfg}: oracle on {len(rows)} of {w.T} rows done", flush=True)
    ridx = torch.from_numpy(rows.astype(np.int64)).to("cuda")
    tol = TOL[w.dtype]
    scale = np.max(np.abs(y))

    def check(got, ref, what):
        assert maxnorm_rel(got, ref) <= tol, what
        # per element as well: one bf16 rounding plus accumulation noise
        assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 2.0 ** -12 * scale), what

    check(to_f64(db.q[ridx]), y[:, : w.Nq], "q_out")
    sl = w.slot_mapping[rows]
    has = sl >= 0
    sidx = torch.from_numpy(sl[has]).to("cuda")
    check(to_f64(db.kc[sidx]), y[has][:, w.Nq: w.Nq + w.Nkv], "k_cache")
    check(to_f64(db.vc[sidx]), y[has][:, w.Nq + w.Nkv:], "v_cache")
    # adapted rows really differ from the base projection (the delta is not lost)
    if act[rows].any():
        ar = rows[act[rows] == 1][:4]
        yb = oracle.base_rows(x, W, ar)
        if bias64 is not None:
            yb = yb + bias64
        ya = y[np.isin(rows, ar)]
        assert maxnorm_rel(ya, yb) > 0.05
    del x, W, A, B, y

    # exactly the mapped slots changed
    changed_k = (_bits(db.kc) != _bits(db.k0)).any(dim=1)
    changed_v = (_bits(db.vc) != _bits(db.v0)).any(dim=1)
    want = torch.zeros(w.n_slots, dtype=torch.bool, device="cuda")
    want[torch.from_numpy(w.slot_mapping[w.slot_mapping >= 0]).to("cuda")] = True
    assert torch.equal(changed_k, want) and torch.equal(changed_v, want)
    if w.cached_prefix_slots is not None:
        pre = torch.from_numpy(w.cached_prefix_slots).to("cuda")
        assert torch.equal(_bits(db.kc[pre]), _bits(db.k0[pre])) and torch.equal(_bits(db.vc[pre]), _bits(db.v0[pre]))

    # pre-activation rows are bit-identical to a base-only call; the call is deterministic
    q1, k1, v1 = db.q.clone(), db.kc.clone(), db.vc.clone()
    db.reset()
    db.forward()
    assert torch.equal(_bits(db.q), _bits(q1)) and torch.equal(_bits(db.kc), _bits(k1))
    assert torch.equal(_bits(db.vc), _bits(v1))
    db.reset()
    db.forward(aid=torch.full_like(db.aid, -1))
    pre_rows = torch.from_numpy(np.nonzero(act == 0)[0]).to("cuda")
    assert torch.equal(_bits(db.q[pre_rows]), _bits(q1[pre_rows]))
    pre_slots = torch.from_numpy(w.slot_mapping[(act == 0) & (w.slot_mapping >= 0)]).to("cuda")
    assert torch.equal(_bits(db.kc[pre_slots]), _bits(k1[pre_slots]))
    assert torch.equal(_bits(db.vc[pre_slots]), _bits(v1[pre_slots]))
    act_rows = torch.from_numpy(np.nonzero(act == 1)[0]).to("cuda")
    if act_rows.numel():
        assert not torch.equal(_bits(db.q[act_rows]), _bits(q1[act_rows]))
