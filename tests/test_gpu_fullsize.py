"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: sampled
token rows against the fp64 oracle (every activation boundary +-2, segment ends, spread rows),
plus properties that hold at any size (exact integer results, untouched cache slots,
bit-identity of pre-activation rows with a base-only run, determinism)."""
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


@pytest.mark.parametrize("cfg,n_sample", [(2, 96), (3, 256), (4, 40), (5, 96)])
def test_full_size_config(cfg, n_sample):
    w = wl.CONFIGS[cfg]()
    print(f"[case] config {cfg}: {w.name} T={w.T} H={w.hidden} N={w.N} L={w.n_adapters} r={w.rank}", flush=True)
    db = DeviceBatch(w, cache_fill=False)
    assert db.validate() == ab.ALORA_OK
    db.forward()

    # integer results, exact
    mask, act = oracle.classify(w.token_adapter_ids, w.token_seg_ids, w.token_positions, w.activation_start)
    perm, off = oracle.group(w.token_adapter_ids, act, w.n_adapters)
    check_grouping(*ab.workspace_int_views(db.dims, db.ws), act, perm, off)

    # sampled rows against the oracle
    rows = wl.sample_rows(w, n_sample)
    x, W, A, B = host_operands(w)
    y = oracle.alora_rows(x, W, A, B, w.token_adapter_ids, act, rows)
    del x, W
    ridx = torch.from_numpy(rows.astype(np.int64)).to("cuda")
    tol = TOL[w.dtype]
    assert maxnorm_rel(to_f64(db.q[ridx]), y[:, : w.Nq]) <= tol
    sl = w.slot_mapping[rows]
    has = sl >= 0
    sidx = torch.from_numpy(sl[has]).to("cuda")
    assert maxnorm_rel(to_f64(db.kc[sidx]), y[has][:, w.Nq: w.Nq + w.Nkv]) <= tol
    assert maxnorm_rel(to_f64(db.vc[sidx]), y[has][:, w.Nq + w.Nkv:]) <= tol
    # per element as well: one bf16 rounding plus accumulation noise
    scale = np.max(np.abs(y))
    assert np.all(np.abs(to_f64(db.q[ridx]) - y[:, : w.Nq]) <= 2.0 ** -8 * np.abs(y[:, : w.Nq]) + 2.0 ** -12 * scale)
    # adapted sample rows really differ from the base projection (the delta is not lost)
    if act[rows].any():
        xs, Ws, _, _ = host_operands(w)
        ar = rows[act[rows] == 1][:4]
        yb = oracle.base_rows(xs, Ws, ar)
        del xs, Ws
        ya = y[np.isin(rows, ar)]
        assert maxnorm_rel(ya, yb) > 0.05

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
