"""The C-ABI library loads, exports every symbol the headers under include/ declare, and its host-side
argument checks answer without touching a GPU (no compute call is made here)."""
import ctypes
import os
import re

import pytest

from paper_2512_17910_amd import binding as ab

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "alora_qkv.h")


def _declared_functions():
    """Every function declared in any header under include/."""
    import glob
    names = set()
    for h in glob.glob(os.path.join(ROOT, "include", "*.h")):
        src = open(h).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names |= set(re.findall(r"\b(alora_[a-z_]+)\s*\(", src))
    return sorted(names)


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert {"alora_qkv_forward", "alora_qkv_workspace_bytes", "alora_qkv_classify_group",
            "alora_qkv_validate", "alora_status_string", "alora_qkv_graph_create", "alora_planner_admit",
            "alora_planner_commit"} <= set(names)
    L = ab.lib()
    for n in names:
        assert hasattr(L, n), f"{n} declared in the header but not exported"


def test_header_constants_match_binding():
    src = open(HEADER).read()
    for name in ("ALORA_F32", "ALORA_BF16", "ALORA_MAX_ADAPTERS", "ALORA_MAX_RANK", "ALORA_OK"):
        m = re.search(rf"#define {name} \(?(-?\d+)\)?", src)
        assert m and int(m.group(1)) == getattr(ab, name)
    for name in ("ALORA_EINVAL", "ALORA_ESHAPE", "ALORA_EWORKSPACE", "ALORA_EHIP", "ALORA_EDATA", "ALORA_ENOMEM"):
        m = re.search(rf"#define {name} \((-?\d+)\)", src)
        assert m and int(m.group(1)) == getattr(ab, name)


def _dims(**kw):
    d = dict(dtype=ab.ALORA_BF16, T=128, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, n_adapters=2,
             rank=16, n_segments=2, n_slots=256)
    d.update(kw)
    dims = ab.make_dims(**d)
    dims.token_seg_ids = 0x10000
    dims.token_positions = 0x20000
    return dims


def test_workspace_size_and_layout():
    d = _dims()
    n = ab.alora_qkv_workspace_bytes(d)
    lay = ab.alora_qkv_workspace_layout(d)
    assert n == lay.total_bytes and n % 256 == 0
    assert lay.active_off % 256 == 0 and lay.perm_off >= lay.active_off + d.T
    assert lay.offsets_off >= lay.perm_off + 4 * d.T
    assert ab.alora_qkv_workspace_bytes(_dims(T=0)) >= 256
    assert ab.alora_qkv_workspace_bytes(_dims(T=4096)) > n


@pytest.mark.parametrize("kw,status", [
    (dict(dtype=7), ab.ALORA_EINVAL),
    (dict(T=-1), ab.ALORA_EINVAL),
    (dict(hidden=100), ab.ALORA_ESHAPE),            # bf16 needs hidden % 64 == 0
    (dict(head_dim=3), ab.ALORA_ESHAPE),            # Nq % 8
    (dict(rank=12), ab.ALORA_ESHAPE),               # bf16 rank % 8
    (dict(rank=72), ab.ALORA_ESHAPE),
    (dict(n_adapters=129), ab.ALORA_ESHAPE),
    (dict(dtype=ab.ALORA_F32, hidden=6), ab.ALORA_ESHAPE),
])
def test_bad_dims_are_rejected(kw, status):
    out = ctypes.c_size_t(0)
    d = _dims(**kw)
    assert ab.lib().alora_qkv_workspace_bytes(ctypes.byref(d), ctypes.byref(out)) == status


def test_forward_rejects_bad_arguments_before_any_launch():
    """Fake (never dereferenced) pointers: every call must fail in the host-side checks."""
    L = ab.lib()
    d = _dims()
    need = ab.alora_qkv_workspace_bytes(d)
    P = 0x100000  # 16-byte and 256-byte aligned dummy address
    tab = (ctypes.c_void_p * 2)(P, P)

    def call(x=P, aid=P, start=P, W=P, A=tab, B=tab, q=P, kc=P, vc=P, slot=P, bs=16, dims=d, ws=P, wsb=need):
        return L.alora_qkv_forward(x, aid, start, W, A, B, q, kc, vc, slot, bs, ctypes.byref(dims), ws, wsb, None)

    assert call(x=None) == ab.ALORA_EINVAL
    assert call(W=None) == ab.ALORA_EINVAL
    assert call(q=None) == ab.ALORA_EINVAL
    assert call(slot=None) == ab.ALORA_EINVAL
    assert call(kc=None) == ab.ALORA_EINVAL
    assert call(A=None) == ab.ALORA_EINVAL
    assert call(x=P + 2) == ab.ALORA_EINVAL
    assert call(bs=0) == ab.ALORA_EINVAL
    assert call(bs=24) == ab.ALORA_ESHAPE            # 256 slots not a multiple of 24
    assert call(ws=None) == ab.ALORA_EWORKSPACE
    assert call(ws=P + 16) == ab.ALORA_EWORKSPACE
    assert call(wsb=need - 1) == ab.ALORA_EWORKSPACE
    tab_bad = (ctypes.c_void_p * 2)(P, None)
    assert call(B=tab_bad) == ab.ALORA_EINVAL
    assert call(dims=_dims(rank=12)) == ab.ALORA_ESHAPE
    # T == 0 is a successful no-op that needs no data pointers
    assert call(x=None, aid=None, W=None, q=None, slot=None, dims=_dims(T=0)) == ab.ALORA_OK
    assert L.alora_status_string(ab.ALORA_ESHAPE).decode().startswith("unsupported shape")
    assert L.alora_qkv_version() >= 100


def _attn_dims(**kw):
    d = dict(dtype=ab.ALORA_BF16, n_tokens=8, n_q_heads=8, n_kv_heads=2, head_dim=128, n_seqs=2, max_blocks=4,
             block_size=16, n_slots=128, scale=0.0)
    d.update(kw)
    return ab.AloraAttnDims(**d)


def test_paged_attention_argument_checks_answer_on_the_host():
    L = ab.lib()
    p = lambda v: ctypes.c_void_p(v)
    good = [p(0x1000), p(0x2000), p(0x3000), p(0x4000), p(0x5000), p(0x6000), p(0x7000)]
    call = lambda args, d: L.alora_paged_attention(*args, ctypes.byref(d), None)
    assert call(good, _attn_dims(head_dim=96)) == ab.ALORA_ESHAPE
    assert call(good, _attn_dims(n_q_heads=6)) == ab.ALORA_ESHAPE           # 3 query heads per K/V head
    assert call(good, _attn_dims(n_q_heads=7)) == ab.ALORA_ESHAPE
    assert call(good, _attn_dims(block_size=0)) == ab.ALORA_EINVAL
    assert call(good, _attn_dims(dtype=5)) == ab.ALORA_EINVAL
    assert call(good, _attn_dims(scale=-1.0)) == ab.ALORA_EINVAL
    assert call(good, _attn_dims(scale=float("nan"))) == ab.ALORA_EINVAL
    assert call(good, _attn_dims(n_tokens=0)) == ab.ALORA_OK                 # nothing to do, nothing launched
    for i in range(7):
        args = list(good)
        args[i] = p(None)
        assert call(args, _attn_dims()) == ab.ALORA_EINVAL
    args = list(good)
    args[0] = p(0x1008)                                                       # q not 16-byte aligned
    assert call(args, _attn_dims()) == ab.ALORA_EINVAL
    assert L.alora_paged_attention(*good, None, None) == ab.ALORA_EINVAL
    assert L.alora_paged_attention_validate(p(0x4000), p(0x5000), p(0x6000), ctypes.byref(_attn_dims(head_dim=32))) == ab.ALORA_ESHAPE
    assert ctypes.sizeof(ab.AloraAttnDims) == 48


def test_bench_refuses_more_than_one_gpu():
    """This build shows one GPU's share: asking bench.py for more exits with a message before touching a GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_model_of_the_ranged_shrink_combine():
    """Host-side model of what the ranged shrink does with a block's partial results: every range of the
    hidden dimension accumulates in fp32, the partials are added in RANGE ORDER whichever range finishes last,
    and the sum is handed on as hi = bf16(S), lo = bf16(S - hi).  On small integers every fp32 sum is exact,
    so the model must equal the exact x . A for any number of ranges and any arrival order, and hi + lo must
    give S back exactly while S needs at most 16 significant bits."""
    import numpy as np
    from paper_2512_17910_amd import workloads as wl
    rng = np.random.default_rng(5)
    H, r, rows = 512, 8, 32
    x = rng.integers(-3, 4, (rows, H)).astype(np.float32)
    A = rng.integers(-3, 4, (H, r)).astype(np.float32)
    exact = x.astype(np.int64) @ A.astype(np.int64)
    for n_ranges in (1, 2, 4, 8):
        kper = H // n_ranges
        parts = []
        for g in range(n_ranges):
            acc = np.zeros((rows, r), np.float32)
            for k in range(g * kper, (g + 1) * kper):          # fp32 accumulation, k ascending
                acc = acc + x[:, k:k + 1] * A[k:k + 1, :]
            parts.append(acc)
        for arrival in (list(range(n_ranges)), list(reversed(range(n_ranges)))):
            # whoever arrives last adds the partials in range order, not in arrival order
            S = np.zeros((rows, r), np.float32)
            for g in range(n_ranges):
                S = S + parts[g]
            assert arrival[-1] in range(n_ranges) and np.array_equal(S.astype(np.int64), exact)
        hi = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(S))
        lo = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(S - hi))
        assert np.array_equal(hi + lo, S)
