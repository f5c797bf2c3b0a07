"""CPU fp64 oracle for the masked multi-adapter aLoRA QKV projection + paged K/V write.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  The GPU library never calls into this package and the two share no code.

The arithmetic lives in alora_oracle.c (plain C, fp64, index-order sums); this module
compiles it with gcc, marshals numpy arrays through ctypes and strings the steps together
in the order the paper gives them (App. B mask -> Algorithm 1 / Sec. 2.3 projection ->
paged store).  All of it is pinned by tests/test_oracle_*.py; nothing is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "alora_oracle.c")
_SO = os.path.join(_HERE, "_alora_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction: sums stay in index order)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
               "-o", _SO, _SRC]
        subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(_SO)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr_table(mats: Sequence[np.ndarray]):
    arr = (ctypes.c_void_p * max(len(mats), 1))()
    for i, m in enumerate(mats):
        arr[i] = m.ctypes.data
    return arr


def classify(aid, seg, pos, start):
    """(paper_mask, active) per token row; App. B mask and its use in Algorithm 1."""
    aid, seg, pos, start = _i32(aid), _i32(seg), _i32(pos), _i32(start)
    T = aid.shape[0]
    mask = np.zeros(T, dtype=np.uint8)
    act = np.zeros(T, dtype=np.uint8)
    _load().oracle_classify(ctypes.c_int64(T), _p(aid), _p(seg), _p(pos), _p(start), _p(mask), _p(act))
    return mask, act


def group(aid, active, n_adapters: int):
    """Stable grouping of active rows by adapter -> (perm [T_act], offsets [L+1])."""
    aid = _i32(aid)
    active = np.ascontiguousarray(active, dtype=np.uint8)
    T = aid.shape[0]
    perm = np.zeros(max(int(active.sum()), 1), dtype=np.int32)
    offsets = np.zeros(n_adapters + 1, dtype=np.int32)
    _load().oracle_group(ctypes.c_int64(T), ctypes.c_int32(n_adapters), _p(aid), _p(active), _p(perm), _p(offsets))
    return perm[: int(active.sum())], offsets


def base_rows(x, W, rows) -> np.ndarray:
    x, W, rows = _f64(x), _f64(W), _i32(rows)
    H, N = W.shape
    assert x.shape[1] == H
    y = np.zeros((rows.shape[0], N), dtype=np.float64)
    _load().oracle_base_rows(ctypes.c_int64(rows.shape[0]), _p(rows), ctypes.c_int32(H), ctypes.c_int32(N),
                             _p(x), _p(W), _p(y))
    return y


def _adapter_args(A, B, H, N):
    A = [_f64(a) for a in A]
    B = [_f64(b) for b in B]
    r = A[0].shape[1] if A else 0
    assert r <= 256
    for a, b in zip(A, B):
        assert a.shape == (H, r) and b.shape == (r, N)
    return A, B, r


def alora_rows(x, W, A, B, aid, active, rows) -> np.ndarray:
    """Select form of the Sec. 2.3 block equations on the given token rows."""
    x, W, rows, aid = _f64(x), _f64(W), _i32(rows), _i32(aid)
    active = np.ascontiguousarray(active, dtype=np.uint8)
    H, N = W.shape
    A, B, r = _adapter_args(A, B, H, N)
    y = np.zeros((rows.shape[0], N), dtype=np.float64)
    _load().oracle_alora_rows(ctypes.c_int64(rows.shape[0]), _p(rows), ctypes.c_int32(H), ctypes.c_int32(N),
                              ctypes.c_int32(r), _p(x), _p(W), _ptr_table(A), _ptr_table(B),
                              _p(aid), _p(active), _p(y))
    return y


def alora_rows_var(x, W, A, B, aid, active, rows, bias=None) -> np.ndarray:
    """alora_rows with the layer's bias (Algorithm 1: l.apply(x, b)) and one rank per adapter
    (A[i] is [H, r_i], B[i] is [r_i, N]; Sec. 4.1)."""
    x, W, rows, aid = _f64(x), _f64(W), _i32(rows), _i32(aid)
    active = np.ascontiguousarray(active, dtype=np.uint8)
    H, N = W.shape
    A = [_f64(a) for a in A]
    B = [_f64(b) for b in B]
    ranks = _i32([a.shape[1] for a in A] or [0])
    for a, b, r in zip(A, B, ranks):
        assert a.shape == (H, r) and b.shape == (r, N) and r <= 256
    bias_p = None
    if bias is not None:
        bias = _f64(bias)
        assert bias.shape == (N,)
        bias_p = _p(bias)
    y = np.zeros((rows.shape[0], N), dtype=np.float64)
    _load().oracle_alora_rows_var(ctypes.c_int64(rows.shape[0]), _p(rows), ctypes.c_int32(H), ctypes.c_int32(N),
                                  _p(ranks), _p(x), _p(W), bias_p, _ptr_table(A), _ptr_table(B),
                                  _p(aid), _p(active), _p(y))
    return y


def alora_rows_per_module(x, W_mod, A_mod, B_mod, aid, active, rows) -> np.ndarray:
    """Sec. 2.3 as it is written: one block equation per module.  W_mod = (W^Q, W^K, W^V); A_mod[m][i] is
    adapter i's factor [H, r] of module m and B_mod[m][i] its factor [r, N_m].  Each module is projected on
    its own (three calls of the single-module routine); the result is [Q | K | V] per row."""
    assert len(W_mod) == len(A_mod) == len(B_mod) == 3
    return np.concatenate([alora_rows(x, W_mod[m], A_mod[m], B_mod[m], aid, active, rows) for m in range(3)], axis=1)


def blend_rows(x, W, A, B, aid, paper_mask, rows) -> np.ndarray:
    """Algorithm 1 taken literally (clone, add_adapter, blend with the mask)."""
    x, W, rows, aid = _f64(x), _f64(W), _i32(rows), _i32(aid)
    paper_mask = np.ascontiguousarray(paper_mask, dtype=np.uint8)
    H, N = W.shape
    A, B, r = _adapter_args(A, B, H, N)
    y = np.zeros((rows.shape[0], N), dtype=np.float64)
    _load().oracle_blend_rows(ctypes.c_int64(rows.shape[0]), _p(rows), ctypes.c_int32(H), ctypes.c_int32(N),
                              ctypes.c_int32(r), _p(x), _p(W), _ptr_table(A), _ptr_table(B),
                              _p(aid), _p(paper_mask), _p(y))
    return y


def slot_coords(slot, block_size: int):
    slot = np.ascontiguousarray(slot, dtype=np.int64)
    T = slot.shape[0]
    blk = np.zeros(T, dtype=np.int64)
    off = np.zeros(T, dtype=np.int32)
    _load().oracle_slot_coords(ctypes.c_int64(T), _p(slot), ctypes.c_int32(block_size), _p(blk), _p(off))
    return blk, off


def store_rows(y, rows, Nq: int, Nkv: int, slot, block_size: int, q_out, k_cache, v_cache) -> None:
    """Write projected rows into q_out [T,Nq] and the paged caches [n_slots,Nkv] in place."""
    y, rows = _f64(y), _i32(rows)
    slot = np.ascontiguousarray(slot, dtype=np.int64)
    for a in (q_out, k_cache, v_cache):
        assert a.dtype == np.float64 and a.flags.c_contiguous
    _load().oracle_store_rows(ctypes.c_int64(rows.shape[0]), _p(rows), ctypes.c_int32(Nq), ctypes.c_int32(Nkv),
                              _p(y), _p(slot), ctypes.c_int32(block_size), _p(q_out), _p(k_cache), _p(v_cache))


@dataclass
class ForwardResult:
    paper_mask: np.ndarray   # uint8 [T], 1 = pre-activation (keep base)
    active: np.ndarray       # uint8 [T], 1 = row receives its adapter's delta
    perm: np.ndarray         # int32 [T_act]
    offsets: np.ndarray      # int32 [L+1]
    q_out: np.ndarray        # float64 [T,Nq]
    k_cache: np.ndarray      # float64 [n_slots,Nkv]
    v_cache: np.ndarray      # float64 [n_slots,Nkv]
    written_slots: np.ndarray  # sorted int64


def alora_qkv_forward(x, token_adapter_ids, token_seg_ids, token_positions, activation_start,
                      W, A, B, slot_mapping, block_size: int, Nq: int, Nkv: int,
                      k_cache: np.ndarray, v_cache: np.ndarray, bias=None) -> ForwardResult:
    """The whole path on every row: mask, grouping, projection, q_out and paged K/V store.

    k_cache / v_cache are float64 [n_slots, Nkv] holding the cache's previous contents; copies
    are updated and returned.
    """
    x = _f64(x)
    T = x.shape[0]
    mask, act = classify(token_adapter_ids, token_seg_ids, token_positions, activation_start)
    perm, offsets = group(token_adapter_ids, act, len(A))
    rows = np.arange(T, dtype=np.int32)
    uniform = len({np.asarray(a).shape[1] for a in A}) <= 1
    if bias is None and uniform:
        y = alora_rows(x, W, A, B, token_adapter_ids, act, rows)
    else:
        y = alora_rows_var(x, W, A, B, token_adapter_ids, act, rows, bias)
    q = np.zeros((T, Nq), dtype=np.float64)
    kc, vc = _f64(k_cache).copy(), _f64(v_cache).copy()
    store_rows(y, rows, Nq, Nkv, slot_mapping, block_size, q, kc, vc)
    sm = np.asarray(slot_mapping, dtype=np.int64)
    return ForwardResult(mask, act, perm, offsets, q, kc, vc, np.sort(sm[sm >= 0]))
