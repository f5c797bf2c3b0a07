"""Harness plumbing shared by the benchmark, the smoke run and the GPU tests: move a Workload to the
device, call the C ABI through the binding, bring results back as exactly widened fp64.  No arithmetic
of the method lives here (the library's kernels compute; the oracle checks)."""
from __future__ import annotations

import numpy as np
import torch

from paper_2512_17910_amd import binding as ab
from paper_2512_17910_amd import workloads as wl

DEV = "cuda"

# parity gates (max-norm relative error per output tensor, versus the fp64 oracle)
TOL = {"f32": 1e-5, "bf16": 2e-2}


def to_dev(a: np.ndarray, dtype: str):
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def to_f64(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return wl.bf16_bits_to_f32(bits).astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


def raw_bits(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.contiguous().view(torch.int32).cpu().numpy().view(np.uint32)


class DeviceBatch:
    """A Workload resident on the GPU plus the buffers one forward call needs."""

    def __init__(self, w: wl.Workload, cache_fill=True):
        self.w = w
        dt = w.dtype
        self.x = to_dev(w.x, dt)
        self.W = to_dev(w.W, dt)
        self.A = [to_dev(a, dt) for a in w.A]
        self.B = [to_dev(b, dt) for b in w.B]
        self.aid = torch.from_numpy(w.token_adapter_ids).to(DEV)
        self.seg = torch.from_numpy(w.token_seg_ids).to(DEV)
        self.pos = torch.from_numpy(w.token_positions).to(DEV)
        self.start = torch.from_numpy(w.activation_start).to(DEV)
        self.slot = torch.from_numpy(w.slot_mapping).to(DEV)
        tdt = torch.bfloat16 if dt == "bf16" else torch.float32
        self.q = torch.zeros((w.T, w.Nq), dtype=tdt, device=DEV)
        if cache_fill:
            self.k0 = to_dev(wl.cache_fill(w.n_slots, w.Nkv, dt, 0), dt)
            self.v0 = to_dev(wl.cache_fill(w.n_slots, w.Nkv, dt, 1), dt)
        else:  # large caches: a cheap on-device pattern instead of host-generated values
            self.k0 = torch.full((w.n_slots, w.Nkv), 0.375, dtype=tdt, device=DEV)
            self.v0 = torch.full((w.n_slots, w.Nkv), -0.625, dtype=tdt, device=DEV)
        self.kc = self.k0.clone()
        self.vc = self.v0.clone()
        self.dims = ab.make_dims(ab.ALORA_BF16 if dt == "bf16" else ab.ALORA_F32, w.T, w.hidden, w.n_q_heads,
                                 w.n_kv_heads, w.head_dim, w.n_adapters, w.rank, w.n_segments, w.n_slots,
                                 self.seg, self.pos)
        self.ws = ab.alloc_workspace(self.dims)
        self.bias = to_dev(w.bias, dt) if w.bias is not None else None

    def reset(self):
        self.q.zero_()
        self.kc.copy_(self.k0)
        self.vc.copy_(self.v0)

    def forward(self, aid=None, A=None, B=None):
        if self.bias is not None or self.w.adapter_ranks is not None:
            ab.alora_qkv_forward_ex(self.x, self.aid if aid is None else aid, self.start, self.W,
                                    self.A if A is None else A, self.B if B is None else B,
                                    self.q, self.kc, self.vc, self.slot, self.w.block_size, self.dims, self.ws,
                                    bias=self.bias, adapter_ranks=self.w.adapter_ranks)
            torch.cuda.synchronize()
            return
        ab.alora_qkv_forward(self.x, self.aid if aid is None else aid, self.start, self.W,
                             self.A if A is None else A, self.B if B is None else B,
                             self.q, self.kc, self.vc, self.slot, self.w.block_size, self.dims, self.ws)
        torch.cuda.synchronize()

    def validate(self) -> int:
        return ab.alora_qkv_validate(self.aid, self.start, self.slot, self.w.block_size, self.dims)


def host_operands(w: wl.Workload):
    """Workload values widened exactly to fp64 (what the oracle consumes)."""
    x = wl.widen_f64(w.x, w.dtype)
    W = wl.widen_f64(w.W, w.dtype)
    A = [wl.widen_f64(a, w.dtype) for a in w.A]
    B = [wl.widen_f64(b, w.dtype) for b in w.B]
    return x, W, A, B


def maxnorm_rel(got: np.ndarray, ref: np.ndarray) -> float:
    denom = np.max(np.abs(ref)) if ref.size else 1.0
    if denom == 0:
        denom = 1.0
    return float(np.max(np.abs(got - ref)) / denom) if ref.size else 0.0


def check_grouping(act_g, perm_g, off_g, ref_active, ref_perm, ref_offsets) -> None:
    """Integer results of the classification/grouping step against the oracle, bit for bit:
    flags, adapter groups in stable order, and the trailing group of rows that keep the base output."""
    act_g, perm_g, off_g = act_g.cpu().numpy(), perm_g.cpu().numpy(), off_g.cpu().numpy()
    T, L = ref_active.shape[0], ref_offsets.shape[0] - 1
    assert np.array_equal(act_g, ref_active)
    assert np.array_equal(off_g[: L + 1], ref_offsets)
    assert off_g[L + 1] == T
    assert np.array_equal(perm_g[: ref_perm.size], ref_perm)
    assert np.array_equal(perm_g[ref_perm.size: T], np.nonzero(ref_active == 0)[0])
