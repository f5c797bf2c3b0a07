"""ctypes binding of the block cache / suffix planner (include/alora_planner.h).  Marshalling only:
numpy arrays in, numpy arrays out; every decision is taken by the C++ planner of the library."""
from __future__ import annotations

import ctypes
from typing import Sequence

import numpy as np

from .binding import AloraError, lib

ALORA_ENOBLOCKS = -7


class PlanBatch(ctypes.Structure):
    _fields_ = [("token_positions", ctypes.c_void_p), ("token_seg_ids", ctypes.c_void_p),
                ("token_adapter_ids", ctypes.c_void_p), ("slot_mapping", ctypes.c_void_p),
                ("activation_start", ctypes.c_void_p),
                ("row_cap", ctypes.c_int32), ("seg_cap", ctypes.c_int32),
                ("n_rows", ctypes.c_int32), ("n_segs", ctypes.c_int32)]


_declared = False
_planner_lib = None   # a separately built planner (the host-only translation unit under CPU sanitizers); None: the library


def use_planner_library(handle) -> None:
    """Point this binding at another build of the planner's C ABI (ctypes handle), or back at the library (None)."""
    global _planner_lib, _declared
    _planner_lib = handle
    _declared = False


def _L():
    global _declared
    L = _planner_lib if _planner_lib is not None else lib()
    if not _declared:
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        L.alora_planner_create.argtypes = [i32, i64, ctypes.POINTER(vp)]
        L.alora_planner_destroy.argtypes = [vp]
        L.alora_planner_admit.argtypes = [vp, i64, vp, i32, i32, i32, ctypes.POINTER(PlanBatch), ctypes.POINTER(i32)]
        L.alora_planner_append.argtypes = [vp, i64, vp, i32, ctypes.POINTER(PlanBatch)]
        L.alora_planner_commit.argtypes = [vp, i64]
        L.alora_planner_finish.argtypes = [vp, i64]
        L.alora_planner_block_table.argtypes = [vp, i64, vp, i32, ctypes.POINTER(i32)]
        L.alora_planner_free_blocks.argtypes = [vp]
        L.alora_planner_free_blocks.restype = i64
        for n in ("create", "destroy", "admit", "append", "commit", "finish", "block_table"):
            getattr(L, "alora_planner_" + n).restype = ctypes.c_int
        _declared = True
    return L


class Batch:
    """Host arrays one forward call's metadata is planned into."""

    def __init__(self, row_cap: int, seg_cap: int):
        self.token_positions = np.zeros(row_cap, np.int32)
        self.token_seg_ids = np.zeros(row_cap, np.int32)
        self.token_adapter_ids = np.zeros(row_cap, np.int32)
        self.slot_mapping = np.zeros(row_cap, np.int64)
        self.activation_start = np.zeros(seg_cap, np.int32)
        self.c = PlanBatch(self.token_positions.ctypes.data, self.token_seg_ids.ctypes.data,
                           self.token_adapter_ids.ctypes.data, self.slot_mapping.ctypes.data,
                           self.activation_start.ctypes.data, row_cap, seg_cap, 0, 0)

    @property
    def n_rows(self) -> int:
        return int(self.c.n_rows)

    @property
    def n_segs(self) -> int:
        return int(self.c.n_segs)

    def rows(self):
        n = self.n_rows
        return (self.token_positions[:n], self.token_seg_ids[:n], self.token_adapter_ids[:n], self.slot_mapping[:n],
                self.activation_start[:self.n_segs])


class Planner:
    def __init__(self, block_size: int, n_blocks: int):
        h = ctypes.c_void_p(None)
        s = _L().alora_planner_create(block_size, n_blocks, ctypes.byref(h))
        if s:
            raise AloraError(s, "alora_planner_create")
        self._h = h
        self.block_size = block_size

    def close(self) -> None:
        if self._h:
            _L().alora_planner_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    @staticmethod
    def _tok(tokens: Sequence[int]) -> np.ndarray:
        return np.ascontiguousarray(tokens, dtype=np.int32)

    def admit(self, req_id: int, tokens, adapter_id: int, activation_start: int, batch: Batch) -> int:
        """Returns the number of tokens taken from the cache."""
        t = self._tok(tokens)
        cached = ctypes.c_int32(0)
        s = _L().alora_planner_admit(self._h, req_id, t.ctypes.data, t.size, adapter_id, activation_start,
                                     ctypes.byref(batch.c), ctypes.byref(cached))
        if s:
            raise AloraError(s, "alora_planner_admit")
        return int(cached.value)

    def append(self, req_id: int, new_tokens, batch: Batch) -> None:
        t = self._tok(new_tokens)
        s = _L().alora_planner_append(self._h, req_id, t.ctypes.data, t.size, ctypes.byref(batch.c))
        if s:
            raise AloraError(s, "alora_planner_append")

    def commit(self, req_id: int) -> None:
        s = _L().alora_planner_commit(self._h, req_id)
        if s:
            raise AloraError(s, "alora_planner_commit")

    def finish(self, req_id: int) -> None:
        s = _L().alora_planner_finish(self._h, req_id)
        if s:
            raise AloraError(s, "alora_planner_finish")

    def block_table(self, req_id: int) -> np.ndarray:
        n = ctypes.c_int32(0)
        s = _L().alora_planner_block_table(self._h, req_id, None, 0, ctypes.byref(n))
        if s:
            raise AloraError(s, "alora_planner_block_table")
        out = np.zeros(n.value, np.int32)
        s = _L().alora_planner_block_table(self._h, req_id, out.ctypes.data, out.size, ctypes.byref(n))
        if s:
            raise AloraError(s, "alora_planner_block_table")
        return out

    def free_blocks(self) -> int:
        return int(_L().alora_planner_free_blocks(self._h))
