"""Thin Python binding over libalora_qkv.so (C ABI declared in include/alora_qkv.h).

Argument marshalling only: torch tensors supply device memory and the stream; every step of
the path runs in the library's HIP kernels.  There is no fallback: if the library is missing
the import of any entry point raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libalora_qkv.so")

ALORA_F32, ALORA_BF16 = 0, 1
ALORA_OK, ALORA_EINVAL, ALORA_ESHAPE, ALORA_EWORKSPACE, ALORA_EHIP, ALORA_EDATA, ALORA_ENOMEM = 0, -1, -2, -3, -4, -5, -6
ALORA_ETOOBIG = -8
ALORA_MAX_ADAPTERS, ALORA_MAX_RANK = 128, 64


class AloraDims(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("T", ctypes.c_int32), ("hidden", ctypes.c_int32),
                ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("n_adapters", ctypes.c_int32), ("rank", ctypes.c_int32), ("n_segments", ctypes.c_int32),
                ("n_slots", ctypes.c_int64), ("token_seg_ids", ctypes.c_void_p),
                ("token_positions", ctypes.c_void_p)]


class AloraWsLayout(ctypes.Structure):
    _fields_ = [("active_off", ctypes.c_size_t), ("perm_off", ctypes.c_size_t),
                ("offsets_off", ctypes.c_size_t), ("total_bytes", ctypes.c_size_t)]


class AloraExtras(ctypes.Structure):
    _fields_ = [("bias", ctypes.c_void_p), ("adapter_ranks", ctypes.c_void_p), ("reuse_grouping", ctypes.c_int32),
                ("rope_cos", ctypes.c_void_p), ("rope_sin", ctypes.c_void_p), ("rope_positions", ctypes.c_int32)]


class AloraAttnDims(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("n_tokens", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("n_seqs", ctypes.c_int32),
                ("max_blocks", ctypes.c_int32), ("block_size", ctypes.c_int32), ("n_slots", ctypes.c_int64),
                ("scale", ctypes.c_float)]


class AloraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().alora_status_string(status).decode()
        if status == ALORA_EHIP:
            msg += f" [hipError {lib().alora_last_hip_error()}]"
        super().__init__(f"{where}: {msg} ({status})")


_lib = None


_lib_path = LIB_PATH


def use_probe_library(path: str) -> None:
    """Make this process load a probe build of the library (see probe.py) instead of the product build.  Only
    before the first call into the library, and only the probe script does it: a probe build computes wrong
    results on purpose."""
    global _lib_path
    if _lib is not None:
        raise RuntimeError("the library is already loaded")
    _lib_path = path


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_lib_path):
            raise ImportError(f"{_lib_path} is missing: build it with `python -m paper_2512_17910_amd.build` "
                              "(there is no non-HIP fallback)")
        # torch first: its HIP runtime must be the one this process uses (a library loaded before it would
        # bring the system's copy of the runtime in beside torch's, and the two do not share devices)
        import torch  # noqa: F401
        L = ctypes.CDLL(_lib_path)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        L.alora_qkv_workspace_bytes.argtypes = [ctypes.POINTER(AloraDims), ctypes.POINTER(sz)]
        L.alora_qkv_workspace_layout.argtypes = [ctypes.POINTER(AloraDims), ctypes.POINTER(AloraWsLayout)]
        L.alora_qkv_classify_group.argtypes = [vp, vp, ctypes.POINTER(AloraDims), vp, sz, vp]
        L.alora_qkv_forward.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32,
                                        ctypes.POINTER(AloraDims), vp, sz, vp]
        L.alora_qkv_validate.argtypes = [vp, vp, vp, i32, ctypes.POINTER(AloraDims)]
        L.alora_qkv_forward_ex.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32,
                                           ctypes.POINTER(AloraDims), ctypes.POINTER(AloraExtras), vp, sz, vp]
        L.alora_qkv_graph_create.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32,
                                             ctypes.POINTER(AloraDims), ctypes.POINTER(AloraExtras), vp, sz,
                                             ctypes.POINTER(vp)]
        L.alora_qkv_forward_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32,
                                               ctypes.POINTER(AloraDims), ctypes.POINTER(AloraExtras), vp]
        L.alora_qkv_forward_static.restype = ctypes.c_int
        L.alora_qkv_static_scratch_bytes.argtypes = []
        L.alora_qkv_static_scratch_bytes.restype = sz
        L.alora_qkv_graph_launch.argtypes = [vp, vp]
        L.alora_qkv_graph_destroy.argtypes = [vp]
        L.alora_paged_attention.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.POINTER(AloraAttnDims), vp]
        L.alora_paged_attention_validate.argtypes = [vp, vp, vp, ctypes.POINTER(AloraAttnDims)]
        L.alora_paged_attention_suffix.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.POINTER(AloraAttnDims), vp]
        L.alora_paged_attention_split.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.POINTER(AloraAttnDims), vp, sz, vp]
        L.alora_paged_attention_workspace_bytes.argtypes = [ctypes.POINTER(AloraAttnDims), ctypes.POINTER(sz)]
        L.alora_paged_attention_suffix_split.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.POINTER(AloraAttnDims), vp, sz, vp]
        L.alora_paged_attention_suffix_workspace_bytes.argtypes = [ctypes.POINTER(AloraAttnDims), ctypes.POINTER(sz)]
        L.alora_status_string.argtypes = [ctypes.c_int]
        L.alora_status_string.restype = ctypes.c_char_p
        L.alora_qkv_set_tuning.argtypes = [ctypes.c_int, ctypes.c_int]
        L.alora_qkv_set_tuning.restype = ctypes.c_int
        L.alora_qkv_profile_begin.argtypes = [ctypes.c_int]
        L.alora_qkv_profile_begin_every.argtypes = [ctypes.c_int, ctypes.c_int]
        L.alora_qkv_profile_begin_every.restype = ctypes.c_int
        L.alora_qkv_profile_end.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int)]
        for name in ("alora_qkv_profile_begin", "alora_qkv_profile_end", "alora_qkv_workspace_bytes", "alora_qkv_workspace_layout", "alora_qkv_classify_group",
                     "alora_qkv_forward", "alora_qkv_validate", "alora_last_hip_error", "alora_qkv_version",
                     "alora_qkv_forward_ex", "alora_qkv_graph_create", "alora_qkv_graph_launch", "alora_qkv_graph_destroy",
                     "alora_paged_attention", "alora_paged_attention_validate", "alora_paged_attention_split", "alora_paged_attention_suffix",
                     "alora_paged_attention_workspace_bytes", "alora_paged_attention_suffix_split",
                     "alora_paged_attention_suffix_workspace_bytes"):
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return ALORA_BF16
    if t.dtype == torch.float32:
        return ALORA_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def make_dims(dtype: int, T: int, hidden: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
              n_adapters: int, rank: int, n_segments: int, n_slots: int,
              token_seg_ids=None, token_positions=None) -> AloraDims:
    return AloraDims(dtype, T, hidden, n_q_heads, n_kv_heads, head_dim, n_adapters, rank, n_segments,
                     n_slots, _ptr(token_seg_ids), _ptr(token_positions))


def alora_qkv_workspace_bytes(dims: AloraDims) -> int:
    out = ctypes.c_size_t(0)
    s = lib().alora_qkv_workspace_bytes(ctypes.byref(dims), ctypes.byref(out))
    if s:
        raise AloraError(s, "alora_qkv_workspace_bytes")
    return int(out.value)


def alora_qkv_workspace_layout(dims: AloraDims) -> AloraWsLayout:
    out = AloraWsLayout()
    s = lib().alora_qkv_workspace_layout(ctypes.byref(dims), ctypes.byref(out))
    if s:
        raise AloraError(s, "alora_qkv_workspace_layout")
    return out


def _stream_handle(stream) -> Optional[int]:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def alloc_workspace(dims: AloraDims, device="cuda"):
    import torch
    return torch.empty(alora_qkv_workspace_bytes(dims), dtype=torch.uint8, device=device)


def _ptr_array(tensors: Sequence):
    arr = (ctypes.c_void_p * max(len(tensors), 1))()
    for i, t in enumerate(tensors):
        arr[i] = t.data_ptr()
    return arr


def alora_qkv_classify_group(token_adapter_ids, activation_start, dims: AloraDims, workspace, stream=None):
    """Runs the classification/grouping step; returns (active, perm, offsets) views of the workspace.
    perm's first offsets[-1] entries are meaningful."""
    import torch
    s = lib().alora_qkv_classify_group(_ptr(token_adapter_ids), _ptr(activation_start), ctypes.byref(dims),
                                       _ptr(workspace), workspace.numel(), _stream_handle(stream))
    if s:
        raise AloraError(s, "alora_qkv_classify_group")
    return workspace_int_views(dims, workspace)


def workspace_int_views(dims: AloraDims, workspace):
    import torch
    lay = alora_qkv_workspace_layout(dims)
    T, L = dims.T, dims.n_adapters
    active = workspace[lay.active_off: lay.active_off + T]
    perm = workspace[lay.perm_off: lay.perm_off + 4 * T].view(torch.int32)
    offsets = workspace[lay.offsets_off: lay.offsets_off + 4 * (L + 2)].view(torch.int32)
    return active, perm, offsets


def alora_qkv_forward(x, token_adapter_ids, activation_start, W_qkv, A: Sequence, B: Sequence,
                      q_out, k_cache, v_cache, slot_mapping, block_size: int, dims: AloraDims,
                      workspace, stream=None) -> None:
    """Enqueue the whole path on `stream` (default: torch's current stream).  Returns nothing;
    q_out and the mapped cache slots are written asynchronously."""
    s = lib().alora_qkv_forward(_ptr(x), _ptr(token_adapter_ids), _ptr(activation_start), _ptr(W_qkv),
                                _ptr_array(A), _ptr_array(B), _ptr(q_out), _ptr(k_cache), _ptr(v_cache),
                                _ptr(slot_mapping), block_size, ctypes.byref(dims), _ptr(workspace),
                                workspace.numel() if workspace is not None else 0, _stream_handle(stream))
    if s:
        raise AloraError(s, "alora_qkv_forward")


def alora_qkv_forward_ex(x, token_adapter_ids, activation_start, W_qkv, A: Sequence, B: Sequence,
                         q_out, k_cache, v_cache, slot_mapping, block_size: int, dims: AloraDims,
                         workspace, bias=None, adapter_ranks=None, stream=None, reuse_grouping: bool = False,
                         rope=None) -> None:
    """alora_qkv_forward with a layer bias [N] (device tensor) and/or one rank per adapter (host ints);
    reuse_grouping: use the classification/grouping an earlier call left in this workspace for the same
    token batch (the per-layer call of a model whose layers share one batch); rope: (cos, sin) fp32 device
    tensors [positions, head_dim / 2]: rotary embedding of q and k fused into the store."""
    ex = AloraExtras(_ptr(bias), None, 1 if reuse_grouping else 0, None, None, 0)
    if rope is not None:
        ex.rope_cos, ex.rope_sin, ex.rope_positions = _ptr(rope[0]), _ptr(rope[1]), int(rope[0].shape[0])
    keep = None
    if adapter_ranks is not None:
        keep = (ctypes.c_int32 * len(adapter_ranks))(*[int(r) for r in adapter_ranks])
        ex.adapter_ranks = ctypes.cast(keep, ctypes.c_void_p)
    s = lib().alora_qkv_forward_ex(_ptr(x), _ptr(token_adapter_ids), _ptr(activation_start), _ptr(W_qkv),
                                   _ptr_array(A), _ptr_array(B), _ptr(q_out), _ptr(k_cache), _ptr(v_cache),
                                   _ptr(slot_mapping), block_size, ctypes.byref(dims), ctypes.byref(ex),
                                   _ptr(workspace), workspace.numel() if workspace is not None else 0,
                                   _stream_handle(stream))
    if s:
        raise AloraError(s, "alora_qkv_forward_ex")


def alora_qkv_forward_static(x, token_adapter_ids, activation_start, W_qkv, A: Sequence, B: Sequence,
                             q_out, k_cache, v_cache, slot_mapping, block_size: int, dims: AloraDims,
                             bias=None, adapter_ranks=None, stream=None, rope=None) -> None:
    """alora_qkv_forward_ex on the library's static device scratch: no workspace argument, no allocation."""
    ex = AloraExtras(_ptr(bias), None, 0, None, None, 0)
    if rope is not None:
        ex.rope_cos, ex.rope_sin, ex.rope_positions = _ptr(rope[0]), _ptr(rope[1]), int(rope[0].shape[0])
    keep = None
    if adapter_ranks is not None:
        keep = (ctypes.c_int32 * len(adapter_ranks))(*[int(r) for r in adapter_ranks])
        ex.adapter_ranks = ctypes.cast(keep, ctypes.c_void_p)
    s = lib().alora_qkv_forward_static(_ptr(x), _ptr(token_adapter_ids), _ptr(activation_start), _ptr(W_qkv),
                                       _ptr_array(A), _ptr_array(B), _ptr(q_out), _ptr(k_cache), _ptr(v_cache),
                                       _ptr(slot_mapping), block_size, ctypes.byref(dims), ctypes.byref(ex),
                                       _stream_handle(stream))
    if s:
        raise AloraError(s, "alora_qkv_forward_static")


def alora_qkv_static_scratch_bytes() -> int:
    return int(lib().alora_qkv_static_scratch_bytes())


def alora_qkv_graph_create(x, token_adapter_ids, activation_start, W_qkv, A: Sequence, B: Sequence,
                           q_out, k_cache, v_cache, slot_mapping, block_size: int, dims: AloraDims, workspace,
                           bias=None, adapter_ranks=None, rope=None):
    """Record one forward call with these buffers into a HIP graph; returns an opaque handle for
    alora_qkv_graph_launch / alora_qkv_graph_destroy.  The caller keeps every tensor alive and rewrites
    their contents in place between launches."""
    h = ctypes.c_void_p(None)
    ex = AloraExtras(_ptr(bias), None, 0, None, None, 0)
    if rope is not None:
        ex.rope_cos, ex.rope_sin, ex.rope_positions = _ptr(rope[0]), _ptr(rope[1]), int(rope[0].shape[0])
    keep = None
    if adapter_ranks is not None:
        keep = (ctypes.c_int32 * len(adapter_ranks))(*[int(r) for r in adapter_ranks])
        ex.adapter_ranks = ctypes.cast(keep, ctypes.c_void_p)
    s = lib().alora_qkv_graph_create(_ptr(x), _ptr(token_adapter_ids), _ptr(activation_start), _ptr(W_qkv),
                                     _ptr_array(A), _ptr_array(B), _ptr(q_out), _ptr(k_cache), _ptr(v_cache),
                                     _ptr(slot_mapping), block_size, ctypes.byref(dims), ctypes.byref(ex),
                                     _ptr(workspace),
                                     workspace.numel() if workspace is not None else 0, ctypes.byref(h))
    if s:
        raise AloraError(s, "alora_qkv_graph_create")
    return h


def alora_qkv_graph_launch(graph, stream=None) -> None:
    s = lib().alora_qkv_graph_launch(graph, _stream_handle(stream))
    if s:
        raise AloraError(s, "alora_qkv_graph_launch")


def alora_qkv_graph_destroy(graph) -> None:
    s = lib().alora_qkv_graph_destroy(graph)
    if s:
        raise AloraError(s, "alora_qkv_graph_destroy")


def alora_qkv_validate(token_adapter_ids, activation_start, slot_mapping, block_size: int, dims: AloraDims) -> int:
    return int(lib().alora_qkv_validate(_ptr(token_adapter_ids), _ptr(activation_start), _ptr(slot_mapping),
                                        block_size, ctypes.byref(dims)))


def alora_qkv_profile_begin(max_calls: int, every: int = 1) -> None:
    """Measure the dominant kernel of every `every`-th forward call, at most max_calls of them."""
    s = lib().alora_qkv_profile_begin_every(max_calls, every)
    if s:
        raise AloraError(s, "alora_qkv_profile_begin")


def alora_qkv_profile_end():
    """(average milliseconds of the dominant kernel, number of measured calls)."""
    ms, n = ctypes.c_double(0.0), ctypes.c_int(0)
    s = lib().alora_qkv_profile_end(ctypes.byref(ms), ctypes.byref(n))
    if s:
        raise AloraError(s, "alora_qkv_profile_end")
    return float(ms.value), int(n.value)


def alora_qkv_set_tuning(feature_tiles: int = 0, splits: int = 0) -> None:
    """Override the automatic tiling of the bf16 path (0, 0 restores it); see alora_qkv.h."""
    s = lib().alora_qkv_set_tuning(feature_tiles, splits)
    if s:
        raise AloraError(s, "alora_qkv_set_tuning")


def make_attn_dims(q, k_cache, block_tables, n_q_heads: int, n_kv_heads: int, head_dim: int, block_size: int,
                   scale: float = 0.0) -> AloraAttnDims:
    """Dimensions of an alora_paged_attention call, read off the tensors."""
    return AloraAttnDims(_dtype_code(q), q.shape[0], n_q_heads, n_kv_heads, head_dim, block_tables.shape[0],
                         block_tables.shape[1], block_size, k_cache.shape[0], scale)


def alora_paged_attention(q, k_cache, v_cache, block_tables, token_seq_ids, token_positions, out,
                          dims: AloraAttnDims, stream=None) -> None:
    """Enqueue causal softmax attention of the rows of q over the paged cache (include/alora_attention.h)."""
    s = lib().alora_paged_attention(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables), _ptr(token_seq_ids),
                                    _ptr(token_positions), _ptr(out), ctypes.byref(dims), _stream_handle(stream))
    if s:
        raise AloraError(s, "alora_paged_attention")


def alora_paged_attention_validate(block_tables, token_seq_ids, token_positions, dims: AloraAttnDims) -> int:
    return int(lib().alora_paged_attention_validate(_ptr(block_tables), _ptr(token_seq_ids), _ptr(token_positions),
                                                    ctypes.byref(dims)))


def alora_paged_attention_workspace_bytes(dims: AloraAttnDims) -> int:
    out = ctypes.c_size_t(0)
    s = lib().alora_paged_attention_workspace_bytes(ctypes.byref(dims), ctypes.byref(out))
    if s:
        raise AloraError(s, "alora_paged_attention_workspace_bytes")
    return int(out.value)


def alora_paged_attention_split(q, k_cache, v_cache, block_tables, token_seq_ids, token_positions, out,
                                dims: AloraAttnDims, workspace, stream=None) -> None:
    """alora_paged_attention with every row's context cut into parts (small batches, long contexts)."""
    s = lib().alora_paged_attention_split(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables), _ptr(token_seq_ids),
                                          _ptr(token_positions), _ptr(out), ctypes.byref(dims), _ptr(workspace),
                                          workspace.numel() if workspace is not None else 0, _stream_handle(stream))
    if s:
        raise AloraError(s, "alora_paged_attention_split")


def alora_paged_attention_suffix(q, k_cache, v_cache, block_tables, token_seq_ids, token_positions, out,
                                 dims: AloraAttnDims, stream=None) -> None:
    """alora_paged_attention for the rows of a projected suffix: consecutive rows of a sequence share the loads
    of their context (bf16, head_dim 128)."""
    s = lib().alora_paged_attention_suffix(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables), _ptr(token_seq_ids),
                                           _ptr(token_positions), _ptr(out), ctypes.byref(dims), _stream_handle(stream))
    if s:
        raise AloraError(s, "alora_paged_attention_suffix")


def alora_paged_attention_suffix_workspace_bytes(dims: AloraAttnDims) -> int:
    out = ctypes.c_size_t(0)
    s = lib().alora_paged_attention_suffix_workspace_bytes(ctypes.byref(dims), ctypes.byref(out))
    if s:
        raise AloraError(s, "alora_paged_attention_suffix_workspace_bytes")
    return int(out.value)


def alora_paged_attention_suffix_split(q, k_cache, v_cache, block_tables, token_seq_ids, token_positions, out,
                                       dims: AloraAttnDims, workspace, stream=None) -> None:
    """alora_paged_attention_suffix with every row block's context cut into parts (few row blocks, long contexts)."""
    s = lib().alora_paged_attention_suffix_split(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
                                                 _ptr(token_seq_ids), _ptr(token_positions), _ptr(out), ctypes.byref(dims),
                                                 _ptr(workspace), workspace.numel() if workspace is not None else 0,
                                                 _stream_handle(stream))
    if s:
        raise AloraError(s, "alora_paged_attention_suffix_split")
