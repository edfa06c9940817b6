"""ctypes binding of libkvblade.so: the same names as the C ABI, argument marshalling only.

Every step of the path runs in the native library; there is no Python or CPU fallback.  If the
library has not been built (python -m paper_2604_26557_amd.build) loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
# KVBLADE_LIB names another build of the same library (e.g. one whose host code is instrumented by sanitizers)
LIB_PATH = os.environ.get("KVBLADE_LIB") or os.path.join(_PKG, "libkvblade.so")

KV_OK, KV_EINVAL, KV_EALIGN, KV_ERANGE, KV_ENOSPC, KV_EHIP = 0, -1, -2, -3, -4, -5
KV_F16, KV_BF16 = 0, 1
KV_TOKEN_MAJOR, KV_PER_SEQ = 0, 1
KV_PATH_DIRECT, KV_PATH_PAGECACHE = 0, 1
KV_K, KV_V, KV_KV = 0, 1, 2
KV_LAYOUT_BHSD, KV_LAYOUT_PAGED = 0, 1
KV_SEQ_ALL = -1
KV_UNBOUNDED = 2**64 - 1
KV_OUT_F32, KV_OUT_SAME = 0, 1
KV_DIR_OFFLOAD, KV_DIR_RELOAD, KV_DIR_RELOAD_ATTN = 0, 1, 2
KV_KERNEL_PACK, KV_KERNEL_UNPACK, KV_KERNEL_ATTN_PARTIAL, KV_KERNEL_ATTN_COMBINE = 0, 1, 2, 3
KV_PIPE_TIME_KERNELS = 1
KV_PIPE_SERIALIZE = 2
KV_PIPE_ATTN_FROM_EXTENT = 4
KV_PIPE_NO_PACING = 8
KV_ATTN_SCRATCH_BYTES = 8 << 20
KV_COPY_AUTO, KV_COPY_MEMCPY, KV_COPY_KERNEL = 0, 1, 2
KV_ORDER_CROSS, KV_ORDER_INTRA = 0, 1

EXPORTS = [
    "kv_layout_plan", "kv_plan_destroy", "kv_plan_info", "kv_plan_tensor", "kv_plan_seq_base",
    "kv_plan_translate", "kv_plan_chunk_cmds", "kv_plan_range_cmds", "kv_offload_pack", "kv_reload_unpack", "kv_decode_attn",
    "kv_decode_attn_workspace", "kv_pipeline_run", "kv_last_hip_error", "kv_strerror", "kv_abi_version",
    "kv_append_tokens", "kv_budget", "kv_plan_trim", "kv_adapt_init", "kv_adapt_order", "kv_adapt_update",
    "kv_abi_sizeof", "kv_budget_sample", "kv_decode_attn_static", "kv_offload_pack_layers", "kv_reload_unpack_layers",
    "kv_decode_attn_splits",
]


class kv_plan_desc_t(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_kv_heads", C.c_int32), ("n_q_heads", C.c_int32),
                ("head_dim", C.c_int32), ("batch", C.c_int32), ("dtype", C.c_int32),
                ("sector_bytes", C.c_int32), ("chunk_tokens", C.c_int32), ("extent_mode", C.c_int32),
                ("reserved", C.c_int32), ("seq_cap", C.POINTER(C.c_int32)),
                ("lba_start", C.c_uint64), ("region_blocks", C.c_uint64),
                ("pc_budget_bytes", C.c_uint64), ("pageable_bytes", C.c_uint64)]


class kv_plan_info_t(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_kv_heads", C.c_int32), ("n_q_heads", C.c_int32),
                ("head_dim", C.c_int32), ("batch", C.c_int32), ("dtype", C.c_int32),
                ("sector_bytes", C.c_int32), ("chunk_tokens", C.c_int32), ("extent_mode", C.c_int32),
                ("n_pagecache_layers", C.c_int32), ("row_bytes", C.c_uint64), ("tensor_blocks", C.c_uint64),
                ("tensor_payload_bytes", C.c_uint64), ("region_bytes_needed", C.c_uint64),
                ("pageable_bytes_needed", C.c_uint64)]


class kv_extent_t(C.Structure):
    _fields_ = [("path", C.c_int32), ("reserved", C.c_int32), ("lba_start", C.c_uint64),
                ("n_blocks", C.c_uint64), ("file_off", C.c_uint64), ("bytes", C.c_uint64)]


class kv_cmd_t(C.Structure):
    _fields_ = [("slba", C.c_uint64), ("buf_off", C.c_uint64), ("nlb", C.c_uint32), ("tok0", C.c_uint32),
                ("ntok", C.c_uint32), ("reserved", C.c_uint32)]


class kv_view_t(C.Structure):
    _fields_ = [("layout", C.c_int32), ("n_layers", C.c_int32),
                ("k_layers", C.POINTER(C.c_void_p)), ("v_layers", C.POINTER(C.c_void_p)),
                ("layer_bytes", C.c_uint64),
                ("stride_b", C.c_int64), ("stride_h", C.c_int64), ("stride_s", C.c_int64),
                ("s_alloc", C.c_int32), ("block_tokens", C.c_int32), ("n_pool_blocks", C.c_int32),
                ("max_blocks_per_seq", C.c_int32), ("block_table", C.c_void_p),
                ("seq_lens_host", C.POINTER(C.c_int32)), ("seq_lens_dev", C.c_void_p),
                ("seq_off_host", C.POINTER(C.c_int64)), ("seq_off_dev", C.c_void_p)]


class kv_attn_args_t(C.Structure):
    _fields_ = [("q_layers", C.POINTER(C.c_void_p)), ("out_layers", C.POINTER(C.c_void_p)),
                ("out_dtype", C.c_int32), ("n_splits", C.c_int32)]


class kv_chunk_trace_t(C.Structure):
    _fields_ = [("host_off", C.c_uint64), ("bytes", C.c_uint64), ("layer", C.c_uint16), ("kind", C.c_uint8),
                ("path", C.c_uint8), ("reserved", C.c_uint32), ("t_issue_s", C.c_double), ("t_done_s", C.c_double)]


class kv_pipe_opts_t(C.Structure):
    _fields_ = [("span_chunks", C.c_int32), ("host_workers", C.c_int32), ("flags", C.c_uint32),
                ("copy_streams", C.c_int32), ("d2h_mode", C.c_int32), ("h2d_mode", C.c_int32),
                ("order_pagecache", C.c_int32), ("order_direct", C.c_int32), ("max_cmd_bytes", C.c_uint64),
                ("caller_stream", C.c_void_p), ("trace", C.POINTER(kv_chunk_trace_t)), ("trace_cap", C.c_uint32),
                ("reserved", C.c_uint32)]


class kv_pipe_stats_t(C.Structure):
    _fields_ = [("wall_s", C.c_double), ("bytes_direct", C.c_uint64), ("bytes_pagecache", C.c_uint64),
                ("n_chunks", C.c_uint32), ("n_spans", C.c_uint32), ("max_in_flight", C.c_uint32),
                ("group_seconds", C.c_double * 2),
                ("kernel_launches", C.c_uint32 * 4), ("kernel_ms", C.c_float * 4),
                ("lba_seq_breaks", C.c_uint32), ("n_traced", C.c_uint32),
                ("host_copy_wait_s", C.c_double), ("harvest_wait_s", C.c_double), ("pace_GBps", C.c_double)]


class kv_adapt_t(C.Structure):
    _fields_ = [("iteration", C.c_int32), ("chosen", C.c_int32 * 2), ("gbps", (C.c_double * 2) * 2)]


class kv_append_stats_t(C.Structure):
    _fields_ = [("n_cmds", C.c_uint32), ("n_rmw_reads", C.c_uint32), ("blocks_written", C.c_uint64)]


_lib = None


def lib() -> C.CDLL:
    """Load the native library; raise if it is missing (there is no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_2604_26557_amd.build`")
        # PyTorch ships its own copy of the HIP runtime under the same soname.  Device memory and
        # streams come from PyTorch, so its copy must be the one in the process: import it first,
        # and this library's dependency then resolves to the runtime that is already loaded.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp, i = C.c_void_p, C.c_int
        L.kv_layout_plan.argtypes = [C.POINTER(kv_plan_desc_t), C.POINTER(vp)]
        L.kv_plan_destroy.argtypes = [vp]
        L.kv_plan_destroy.restype = None
        L.kv_plan_info.argtypes = [vp, C.POINTER(kv_plan_info_t)]
        L.kv_plan_tensor.argtypes = [vp, i, i, C.POINTER(kv_extent_t)]
        L.kv_plan_seq_base.argtypes = [vp, i, C.POINTER(C.c_uint64)]
        L.kv_plan_translate.argtypes = [vp, i, i, i, i, i, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
        L.kv_plan_chunk_cmds.argtypes = [vp, i, i, i, i, C.POINTER(kv_cmd_t), i, C.POINTER(i)]
        L.kv_plan_range_cmds.argtypes = [vp, i, i, i, i, i, C.c_uint64, C.POINTER(kv_cmd_t), i, C.POINTER(i)]
        L.kv_offload_pack.argtypes = [vp, i, i, C.POINTER(kv_view_t), i, i, i, vp, C.c_size_t, vp]
        L.kv_reload_unpack.argtypes = [vp, i, i, vp, C.c_size_t, C.POINTER(kv_view_t), i, i, i, vp]
        L.kv_offload_pack_layers.argtypes = [vp, i, i, C.POINTER(kv_view_t), vp, C.c_size_t, vp]
        L.kv_reload_unpack_layers.argtypes = [vp, i, i, vp, C.c_size_t, C.POINTER(kv_view_t), vp]
        L.kv_decode_attn.argtypes = [vp, C.POINTER(kv_view_t), i, vp, vp, i, i, vp, C.c_size_t, vp]
        L.kv_decode_attn_static.argtypes = [vp, C.POINTER(kv_view_t), i, vp, vp, i, i, vp]
        L.kv_decode_attn_splits.argtypes = [vp, C.POINTER(C.c_int32), i, C.POINTER(i), C.POINTER(i), C.POINTER(i)]
        L.kv_decode_attn_workspace.argtypes = [vp, i, i]
        L.kv_decode_attn_workspace.restype = C.c_size_t
        L.kv_pipeline_run.argtypes = [vp, i, i, i, C.POINTER(kv_view_t), vp, C.c_size_t, vp, C.c_size_t, i, i,
                                      C.POINTER(kv_attn_args_t), C.POINTER(kv_pipe_opts_t),
                                      C.POINTER(kv_pipe_stats_t)]
        L.kv_append_tokens.argtypes = [vp, i, i, C.POINTER(kv_view_t), vp, C.c_size_t, vp, C.c_size_t, vp,
                                       C.POINTER(kv_append_stats_t)]
        L.kv_budget.argtypes = [C.c_int64, C.c_int64, C.c_int64, C.c_int32, C.c_int64, C.POINTER(C.c_int64),
                                C.POINTER(C.c_int64)]
        L.kv_budget_sample.argtypes = [C.c_char_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        L.kv_plan_trim.argtypes = [vp, i, i, vp, C.c_size_t, vp, C.c_size_t, C.POINTER(C.c_uint64),
                                   C.POINTER(C.c_uint64)]
        L.kv_adapt_init.argtypes = [C.POINTER(kv_adapt_t)]
        L.kv_adapt_order.argtypes = [C.POINTER(kv_adapt_t), i]
        L.kv_adapt_update.argtypes = [C.POINTER(kv_adapt_t), C.POINTER(kv_pipe_stats_t)]
        L.kv_strerror.restype = C.c_char_p
        L.kv_strerror.argtypes = [i]
        L.kv_abi_sizeof.argtypes = [i]
        L.kv_abi_sizeof.restype = C.c_size_t
        for name in EXPORTS:
            getattr(L, name)
        # the ctypes mirrors must have the library's own struct sizes
        for which, t in enumerate((kv_plan_desc_t, kv_plan_info_t, kv_extent_t, kv_cmd_t, kv_view_t, kv_attn_args_t,
                                   kv_pipe_opts_t, kv_pipe_stats_t, kv_append_stats_t, kv_adapt_t,
                                   kv_chunk_trace_t)):
            if L.kv_abi_sizeof(which) != C.sizeof(t):
                raise RuntimeError(f"{t.__name__}: binding has {C.sizeof(t)} bytes, library {L.kv_abi_sizeof(which)}")
        _lib = L
    return _lib


class KVError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().kv_strerror(code).decode()
        if code == KV_EHIP:
            msg += f" (hipError {lib().kv_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{code}]")


def _check(code: int, where: str) -> None:
    if code != KV_OK:
        raise KVError(code, where)


# ------------------------------------------------------------------------------------------ plan
class Plan:
    """Owner of a kv_plan_t*."""

    def __init__(self, handle: int):
        self.handle = C.c_void_p(handle)
        self.info = kv_plan_info(self)

    def close(self):
        if self.handle:
            lib().kv_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def kv_layout_plan(n_layers: int, n_kv_heads: int, n_q_heads: int, head_dim: int, seq_cap: Sequence[int],
                   dtype: int, sector_bytes: int, chunk_tokens: int, extent_mode: int = KV_TOKEN_MAJOR,
                   lba_start: int = 0, region_blocks: int = KV_UNBOUNDED, pc_budget_bytes: int = 0,
                   pageable_bytes: int = KV_UNBOUNDED) -> Plan:
    cap = (C.c_int32 * len(seq_cap))(*[int(c) for c in seq_cap])
    d = kv_plan_desc_t(n_layers, n_kv_heads, n_q_heads, head_dim, len(seq_cap), dtype, sector_bytes,
                       chunk_tokens, extent_mode, 0, cap, lba_start, region_blocks, pc_budget_bytes,
                       pageable_bytes)
    h = C.c_void_p()
    _check(lib().kv_layout_plan(C.byref(d), C.byref(h)), "kv_layout_plan")
    return Plan(h.value)


def kv_plan_info(plan: Plan) -> kv_plan_info_t:
    o = kv_plan_info_t()
    _check(lib().kv_plan_info(plan.handle, C.byref(o)), "kv_plan_info")
    return o


def kv_plan_tensor(plan: Plan, layer: int, kind: int) -> kv_extent_t:
    o = kv_extent_t()
    _check(lib().kv_plan_tensor(plan.handle, layer, kind, C.byref(o)), "kv_plan_tensor")
    return o


def kv_plan_seq_base(plan: Plan, seq: int) -> int:
    o = C.c_uint64()
    _check(lib().kv_plan_seq_base(plan.handle, seq, C.byref(o)), "kv_plan_seq_base")
    return int(o.value)


def kv_plan_translate(plan: Plan, layer: int, kind: int, seq: int, tok0: int, ntok: int):
    s, r = C.c_uint64(), C.c_uint64()
    _check(lib().kv_plan_translate(plan.handle, layer, kind, seq, tok0, ntok, C.byref(s), C.byref(r)),
           "kv_plan_translate")
    return int(s.value), int(r.value)


def kv_plan_chunk_cmds(plan: Plan, layer: int, kind: int, seq: int, chunk_tokens: int = 0) -> List[kv_cmd_t]:
    n = C.c_int()
    _check(lib().kv_plan_chunk_cmds(plan.handle, layer, kind, seq, chunk_tokens, None, 0, C.byref(n)),
           "kv_plan_chunk_cmds")
    arr = (kv_cmd_t * max(1, n.value))()
    _check(lib().kv_plan_chunk_cmds(plan.handle, layer, kind, seq, chunk_tokens, arr, n.value, C.byref(n)),
           "kv_plan_chunk_cmds")
    return list(arr[:n.value])


def kv_plan_range_cmds(plan: Plan, layer: int, kind: int, seq: int, tok0: int, ntok: int,
                       mdts_bytes: int = 0) -> List[kv_cmd_t]:
    n = C.c_int()
    _check(lib().kv_plan_range_cmds(plan.handle, layer, kind, seq, tok0, ntok, mdts_bytes, None, 0, C.byref(n)),
           "kv_plan_range_cmds")
    arr = (kv_cmd_t * max(1, n.value))()
    _check(lib().kv_plan_range_cmds(plan.handle, layer, kind, seq, tok0, ntok, mdts_bytes, arr, n.value,
                                    C.byref(n)), "kv_plan_range_cmds")
    return list(arr[:n.value])


# ------------------------------------------------------------------------------------------ views
class View:
    """kv_view_t plus the Python objects that keep its host arrays and device tensors alive."""

    def __init__(self, struct: kv_view_t, keep):
        self.struct = struct
        self._keep = keep

    def ref(self):
        return C.byref(self.struct)


def _ptr_array(tensors) -> C.Array:
    return (C.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])


def bhsd_view(k_layers, v_layers, seq_lens: Sequence[int], seq_lens_dev=None) -> View:
    """View over per-layer torch tensors [B, H, S_alloc, D] (device, last dim contiguous)."""
    t0 = k_layers[0]
    assert t0.dim() == 4 and t0.stride(3) == 1
    for t in list(k_layers) + list(v_layers):
        assert t.shape == t0.shape and t.stride() == t0.stride() and t.dtype == t0.dtype
    kp, vp = _ptr_array(k_layers), _ptr_array(v_layers)
    lens = (C.c_int32 * len(seq_lens))(*[int(x) for x in seq_lens])
    span = sum((t0.shape[i] - 1) * t0.stride(i) for i in range(4)) + 1
    s = kv_view_t()
    s.layout, s.n_layers = KV_LAYOUT_BHSD, len(k_layers)
    s.k_layers, s.v_layers = kp, vp
    s.layer_bytes = span * t0.element_size()
    s.stride_b, s.stride_h, s.stride_s = t0.stride(0), t0.stride(1), t0.stride(2)
    s.s_alloc = t0.shape[2]
    s.seq_lens_host = lens
    s.seq_lens_dev = seq_lens_dev.data_ptr() if seq_lens_dev is not None else None
    return View(s, (k_layers, v_layers, kp, vp, lens, seq_lens_dev))


def paged_view(k_pools, v_pools, block_table_dev, seq_lens: Sequence[int], seq_lens_dev=None) -> View:
    """View over per-layer block pools [n_pool, H, block_tokens, D] (device, contiguous) and a
    device block table [B, max_blocks] int32."""
    t0 = k_pools[0]
    assert t0.dim() == 4 and t0.is_contiguous() and block_table_dev.is_contiguous()
    for t in list(k_pools) + list(v_pools):
        assert t.shape == t0.shape and t.is_contiguous() and t.dtype == t0.dtype
    kp, vp = _ptr_array(k_pools), _ptr_array(v_pools)
    lens = (C.c_int32 * len(seq_lens))(*[int(x) for x in seq_lens])
    s = kv_view_t()
    s.layout, s.n_layers = KV_LAYOUT_PAGED, len(k_pools)
    s.k_layers, s.v_layers = kp, vp
    s.layer_bytes = t0.numel() * t0.element_size()
    s.block_tokens = t0.shape[2]
    s.n_pool_blocks = t0.shape[0]
    s.max_blocks_per_seq = block_table_dev.shape[1]
    s.block_table = block_table_dev.data_ptr()
    s.seq_lens_host = lens
    s.seq_lens_dev = seq_lens_dev.data_ptr() if seq_lens_dev is not None else None
    return View(s, (k_pools, v_pools, kp, vp, lens, block_table_dev, seq_lens_dev))


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        return None
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _caller_stream(stream) -> Optional[int]:
    """The stream handed to the blocking calls: the given one, else PyTorch's current stream."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return _stream_ptr(stream)


# ------------------------------------------------------------------------------------------ kernels
def kv_offload_pack(plan: Plan, layer: int, kind: int, src: View, seq: int, tok0: int, ntok: int, dst,
                    stream=None) -> None:
    """dst: torch uint8 device tensor receiving the bytes."""
    _check(lib().kv_offload_pack(plan.handle, layer, kind, src.ref(), seq, tok0, ntok, dst.data_ptr(),
                                 dst.numel() * dst.element_size(), _caller_stream(stream)), "kv_offload_pack")


def kv_reload_unpack(plan: Plan, layer: int, kind: int, src, dst: View, seq: int, tok0: int, ntok: int,
                     stream=None) -> None:
    _check(lib().kv_reload_unpack(plan.handle, layer, kind, src.data_ptr(), src.numel() * src.element_size(),
                                  dst.ref(), seq, tok0, ntok, _caller_stream(stream)), "kv_reload_unpack")


def kv_offload_pack_layers(plan: Plan, layer_begin: int, layer_end: int, src: View, dst, stream=None) -> None:
    _check(lib().kv_offload_pack_layers(plan.handle, layer_begin, layer_end, src.ref(), dst.data_ptr(),
                                        dst.numel() * dst.element_size(), _caller_stream(stream)),
           "kv_offload_pack_layers")


def kv_reload_unpack_layers(plan: Plan, layer_begin: int, layer_end: int, src, dst: View, stream=None) -> None:
    _check(lib().kv_reload_unpack_layers(plan.handle, layer_begin, layer_end, src.data_ptr(),
                                         src.numel() * src.element_size(), dst.ref(), _caller_stream(stream)),
           "kv_reload_unpack_layers")


def kv_decode_attn_splits(plan: Plan, seq_lens: Sequence[int], n_splits: int = 0):
    """(split count of the partial layout, first[B+1], tokens[B]) as kv_decode_attn would split these lengths."""
    B = len(seq_lens)
    lens = (C.c_int32 * B)(*[int(x) for x in seq_lens])
    ns = C.c_int()
    first = (C.c_int * (B + 1))()
    tokens = (C.c_int * B)()
    _check(lib().kv_decode_attn_splits(plan.handle, lens, n_splits, C.byref(ns), first, tokens), "kv_decode_attn_splits")
    return int(ns.value), list(first), list(tokens)


def kv_decode_attn_workspace(plan: Plan, n_splits: int, max_len: int) -> int:
    return int(lib().kv_decode_attn_workspace(plan.handle, n_splits, max_len))


def kv_decode_attn(plan: Plan, kv: View, layer: int, q, out, out_dtype: int, n_splits: int, workspace,
                   stream=None) -> None:
    _check(lib().kv_decode_attn(plan.handle, kv.ref(), layer, q.data_ptr(), out.data_ptr(), out_dtype, n_splits,
                                workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                _caller_stream(stream)), "kv_decode_attn")


def kv_decode_attn_static(plan: Plan, kv: View, layer: int, q, out, out_dtype: int, n_splits: int = 0,
                          stream=None) -> None:
    """kv_decode_attn without a workspace argument: the library's own static device array holds the partials."""
    _check(lib().kv_decode_attn_static(plan.handle, kv.ref(), layer, q.data_ptr(), out.data_ptr(), out_dtype,
                                       n_splits, _caller_stream(stream)), "kv_decode_attn_static")


# ------------------------------------------------------------------------------------------ pipeline
def kv_pipeline_run(plan: Plan, direction: int, layer_begin: int, layer_end: int, view: View,
                    lba_region=None, pageable=None, chunk_tokens: int = 0, depth: int = 2,
                    q_layers=None, out_layers=None, out_dtype: int = KV_OUT_F32, n_splits: int = 0,
                    span_chunks: int = 0, host_workers: int = 0, time_kernels: bool = False,
                    copy_streams: int = 0, d2h_mode: int = KV_COPY_AUTO, h2d_mode: int = KV_COPY_AUTO,
                    serialize: bool = False, attn_from_extent: bool = False,
                    order_pagecache: int = KV_ORDER_CROSS, order_direct: int = KV_ORDER_CROSS,
                    max_cmd_bytes: int = 0, stream=None, trace_cap: int = 0, pacing: bool = True) -> kv_pipe_stats_t:
    """lba_region: pinned torch uint8 CPU tensor; pageable: ordinary torch uint8 CPU tensor or NumPy array.
    stream: the stream the view's buffers were produced on (default: PyTorch's current stream); the call's
    kernels are queued on it.  trace_cap > 0: the returned stats carry `.trace`, the list of the first
    trace_cap chunk commands as kv_chunk_trace_t."""
    def host(buf):
        if buf is None:
            return None, 0
        if isinstance(buf, np.ndarray):
            return buf.ctypes.data, buf.nbytes
        return buf.data_ptr(), buf.numel() * buf.element_size()

    rp, rb = host(lba_region)
    pp, pb = host(pageable)
    attn = None
    keep = None
    if q_layers is not None:
        qa, oa = _ptr_array(q_layers), _ptr_array(out_layers)
        attn = kv_attn_args_t(qa, oa, out_dtype, n_splits)
        keep = (qa, oa)
    opts = kv_pipe_opts_t(span_chunks, host_workers, (KV_PIPE_TIME_KERNELS if time_kernels else 0) | (KV_PIPE_SERIALIZE if serialize else 0)
                          | (KV_PIPE_ATTN_FROM_EXTENT if attn_from_extent else 0) | (0 if pacing else KV_PIPE_NO_PACING), copy_streams,
                          d2h_mode, h2d_mode, order_pagecache, order_direct, max_cmd_bytes, _caller_stream(stream))
    trace = (kv_chunk_trace_t * trace_cap)() if trace_cap > 0 else None
    if trace is not None:
        opts.trace = C.cast(trace, C.POINTER(kv_chunk_trace_t))
        opts.trace_cap = trace_cap
    st = kv_pipe_stats_t()
    rc = lib().kv_pipeline_run(plan.handle, direction, layer_begin, layer_end, view.ref(), rp, rb, pp, pb,
                               chunk_tokens, depth, C.byref(attn) if attn is not None else None, C.byref(opts),
                               C.byref(st))
    del keep
    _check(rc, "kv_pipeline_run")
    if trace is not None:
        st.trace = [trace[i] for i in range(st.n_traced)]
        st._trace_buf = trace
    return st


def _host_buf(buf):
    if buf is None:
        return None, 0
    if isinstance(buf, np.ndarray):
        return buf.ctypes.data, buf.nbytes
    return buf.data_ptr(), buf.numel() * buf.element_size()


def kv_append_tokens(plan: Plan, layer_begin: int, layer_end: int, view: View, lba_region=None,
                     pageable=None, stream=None) -> kv_append_stats_t:
    rp, rb = _host_buf(lba_region)
    pp, pb = _host_buf(pageable)
    st = kv_append_stats_t()
    _check(lib().kv_append_tokens(plan.handle, layer_begin, layer_end, view.ref(), rp, rb, pp, pb,
                                  _caller_stream(stream), C.byref(st)), "kv_append_tokens")
    return st


def kv_budget_sample(root: str = ""):
    """(M_avail, M_max, M_anon+shmem) in bytes, sampled now (Eq. 1's inputs)."""
    a, b, c = C.c_int64(), C.c_int64(), C.c_int64()
    _check(lib().kv_budget_sample(root.encode(), C.byref(a), C.byref(b), C.byref(c)), "kv_budget_sample")
    return int(a.value), int(b.value), int(c.value)


def kv_budget(m_avail: int, m_max: int, m_anon_shmem: int, n_threads: int, m_pin: int):
    a, b = C.c_int64(), C.c_int64()
    _check(lib().kv_budget(m_avail, m_max, m_anon_shmem, n_threads, m_pin, C.byref(a), C.byref(b)), "kv_budget")
    return int(a.value), int(b.value)


def kv_plan_trim(plan: Plan, layer_begin: int, layer_end: int, lba_region=None, pageable=None):
    rp, rb = _host_buf(lba_region)
    pp, pb = _host_buf(pageable)
    n, k = C.c_uint64(), C.c_uint64()
    _check(lib().kv_plan_trim(plan.handle, layer_begin, layer_end, rp, rb, pp, pb, C.byref(n), C.byref(k)),
           "kv_plan_trim")
    return int(n.value), int(k.value)


def kv_adapt_init() -> kv_adapt_t:
    a = kv_adapt_t()
    _check(lib().kv_adapt_init(C.byref(a)), "kv_adapt_init")
    return a


def kv_adapt_order(a: kv_adapt_t, group: int) -> int:
    r = lib().kv_adapt_order(C.byref(a), group)
    if r < 0:
        raise KVError(r, "kv_adapt_order")
    return r


def kv_adapt_update(a: kv_adapt_t, stats: kv_pipe_stats_t) -> None:
    _check(lib().kv_adapt_update(C.byref(a), C.byref(stats)), "kv_adapt_update")
