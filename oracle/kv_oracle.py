"""ctypes front end of kv_oracle.c -- TEST INFRASTRUCTURE, not product code.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this.
It marshals NumPy arrays to the plain C definitions and composes them into a whole
layout plan (Alg. 1 then Eq. 3-6).  Arithmetic of its own, each pinned in
tests/test_oracle_plan.py: byte counts from shapes (`Plan.row_bytes`, `region_bytes`,
`pageable_bytes`), the byte offset of an extent in its host buffer (`ext_byte_off`), and the
first sector handed to Alg. 2 by `token_range` (start LBA on the direct path; arena byte
offset / sector size on the page-cache path; plus the sequence's base in per-sequence mode).

`omp=True` on pack / unpack / attention runs the all-core build of the same C file (the
benchmark's second CPU-baseline figure); everything else, and every test of the GPU path,
uses the defining one-thread build.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kv_oracle.c")
_LIB = os.path.join(_HERE, "libkv_oracle.so")

OK, EINVAL, EALIGN, ERANGE = 0, -1, -2, -3


_LIB_OMP = os.path.join(_HERE, "libkv_oracle_omp.so")


def build(force: bool = False, omp: bool = False) -> str:
    """Compile kv_oracle.c with gcc: plain -O2, one thread (the defining build), or the same with -fopenmp."""
    out = _LIB_OMP if omp else _LIB
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra"]
                              + (["-fopenmp"] if omp else []) + ["-o", out, _SRC, "-lm"])
    return out


class _Src(C.Structure):
    _fields_ = [("paged", C.c_int32),
                ("stride_b", C.c_int64), ("stride_h", C.c_int64), ("stride_s", C.c_int64),
                ("block_table", C.c_void_p), ("max_blocks", C.c_int64),
                ("block_tokens", C.c_int64), ("H", C.c_int64), ("D", C.c_int64)]


_libs = {}


def lib(omp: bool = False):
    if omp not in _libs:
        # KV_ORACLE_LIB names another build of kv_oracle.c (e.g. one instrumented by sanitizers) for the one-thread role
        other = None if omp else os.environ.get("KV_ORACLE_LIB")
        _libs[omp] = _load(other or build(omp=omp))
    return _libs[omp]


def threads(omp: bool = False) -> int:
    """Threads the loops of that build are shared among (1 for the defining build)."""
    return int(lib(omp).orc_threads())


def _load(path):
    _lib = C.CDLL(path)
    _lib.orc_threads.restype = C.c_int
    _lib.orc_threads.argtypes = []
    _lib.orc_residency.restype = C.c_int64
    _lib.orc_residency.argtypes = [C.c_uint64, C.c_uint64, C.c_int64, C.c_void_p]
    _lib.orc_tensor_blocks.restype = C.c_int
    _lib.orc_tensor_blocks.argtypes = [C.c_int, C.c_int64, C.c_void_p, C.c_int64, C.c_int64, C.c_int64,
                                       C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p]
    _lib.orc_bind.restype = None
    _lib.orc_bind.argtypes = [C.c_int64, C.c_void_p, C.c_uint64, C.c_uint64, C.c_uint64,
                              C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    _lib.orc_translate.restype = C.c_int
    _lib.orc_translate.argtypes = [C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_uint64,
                                   C.c_void_p, C.c_void_p]
    _lib.orc_chunk_size.restype = C.c_uint64
    _lib.orc_chunk_size.argtypes = [C.c_uint64, C.c_uint64]
    _lib.orc_chunk_cmds.restype = C.c_int64
    _lib.orc_chunk_cmds.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint64, C.c_int64,
                                    C.c_void_p, C.c_void_p, C.c_void_p]
    _lib.orc_pack.restype = None
    _lib.orc_pack.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_void_p, C.c_void_p,
                              C.c_uint64, C.c_uint64, C.c_void_p]
    _lib.orc_unpack.restype = None
    _lib.orc_unpack.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_void_p, C.c_void_p,
                                C.c_uint64, C.c_void_p]
    _lib.orc_attention.restype = C.c_int
    _lib.orc_attention.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int64,
                                   C.c_int64, C.c_void_p, C.c_void_p]
    _lib.orc_budget.restype = None
    _lib.orc_budget.argtypes = [C.c_int64] * 5 + [C.c_void_p, C.c_void_p]
    _lib.orc_trim.restype = None
    _lib.orc_trim.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_uint64]
    _lib.orc_adapt_order.restype = C.c_int
    _lib.orc_adapt_order.argtypes = [C.c_int64, C.c_double, C.c_double]
    _lib.orc_f16_to_double.restype = C.c_double
    _lib.orc_f16_to_double.argtypes = [C.c_uint16]
    _lib.orc_bf16_to_double.restype = C.c_double
    _lib.orc_bf16_to_double.argtypes = [C.c_uint16]
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


# ---------------------------------------------------------------- plan pieces
def budget(M_avail: int, M_max: int, M_anon_shmem: int, N_threads: int, M_pin: int):
    """Eq. 1-2.  Returns (M_star, B_pc)."""
    a, b = C.c_int64(), C.c_int64()
    lib().orc_budget(M_avail, M_max, M_anon_shmem, N_threads, M_pin, C.byref(a), C.byref(b))
    return int(a.value), int(b.value)


def trim(buf: np.ndarray, off: int, n_blocks: int, lba_size: int) -> None:
    assert buf.dtype == np.uint8 and off + n_blocks * lba_size <= buf.size
    lib().orc_trim(_p(buf), off, n_blocks, lba_size)


def adapt_order(iteration: int, thr_intra: float, thr_cross: float) -> int:
    """Sec. IV-C: strategy (1 = overlap-intra, 0 = overlap-cross) of the 1-based decode iteration about to run."""
    return int(lib().orc_adapt_order(iteration, thr_intra, thr_cross))


def residency(X: int, S_kpu: int, L: int):
    x = np.zeros(L, dtype=np.int32)
    n1 = lib().orc_residency(X, S_kpu, L, _p(x))
    return int(n1), x


def tensor_blocks(per_seq: bool, cap: Sequence[int], H: int, D: int, e: int, lba_size: int):
    cap = np.asarray(cap, dtype=np.int32)
    nb, pay = C.c_uint64(), C.c_uint64()
    base = np.zeros(len(cap), dtype=np.uint64)
    rc = lib().orc_tensor_blocks(int(per_seq), len(cap), _p(cap), H, D, e, lba_size,
                                 C.byref(nb), _p(base), C.byref(pay))
    if rc:
        raise ValueError(rc)
    return int(nb.value), base, int(pay.value)


def bind(L: int, x: np.ndarray, n_blocks_per_tensor: int, lba_size: int, lba_start_first: int):
    path = np.zeros(2 * L, dtype=np.int32)
    lba = np.zeros(2 * L, dtype=np.uint64)
    nb = np.zeros(2 * L, dtype=np.uint64)
    off = np.zeros(2 * L, dtype=np.uint64)
    x = np.ascontiguousarray(x, dtype=np.int32)
    lib().orc_bind(L, _p(x), n_blocks_per_tensor, lba_size, lba_start_first, _p(path), _p(lba), _p(nb), _p(off))
    return path, lba, nb, off


def translate(lba_start: int, shape_src, shape_tgt, idx, e: int, lba_size: int):
    """Alg. 2.  Returns (rc, slba_star, req_bytes)."""
    f = np.asarray(shape_src, dtype=np.int64)
    d = np.asarray(shape_tgt, dtype=np.int64)
    i = np.asarray(idx, dtype=np.int64)
    s, r = C.c_uint64(), C.c_uint64()
    rc = lib().orc_translate(lba_start, _p(f), _p(d), _p(i), e, lba_size, C.byref(s), C.byref(r))
    return rc, int(s.value), int(r.value)


def chunk_size(mdts_bytes: int, lba_size: int) -> int:
    """Eq. 7: align_down(MDTS, lba_size)."""
    return int(lib().orc_chunk_size(mdts_bytes, lba_size))


def chunk_cmds(slba_star: int, req_bytes: int, chunk_bytes: int, lba_size: int):
    """Eq. 7-11.  Returns a list of (slba, nlb, dbuf_off)."""
    n = lib().orc_chunk_cmds(slba_star, req_bytes, chunk_bytes, lba_size, 0, None, None, None)
    if n < 0:
        raise ValueError(n)
    slba = np.zeros(n, dtype=np.uint64)
    nlb = np.zeros(n, dtype=np.uint32)
    off = np.zeros(n, dtype=np.uint64)
    lib().orc_chunk_cmds(slba_star, req_bytes, chunk_bytes, lba_size, n, _p(slba), _p(nlb), _p(off))
    return [(int(a), int(b), int(c)) for a, b, c in zip(slba, nlb, off)]


# ---------------------------------------------------------------- layouts
@dataclass
class Source:
    """Attention-side layout description (strided [B,H,S,D] or paged block pool)."""
    H: int
    D: int
    paged: bool = False
    stride_b: int = 0
    stride_h: int = 0
    stride_s: int = 0
    block_table: Optional[np.ndarray] = None   # int32 [B, max_blocks]
    block_tokens: int = 16

    def c(self) -> _Src:
        s = _Src()
        s.paged = int(self.paged)
        s.stride_b, s.stride_h, s.stride_s = self.stride_b, self.stride_h, self.stride_s
        if self.paged:
            self._bt = np.ascontiguousarray(self.block_table, dtype=np.int32)
            s.block_table = self._bt.ctypes.data
            s.max_blocks = self._bt.shape[1]
        else:
            s.block_table = None
            s.max_blocks = 0
        s.block_tokens = self.block_tokens
        s.H, s.D = self.H, self.D
        return s


def bhsd_source(shape, H=None, D=None) -> Source:
    """Contiguous [B,H,S,D]."""
    B, Hh, S, Dd = shape
    return Source(H=Hh, D=Dd, stride_b=Hh * S * Dd, stride_h=S * Dd, stride_s=Dd)


def u16(t) -> np.ndarray:
    """Raw 16-bit view of a torch fp16/bf16 CPU tensor or a NumPy array (no copy)."""
    if isinstance(t, np.ndarray):
        return t.view(np.uint16)
    import torch
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def pack(src: Source, data: np.ndarray, per_seq: bool, lens: Sequence[int], seq_base: np.ndarray,
         n_blocks: int, lba_size: int, ext: np.ndarray, omp: bool = False) -> None:
    """Write one tensor's whole extent (payload + zero pad) into ext (uint8, n_blocks*lba_size)."""
    assert ext.dtype == np.uint8 and ext.flags.c_contiguous and ext.size >= n_blocks * lba_size
    lens = np.asarray(lens, dtype=np.int32)
    seq_base = np.ascontiguousarray(seq_base, dtype=np.uint64)
    s = src.c()
    lib(omp).orc_pack(C.byref(s), _p(data), int(per_seq), len(lens), _p(lens), _p(seq_base), n_blocks, lba_size, _p(ext))


def unpack(src: Source, data: np.ndarray, per_seq: bool, lens: Sequence[int], seq_base: np.ndarray,
           lba_size: int, ext: np.ndarray, omp: bool = False) -> None:
    assert ext.dtype == np.uint8 and ext.flags.c_contiguous and data.flags.writeable
    lens = np.asarray(lens, dtype=np.int32)
    seq_base = np.ascontiguousarray(seq_base, dtype=np.uint64)
    s = src.c()
    lib(omp).orc_unpack(C.byref(s), _p(data), int(per_seq), len(lens), _p(lens), _p(seq_base), lba_size, _p(ext))


def attention(src: Source, K: np.ndarray, V: np.ndarray, q: np.ndarray, is_bf16: bool,
              lens: Sequence[int], Hq: int, omp: bool = False) -> np.ndarray:
    """One decode-attention step in double.  q is uint16 [B,Hq,D]; returns float64 [B,Hq,D]."""
    lens = np.asarray(lens, dtype=np.int32)
    B = len(lens)
    out = np.zeros((B, Hq, src.D), dtype=np.float64)
    s = src.c()
    q = np.ascontiguousarray(q)
    rc = lib(omp).orc_attention(C.byref(s), _p(K), _p(V), _p(q), int(is_bf16), B, Hq, _p(lens), _p(out))
    if rc:
        raise ValueError(rc)
    return out


def decode16(bits: np.ndarray, is_bf16: bool) -> np.ndarray:
    f = lib().orc_bf16_to_double if is_bf16 else lib().orc_f16_to_double
    return np.array([f(int(b)) for b in bits.ravel()], dtype=np.float64).reshape(bits.shape)


# ---------------------------------------------------------------- whole plan
@dataclass
class Plan:
    L: int
    H: int
    Hq: int
    D: int
    B: int
    e: int
    lba_size: int
    per_seq: bool
    cap: List[int]
    n1: int
    x: np.ndarray
    n_blocks_tensor: int
    payload_bytes: int
    seq_base: np.ndarray
    path: np.ndarray
    lba_start: np.ndarray
    n_blocks: np.ndarray
    file_off: np.ndarray
    lba_start_first: int

    @property
    def row_bytes(self) -> int:
        """Bytes of one token row of an extent: (B*H*D*e) token-major, (H*D*e) per sequence."""
        return (self.H if self.per_seq else self.B * self.H) * self.D * self.e

    @property
    def direct_blocks(self) -> int:
        return int(sum(int(n) for n, p in zip(self.n_blocks, self.path) if p == 0))

    @property
    def region_bytes(self) -> int:
        """Bytes an LBA-addressed region based at LBA 0 must span."""
        return (self.lba_start_first + self.direct_blocks) * self.lba_size

    @property
    def pageable_bytes(self) -> int:
        return int(sum(int(n) for n, p in zip(self.n_blocks, self.path) if p == 1)) * self.lba_size

    def ext_byte_off(self, n: int) -> int:
        """Byte offset of tensor n's extent in its host buffer (region or arena)."""
        if self.path[n] == 0:
            return int(self.lba_start[n]) * self.lba_size
        return int(self.file_off[n])


def layout_plan(L: int, H: int, Hq: int, D: int, cap: Sequence[int], e: int, lba_size: int,
                per_seq: bool, X: int, lba_start_first: int) -> Plan:
    """Alg. 1 then Eq. 3-6 over all 2L tensors.  S_kpu is the occupied (padded) extent size."""
    cap = [int(c) for c in cap]
    nb, base, pay = tensor_blocks(per_seq, cap, H, D, e, lba_size)
    n1, x = residency(X, nb * lba_size, L)
    path, lba, nbs, off = bind(L, x, nb, lba_size, lba_start_first)
    return Plan(L, H, Hq, D, len(cap), e, lba_size, per_seq, cap, n1, x, nb, pay, base,
                path, lba, nbs, off, lba_start_first)


def token_range(plan: Plan, n: int, b: int, tok0: int, ntok: int):
    """Alg. 2 for a run of whole token rows of tensor n (sequence b in per-sequence mode)."""
    if plan.per_seq:
        d = (plan.cap[b], plan.H, plan.D)
        f = (ntok, plan.H, plan.D)
        start = int(plan.seq_base[b])
    else:
        d = (plan.cap[0], plan.B * plan.H, plan.D)
        f = (ntok, plan.B * plan.H, plan.D)
        start = 0
    first = (int(plan.lba_start[n]) if plan.path[n] == 0 else int(plan.file_off[n]) // plan.lba_size) + start
    return translate(first, f, d, (tok0, 0, 0), plan.e, plan.lba_size)
