"""ctypes binding of libpowattn.so: same names as the C ABI in include/powattn.h.

Only argument marshalling lives here (tensor -> pointer, current stream,
status -> exception, output allocation through torch).  Every step of the
attention path runs in the library's HIP kernels; if the library has not been
built this module raises instead of computing anything itself.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("POWATTN_LIB") or os.path.join(_HERE, "libpowattn.so")

OK, INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, HIP_ERROR = 0, 1, 2, 3, 4
POWER, DENSE = 1, 2
BF16, F32 = 0, 1

EXPORTS = (
    "powattn_version", "powattn_strerror", "powattn_num_blocks", "powattn_max_k",
    "powattn_row_host", "powattn_mask_build", "powattn_prefill",
    "powattn_prefill_chunk", "powattn_prefill_chunk_paged", "powattn_prefill_batch_paged", "powattn_prefill_varlen", "powattn_decode_workspace_bytes", "powattn_decode",
    "powattn_decode_static", "powattn_decode_paged", "powattn_backward_workspace_bytes", "powattn_backward",
)


class PowattnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({strerror(status)})")


class _CPattern(ctypes.Structure):
    _fields_ = [("block", ctypes.c_int32), ("window", ctypes.c_int32),
                ("sink", ctypes.c_int32), ("flags", ctypes.c_uint32)]


@dataclass(frozen=True)
class Pattern:
    """powattn_pattern: B, W, S of Algorithm 1 plus the flag bits."""
    block: int
    window: int
    sink: int = 1
    flags: int = POWER

    def c(self) -> _CPattern:
        return _CPattern(self.block, self.window, self.sink, self.flags)


_lib = None


def lib() -> ctypes.CDLL:
    """Loads the built library (never builds it, never falls back)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2503_03588_amd.build` "
            "(there is no fallback path)")
    L = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER(_CPattern)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    L.powattn_version.restype = ctypes.c_int
    L.powattn_version.argtypes = []
    L.powattn_strerror.restype = ctypes.c_char_p
    L.powattn_strerror.argtypes = [ctypes.c_int]
    L.powattn_num_blocks.restype = i64
    L.powattn_num_blocks.argtypes = [P, i64]
    L.powattn_max_k.restype = i32
    L.powattn_max_k.argtypes = [P, i64]
    L.powattn_row_host.restype = i32
    L.powattn_row_host.argtypes = [P, i64, ctypes.POINTER(i32), i32]
    L.powattn_mask_build.restype = ctypes.c_int
    L.powattn_mask_build.argtypes = [P, i64, vp, vp, i32, vp, vp]
    L.powattn_prefill.restype = ctypes.c_int
    L.powattn_prefill.argtypes = [P, vp, vp, i32, vp, vp, vp, vp, vp, i32, i32, i32, i64, i32, i32, f32, vp]
    L.powattn_prefill_chunk.restype = ctypes.c_int
    L.powattn_prefill_chunk.argtypes = [P, vp, vp, i32, vp, vp, vp, vp, vp, i32, i32, i32, i64, i64, i64, i32, i32, f32, vp]
    L.powattn_prefill_chunk_paged.restype = ctypes.c_int
    L.powattn_prefill_chunk_paged.argtypes = [P, vp, vp, i32, vp, vp, vp, vp, i32, i64, vp, vp, i32, i32, i32, i64, i64,
                                              i32, i32, f32, vp]
    L.powattn_prefill_batch_paged.restype = ctypes.c_int
    L.powattn_prefill_batch_paged.argtypes = [P, vp, vp, i32, vp, vp, vp, vp, i32, i64, vp, vp, i64, vp, vp, i32, i32, i32,
                                              i32, i32, f32, vp]
    L.powattn_prefill_varlen.restype = ctypes.c_int
    L.powattn_prefill_varlen.argtypes = [P, vp, vp, i32, vp, vp, vp, vp, vp, i32, i32, i32, vp, i64,
                                         i32, i32, f32, vp]
    L.powattn_decode_workspace_bytes.restype = ctypes.c_size_t
    L.powattn_decode_workspace_bytes.argtypes = [P, i32, i32, i32, i32, i64]
    L.powattn_decode.restype = ctypes.c_int
    L.powattn_decode.argtypes = [P, vp, vp, vp, vp, i64, vp, vp, i32, i32, i32, i32, i32, f32,
                                 vp, ctypes.c_size_t, vp]
    L.powattn_decode_static.restype = ctypes.c_int
    L.powattn_decode_static.argtypes = [P, vp, vp, vp, vp, i64, vp, vp, i32, i32, i32, i32, i32, f32, vp]
    L.powattn_decode_paged.restype = ctypes.c_int
    L.powattn_decode_paged.argtypes = [P, vp, vp, vp, i64, vp, i32, vp, vp, vp, i32, i32, i32, i32, i32, f32,
                                       vp, ctypes.c_size_t, vp]
    L.powattn_backward_workspace_bytes.restype = ctypes.c_size_t
    L.powattn_backward_workspace_bytes.argtypes = [P, i32, i32, i32, i64, i32]
    L.powattn_backward.restype = ctypes.c_int
    L.powattn_backward.argtypes = [P, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i64, i32, i32,
                                   f32, vp, ctypes.c_size_t, vp]
    _lib = L
    return L


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream(stream=None):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise ValueError(f"unsupported dtype {t.dtype}")


def _check(status: int, where: str):
    if status != OK:
        raise PowattnError(status, where)


# ---- host-only queries --------------------------------------------------------
def version() -> int:
    return lib().powattn_version()


def strerror(status: int) -> str:
    return lib().powattn_strerror(status).decode()


def num_blocks(pattern: Pattern, seq_len: int) -> int:
    n = lib().powattn_num_blocks(ctypes.byref(pattern.c()), seq_len)
    if n < 0:
        raise PowattnError(-n, "powattn_num_blocks")
    return n


def max_k(pattern: Pattern, seq_len: int) -> int:
    n = lib().powattn_max_k(ctypes.byref(pattern.c()), seq_len)
    if n < 0:
        raise PowattnError(-n, "powattn_max_k")
    return n


def row_host(pattern: Pattern, q_block: int):
    L = lib()
    cp = pattern.c()
    n = L.powattn_row_host(ctypes.byref(cp), q_block, None, 0)
    if n < 0:
        raise PowattnError(-n, "powattn_row_host")
    buf = (ctypes.c_int32 * max(n, 1))()
    n2 = L.powattn_row_host(ctypes.byref(cp), q_block, buf, n)
    if n2 < 0:
        raise PowattnError(-n2, "powattn_row_host")
    return list(buf[:n2])


def decode_workspace_bytes(pattern: Pattern, batch, n_q_heads, n_kv_heads, head_dim, cache_capacity) -> int:
    return lib().powattn_decode_workspace_bytes(ctypes.byref(pattern.c()), batch, n_q_heads, n_kv_heads,
                                                head_dim, cache_capacity)


def decode_workspace(pattern: Pattern, batch, n_q_heads, n_kv_heads, head_dim, cache_capacity, device="cuda"):
    """An uninitialised workspace of the size powattn_decode asks for."""
    need = decode_workspace_bytes(pattern, batch, n_q_heads, n_kv_heads, head_dim, cache_capacity)
    if need == 0:
        raise PowattnError(INVALID_ARG, "powattn_decode_workspace_bytes")
    return torch.empty((need,), dtype=torch.uint8, device=device)


# ---- device entry points ---------------------------------------------------------
def mask_build(pattern: Pattern, seq_len: int, kv_cnt=None, kv_idx=None, block_mask=None,
               want_block_mask=False, device="cuda", stream=None):
    """powattn_mask_build.  Allocates the outputs when they are not given.
    Returns (kv_cnt int32 [nb], kv_idx int32 [nb, max_k], block_mask uint8 [nb, nb] or None)."""
    nb = num_blocks(pattern, seq_len)
    if kv_idx is None:
        mk = max_k(pattern, seq_len)
        kv_idx = torch.empty((nb, mk), dtype=torch.int32, device=device)
    if kv_cnt is None:
        kv_cnt = torch.empty((nb,), dtype=torch.int32, device=device)
    if block_mask is None and want_block_mask:
        block_mask = torch.empty((nb, nb), dtype=torch.uint8, device=device)
    st = lib().powattn_mask_build(ctypes.byref(pattern.c()), seq_len, _ptr(kv_cnt), _ptr(kv_idx),
                                  kv_idx.shape[1], _ptr(block_mask), _stream(stream))
    _check(st, "powattn_mask_build")
    return kv_cnt, kv_idx, block_mask


def prefill(pattern: Pattern, kv_cnt, kv_idx, q, k, v, o=None, lse=None, softmax_scale=0.0,
            want_lse=True, stream=None):
    """powattn_prefill.  q/o: [b,Hq,N,D]; k/v: [b,Hkv,N,D].  Returns (o, lse)."""
    batch, hq, n, d = q.shape
    hkv = k.shape[1]
    if k.shape != (batch, hkv, n, d) or v.shape != k.shape:
        raise ValueError("k/v shape mismatch")
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q/k/v dtype mismatch")
    if o is None:
        o = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty((batch, hq, n), dtype=torch.float32, device=q.device)
    mk = kv_idx.shape[1] if kv_idx is not None else 0
    if kv_idx is not None and kv_cnt.shape[0] * pattern.block < n:
        raise ValueError("block lists shorter than the sequence")
    st = lib().powattn_prefill(ctypes.byref(pattern.c()), _ptr(kv_cnt), _ptr(kv_idx), mk,
                               _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse),
                               batch, hq, hkv, n, d, _dtype_code(q), float(softmax_scale), _stream(stream))
    _check(st, "powattn_prefill")
    return o, lse


def prefill_chunk(pattern: Pattern, kv_cnt, kv_idx, q, k_cache, v_cache, q_start, o=None, lse=None,
                  softmax_scale=0.0, want_lse=True, stream=None):
    """powattn_prefill_chunk.  q/o: [b,Hq,q_len,D] at positions q_start..; caches: [b,Hkv,capacity,D] holding
    positions 0..q_start+q_len-1.  Returns (o, lse)."""
    batch, hq, q_len, d = q.shape
    hkv, cap = k_cache.shape[1], k_cache.shape[2]
    if k_cache.shape != (batch, hkv, cap, d) or v_cache.shape != k_cache.shape:
        raise ValueError("cache shape mismatch")
    if k_cache.dtype != q.dtype or v_cache.dtype != q.dtype:
        raise ValueError("q/k/v dtype mismatch")
    if o is None:
        o = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty((batch, hq, q_len), dtype=torch.float32, device=q.device)
    mk = kv_idx.shape[1] if kv_idx is not None else 0
    if kv_idx is not None and kv_cnt.shape[0] * pattern.block < q_start + q_len:
        raise ValueError("block lists shorter than the context")
    st = lib().powattn_prefill_chunk(ctypes.byref(pattern.c()), _ptr(kv_cnt), _ptr(kv_idx), mk,
                                     _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(o), _ptr(lse),
                                     batch, hq, hkv, int(q_start), q_len, cap, d, _dtype_code(q),
                                     float(softmax_scale), _stream(stream))
    _check(st, "powattn_prefill_chunk")
    return o, lse


def prefill_chunk_paged(pattern: Pattern, kv_cnt, kv_idx, q, k_pages, v_pages, block_table, q_start, o=None, lse=None,
                        softmax_scale=0.0, want_lse=True, stream=None):
    """powattn_prefill_chunk_paged.  q/o: [b,Hq,q_len,D] at positions q_start..; pages: [n_pages,Hkv,block,D];
    block_table int32 [b, table_stride].  Returns (o, lse)."""
    batch, hq, q_len, d = q.shape
    n_pages, hkv, blk = k_pages.shape[0], k_pages.shape[1], k_pages.shape[2]
    if k_pages.shape != (n_pages, hkv, blk, d) or v_pages.shape != k_pages.shape:
        raise ValueError("page pool shape mismatch")
    if blk != pattern.block:
        raise ValueError("a page holds one block of the pattern")
    if k_pages.dtype != q.dtype or v_pages.dtype != q.dtype:
        raise ValueError("q/k/v dtype mismatch")
    if block_table.dtype != torch.int32 or block_table.dim() != 2 or block_table.shape[0] != batch:
        raise ValueError("block_table must be int32 [batch, table_stride]")
    if not block_table.is_contiguous():
        raise ValueError("block_table must be contiguous")
    if kv_idx is None or kv_cnt is None:
        raise ValueError("the paged form needs block lists")
    if kv_cnt.shape[0] * pattern.block < q_start + q_len:
        raise ValueError("block lists shorter than the context")
    if o is None:
        o = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty((batch, hq, q_len), dtype=torch.float32, device=q.device)
    st = lib().powattn_prefill_chunk_paged(ctypes.byref(pattern.c()), _ptr(kv_cnt), _ptr(kv_idx), kv_idx.shape[1],
                                           _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table),
                                           block_table.shape[1], n_pages, _ptr(o), _ptr(lse),
                                           batch, hq, hkv, int(q_start), q_len, d, _dtype_code(q),
                                           float(softmax_scale), _stream(stream))
    _check(st, "powattn_prefill_chunk_paged")
    return o, lse


def prefill_batch_paged(pattern: Pattern, kv_cnt, kv_idx, q, k_pages, v_pages, block_table, q_start, q_len, o=None,
                        lse=None, softmax_scale=0.0, want_lse=True, stream=None):
    """powattn_prefill_batch_paged.  q/o: [b,Hq,q_rows,D]; pages: [n_pages,Hkv,block,D]; block_table int32
    [b, table_stride]; q_start, q_len int32 [b] on the device.  Returns (o, lse); rows at or beyond a sequence's
    q_len are left as they were."""
    batch, hq, q_rows, d = q.shape
    n_pages, hkv, blk = k_pages.shape[0], k_pages.shape[1], k_pages.shape[2]
    if k_pages.shape != (n_pages, hkv, blk, d) or v_pages.shape != k_pages.shape:
        raise ValueError("page pool shape mismatch")
    if blk != pattern.block:
        raise ValueError("a page holds one block of the pattern")
    if k_pages.dtype != q.dtype or v_pages.dtype != q.dtype:
        raise ValueError("q/k/v dtype mismatch")
    if block_table.dtype != torch.int32 or block_table.dim() != 2 or block_table.shape[0] != batch:
        raise ValueError("block_table must be int32 [batch, table_stride]")
    if not block_table.is_contiguous():
        raise ValueError("block_table must be contiguous")
    for t in (q_start, q_len):
        if t.dtype != torch.int32 or t.shape != (batch,) or t.device != q.device:
            raise ValueError("q_start and q_len must be int32 [batch] on the device of q")
    if kv_idx is None or kv_cnt is None:
        raise ValueError("the paged form needs block lists")
    if kv_cnt.shape[0] < block_table.shape[1]:
        raise ValueError("block lists shorter than the longest context the block table can describe")
    if o is None:
        o = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty((batch, hq, q_rows), dtype=torch.float32, device=q.device)
    st = lib().powattn_prefill_batch_paged(ctypes.byref(pattern.c()), _ptr(kv_cnt), _ptr(kv_idx), kv_idx.shape[1],
                                           _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table),
                                           block_table.shape[1], n_pages, _ptr(q_start), _ptr(q_len), q_rows,
                                           _ptr(o), _ptr(lse), batch, hq, hkv, d, _dtype_code(q),
                                           float(softmax_scale), _stream(stream))
    _check(st, "powattn_prefill_batch_paged")
    return o, lse


def decode(pattern: Pattern, q, k_cache, v_cache, kv_len, o=None, lse=None, softmax_scale=0.0,
           workspace=None, want_lse=True, stream=None):
    """powattn_decode.  q/o: [b,Hq,D]; caches: [b,Hkv,capacity,D]; kv_len int32 [b].  Returns (o, lse)."""
    batch, hq, d = q.shape
    hkv, cap = k_cache.shape[1], k_cache.shape[2]
    if k_cache.shape != (batch, hkv, cap, d) or v_cache.shape != k_cache.shape:
        raise ValueError("cache shape mismatch")
    if kv_len.dtype != torch.int32 or kv_len.shape != (batch,):
        raise ValueError("kv_len must be int32 [batch]")
    if o is None:
        o = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty((batch, hq), dtype=torch.float32, device=q.device)
    if workspace is None:
        need = decode_workspace_bytes(pattern, batch, hq, hkv, d, cap)
        workspace = decode_workspace(pattern, batch, hq, hkv, d, cap, q.device)
    st = lib().powattn_decode(ctypes.byref(pattern.c()), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(kv_len),
                              cap, _ptr(o), _ptr(lse), batch, hq, hkv, d, _dtype_code(q),
                              float(softmax_scale), _ptr(workspace), workspace.numel() * workspace.element_size(),
                              _stream(stream))
    _check(st, "powattn_decode")
    return o, lse


def decode_static(pattern: Pattern, q, k_cache, v_cache, kv_len, o, lse=None, softmax_scale=0.0, stream=None):
    """powattn_decode_static: powattn_decode on the library's own scratch buffer.  The caller passes every
    tensor, o (and lse, if wanted) included: nothing is allocated here or in the library.  Returns (o, lse)."""
    batch, hq, d = q.shape
    hkv, cap = k_cache.shape[1], k_cache.shape[2]
    if k_cache.shape != (batch, hkv, cap, d) or v_cache.shape != k_cache.shape:
        raise ValueError("cache shape mismatch")
    if kv_len.dtype != torch.int32 or kv_len.shape != (batch,):
        raise ValueError("kv_len must be int32 [batch]")
    if o.shape != q.shape or o.dtype != q.dtype:
        raise ValueError("o must have the shape and dtype of q")
    st = lib().powattn_decode_static(ctypes.byref(pattern.c()), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(kv_len),
                                     cap, _ptr(o), _ptr(lse), batch, hq, hkv, d, _dtype_code(q),
                                     float(softmax_scale), _stream(stream))
    _check(st, "powattn_decode_static")
    return o, lse


def decode_paged(pattern: Pattern, q, k_pages, v_pages, block_table, kv_len, o=None, lse=None, softmax_scale=0.0,
                 workspace=None, want_lse=True, stream=None):
    """powattn_decode_paged.  q/o: [b,Hq,D]; pages: [n_pages,Hkv,block,D]; block_table int32 [b, table_stride];
    kv_len int32 [b].  Returns (o, lse)."""
    batch, hq, d = q.shape
    n_pages, hkv, blk = k_pages.shape[0], k_pages.shape[1], k_pages.shape[2]
    if k_pages.shape != (n_pages, hkv, blk, d) or v_pages.shape != k_pages.shape:
        raise ValueError("page pool shape mismatch")
    if blk != pattern.block:
        raise ValueError("a page holds one block of the pattern")
    if block_table.dtype != torch.int32 or block_table.dim() != 2 or block_table.shape[0] != batch:
        raise ValueError("block_table must be int32 [batch, table_stride]")
    if not block_table.is_contiguous():
        raise ValueError("block_table must be contiguous")
    if kv_len.dtype != torch.int32 or kv_len.shape != (batch,):
        raise ValueError("kv_len must be int32 [batch]")
    stride = block_table.shape[1]
    if o is None:
        o = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty((batch, hq), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = decode_workspace(pattern, batch, hq, hkv, d, stride * blk, q.device)
    st = lib().powattn_decode_paged(ctypes.byref(pattern.c()), _ptr(q), _ptr(k_pages), _ptr(v_pages), n_pages,
                                    _ptr(block_table), stride, _ptr(kv_len), _ptr(o), _ptr(lse),
                                    batch, hq, hkv, d, _dtype_code(q), float(softmax_scale),
                                    _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "powattn_decode_paged")
    return o, lse


def backward_workspace_bytes(pattern: Pattern, batch, n_q_heads, n_kv_heads, seq_len, head_dim) -> int:
    return lib().powattn_backward_workspace_bytes(ctypes.byref(pattern.c()), batch, n_q_heads, n_kv_heads,
                                                  seq_len, head_dim)


def backward(pattern: Pattern, kv_cnt, kv_idx, q, k, v, o, lse, d_o, dq=None, dk=None, dv=None, softmax_scale=0.0,
             workspace=None, stream=None):
    """powattn_backward.  q/o/d_o/dq: [b,Hq,N,D]; k/v/dk/dv: [b,Hkv,N,D]; lse float32 [b,Hq,N].
    Returns (dq, dk, dv)."""
    batch, hq, n, d = q.shape
    hkv = k.shape[1]
    if k.shape != (batch, hkv, n, d) or v.shape != k.shape:
        raise ValueError("k/v shape mismatch")
    if o.shape != q.shape or d_o.shape != q.shape or lse.shape != (batch, hq, n):
        raise ValueError("o/d_o/lse shape mismatch")
    if lse.dtype != torch.float32:
        raise ValueError("lse must be float32")
    for t in (k, v, o, d_o):
        if t.dtype != q.dtype:
            raise ValueError("dtype mismatch")
    if dq is None:
        dq = torch.empty_like(q)
    if dk is None:
        dk = torch.empty_like(k)
    if dv is None:
        dv = torch.empty_like(v)
    if workspace is None:
        need = backward_workspace_bytes(pattern, batch, hq, hkv, n, d)
        if need == 0:
            raise PowattnError(INVALID_ARG, "powattn_backward_workspace_bytes")
        workspace = torch.empty((need,), dtype=torch.uint8, device=q.device)
    st = lib().powattn_backward(ctypes.byref(pattern.c()), _ptr(kv_cnt), _ptr(kv_idx), kv_idx.shape[1],
                                _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(dq), _ptr(dk), _ptr(dv),
                                batch, hq, hkv, n, d, _dtype_code(q), float(softmax_scale),
                                _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "powattn_backward")
    return dq, dk, dv


def prefill_varlen(pattern: Pattern, kv_cnt, kv_idx, q, k, v, seq_lens, o=None, lse=None, softmax_scale=0.0,
                   want_lse=True, stream=None):
    """powattn_prefill_varlen.  q/o: [b,Hq,Np,D]; k/v: [b,Hkv,Np,D] padded to Np rows; seq_lens: int32 device
    tensor [b].  Rows beyond a sequence's length keep whatever o/lse held.  Returns (o, lse)."""
    batch, hq, npad, d = q.shape
    hkv = k.shape[1]
    if k.shape != (batch, hkv, npad, d) or v.shape != k.shape:
        raise ValueError("k/v shape mismatch")
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q/k/v dtype mismatch")
    if seq_lens.dtype != torch.int32 or seq_lens.shape != (batch,) or seq_lens.device != q.device:
        raise ValueError("seq_lens must be an int32 tensor [batch] on the device of q")
    if kv_idx is not None and kv_cnt.shape[0] * pattern.block < npad:
        raise ValueError("block lists shorter than the padded length")
    if o is None:
        o = torch.zeros_like(q)
    if lse is None and want_lse:
        lse = torch.zeros((batch, hq, npad), dtype=torch.float32, device=q.device)
    mk = kv_idx.shape[1] if kv_idx is not None else 0
    st = lib().powattn_prefill_varlen(ctypes.byref(pattern.c()), _ptr(kv_cnt), _ptr(kv_idx), mk,
                                      _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), batch, hq, hkv, _ptr(seq_lens),
                                      npad, d, _dtype_code(q), float(softmax_scale), _stream(stream))
    _check(st, "powattn_prefill_varlen")
    return o, lse
