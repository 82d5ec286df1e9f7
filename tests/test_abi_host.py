"""Host-only checks of the C ABI: the library loads, exports every function the
header declares, answers the host-side queries like the oracle does, and turns
bad arguments into status codes before anything could be launched (CPU only:
no call here reaches a kernel launch)."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import powattn_oracle as orc
from paper_2503_03588_amd import binding as pa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # a non-null "device pointer" that is never dereferenced on these paths


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(pa.LIB_PATH):
        pytest.fail("libpowattn.so has not been built (python -m paper_2503_03588_amd.build)")
    return pa.lib()


def test_every_declared_function_is_exported(L):
    text = open(os.path.join(ROOT, "include", "powattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(powattn_[a-z_0-9]+)\s*\(", text))
    assert declared == set(pa.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name


def test_version_and_strerror(L):
    assert pa.version() >= 100
    assert pa.strerror(pa.OK) == "ok"
    for st in (pa.INVALID_ARG, pa.UNSUPPORTED, pa.WORKSPACE_TOO_SMALL, pa.HIP_ERROR, 77):
        assert isinstance(pa.strerror(st), str) and pa.strerror(st)


@pytest.mark.parametrize("n,B,W,S,flags", [
    (1024, 64, 2, 1, pa.POWER), (1024, 64, 2, 0, pa.POWER), (32768, 64, 4, 1, pa.POWER),
    (131072, 128, 4, 1, pa.POWER), (32768, 256, 5, 1, pa.POWER), (32768, 256, 9, 1, 0),
    (1000, 64, 0, 0, pa.POWER), (5000, 16, 3, 5, pa.POWER), (777, 16, 2, 1, pa.DENSE),
])
def test_host_rows_and_capacity_match_oracle(L, n, B, W, S, flags):
    pat = pa.Pattern(B, W, S, flags)
    opat = orc.Pattern(B, W, S, power=bool(flags & pa.POWER), dense=bool(flags & pa.DENSE))
    cnt, idx, mk = orc.block_lists(n, opat)
    assert pa.num_blocks(pat, n) == cnt.shape[0]
    assert pa.max_k(pat, n) == mk
    for i in sorted(set([0, 1, 2, 3, cnt.shape[0] // 2, cnt.shape[0] - 2, cnt.shape[0] - 1])):
        if 0 <= i < cnt.shape[0]:
            assert pa.row_host(pat, i) == idx[i, : cnt[i]].tolist()


def test_row_host_capacity_error(L):
    cp = pa.Pattern(64, 4, 1).c()
    buf = (ctypes.c_int32 * 4)()
    assert L.powattn_row_host(ctypes.byref(cp), 1023, buf, 4) == -pa.WORKSPACE_TOO_SMALL
    assert L.powattn_row_host(ctypes.byref(cp), -1, buf, 4) == -pa.INVALID_ARG
    assert L.powattn_row_host(None, 3, buf, 4) == -pa.INVALID_ARG


def test_bad_patterns(L):
    for pat in (pa.Pattern(0, 2, 1), pa.Pattern(64, -1, 1), pa.Pattern(64, 2, -1),
                pa.Pattern(64, 2, 1, flags=8), pa.Pattern(64, 0, 1, flags=0)):
        cp = pat.c()
        assert L.powattn_max_k(ctypes.byref(cp), 1024) == -pa.INVALID_ARG
        assert L.powattn_mask_build(ctypes.byref(cp), 1024, FAKE, FAKE, 16, None, None) == pa.INVALID_ARG
    cp = pa.Pattern(64, 2, 1).c()
    assert L.powattn_num_blocks(ctypes.byref(cp), 0) == -pa.INVALID_ARG


def test_mask_build_argument_errors(L):
    cp = pa.Pattern(64, 4, 1).c()
    assert L.powattn_mask_build(None, 1024, FAKE, FAKE, 16, None, None) == pa.INVALID_ARG
    assert L.powattn_mask_build(ctypes.byref(cp), 1024, None, FAKE, 16, None, None) == pa.INVALID_ARG
    assert L.powattn_mask_build(ctypes.byref(cp), 1024, FAKE, None, 16, None, None) == pa.INVALID_ARG
    assert L.powattn_mask_build(ctypes.byref(cp), -5, FAKE, FAKE, 16, None, None) == pa.INVALID_ARG
    assert L.powattn_mask_build(ctypes.byref(cp), 65536, FAKE, FAKE, 12, None, None) == pa.WORKSPACE_TOO_SMALL


def _prefill(L, pat=None, cnt=FAKE, idx=FAKE, max_k=13, q=FAKE, k=FAKE, v=FAKE, o=FAKE, lse=None,
             batch=1, hq=4, hkv=2, n=1024, d=128, dtype=pa.BF16, scale=0.0):
    cp = (pat or pa.Pattern(64, 4, 1)).c()
    return L.powattn_prefill(ctypes.byref(cp), cnt, idx, max_k, q, k, v, o, lse, batch, hq, hkv, n, d, dtype,
                             scale, None)


def test_prefill_argument_errors(L):
    assert _prefill(L, q=None) == pa.INVALID_ARG
    assert _prefill(L, k=None) == pa.INVALID_ARG
    assert _prefill(L, v=None) == pa.INVALID_ARG
    assert _prefill(L, o=None) == pa.INVALID_ARG
    assert _prefill(L, cnt=None) == pa.INVALID_ARG
    assert _prefill(L, idx=None) == pa.INVALID_ARG
    assert _prefill(L, max_k=0) == pa.INVALID_ARG
    assert _prefill(L, hq=6, hkv=4) == pa.INVALID_ARG
    assert _prefill(L, batch=0) == pa.INVALID_ARG
    assert _prefill(L, n=0) == pa.INVALID_ARG
    assert _prefill(L, scale=float("nan")) == pa.INVALID_ARG
    assert _prefill(L, d=96) == pa.UNSUPPORTED
    assert _prefill(L, dtype=5) == pa.UNSUPPORTED
    assert _prefill(L, pat=pa.Pattern(48, 4, 1)) == pa.UNSUPPORTED            # bf16 needs a multiple of 64
    assert _prefill(L, pat=pa.Pattern(24, 4, 1), dtype=pa.F32) == pa.UNSUPPORTED


def _decode(L, pat=None, q=FAKE, k=FAKE, v=FAKE, kv_len=FAKE, cap=65536, o=FAKE, lse=None, batch=2, hq=8,
            hkv=2, d=128, dtype=pa.BF16, scale=0.0, ws=FAKE, ws_bytes=None):
    p = pat or pa.Pattern(64, 4, 1)
    cp = p.c()
    if ws_bytes is None:
        ws_bytes = L.powattn_decode_workspace_bytes(ctypes.byref(cp), batch, hq, hkv, d, cap)
    return L.powattn_decode(ctypes.byref(cp), q, k, v, kv_len, cap, o, lse, batch, hq, hkv, d, dtype, scale,
                            ws, ws_bytes, None)


def _chunk(L, pat=None, cnt=FAKE, idx=FAKE, max_k=13, q=FAKE, k=FAKE, v=FAKE, o=FAKE, lse=None,
           batch=1, hq=4, hkv=2, q_start=1024, q_len=512, cap=4096, d=128, dtype=pa.BF16, scale=0.0):
    cp = (pat or pa.Pattern(64, 4, 1)).c()
    return L.powattn_prefill_chunk(ctypes.byref(cp), cnt, idx, max_k, q, k, v, o, lse, batch, hq, hkv,
                                   q_start, q_len, cap, d, dtype, scale, None)


def test_prefill_chunk_argument_errors(L):
    assert _chunk(L, q=None) == pa.INVALID_ARG
    assert _chunk(L, k=None) == pa.INVALID_ARG
    assert _chunk(L, o=None) == pa.INVALID_ARG
    assert _chunk(L, cnt=None) == pa.INVALID_ARG
    assert _chunk(L, max_k=0) == pa.INVALID_ARG
    assert _chunk(L, hq=6, hkv=4) == pa.INVALID_ARG
    assert _chunk(L, q_start=-64) == pa.INVALID_ARG
    assert _chunk(L, q_len=0) == pa.INVALID_ARG
    assert _chunk(L, q_start=4032, q_len=128) == pa.INVALID_ARG  # runs past the cache capacity
    assert _chunk(L, scale=float("nan")) == pa.INVALID_ARG
    assert _chunk(L, dtype=pa.F32) == pa.UNSUPPORTED
    assert _chunk(L, d=96) == pa.UNSUPPORTED
    assert _chunk(L, pat=pa.Pattern(48, 4, 1), q_start=960) == pa.UNSUPPORTED
    # the dense pattern needs no lists
    assert _chunk(L, pat=pa.Pattern(64, 1, 0, flags=pa.DENSE), cnt=None, idx=None, max_k=0, q=None) == pa.INVALID_ARG


def _chunk_paged(L, pat=None, cnt=FAKE, idx=FAKE, max_k=13, q=FAKE, k=FAKE, v=FAKE, table=FAKE, stride=64, n_pages=100,
                 o=FAKE, lse=None, batch=1, hq=4, hkv=2, q_start=1024, q_len=512, d=128, dtype=pa.BF16, scale=0.0):
    cp = (pat or pa.Pattern(64, 4, 1)).c()
    return L.powattn_prefill_chunk_paged(ctypes.byref(cp), cnt, idx, max_k, q, k, v, table, stride, n_pages, o, lse,
                                         batch, hq, hkv, q_start, q_len, d, dtype, scale, None)


def test_prefill_chunk_paged_argument_errors(L):
    # every case is refused on the host, before any launch
    assert _chunk_paged(L, q=None) == pa.INVALID_ARG
    assert _chunk_paged(L, k=None) == pa.INVALID_ARG
    assert _chunk_paged(L, v=None) == pa.INVALID_ARG
    assert _chunk_paged(L, o=None) == pa.INVALID_ARG
    assert _chunk_paged(L, table=None) == pa.INVALID_ARG
    assert _chunk_paged(L, cnt=None) == pa.INVALID_ARG
    assert _chunk_paged(L, max_k=0) == pa.INVALID_ARG
    assert _chunk_paged(L, stride=0) == pa.INVALID_ARG
    assert _chunk_paged(L, n_pages=0) == pa.INVALID_ARG
    assert _chunk_paged(L, hq=6, hkv=4) == pa.INVALID_ARG
    assert _chunk_paged(L, q_start=-1) == pa.INVALID_ARG
    assert _chunk_paged(L, q_len=0) == pa.INVALID_ARG
    assert _chunk_paged(L, q_start=4000, q_len=128) == pa.INVALID_ARG         # runs past the table (64 blocks of 64)
    assert _chunk_paged(L, scale=float("nan")) == pa.INVALID_ARG
    assert _chunk_paged(L, dtype=pa.F32) == pa.UNSUPPORTED
    assert _chunk_paged(L, d=96) == pa.UNSUPPORTED
    assert _chunk_paged(L, pat=pa.Pattern(48, 4, 1), q_start=960) == pa.UNSUPPORTED
    assert _chunk_paged(L, pat=pa.Pattern(64, 1, 0, flags=pa.DENSE)) == pa.UNSUPPORTED
    assert _chunk_paged(L, max_k=64) == pa.UNSUPPORTED                         # list rows of at most 63 entries
    assert _chunk_paged(L, n_pages=2 ** 31) == pa.UNSUPPORTED                  # pool rows are kept in 32 bits


def _batch_paged(L, pat=None, cnt=FAKE, idx=FAKE, max_k=13, q=FAKE, k=FAKE, v=FAKE, table=FAKE, stride=64, n_pages=100,
                 starts=FAKE, lens=FAKE, q_rows=512, o=FAKE, lse=None, batch=2, hq=4, hkv=2, d=128, dtype=pa.BF16, scale=0.0):
    cp = (pat or pa.Pattern(64, 4, 1)).c()
    return L.powattn_prefill_batch_paged(ctypes.byref(cp), cnt, idx, max_k, q, k, v, table, stride, n_pages, starts, lens,
                                         q_rows, o, lse, batch, hq, hkv, d, dtype, scale, None)


def test_prefill_batch_paged_argument_errors(L):
    for name in ("q", "k", "v", "o", "table", "starts", "lens", "cnt", "idx"):
        assert _batch_paged(L, **{name: None}) == pa.INVALID_ARG, name
    assert _batch_paged(L, max_k=0) == pa.INVALID_ARG
    assert _batch_paged(L, stride=0) == pa.INVALID_ARG
    assert _batch_paged(L, n_pages=0) == pa.INVALID_ARG
    assert _batch_paged(L, q_rows=0) == pa.INVALID_ARG
    assert _batch_paged(L, q_rows=64 * 64 + 1) == pa.INVALID_ARG                # more rows than the table describes
    assert _batch_paged(L, batch=0) == pa.INVALID_ARG
    assert _batch_paged(L, hq=6, hkv=4) == pa.INVALID_ARG
    assert _batch_paged(L, scale=float("nan")) == pa.INVALID_ARG
    assert _batch_paged(L, dtype=pa.F32) == pa.UNSUPPORTED
    assert _batch_paged(L, d=96) == pa.UNSUPPORTED
    assert _batch_paged(L, pat=pa.Pattern(48, 4, 1)) == pa.UNSUPPORTED
    assert _batch_paged(L, pat=pa.Pattern(64, 1, 0, flags=pa.DENSE)) == pa.UNSUPPORTED
    assert _batch_paged(L, max_k=64) == pa.UNSUPPORTED
    assert _batch_paged(L, n_pages=2 ** 31) == pa.UNSUPPORTED


def test_prefill_varlen_argument_errors(L):
    cp = pa.Pattern(64, 4, 1).c()

    def call(q=FAKE, lens_=FAKE, npad=2048, hq=4, hkv=2, d=128, dtype=pa.BF16, max_k=13, cnt=FAKE, pat=cp):
        # the lengths live in device memory: the host checks the pointer only (the kernel clamps the values)
        return L.powattn_prefill_varlen(ctypes.byref(pat), cnt, FAKE, max_k, q, FAKE, FAKE, FAKE, None, 2, hq, hkv,
                                        lens_, npad, d, dtype, 0.0, None)
    assert call(q=None) == pa.INVALID_ARG
    assert call(lens_=None) == pa.INVALID_ARG
    assert call(cnt=None) == pa.INVALID_ARG
    assert call(npad=0) == pa.INVALID_ARG
    assert call(hq=6, hkv=4) == pa.INVALID_ARG
    assert call(dtype=pa.F32) == pa.UNSUPPORTED
    assert call(d=96) == pa.UNSUPPORTED
    assert call(pat=pa.Pattern(48, 4, 1).c()) == pa.UNSUPPORTED


def test_decode_argument_errors(L):
    assert _decode(L, q=None) == pa.INVALID_ARG
    assert _decode(L, k=None) == pa.INVALID_ARG
    assert _decode(L, v=None) == pa.INVALID_ARG
    assert _decode(L, kv_len=None) == pa.INVALID_ARG
    assert _decode(L, o=None) == pa.INVALID_ARG
    assert _decode(L, cap=0) == pa.INVALID_ARG
    assert _decode(L, hq=6, hkv=4) == pa.INVALID_ARG
    assert _decode(L, d=80) == pa.UNSUPPORTED
    assert _decode(L, dtype=pa.F32) == pa.UNSUPPORTED
    assert _decode(L, pat=pa.Pattern(32, 4, 1)) == pa.UNSUPPORTED
    assert _decode(L, ws=None) == pa.WORKSPACE_TOO_SMALL
    assert _decode(L, ws_bytes=64) == pa.WORKSPACE_TOO_SMALL
    assert _decode(L, ws=FAKE + 8) == pa.INVALID_ARG                          # misaligned workspace


def test_decode_static_argument_errors_are_found_before_the_device_is_touched(L):
    def call(pat=None, q=FAKE, k=FAKE, v=FAKE, kv_len=FAKE, cap=65536, o=FAKE, batch=2, hq=8, hkv=2, d=128,
             dtype=pa.BF16, scale=0.0):
        cp = (pat or pa.Pattern(64, 4, 1)).c()
        return L.powattn_decode_static(ctypes.byref(cp), q, k, v, kv_len, cap, o, None, batch, hq, hkv, d, dtype,
                                       scale, None)
    assert call(q=None) == pa.INVALID_ARG
    assert call(kv_len=None) == pa.INVALID_ARG
    assert call(o=None) == pa.INVALID_ARG
    assert call(cap=0) == pa.INVALID_ARG
    assert call(hq=6, hkv=4) == pa.INVALID_ARG
    assert call(d=80) == pa.UNSUPPORTED
    assert call(dtype=pa.F32) == pa.UNSUPPORTED
    assert call(scale=float("nan")) == pa.INVALID_ARG
    # a shape whose partial results do not fit the library's static buffer (32 MiB) is refused
    assert pa.decode_workspace_bytes(pa.Pattern(64, 4, 1), 1024, 32, 8, 128, 65536) > (32 << 20)
    assert call(batch=1024, hq=32, hkv=8) == pa.WORKSPACE_TOO_SMALL


def _paged(L, pat=None, q=FAKE, k=FAKE, v=FAKE, n_pages=100, table=FAKE, stride=64, kv_len=FAKE, o=FAKE, lse=None,
           batch=2, hq=8, hkv=2, d=128, dtype=pa.BF16, scale=0.0, ws=FAKE, ws_bytes=None):
    p = pat or pa.Pattern(64, 4, 1)
    cp = p.c()
    if ws_bytes is None:
        ws_bytes = L.powattn_decode_workspace_bytes(ctypes.byref(cp), batch, hq, hkv, d, max(stride, 1) * p.block)
    return L.powattn_decode_paged(ctypes.byref(cp), q, k, v, n_pages, table, stride, kv_len, o, lse,
                                  batch, hq, hkv, d, dtype, scale, ws, ws_bytes, None)


def test_decode_paged_argument_errors(L):
    assert _paged(L, q=None) == pa.INVALID_ARG
    assert _paged(L, k=None) == pa.INVALID_ARG
    assert _paged(L, v=None) == pa.INVALID_ARG
    assert _paged(L, table=None) == pa.INVALID_ARG
    assert _paged(L, kv_len=None) == pa.INVALID_ARG
    assert _paged(L, o=None) == pa.INVALID_ARG
    assert _paged(L, n_pages=0) == pa.INVALID_ARG
    assert _paged(L, stride=0) == pa.INVALID_ARG
    assert _paged(L, hq=6, hkv=4) == pa.INVALID_ARG
    assert _paged(L, scale=float("nan")) == pa.INVALID_ARG
    assert _paged(L, d=80) == pa.UNSUPPORTED
    assert _paged(L, dtype=pa.F32) == pa.UNSUPPORTED
    assert _paged(L, pat=pa.Pattern(32, 4, 1)) == pa.UNSUPPORTED
    assert _paged(L, ws=None) == pa.WORKSPACE_TOO_SMALL
    assert _paged(L, ws_bytes=64) == pa.WORKSPACE_TOO_SMALL
    assert _paged(L, ws=FAKE + 8) == pa.INVALID_ARG


def _backward(L, pat=None, cnt=FAKE, idx=FAKE, max_k=13, q=FAKE, k=FAKE, v=FAKE, o=FAKE, lse=FAKE, do=FAKE,
              dq=FAKE, dk=FAKE, dv=FAKE, batch=1, hq=4, hkv=2, n=4096, d=128, dtype=pa.BF16, scale=0.0,
              ws=FAKE, ws_bytes=None):
    p = pat or pa.Pattern(64, 4, 1)
    cp = p.c()
    if ws_bytes is None:
        ws_bytes = L.powattn_backward_workspace_bytes(ctypes.byref(cp), batch, hq, hkv, n, d)
    return L.powattn_backward(ctypes.byref(cp), cnt, idx, max_k, q, k, v, o, lse, do, dq, dk, dv, batch, hq, hkv,
                              n, d, dtype, scale, ws, ws_bytes, None)


def test_backward_argument_errors(L):
    for name in ("cnt", "idx", "q", "k", "v", "o", "lse", "do", "dq", "dk", "dv"):
        assert _backward(L, **{name: None}) == pa.INVALID_ARG, name
    assert _backward(L, hq=6, hkv=4) == pa.INVALID_ARG
    assert _backward(L, n=0) == pa.INVALID_ARG
    assert _backward(L, scale=float("nan")) == pa.INVALID_ARG
    assert _backward(L, max_k=5) == pa.WORKSPACE_TOO_SMALL              # shorter than the pattern's rows
    assert _backward(L, dtype=pa.F32) == pa.UNSUPPORTED
    assert _backward(L, d=96) == pa.UNSUPPORTED
    assert _backward(L, pat=pa.Pattern(192, 4, 1)) == pa.UNSUPPORTED
    assert _backward(L, pat=pa.Pattern(64, 1, 0, flags=pa.DENSE)) == pa.UNSUPPORTED
    assert _backward(L, ws=None) == pa.WORKSPACE_TOO_SMALL
    assert _backward(L, ws_bytes=64) == pa.WORKSPACE_TOO_SMALL
    assert _backward(L, ws=FAKE + 8) == pa.INVALID_ARG
    cp = pa.Pattern(64, 4, 1).c()
    n = L.powattn_backward_workspace_bytes(ctypes.byref(cp), 1, 32, 8, 131072, 128)
    assert n >= 2 * 32 * 131072 * 4 + 2 * 8 * 64 * 128 * 4 and n % 256 == 0
    assert L.powattn_backward_workspace_bytes(ctypes.byref(cp), 0, 32, 8, 131072, 128) == 0


def test_decode_workspace_size(L):
    pat = pa.Pattern(64, 4, 1)
    n = pa.decode_workspace_bytes(pat, 16, 32, 8, 128, 65536)
    assert n > 0 and n % 256 == 0
    assert pa.decode_workspace_bytes(pat, 16, 32, 8, 128, 131072) >= n
    assert pa.decode_workspace_bytes(pat, 0, 32, 8, 128, 65536) == 0
    assert pa.decode_workspace_bytes(pat, 16, 30, 8, 128, 65536) == 0


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(pa, "_lib", None)
    monkeypatch.setattr(pa, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        pa.version()
