"""Python face of the CPU checker (TEST INFRASTRUCTURE ONLY).

Thin ctypes wrappers around oracle/hetis_oracle.c: numpy arrays in, fp64 numpy
arrays out.  Only tests, the smoke check and the benchmark's cpu_baseline leg
may import this package; the GPU library never does, and nothing here imports
the GPU package.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from .build_oracle import build as _build

_lib = None


class _Shape(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("block_size", C.c_int32),
                ("max_blocks_per_seq", C.c_int32),
                ("kv_stride_block", C.c_int64), ("kv_stride_head", C.c_int64)]


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build(force=False))
        _lib.oracle_half_to_double.restype = C.c_double
        _lib.oracle_half_to_double.argtypes = [C.c_uint16]
        for name in ("oracle_attn_decode", "oracle_attn_partial", "oracle_attn_merge",
                     "oracle_max_threads"):
            getattr(_lib, name).restype = C.c_int
    return _lib


def _u16(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16
    return a


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def _shape(q, k_cache, block_table):
    B, Hq, D = q.shape
    nb, Hkv, bs, D2 = k_cache.shape
    assert D == D2 and Hq % Hkv == 0
    return _Shape(B, Hq, Hkv, D, bs, block_table.shape[1], Hkv * bs * D, bs * D)


def half_to_double(bits: int) -> float:
    return lib().oracle_half_to_double(int(bits))


def max_threads() -> int:
    return lib().oracle_max_threads()


def attn_decode(q, k_cache, v_cache, block_table, seq_lens, head_ids, scale,
                n_threads: int = 0, fill=np.nan):
    """fp64 [B, Hq, D]; rows of heads not selected keep `fill`."""
    q, k, v = _u16(q), _u16(k_cache), _u16(v_cache)
    bt, sl, hid = _i32(block_table), _i32(seq_lens), _i32(head_ids)
    shp = _shape(q, k, bt)
    out = np.full(q.shape, fill, dtype=np.float64)
    rc = lib().oracle_attn_decode(C.byref(shp), _ptr(q), _ptr(k), _ptr(v), _ptr(bt), _ptr(sl),
                                  _ptr(hid), C.c_int32(len(hid)), C.c_double(scale), _ptr(out),
                                  C.c_int32(n_threads))
    if rc != 0:
        raise RuntimeError(f"oracle_attn_decode failed: {rc}")
    return out


def attn_partial(q, k_cache, v_cache, block_table, seq_lens, head_ids, scale, chunk_tokens,
                 max_chunks, fill=np.nan):
    """(o_partial fp64 [B, S*r, C, D], lse_partial fp64 [B, S*r, C])."""
    q, k, v = _u16(q), _u16(k_cache), _u16(v_cache)
    bt, sl, hid = _i32(block_table), _i32(seq_lens), _i32(head_ids)
    shp = _shape(q, k, bt)
    rows = len(hid) * (shp.n_q_heads // shp.n_kv_heads)
    o = np.full((shp.batch, rows, max_chunks, shp.head_dim), fill, dtype=np.float64)
    lse = np.full((shp.batch, rows, max_chunks), fill, dtype=np.float64)
    rc = lib().oracle_attn_partial(C.byref(shp), _ptr(q), _ptr(k), _ptr(v), _ptr(bt), _ptr(sl),
                                   _ptr(hid), C.c_int32(len(hid)), C.c_double(scale),
                                   C.c_int32(chunk_tokens), C.c_int32(max_chunks), _ptr(o),
                                   _ptr(lse))
    if rc != 0:
        raise RuntimeError(f"oracle_attn_partial failed: {rc}")
    return o, lse


def attn_merge(o_partial, lse_partial, seq_lens, head_ids, n_q_heads, n_kv_heads, chunk_tokens,
               fill=np.nan):
    """fp64 [B, Hq, D] from partials laid out as attn_partial returns them."""
    o = np.ascontiguousarray(o_partial, dtype=np.float64)
    lse = np.ascontiguousarray(lse_partial, dtype=np.float64)
    sl, hid = _i32(seq_lens), _i32(head_ids)
    B, rows, max_chunks, D = o.shape
    shp = _Shape(B, n_q_heads, n_kv_heads, D, 16, 0, 0, 0)
    out = np.full((B, n_q_heads, D), fill, dtype=np.float64)
    rc = lib().oracle_attn_merge(C.byref(shp), _ptr(o), _ptr(lse), _ptr(sl), _ptr(hid),
                                 C.c_int32(len(hid)), C.c_int32(chunk_tokens),
                                 C.c_int32(max_chunks), _ptr(out))
    if rc != 0:
        raise RuntimeError(f"oracle_attn_merge failed: {rc}")
    return out
