"""Python face of the CPU checker (TEST INFRASTRUCTURE ONLY).

Thin ctypes wrappers around oracle/hetis_oracle.c (Attention: numpy arrays in,
fp64 numpy arrays out) and oracle/hetis_kv_oracle.c (cache store / fetch / tile
copy: 16-bit arrays in and out).  Only tests, the smoke check and the benchmark's cpu_baseline leg
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
                     "oracle_attn_decode_pairs", "oracle_max_threads", "oracle_kv_store", "oracle_kv_append",
                     "oracle_kv_fetch", "oracle_kv_copy_tiles", "oracle_kv_append_pairs"):
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


def attn_decode_pairs(q, k_tiles, v_tiles, block_table, seq_lens, pair_seq, pair_head, n_kv_heads,
                      scale, fill=np.nan):
    """fp64 [B, Hq, D] for a list of (sequence, KV head) pairs over a pool of single-head tiles
    [num_tiles, 16, D] with one block-table row per pair; rows no pair names keep `fill`."""
    q, k, v = _u16(q), _u16(k_tiles), _u16(v_tiles)
    bt, sl = _i32(block_table), _i32(seq_lens)
    ps, ph = _i32(pair_seq), _i32(pair_head)
    B, Hq, D = q.shape
    nt, bs, D2 = k.shape
    assert D == D2 and bt.shape[0] == len(ps) == len(ph)
    shp = _Shape(B, Hq, n_kv_heads, D, bs, bt.shape[1], bs * D, 0)
    out = np.full(q.shape, fill, dtype=np.float64)
    rc = lib().oracle_attn_decode_pairs(C.byref(shp), _ptr(q), _ptr(k), _ptr(v), _ptr(bt),
                                        _ptr(sl), _ptr(ps), _ptr(ph), C.c_int32(len(ps)),
                                        C.c_double(scale), _ptr(out))
    if rc != 0:
        raise RuntimeError(f"oracle_attn_decode_pairs failed: {rc}")
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


# ---------------------------------------------------------------- cache management

class _Pool(C.Structure):
    _fields_ = [("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("block_size", C.c_int32),
                ("num_blocks", C.c_int32),
                ("kv_stride_block", C.c_int64), ("kv_stride_head", C.c_int64)]


def _cache_geometry(cache, strides):
    """(num_blocks, Hkv, block_size, D, stride_block, stride_head) of a [nb, Hkv, bs, D] pool,
    or of a flat buffer described by strides = (nb, Hkv, bs, D, stride_block, stride_head)."""
    if strides is not None:
        return tuple(int(x) for x in strides)
    nb, Hkv, bs, D = cache.shape
    return nb, Hkv, bs, D, Hkv * bs * D, bs * D


def _opt_i32(a):
    return None if a is None else _i32(a)


def _opt_ptr(a):
    return None if a is None else _ptr(a)


def kv_store(k_cache, v_cache, k_new, v_new, token_seq, token_pos, block_table, head_ids,
             strides=None):
    """Copies of the two caches with rows k_new[n, g], v_new[n, g] stored at
    (token_seq[n], token_pos[n], g) for g in head_ids.  token_seq=None: entry n is sequence n."""
    k, v = _u16(k_cache).copy(), _u16(v_cache).copy()
    kn, vn = _u16(k_new), _u16(v_new)
    nb, Hkv, bs, D, sb, sh = _cache_geometry(k, strides)
    assert kn.shape[1:] == (Hkv, D) and vn.shape == kn.shape
    bt, hid, pos, seq = _i32(block_table), _i32(head_ids), _i32(token_pos), _opt_i32(token_seq)
    shp = _Shape(bt.shape[0], Hkv, Hkv, D, bs, bt.shape[1], sb, sh)
    rc = lib().oracle_kv_store(C.byref(shp), _ptr(kn), _ptr(vn), _opt_ptr(seq), _ptr(pos),
                               C.c_int32(len(pos)), _ptr(bt), _ptr(hid), C.c_int32(len(hid)),
                               C.c_int32(nb), _ptr(k), _ptr(v))
    if rc != 0:
        raise RuntimeError(f"oracle_kv_store failed: {rc}")
    return k, v


def kv_append(k_cache, v_cache, k_new, v_new, block_table, seq_lens, head_ids, strides=None):
    """Copies of the two caches with the new row of every sequence stored at seq_lens[b] - 1."""
    k, v = _u16(k_cache).copy(), _u16(v_cache).copy()
    kn, vn = _u16(k_new), _u16(v_new)
    nb, Hkv, bs, D, sb, sh = _cache_geometry(k, strides)
    bt, hid, sl = _i32(block_table), _i32(head_ids), _i32(seq_lens)
    assert kn.shape == (bt.shape[0], Hkv, D) and vn.shape == kn.shape
    shp = _Shape(bt.shape[0], Hkv, Hkv, D, bs, bt.shape[1], sb, sh)
    rc = lib().oracle_kv_append(C.byref(shp), _ptr(kn), _ptr(vn), _ptr(bt), _ptr(sl), _ptr(hid),
                                C.c_int32(len(hid)), C.c_int32(nb), _ptr(k), _ptr(v))
    if rc != 0:
        raise RuntimeError(f"oracle_kv_append failed: {rc}")
    return k, v


def kv_append_pairs(k_tiles, v_tiles, k_new, v_new, block_table, seq_lens, pair_seq, pair_head):
    """Copies of the two tile pools [num_tiles, 16, D] with the new row of every (sequence, KV
    head) pair stored at seq_lens[b] - 1 through the pair's own block-table row."""
    k, v = _u16(k_tiles).copy(), _u16(v_tiles).copy()
    kn, vn = _u16(k_new), _u16(v_new)
    nt, bs, D = k.shape
    B, Hkv, D2 = kn.shape
    bt, sl, ps, ph = _i32(block_table), _i32(seq_lens), _i32(pair_seq), _i32(pair_head)
    assert D == D2 and vn.shape == kn.shape and bt.shape[0] == len(ps) == len(ph) and len(sl) == B
    shp = _Shape(B, Hkv, Hkv, D, bs, bt.shape[1], bs * D, 0)
    rc = lib().oracle_kv_append_pairs(C.byref(shp), _ptr(kn), _ptr(vn), _ptr(bt), _ptr(sl), _ptr(ps),
                                      _ptr(ph), C.c_int32(len(ps)), C.c_int32(nt), _ptr(k), _ptr(v))
    if rc != 0:
        raise RuntimeError(f"oracle_kv_append_pairs failed: {rc}")
    return k, v


def kv_fetch(k_cache, v_cache, token_seq, token_pos, block_table, head_ids, fill=0xFFFF,
             strides=None):
    """(k_out, v_out) uint16 [n_tokens, Hkv, D]; rows not fetched keep `fill`."""
    k, v = _u16(k_cache), _u16(v_cache)
    nb, Hkv, bs, D, sb, sh = _cache_geometry(k, strides)
    bt, hid, pos, seq = _i32(block_table), _i32(head_ids), _i32(token_pos), _opt_i32(token_seq)
    ko = np.full((len(pos), Hkv, D), fill, dtype=np.uint16)
    vo = np.full((len(pos), Hkv, D), fill, dtype=np.uint16)
    shp = _Shape(bt.shape[0], Hkv, Hkv, D, bs, bt.shape[1], sb, sh)
    rc = lib().oracle_kv_fetch(C.byref(shp), _ptr(k), _ptr(v), _opt_ptr(seq), _ptr(pos),
                               C.c_int32(len(pos)), _ptr(bt), _ptr(hid), C.c_int32(len(hid)),
                               C.c_int32(nb), _ptr(ko), _ptr(vo))
    if rc != 0:
        raise RuntimeError(f"oracle_kv_fetch failed: {rc}")
    return ko, vo


def kv_copy_tiles(src_k, src_v, dst_k, dst_v, src_blocks, dst_blocks, src_heads, dst_heads,
                  src_strides=None, dst_strides=None):
    """Copies of the destination caches with tile (src_blocks[i], src_heads[j]) of the source
    written to (dst_blocks[i], dst_heads[j]) for every i, j."""
    sk, sv = _u16(src_k), _u16(src_v)
    dk, dv = _u16(dst_k).copy(), _u16(dst_v).copy()
    snb, sH, sbs, sD, ssb, ssh = _cache_geometry(sk, src_strides)
    dnb, dH, dbs, dD, dsb, dsh = _cache_geometry(dk, dst_strides)
    sp, dp = _Pool(sH, sD, sbs, snb, ssb, ssh), _Pool(dH, dD, dbs, dnb, dsb, dsh)
    sbk, dbk, sh_, dh_ = _i32(src_blocks), _i32(dst_blocks), _i32(src_heads), _i32(dst_heads)
    assert len(sbk) == len(dbk) and len(sh_) == len(dh_)
    rc = lib().oracle_kv_copy_tiles(C.byref(sp), _ptr(sk), _ptr(sv), C.byref(dp), _ptr(dk),
                                    _ptr(dv), _ptr(sbk), _ptr(dbk), C.c_int32(len(sbk)),
                                    _ptr(sh_), _ptr(dh_), C.c_int32(len(sh_)))
    if rc != 0:
        raise RuntimeError(f"oracle_kv_copy_tiles failed: {rc}")
    return dk, dv


# ---------------------------------------------------------------- Profiler model (Eq. (3))

def profiler_fit(h, g, tau):
    """Least-squares (a, b, c) of tau = a*h + b*g + c (Section 5.1, Eq. (3)) and the mean
    relative accuracy 1 - mean |prediction - tau| / tau on the samples.  The definition,
    written with numpy's least-squares routine on the plain design matrix [h, g, 1]."""
    h, g, tau = (np.asarray(x, dtype=np.float64) for x in (h, g, tau))
    X = np.stack([h, g, np.ones_like(h)], axis=1)
    abc, _, rank, _ = np.linalg.lstsq(X, tau, rcond=None)
    if rank < 3:
        raise ValueError("samples do not determine a, b, c")
    acc = 1.0 - float(np.mean(np.abs(X @ abc - tau) / tau))
    return abc, acc


def profiler_fit_nonneg(h, g, tau):
    """The same least-squares problem under a >= 0 and b >= 0 (the Dispatcher of Section 5.2
    uses a and b as costs), handed to scipy's bounded least-squares routine on columns scaled
    to unit size.  Returns ((a, b, c), accuracy)."""
    from scipy.optimize import lsq_linear
    h, g, tau = (np.asarray(x, dtype=np.float64) for x in (h, g, tau))
    X = np.stack([h, g, np.ones_like(h)], axis=1)
    scale = np.abs(X).max(axis=0)
    if not (scale > 0).all():
        raise ValueError("samples do not determine a, b, c")
    res = lsq_linear(X / scale, tau, bounds=([0.0, 0.0, -np.inf], [np.inf, np.inf, np.inf]),
                     method="bvls", tol=1e-14)
    abc = res.x / scale
    acc = 1.0 - float(np.mean(np.abs(X @ abc - tau) / tau))
    return abc, acc


# ---------------------------------------------------------------- Dispatcher (Eq. (7))

def dispatch(devices, lengths, n_heads, r):
    """See oracle/dispatch_oracle.py."""
    from . import dispatch_oracle
    return dispatch_oracle.dispatch(devices, lengths, n_heads, r)
