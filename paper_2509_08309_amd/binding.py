"""ctypes binding of libhetis_attn.so: same names as include/hetis_attn.h and include/hetis_kv.h.

Argument marshalling only.  Tensors are torch tensors that already live on the
GPU (PyTorch is used for device memory and streams, nothing else); every
function passes raw device pointers to the C ABI and returns its status.  The
library is loaded on first use and loading fails loudly when it has not been
built: there is no CPU fallback of any kind.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
# HETIS_ATTN_LIB (optional) points at another build of the same library, e.g. a tuning variant.
LIB_PATH = os.environ.get("HETIS_ATTN_LIB") or os.path.join(HERE, "libhetis_attn.so")

HETIS_OK = 0
HETIS_ERR_NULL = -1
HETIS_ERR_BAD_SHAPE = -2
HETIS_ERR_UNSUPPORTED = -3
HETIS_ERR_BAD_HEADS = -4
HETIS_ERR_WORKSPACE = -5
HETIS_ERR_LAUNCH = -6
HETIS_ERR_ALLOC = -7
HETIS_ERR_BAD_CONTENT = -8
HETIS_ERR_INFEASIBLE = -9
HETIS_ERR_DEVICE_WAIT = -10
HETIS_ATTN_CONTROL_BYTES = 256
HETIS_ATTN_STATIC_SCRATCH_BYTES = 32 << 20


class hetis_attn_shape(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("block_size", C.c_int32),
                ("max_blocks_per_seq", C.c_int32),
                ("kv_stride_block", C.c_int64), ("kv_stride_head", C.c_int64)]


class hetis_kv_pool(C.Structure):
    _fields_ = [("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("block_size", C.c_int32),
                ("reserved", C.c_int32), ("num_blocks", C.c_int64),
                ("kv_stride_block", C.c_int64), ("kv_stride_head", C.c_int64)]


class hetis_dispatch_device(C.Structure):
    _fields_ = [("a", C.c_double), ("b", C.c_double), ("c", C.c_double), ("gamma", C.c_double),
                ("beta", C.c_double), ("h", C.c_double), ("g", C.c_double),
                ("capacity", C.c_double), ("is_primary", C.c_int32), ("reserved", C.c_int32)]


class HetisError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({hetis_attn_status_string(status)})")


_lib = None


def load(build_if_missing: bool = False):
    """Load the built library; optionally build it first when nothing is built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if build_if_missing:
            from .build import build
            build()
        else:
            raise FileNotFoundError(
                f"{LIB_PATH} is not built; run `python -m paper_2509_08309_amd.build` "
                "(the HIP library is required, there is no fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    shp = C.POINTER(hetis_attn_shape)
    lib.hetis_attn_version.restype = C.c_int
    lib.hetis_attn_version.argtypes = []
    lib.hetis_attn_status_string.restype = C.c_char_p
    lib.hetis_attn_status_string.argtypes = [C.c_int]
    lib.hetis_attn_decode.restype = C.c_int
    lib.hetis_attn_decode.argtypes = [shp, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp]
    lib.hetis_attn_release_workspace.restype = C.c_int
    lib.hetis_attn_release_workspace.argtypes = []
    lib.hetis_attn_reserve_workspace.restype = C.c_int
    lib.hetis_attn_reserve_workspace.argtypes = [C.c_size_t]
    lib.hetis_attn_decode_ws.restype = C.c_int
    lib.hetis_attn_decode_ws.argtypes = [shp, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp, C.c_size_t, vp]
    lib.hetis_attn_decode_step.restype = C.c_int
    lib.hetis_attn_decode_step.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp]
    lib.hetis_attn_decode_step_ws.restype = C.c_int
    lib.hetis_attn_decode_step_ws.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp,
                                              C.c_size_t, vp]
    lib.hetis_attn_decode_static.restype = C.c_int
    lib.hetis_attn_decode_static.argtypes = [shp, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp]
    lib.hetis_attn_decode_workspace_bytes.restype = C.c_int
    lib.hetis_attn_decode_workspace_bytes.argtypes = [shp, i32, C.POINTER(C.c_size_t)]
    lib.hetis_attn_decode_pairs_workspace_bytes.restype = C.c_int
    lib.hetis_attn_decode_pairs_workspace_bytes.argtypes = [shp, i32, C.POINTER(C.c_size_t)]
    lib.hetis_attn_workspace_init.restype = C.c_int
    lib.hetis_attn_workspace_init.argtypes = [vp, C.c_size_t, vp]
    lib.hetis_attn_workspace_status.restype = C.c_int
    lib.hetis_attn_workspace_status.argtypes = [vp, vp, C.POINTER(C.c_uint32)]
    lib.hetis_attn_decode_split_ws.restype = C.c_int
    lib.hetis_attn_decode_split_ws.argtypes = [shp, vp, vp, vp, vp, vp, vp, i32, f32, i32, i32,
                                               vp, vp, vp, vp]
    lib.hetis_attn_decode_pairs_step.restype = C.c_int
    lib.hetis_attn_decode_pairs_step.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp]
    lib.hetis_attn_decode_pairs_step_ws.restype = C.c_int
    lib.hetis_attn_decode_pairs_step_ws.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, f32, vp,
                                                    vp, C.c_size_t, vp]
    lib.hetis_attn_decode_pairs_ws.restype = C.c_int
    lib.hetis_attn_decode_pairs_ws.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp,
                                               C.c_size_t, vp]
    lib.hetis_attn_split_num_chunks.restype = C.c_int
    lib.hetis_attn_split_num_chunks.argtypes = [i32, i32]
    lib.hetis_attn_split_workspace_bytes.restype = C.c_int
    lib.hetis_attn_split_workspace_bytes.argtypes = [shp, i32, i32, i32, C.POINTER(C.c_size_t),
                                                     C.POINTER(C.c_size_t)]
    lib.hetis_attn_decode_split.restype = C.c_int
    lib.hetis_attn_decode_split.argtypes = [shp, vp, vp, vp, vp, vp, vp, i32, f32, i32, i32,
                                            vp, vp, vp]
    lib.hetis_attn_merge.restype = C.c_int
    lib.hetis_attn_merge.argtypes = [shp, vp, vp, vp, vp, i32, i32, i32, vp, vp]
    lib.hetis_attn_profile_events.restype = C.c_int
    lib.hetis_attn_profile_events.argtypes = [vp, vp]
    lib.hetis_attn_validate.restype = C.c_int
    lib.hetis_attn_validate.argtypes = [shp, vp, vp, vp, i32, i64, vp]
    lib.hetis_attn_decode_pairs.restype = C.c_int
    lib.hetis_attn_decode_pairs.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp]
    lib.hetis_attn_validate_pairs.restype = C.c_int
    lib.hetis_attn_validate_pairs.argtypes = [shp, vp, vp, vp, vp, i32, i64, vp]
    lib.hetis_dispatch_solve.restype = C.c_int
    lib.hetis_dispatch_solve.argtypes = [vp, i32, vp, i32, i32, i32, vp, vp, vp, vp]
    lib.hetis_profiler_fit.restype = C.c_int
    lib.hetis_profiler_fit.argtypes = [vp, vp, vp, i32, vp, vp]
    lib.hetis_profiler_fit_nonneg.restype = C.c_int
    lib.hetis_profiler_fit_nonneg.argtypes = [vp, vp, vp, i32, vp, vp]
    lib.hetis_profiler_predict.restype = C.c_int
    lib.hetis_profiler_predict.argtypes = [vp, vp, vp, i32, vp]
    pool = C.POINTER(hetis_kv_pool)
    lib.hetis_kv_append.restype = C.c_int
    lib.hetis_kv_append.argtypes = [shp, vp, vp, vp, vp, vp, i32, i64, vp, vp, vp]
    lib.hetis_kv_append_pairs.restype = C.c_int
    lib.hetis_kv_append_pairs.argtypes = [shp, vp, vp, vp, vp, vp, vp, i32, i64, vp, vp, vp]
    lib.hetis_kv_store.restype = C.c_int
    lib.hetis_kv_store.argtypes = [shp, vp, vp, vp, vp, i32, vp, vp, i32, i64, vp, vp, vp]
    lib.hetis_kv_fetch.restype = C.c_int
    lib.hetis_kv_fetch.argtypes = [shp, vp, vp, vp, vp, i32, vp, vp, i32, i64, vp, vp, vp]
    lib.hetis_kv_copy_tiles.restype = C.c_int
    lib.hetis_kv_copy_tiles.argtypes = [pool, vp, vp, pool, vp, vp, vp, vp, i32, vp, vp, i32, vp]
    lib.hetis_kv_profile_events.restype = C.c_int
    lib.hetis_kv_profile_events.argtypes = [vp, vp]
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor / numpy array / raw int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return t.ctypes.data            # numpy array (host pointer)


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def make_shape(batch, n_q_heads, n_kv_heads, head_dim, max_blocks_per_seq, block_size=16,
               kv_stride_block=0, kv_stride_head=0) -> hetis_attn_shape:
    return hetis_attn_shape(batch, n_q_heads, n_kv_heads, head_dim, block_size,
                            max_blocks_per_seq, kv_stride_block, kv_stride_head)


def hetis_attn_version() -> int:
    return load().hetis_attn_version()


def hetis_attn_status_string(status: int) -> str:
    return load().hetis_attn_status_string(status).decode()


def hetis_attn_decode(shape, q, k_cache, v_cache, block_table, seq_lens, head_ids, n_sel_heads,
                      scale, out, stream=None) -> int:
    return load().hetis_attn_decode(C.byref(shape), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                    _ptr(block_table), _ptr(seq_lens), _ptr(head_ids),
                                    int(n_sel_heads), float(scale), _ptr(out), _stream(stream))


def hetis_attn_decode_ws(shape, q, k_cache, v_cache, block_table, seq_lens, head_ids, n_sel_heads,
                         scale, out, workspace, workspace_bytes, stream=None) -> int:
    return load().hetis_attn_decode_ws(C.byref(shape), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                       _ptr(block_table), _ptr(seq_lens), _ptr(head_ids),
                                       int(n_sel_heads), float(scale), _ptr(out), _ptr(workspace),
                                       int(workspace_bytes), _stream(stream))


def hetis_attn_decode_step(shape, q, k_new, v_new, k_cache, v_cache, block_table, seq_lens, head_ids,
                           n_sel_heads, scale, out, stream=None) -> int:
    return load().hetis_attn_decode_step(C.byref(shape), _ptr(q), _ptr(k_new), _ptr(v_new),
                                         _ptr(k_cache), _ptr(v_cache), _ptr(block_table),
                                         _ptr(seq_lens), _ptr(head_ids), int(n_sel_heads),
                                         float(scale), _ptr(out), _stream(stream))


def hetis_attn_decode_step_ws(shape, q, k_new, v_new, k_cache, v_cache, block_table, seq_lens,
                              head_ids, n_sel_heads, scale, out, workspace, workspace_bytes,
                              stream=None) -> int:
    return load().hetis_attn_decode_step_ws(C.byref(shape), _ptr(q), _ptr(k_new), _ptr(v_new),
                                            _ptr(k_cache), _ptr(v_cache), _ptr(block_table),
                                            _ptr(seq_lens), _ptr(head_ids), int(n_sel_heads),
                                            float(scale), _ptr(out), _ptr(workspace),
                                            int(workspace_bytes), _stream(stream))


def hetis_attn_decode_static(shape, q, k_cache, v_cache, block_table, seq_lens, head_ids,
                             n_sel_heads, scale, out, stream=None) -> int:
    return load().hetis_attn_decode_static(C.byref(shape), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                           _ptr(block_table), _ptr(seq_lens), _ptr(head_ids),
                                           int(n_sel_heads), float(scale), _ptr(out),
                                           _stream(stream))


def hetis_attn_decode_workspace_bytes(shape, n_sel_heads):
    """(status, bytes)."""
    n = C.c_size_t(0)
    rc = load().hetis_attn_decode_workspace_bytes(C.byref(shape), int(n_sel_heads), C.byref(n))
    return rc, n.value


def hetis_attn_decode_pairs_workspace_bytes(shape, n_pairs):
    """(status, bytes)."""
    n = C.c_size_t(0)
    rc = load().hetis_attn_decode_pairs_workspace_bytes(C.byref(shape), int(n_pairs), C.byref(n))
    return rc, n.value


def hetis_attn_workspace_init(workspace, nbytes, stream=None) -> int:
    return load().hetis_attn_workspace_init(_ptr(workspace), int(nbytes), _stream(stream))


def hetis_attn_workspace_status(workspace=None, stream=None):
    """(status, flags); workspace None = the library-owned one of the current device."""
    flags = C.c_uint32(0)
    rc = load().hetis_attn_workspace_status(_ptr(workspace), _stream(stream), C.byref(flags))
    return rc, flags.value


def hetis_attn_reserve_workspace(nbytes: int) -> int:
    return load().hetis_attn_reserve_workspace(int(nbytes))


def hetis_attn_release_workspace() -> int:
    return load().hetis_attn_release_workspace()


def hetis_attn_split_num_chunks(max_seq_len: int, chunk_tokens: int) -> int:
    return load().hetis_attn_split_num_chunks(int(max_seq_len), int(chunk_tokens))


def hetis_attn_split_workspace_bytes(shape, n_sel_heads, max_seq_len, chunk_tokens):
    """(status, o_partial_bytes, lse_partial_bytes)."""
    a, b = C.c_size_t(0), C.c_size_t(0)
    rc = load().hetis_attn_split_workspace_bytes(C.byref(shape), int(n_sel_heads),
                                                 int(max_seq_len), int(chunk_tokens),
                                                 C.byref(a), C.byref(b))
    return rc, a.value, b.value


def hetis_attn_decode_split(shape, q, k_cache, v_cache, block_table, seq_lens, head_ids,
                            n_sel_heads, scale, chunk_tokens, max_seq_len, o_partial,
                            lse_partial, stream=None) -> int:
    return load().hetis_attn_decode_split(C.byref(shape), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                          _ptr(block_table), _ptr(seq_lens), _ptr(head_ids),
                                          int(n_sel_heads), float(scale), int(chunk_tokens),
                                          int(max_seq_len), _ptr(o_partial), _ptr(lse_partial),
                                          _stream(stream))


def hetis_attn_decode_split_ws(shape, q, k_cache, v_cache, block_table, seq_lens, head_ids,
                               n_sel_heads, scale, chunk_tokens, max_seq_len, o_partial,
                               lse_partial, control, stream=None) -> int:
    return load().hetis_attn_decode_split_ws(C.byref(shape), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                             _ptr(block_table), _ptr(seq_lens), _ptr(head_ids),
                                             int(n_sel_heads), float(scale), int(chunk_tokens),
                                             int(max_seq_len), _ptr(o_partial), _ptr(lse_partial),
                                             _ptr(control), _stream(stream))


def hetis_attn_merge(shape, o_partial, lse_partial, seq_lens, head_ids, n_sel_heads,
                     chunk_tokens, max_seq_len, out, stream=None) -> int:
    return load().hetis_attn_merge(C.byref(shape), _ptr(o_partial), _ptr(lse_partial),
                                   _ptr(seq_lens), _ptr(head_ids), int(n_sel_heads),
                                   int(chunk_tokens), int(max_seq_len), _ptr(out),
                                   _stream(stream))


def hetis_attn_profile_events(begin, end) -> int:
    """begin/end: raw hipEvent_t handles (ints, e.g. torch.cuda.Event.cuda_event) or None."""
    return load().hetis_attn_profile_events(begin, end)


def hetis_attn_validate(shape, block_table, seq_lens, head_ids, n_sel_heads, num_blocks,
                        stream=None) -> int:
    return load().hetis_attn_validate(C.byref(shape), _ptr(block_table), _ptr(seq_lens),
                                      _ptr(head_ids), int(n_sel_heads), int(num_blocks),
                                      _stream(stream))


def hetis_attn_decode_pairs(shape, q, k_tiles, v_tiles, block_table, seq_lens, pair_seq, pair_head,
                            n_pairs, scale, out, stream=None) -> int:
    return load().hetis_attn_decode_pairs(C.byref(shape), _ptr(q), _ptr(k_tiles), _ptr(v_tiles),
                                          _ptr(block_table), _ptr(seq_lens), _ptr(pair_seq),
                                          _ptr(pair_head), int(n_pairs), float(scale), _ptr(out),
                                          _stream(stream))


def hetis_attn_decode_pairs_ws(shape, q, k_tiles, v_tiles, block_table, seq_lens, pair_seq,
                               pair_head, n_pairs, scale, out, workspace, workspace_bytes,
                               stream=None) -> int:
    return load().hetis_attn_decode_pairs_ws(C.byref(shape), _ptr(q), _ptr(k_tiles), _ptr(v_tiles),
                                             _ptr(block_table), _ptr(seq_lens), _ptr(pair_seq),
                                             _ptr(pair_head), int(n_pairs), float(scale),
                                             _ptr(out), _ptr(workspace), int(workspace_bytes),
                                             _stream(stream))


def hetis_attn_decode_pairs_step(shape, q, k_new, v_new, k_tiles, v_tiles, block_table, seq_lens,
                                 pair_seq, pair_head, n_pairs, scale, out, stream=None) -> int:
    return load().hetis_attn_decode_pairs_step(C.byref(shape), _ptr(q), _ptr(k_new), _ptr(v_new),
                                               _ptr(k_tiles), _ptr(v_tiles), _ptr(block_table),
                                               _ptr(seq_lens), _ptr(pair_seq), _ptr(pair_head),
                                               int(n_pairs), float(scale), _ptr(out), _stream(stream))


def hetis_attn_decode_pairs_step_ws(shape, q, k_new, v_new, k_tiles, v_tiles, block_table,
                                    seq_lens, pair_seq, pair_head, n_pairs, scale, out, workspace,
                                    workspace_bytes, stream=None) -> int:
    return load().hetis_attn_decode_pairs_step_ws(C.byref(shape), _ptr(q), _ptr(k_new), _ptr(v_new),
                                                  _ptr(k_tiles), _ptr(v_tiles), _ptr(block_table),
                                                  _ptr(seq_lens), _ptr(pair_seq), _ptr(pair_head),
                                                  int(n_pairs), float(scale), _ptr(out),
                                                  _ptr(workspace), int(workspace_bytes),
                                                  _stream(stream))


def hetis_attn_validate_pairs(shape, block_table, seq_lens, pair_seq, pair_head, n_pairs,
                              num_tiles, stream=None) -> int:
    return load().hetis_attn_validate_pairs(C.byref(shape), _ptr(block_table), _ptr(seq_lens),
                                            _ptr(pair_seq), _ptr(pair_head), int(n_pairs),
                                            int(num_tiles), _stream(stream))


def make_pool(n_kv_heads, head_dim, num_blocks, block_size=16, kv_stride_block=0,
              kv_stride_head=0) -> hetis_kv_pool:
    return hetis_kv_pool(n_kv_heads, head_dim, block_size, 0, num_blocks, kv_stride_block,
                         kv_stride_head)


def hetis_kv_append(shape, k_new, v_new, block_table, seq_lens, head_ids, n_sel_heads,
                    num_blocks, k_cache, v_cache, stream=None) -> int:
    return load().hetis_kv_append(C.byref(shape), _ptr(k_new), _ptr(v_new), _ptr(block_table),
                                  _ptr(seq_lens), _ptr(head_ids), int(n_sel_heads),
                                  int(num_blocks), _ptr(k_cache), _ptr(v_cache), _stream(stream))


def hetis_kv_append_pairs(shape, k_new, v_new, block_table, seq_lens, pair_seq, pair_head, n_pairs,
                          num_tiles, k_tiles, v_tiles, stream=None) -> int:
    return load().hetis_kv_append_pairs(C.byref(shape), _ptr(k_new), _ptr(v_new), _ptr(block_table),
                                        _ptr(seq_lens), _ptr(pair_seq), _ptr(pair_head),
                                        int(n_pairs), int(num_tiles), _ptr(k_tiles), _ptr(v_tiles),
                                        _stream(stream))


def hetis_kv_store(shape, k_new, v_new, token_seq, token_pos, n_tokens, block_table, head_ids,
                   n_sel_heads, num_blocks, k_cache, v_cache, stream=None) -> int:
    return load().hetis_kv_store(C.byref(shape), _ptr(k_new), _ptr(v_new), _ptr(token_seq),
                                 _ptr(token_pos), int(n_tokens), _ptr(block_table),
                                 _ptr(head_ids), int(n_sel_heads), int(num_blocks),
                                 _ptr(k_cache), _ptr(v_cache), _stream(stream))


def hetis_kv_fetch(shape, k_cache, v_cache, token_seq, token_pos, n_tokens, block_table,
                   head_ids, n_sel_heads, num_blocks, k_out, v_out, stream=None) -> int:
    return load().hetis_kv_fetch(C.byref(shape), _ptr(k_cache), _ptr(v_cache), _ptr(token_seq),
                                 _ptr(token_pos), int(n_tokens), _ptr(block_table),
                                 _ptr(head_ids), int(n_sel_heads), int(num_blocks), _ptr(k_out),
                                 _ptr(v_out), _stream(stream))


def hetis_kv_copy_tiles(src_pool, src_k, src_v, dst_pool, dst_k, dst_v, src_blocks, dst_blocks,
                        n_pairs, src_heads, dst_heads, n_sel_heads, stream=None) -> int:
    return load().hetis_kv_copy_tiles(
        None if src_pool is None else C.byref(src_pool), _ptr(src_k), _ptr(src_v),
        None if dst_pool is None else C.byref(dst_pool), _ptr(dst_k), _ptr(dst_v),
        _ptr(src_blocks), _ptr(dst_blocks), int(n_pairs), _ptr(src_heads), _ptr(dst_heads),
        int(n_sel_heads), _stream(stream))


def hetis_kv_profile_events(begin, end) -> int:
    """begin/end: raw hipEvent_t handles (ints) or None."""
    return load().hetis_kv_profile_events(begin, end)


def hetis_profiler_fit(h, g, tau, n, abc, accuracy=None) -> int:
    """h, g, tau, abc: contiguous float64 numpy arrays (host); accuracy: ctypes.c_double or None."""
    acc = None if accuracy is None else C.byref(accuracy)
    return load().hetis_profiler_fit(_ptr(h), _ptr(g), _ptr(tau), int(n), _ptr(abc),
                                     C.cast(acc, C.c_void_p) if acc is not None else None)


def hetis_profiler_fit_nonneg(h, g, tau, n, abc, accuracy=None) -> int:
    """As hetis_profiler_fit, under a >= 0 and b >= 0."""
    acc = None if accuracy is None else C.byref(accuracy)
    return load().hetis_profiler_fit_nonneg(_ptr(h), _ptr(g), _ptr(tau), int(n), _ptr(abc),
                                            C.cast(acc, C.c_void_p) if acc is not None else None)


def hetis_profiler_predict(abc, h, g, n, tau_out) -> int:
    return load().hetis_profiler_predict(_ptr(abc), _ptr(h), _ptr(g), int(n), _ptr(tau_out))


def hetis_dispatch_solve(devices, n_devices, lengths, n_requests, n_heads, group, x_frac, x_heads,
                         z_lp=None, z_rounded=None) -> int:
    """devices: ctypes array of hetis_dispatch_device (or None); lengths, x_frac: float64 numpy
    arrays; x_heads: int32 numpy array; z_lp, z_rounded: ctypes.c_double or None."""
    dp = None if devices is None else C.cast(devices, C.c_void_p)
    ref = lambda v: None if v is None else C.cast(C.byref(v), C.c_void_p)
    return load().hetis_dispatch_solve(dp, int(n_devices), _ptr(lengths), int(n_requests),
                                       int(n_heads), int(group), _ptr(x_frac), _ptr(x_heads),
                                       ref(z_lp), ref(z_rounded))


def check(status: int, where: str = "hetis_attn") -> None:
    if status != HETIS_OK:
        raise HetisError(status, where)
