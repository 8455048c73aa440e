"""Host-side checks of the C ABI that need no GPU: exported symbols and argument errors."""
import ctypes as C
import os
import re

import pytest

import paper_2509_08309_amd as H
from paper_2509_08309_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return binding.load(build_if_missing=True)


def declared_functions():
    names = []
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names += re.findall(r"\b(hetis_(?:attn|kv|profiler|dispatch)_\w+)\s*\(", text)
    return sorted(set(names))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert len(names) >= 14 and "hetis_kv_copy_tiles" in names
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/ but not exported"
        assert hasattr(binding, n), f"{n} has no Python binding of the same name"


def test_version_and_status_strings(lib):
    assert H.hetis_attn_version() >= 100
    seen = {H.hetis_attn_status_string(s) for s in range(0, -11, -1)}
    assert len(seen) == 11 and "unknown status" not in seen
    assert H.hetis_attn_status_string(-99) == "unknown status"


P = 0x1000  # a non-null fake pointer: every call below must fail before touching it


def good():
    return H.make_shape(4, 8, 8, 64, 16)


def decode(shape, n_sel=4, **kw):
    a = dict(q=P, k=P, v=P, bt=P, sl=P, hid=P, out=P)
    a.update(kw)
    return H.hetis_attn_decode(shape, a["q"], a["k"], a["v"], a["bt"], a["sl"], a["hid"], n_sel,
                               0.125, a["out"], 0)


@pytest.mark.parametrize("arg", ["q", "k", "v", "bt", "sl", "hid", "out"])
def test_null_pointers(lib, arg):
    assert decode(good(), **{arg: None}) == binding.HETIS_ERR_NULL


def test_null_shape(lib):
    rc = lib.hetis_attn_decode(None, P, P, P, P, P, P, 4, 0.125, P, None)
    assert rc == binding.HETIS_ERR_NULL


@pytest.mark.parametrize("field,value,status", [
    ("batch", 0, binding.HETIS_ERR_BAD_SHAPE),
    ("batch", -3, binding.HETIS_ERR_BAD_SHAPE),
    ("n_q_heads", 0, binding.HETIS_ERR_BAD_SHAPE),
    ("n_kv_heads", 3, binding.HETIS_ERR_BAD_SHAPE),       # 8 % 3 != 0
    ("max_blocks_per_seq", 0, binding.HETIS_ERR_BAD_SHAPE),
    ("kv_stride_head", -8, binding.HETIS_ERR_BAD_SHAPE),
    ("kv_stride_head", 1028, binding.HETIS_ERR_BAD_SHAPE),  # not a multiple of 8
    ("kv_stride_head", 512, binding.HETIS_ERR_BAD_SHAPE),   # smaller than a tile
    ("head_dim", 96, binding.HETIS_ERR_UNSUPPORTED),
    ("head_dim", 256, binding.HETIS_ERR_UNSUPPORTED),
    ("block_size", 32, binding.HETIS_ERR_UNSUPPORTED),
    ("n_kv_heads", 1, binding.HETIS_ERR_BAD_HEADS),        # r = 8 fine, but n_sel = 4 > 1
    ("batch", 70000, binding.HETIS_ERR_UNSUPPORTED),
])
def test_bad_shapes(lib, field, value, status):
    s = good()
    setattr(s, field, value)
    assert decode(s) == status


def test_unsupported_group_size(lib):
    s = H.make_shape(4, 24, 8, 64, 16)       # r = 3
    assert decode(s) == binding.HETIS_ERR_UNSUPPORTED
    s = H.make_shape(4, 128, 8, 64, 16)      # r = 16
    assert decode(s) == binding.HETIS_ERR_UNSUPPORTED


@pytest.mark.parametrize("n_sel", [0, -1, 9])
def test_bad_head_count(lib, n_sel):
    assert decode(good(), n_sel=n_sel) == binding.HETIS_ERR_BAD_HEADS


def test_split_argument_errors(lib):
    s = good()
    assert H.hetis_attn_split_num_chunks(255, 512) == 1
    assert H.hetis_attn_split_num_chunks(32768, 512) == 64
    assert H.hetis_attn_split_num_chunks(513, 512) == 2
    assert H.hetis_attn_split_num_chunks(100, 0) == binding.HETIS_ERR_UNSUPPORTED
    assert H.hetis_attn_split_num_chunks(100, 24) == binding.HETIS_ERR_UNSUPPORTED
    assert H.hetis_attn_split_num_chunks(0, 16) == binding.HETIS_ERR_WORKSPACE
    # a wave keeps the block ids of a chunk in one register: at most 64 blocks = 1024 tokens
    assert H.hetis_attn_split_num_chunks(4096, 1024) == 4
    assert H.hetis_attn_split_num_chunks(4096, 1040) == binding.HETIS_ERR_UNSUPPORTED
    rc, ob, lb = H.hetis_attn_split_workspace_bytes(s, 4, 256, 48)
    assert rc == 0 and ob == 4 * 4 * 6 * 64 * 4 and lb == 4 * 4 * 6 * 4
    assert H.hetis_attn_split_workspace_bytes(s, 4, 257, 48)[0] == binding.HETIS_ERR_WORKSPACE
    assert H.hetis_attn_split_workspace_bytes(s, 4, 256, 40)[0] == binding.HETIS_ERR_UNSUPPORTED
    assert H.hetis_attn_split_workspace_bytes(s, 0, 256, 48)[0] == binding.HETIS_ERR_BAD_HEADS

    def split(chunk=48, msl=256, o=P, lse=P, n_sel=4):
        return H.hetis_attn_decode_split(s, P, P, P, P, P, P, n_sel, 0.125, chunk, msl, o, lse, 0)
    assert split(o=None) == binding.HETIS_ERR_NULL
    assert split(lse=None) == binding.HETIS_ERR_NULL
    assert split(chunk=8) == binding.HETIS_ERR_UNSUPPORTED
    assert split(chunk=2048) == binding.HETIS_ERR_UNSUPPORTED
    assert split(msl=0) == binding.HETIS_ERR_WORKSPACE
    assert split(msl=4096) == binding.HETIS_ERR_WORKSPACE
    assert split(n_sel=9) == binding.HETIS_ERR_BAD_HEADS

    def merge(chunk=48, msl=256, o=P, lse=P, out=P):
        return H.hetis_attn_merge(s, o, lse, P, P, 4, chunk, msl, out, 0)
    assert merge(o=None) == binding.HETIS_ERR_NULL
    assert merge(out=None) == binding.HETIS_ERR_NULL
    assert merge(chunk=-16) == binding.HETIS_ERR_UNSUPPORTED
    assert merge(msl=257) == binding.HETIS_ERR_WORKSPACE


def test_validate_argument_errors(lib):
    s = good()
    assert H.hetis_attn_validate(s, None, P, P, 4, 10, 0) == binding.HETIS_ERR_NULL
    assert H.hetis_attn_validate(s, P, P, P, 4, 0, 0) == binding.HETIS_ERR_BAD_SHAPE
    assert H.hetis_attn_validate(s, P, P, P, 0, 10, 0) == binding.HETIS_ERR_BAD_HEADS


def test_release_workspace_without_gpu_is_ok(lib):
    assert H.hetis_attn_release_workspace() == binding.HETIS_OK
    # nothing was ever allocated: the status of the library-owned workspace needs no HIP call
    assert H.hetis_attn_workspace_status(None, 0) == (binding.HETIS_OK, 0)


WS = 0x10000    # a fake, 256-byte aligned workspace address


def test_workspace_sizes(lib):
    up = lambda x: (x + 255) // 256 * 256
    fixed = 256 + 4 * (1 << 18)
    # 512 or more rows (sequences x selected heads, or pairs): the work is handed out in whole
    # segments.  Rows of up to one segment (4096 tokens) are combined inside a workgroup: a shape
    # whose block table allows no more needs the control words only
    s = H.make_shape(128, 40, 40, 128, 256)
    assert H.hetis_attn_decode_workspace_bytes(s, 13) == (0, 256)
    assert H.hetis_attn_decode_pairs_workspace_bytes(s, 1721) == (0, 256)
    assert H.hetis_attn_decode_workspace_bytes(H.make_shape(256, 64, 8, 128, 256), 3) == (0, 256)
    # longer rows: control words, a fixed area of 2^18 arrival counters, then one partial result
    # of (D + 1) floats per segment and query row; each area rounded up to 256 bytes.
    # up to 32768 tokens = 8 segments
    long = H.make_shape(64, 40, 40, 128, 2048)
    rows = 64 * 40 * 8
    assert H.hetis_attn_decode_workspace_bytes(long, 40) == (0, fixed + rows * 128 * 4 + up(rows * 4))
    # a grouped-query shape with up to 8192 tokens: 2 segments, r = 8 rows each
    rows = 256 * 3 * 2 * 8
    assert H.hetis_attn_decode_workspace_bytes(H.make_shape(256, 64, 8, 128, 512), 3) \
        == (0, fixed + rows * 128 * 4 + up(rows * 4))
    # one block more than a whole number of segments: one more segment
    rows = 300 * 5 * 2 * 1
    assert H.hetis_attn_decode_workspace_bytes(H.make_shape(300, 8, 8, 64, 257), 5) \
        == (0, fixed + rows * 64 * 4 + up(rows * 4))
    assert H.hetis_attn_decode_pairs_workspace_bytes(long, 0) == (0, 256)
    rows = 777 * 8
    assert H.hetis_attn_decode_pairs_workspace_bytes(long, 777) \
        == (0, fixed + rows * 128 * 4 + up(rows * 4))
    # fewer than 512 rows: the work is handed out in single chunks, whose results all pass
    # through the workspace: one slot per chunk of a whole segment (4096 / 256 = 16, grouped-query
    # shapes 4096 / 512 = 8) and segment the block table allows
    rows = 4 * 4 * 16
    assert H.hetis_attn_decode_workspace_bytes(H.make_shape(4, 8, 8, 64, 16), 4) \
        == (0, fixed + rows * 64 * 4 + up(rows * 4))
    rows = 8 * 40 * 8 * 16
    assert H.hetis_attn_decode_workspace_bytes(H.make_shape(8, 40, 40, 128, 2048), 40) \
        == (0, fixed + rows * 128 * 4 + up(rows * 4))
    rows = 3 * 5 * 2 * 16
    assert H.hetis_attn_decode_workspace_bytes(H.make_shape(3, 8, 8, 64, 257), 5) \
        == (0, fixed + rows * 64 * 4 + up(rows * 4))
    rows = 77 * 8 * 16
    assert H.hetis_attn_decode_pairs_workspace_bytes(long, 77) \
        == (0, fixed + rows * 128 * 4 + up(rows * 4))
    rows = 16 * 3 * 2 * 8 * 8
    assert H.hetis_attn_decode_workspace_bytes(H.make_shape(16, 64, 8, 128, 512), 3) \
        == (0, fixed + rows * 128 * 4 + up(rows * 4))
    assert H.hetis_attn_decode_workspace_bytes(s, 0)[0] == binding.HETIS_ERR_BAD_HEADS
    assert H.hetis_attn_decode_workspace_bytes(H.make_shape(4, 8, 8, 96, 16), 4)[0] == binding.HETIS_ERR_UNSUPPORTED
    assert H.hetis_attn_decode_pairs_workspace_bytes(s, -1)[0] == binding.HETIS_ERR_BAD_SHAPE
    assert H.hetis_attn_decode_pairs_workspace_bytes(s, 65536)[0] == binding.HETIS_ERR_UNSUPPORTED
    assert lib.hetis_attn_decode_workspace_bytes(C.byref(s), 13, None) == binding.HETIS_ERR_NULL


def test_decode_step_argument_errors(lib):
    s = good()

    def call(kn=P, vn=P, q=P, n_sel=4, ws=None):
        if ws is None:
            return H.hetis_attn_decode_step(s, q, kn, vn, P, P, P, P, P, n_sel, 0.125, P, 0)
        return H.hetis_attn_decode_step_ws(s, q, kn, vn, P, P, P, P, P, n_sel, 0.125, P, ws[0], ws[1], 0)
    assert call(kn=None) == binding.HETIS_ERR_NULL
    assert call(vn=None) == binding.HETIS_ERR_NULL
    assert call(q=None) == binding.HETIS_ERR_NULL
    assert call(n_sel=0) == binding.HETIS_ERR_BAD_HEADS
    assert call(ws=(None, 256)) == binding.HETIS_ERR_NULL
    assert call(ws=(WS, 128)) == binding.HETIS_ERR_WORKSPACE
    assert call(kn=None, ws=(WS, 256)) == binding.HETIS_ERR_NULL


def test_static_scratch_entry_point_argument_errors(lib):
    s = good()
    call = lambda shape=s, n_sel=4, q=P: H.hetis_attn_decode_static(shape, q, P, P, P, P, P, n_sel,
                                                                    0.125, P, 0)
    assert call(q=None) == binding.HETIS_ERR_NULL
    assert call(n_sel=9) == binding.HETIS_ERR_BAD_HEADS
    assert call(shape=H.make_shape(4, 8, 8, 96, 16)) == binding.HETIS_ERR_UNSUPPORTED
    # a shape whose workspace exceeds the static array is refused before any HIP call
    big = H.make_shape(2048, 40, 40, 128, 2048)
    assert H.hetis_attn_decode_workspace_bytes(big, 40)[1] > binding.HETIS_ATTN_STATIC_SCRATCH_BYTES
    assert call(shape=big, n_sel=40) == binding.HETIS_ERR_WORKSPACE


def test_ws_entry_points_argument_errors(lib):
    s = H.make_shape(4, 8, 8, 64, 600)                                  # up to 9600 tokens: 3 segments
    rc, need = H.hetis_attn_decode_workspace_bytes(s, 4)
    assert rc == 0 and need > 256

    def call(ws=WS, nbytes=need, shape=s, n_sel=4, q=P):
        return H.hetis_attn_decode_ws(shape, q, P, P, P, P, P, n_sel, 0.125, P, ws, nbytes, 0)
    assert call(ws=None) == binding.HETIS_ERR_NULL
    assert call(q=None) == binding.HETIS_ERR_NULL
    # a call with few rows works with less than that (it then hands out whole segments, for
    # which one slot per segment is enough), but not with less than what segments need
    rows = 4 * 4 * 3
    seg_need = 256 + 4 * (1 << 18) + rows * 64 * 4 + (rows * 4 + 255) // 256 * 256
    assert seg_need < need
    assert call(nbytes=seg_need - 1) == binding.HETIS_ERR_WORKSPACE
    assert call(ws=WS + 64) == binding.HETIS_ERR_WORKSPACE              # not 256-byte aligned
    assert call(n_sel=9) == binding.HETIS_ERR_BAD_HEADS
    assert call(shape=H.make_shape(4, 8, 8, 96, 16)) == binding.HETIS_ERR_UNSUPPORTED

    def pairs(ws=WS, nbytes=1 << 20, n_pairs=5, ps=P):
        return H.hetis_attn_decode_pairs_ws(s, P, P, P, P, P, ps, P, n_pairs, 0.125, P, ws, nbytes, 0)
    s = good()
    assert pairs(ws=None) == binding.HETIS_ERR_NULL
    assert pairs(ps=None) == binding.HETIS_ERR_NULL
    assert pairs(nbytes=128) == binding.HETIS_ERR_WORKSPACE
    assert pairs(n_pairs=-1) == binding.HETIS_ERR_BAD_SHAPE
    assert pairs(n_pairs=0) == binding.HETIS_OK                         # nothing to do, no HIP call

    def split(control=WS, o=P):
        return H.hetis_attn_decode_split_ws(s, P, P, P, P, P, P, 4, 0.125, 48, 256, o, P, control, 0)
    assert split(control=None) == binding.HETIS_ERR_NULL
    assert split(o=None) == binding.HETIS_ERR_NULL
    assert split(control=WS + 8) == binding.HETIS_ERR_WORKSPACE

    assert H.hetis_attn_workspace_init(None, 256, 0) == binding.HETIS_ERR_NULL
    assert H.hetis_attn_workspace_init(WS, 128, 0) == binding.HETIS_ERR_WORKSPACE
    assert H.hetis_attn_workspace_init(WS, 264, 0) == binding.HETIS_ERR_WORKSPACE   # not a multiple of 16
    assert H.hetis_attn_workspace_init(WS + 16, 256, 0) == binding.HETIS_ERR_WORKSPACE


def test_product_never_imports_the_checker():
    pkg = os.path.join(ROOT, "paper_2509_08309_amd")
    for root, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(root, fn)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle\b", text, flags=re.M), fn
                assert "hetis_oracle" not in text and "liboracle" not in text, fn


# ---------------------------------------------------------------- cache management entry points

def kv_append(shape, n_sel=4, num_blocks=10, **kw):
    a = dict(kn=P, vn=P, bt=P, sl=P, hid=P, k=P, v=P)
    a.update(kw)
    return H.hetis_kv_append(shape, a["kn"], a["vn"], a["bt"], a["sl"], a["hid"], n_sel,
                             num_blocks, a["k"], a["v"], 0)


def kv_store(shape, n_sel=4, n_tokens=3, num_blocks=10, fetch=False, **kw):
    a = dict(kn=P, vn=P, seq=P, pos=P, bt=P, hid=P, k=P, v=P)
    a.update(kw)
    if fetch:
        return H.hetis_kv_fetch(shape, a["k"], a["v"], a["seq"], a["pos"], n_tokens, a["bt"],
                                a["hid"], n_sel, num_blocks, a["kn"], a["vn"], 0)
    return H.hetis_kv_store(shape, a["kn"], a["vn"], a["seq"], a["pos"], n_tokens, a["bt"],
                            a["hid"], n_sel, num_blocks, a["k"], a["v"], 0)


@pytest.mark.parametrize("arg", ["kn", "vn", "bt", "sl", "hid", "k", "v"])
def test_kv_append_null_pointers(lib, arg):
    assert kv_append(good(), **{arg: None}) == binding.HETIS_ERR_NULL


@pytest.mark.parametrize("fetch", [False, True])
@pytest.mark.parametrize("arg", ["kn", "vn", "pos", "bt", "hid", "k", "v"])
def test_kv_store_fetch_null_pointers(lib, arg, fetch):
    assert kv_store(good(), fetch=fetch, **{arg: None}) == binding.HETIS_ERR_NULL


def test_kv_row_argument_errors(lib):
    assert lib.hetis_kv_append(None, P, P, P, P, P, 4, 10, P, P, None) == binding.HETIS_ERR_NULL
    assert kv_append(good(), n_sel=0) == binding.HETIS_ERR_BAD_HEADS
    assert kv_append(good(), n_sel=9) == binding.HETIS_ERR_BAD_HEADS
    assert kv_append(good(), num_blocks=0) == binding.HETIS_ERR_BAD_SHAPE
    assert kv_append(H.make_shape(4, 8, 8, 96, 16)) == binding.HETIS_ERR_UNSUPPORTED
    assert kv_append(H.make_shape(4, 8, 8, 64, 16, block_size=32)) == binding.HETIS_ERR_UNSUPPORTED
    assert kv_append(H.make_shape(4, 8, 8, 64, 16, kv_stride_head=1028)) == binding.HETIS_ERR_BAD_SHAPE
    for fetch in (False, True):
        assert kv_store(good(), n_tokens=-1, fetch=fetch) == binding.HETIS_ERR_BAD_SHAPE
        # implicit sequence ids need n_tokens <= batch
        assert kv_store(good(), n_tokens=5, seq=None, fetch=fetch) == binding.HETIS_ERR_BAD_SHAPE
        # nothing to do: returns before any HIP call
        assert kv_store(good(), n_tokens=0, fetch=fetch) == binding.HETIS_OK


def kv_copy(sp, dp, n_pairs=3, n_sel=2, **kw):
    a = dict(sk=P, sv=P, dk=P, dv=P, sb=P, db=P, sh=P, dh=P)
    a.update(kw)
    return H.hetis_kv_copy_tiles(sp, a["sk"], a["sv"], dp, a["dk"], a["dv"], a["sb"], a["db"],
                                 n_pairs, a["sh"], a["dh"], n_sel, 0)


@pytest.mark.parametrize("arg", ["sk", "sv", "dk", "dv", "sb", "db", "sh", "dh"])
def test_kv_copy_null_pointers(lib, arg):
    sp, dp = H.make_pool(8, 64, 10), H.make_pool(2, 64, 6)
    assert kv_copy(sp, dp, **{arg: None}) == binding.HETIS_ERR_NULL


def test_kv_copy_argument_errors(lib):
    sp, dp = H.make_pool(8, 64, 10), H.make_pool(2, 64, 6)
    assert kv_copy(None, dp) == binding.HETIS_ERR_NULL
    assert kv_copy(sp, None) == binding.HETIS_ERR_NULL
    assert kv_copy(sp, H.make_pool(2, 128, 6)) == binding.HETIS_ERR_BAD_SHAPE
    assert kv_copy(sp, H.make_pool(2, 64, 0)) == binding.HETIS_ERR_BAD_SHAPE
    assert kv_copy(sp, H.make_pool(2, 80, 6)) == binding.HETIS_ERR_UNSUPPORTED
    assert kv_copy(sp, H.make_pool(2, 64, 6, kv_stride_head=100)) == binding.HETIS_ERR_BAD_SHAPE
    assert kv_copy(sp, dp, n_pairs=-1) == binding.HETIS_ERR_BAD_SHAPE
    assert kv_copy(sp, dp, n_sel=0) == binding.HETIS_ERR_BAD_HEADS
    assert kv_copy(sp, dp, n_sel=1025) == binding.HETIS_ERR_BAD_HEADS
    assert kv_copy(sp, dp, n_pairs=0) == binding.HETIS_OK
    assert H.hetis_kv_profile_events(P, None) == binding.HETIS_ERR_NULL
    assert H.hetis_kv_profile_events(None, None) == binding.HETIS_OK


# ---------------------------------------------------------------- per-request head subsets

def decode_pairs(shape, n_pairs=5, **kw):
    a = dict(q=P, k=P, v=P, bt=P, sl=P, ps=P, ph=P, out=P)
    a.update(kw)
    return H.hetis_attn_decode_pairs(shape, a["q"], a["k"], a["v"], a["bt"], a["sl"], a["ps"],
                                     a["ph"], n_pairs, 0.125, a["out"], 0)


@pytest.mark.parametrize("arg", ["q", "k", "v", "bt", "sl", "ps", "ph", "out"])
def test_pairs_null_pointers(lib, arg):
    assert decode_pairs(good(), **{arg: None}) == binding.HETIS_ERR_NULL


def test_pairs_step_argument_errors(lib):
    s = good()

    def call(kn=P, vn=P, ps=P, n_pairs=5, ws=None):
        if ws is None:
            return H.hetis_attn_decode_pairs_step(s, P, kn, vn, P, P, P, P, ps, P, n_pairs, 0.125, P, 0)
        return H.hetis_attn_decode_pairs_step_ws(s, P, kn, vn, P, P, P, P, ps, P, n_pairs, 0.125, P,
                                                 ws[0], ws[1], 0)
    assert call(kn=None) == binding.HETIS_ERR_NULL
    assert call(vn=None) == binding.HETIS_ERR_NULL
    assert call(ps=None) == binding.HETIS_ERR_NULL
    assert call(n_pairs=-1) == binding.HETIS_ERR_BAD_SHAPE
    assert call(n_pairs=0) == binding.HETIS_OK                          # nothing to do, no HIP call
    assert call(ws=(None, 256)) == binding.HETIS_ERR_NULL
    assert call(ws=(WS, 128)) == binding.HETIS_ERR_WORKSPACE
    assert call(kn=None, ws=(WS, 256)) == binding.HETIS_ERR_NULL


def test_pairs_argument_errors(lib):
    assert decode_pairs(good(), n_pairs=-1) == binding.HETIS_ERR_BAD_SHAPE
    assert decode_pairs(good(), n_pairs=65536) == binding.HETIS_ERR_UNSUPPORTED
    assert decode_pairs(H.make_shape(4, 8, 8, 96, 16)) == binding.HETIS_ERR_UNSUPPORTED
    assert decode_pairs(H.make_shape(4, 8, 3, 64, 16)) == binding.HETIS_ERR_BAD_SHAPE
    assert decode_pairs(H.make_shape(4, 8, 8, 64, 16, kv_stride_block=1000)) == binding.HETIS_ERR_BAD_SHAPE
    assert decode_pairs(H.make_shape(4, 8, 8, 64, 16, kv_stride_block=1028)) == binding.HETIS_ERR_BAD_SHAPE
    assert decode_pairs(good(), n_pairs=0) == binding.HETIS_OK        # nothing to do, no HIP call
    assert H.hetis_attn_validate_pairs(good(), P, P, None, P, 3, 10, 0) == binding.HETIS_ERR_NULL
    assert H.hetis_attn_validate_pairs(good(), P, P, P, P, 3, 0, 0) == binding.HETIS_ERR_BAD_SHAPE
    assert H.hetis_attn_validate_pairs(good(), P, P, P, P, 0, 10, 0) == binding.HETIS_OK


def test_kv_append_pairs_argument_errors(lib):
    def call(shape=None, n_pairs=3, num_tiles=10, **kw):
        a = dict(kn=P, vn=P, bt=P, sl=P, ps=P, ph=P, k=P, v=P)
        a.update(kw)
        return H.hetis_kv_append_pairs(shape or good(), a["kn"], a["vn"], a["bt"], a["sl"], a["ps"],
                                       a["ph"], n_pairs, num_tiles, a["k"], a["v"], 0)
    for arg in ("kn", "vn", "bt", "sl", "ps", "ph", "k", "v"):
        assert call(**{arg: None}) == binding.HETIS_ERR_NULL
    assert call(n_pairs=-1) == binding.HETIS_ERR_BAD_SHAPE
    assert call(num_tiles=0) == binding.HETIS_ERR_BAD_SHAPE
    assert call(shape=H.make_shape(4, 8, 8, 96, 16)) == binding.HETIS_ERR_UNSUPPORTED
    assert call(shape=H.make_shape(4, 8, 8, 64, 16, kv_stride_block=1000)) == binding.HETIS_ERR_BAD_SHAPE
    assert call(n_pairs=0) == binding.HETIS_OK
