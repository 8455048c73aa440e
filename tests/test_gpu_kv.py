"""Parity of the cache-management kernels (through the C ABI) against the CPU checker.

Everything here is byte movement, so the bar is bit-exact: whole caches are compared,
which also proves that nothing outside the addressed rows / tiles was written.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_08309_amd as H
from paper_2509_08309_amd import workloads as W

from gpu_harness import SENTINEL, TOL, Dev, as_f64, bits, check_rows, selected_rows

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def i32(a):
    return torch.from_numpy(np.ascontiguousarray(np.asarray(a, dtype=np.int32))).to(DEV)


def same_bits(t: torch.Tensor, ref_u16: np.ndarray) -> bool:
    """Compare a GPU fp16 tensor with uint16 reference bits on the GPU (full size)."""
    ref = torch.from_numpy(ref_u16.view(np.int16)).to(DEV)
    return bool(torch.equal(t.view(torch.int16).reshape(-1), ref.reshape(-1)))


def u16(t: torch.Tensor) -> np.ndarray:
    return bits(t)


def kv_shape(w, **kw):
    s = w.spec
    return H.make_shape(s.batch, s.n_q_heads, s.n_kv_heads, s.head_dim, w.block_table.shape[1],
                        **kw)


def gpu_append(w, k, v, kn, vn, seq_lens, head_ids, shape=None):
    shape = shape or kv_shape(w)
    H.check(H.hetis_kv_append(shape, kn, vn, i32(w.block_table), i32(seq_lens), i32(head_ids),
                              len(head_ids), w.num_blocks, k, v), "hetis_kv_append")
    torch.cuda.synchronize()


# ------------------------------------------------------------------ append (decode step)

@pytest.mark.parametrize("D,Hq,Hkv,heads", [(64, 8, 8, [1, 3, 4, 6]), (128, 8, 8, [7]),
                                            (128, 16, 2, [1, 0]), (64, 4, 4, [0, 1, 2, 3])])
def test_append_small(D, Hq, Hkv, heads):
    lens = [1, 15, 16, 17, 32, 33, 100, 255, 256, 0, 511]
    w = W.make_custom(lens, Hq, Hkv, D, heads, seed=31, device=DEV)
    kn, vn = W.new_token_rows(w)
    ref_k, ref_v = oracle.kv_append(u16(w.k_cache), u16(w.v_cache), u16(kn), u16(vn),
                                    w.block_table, w.seq_lens, heads)
    k, v = w.k_cache.clone(), w.v_cache.clone()
    gpu_append(w, k, v, kn, vn, w.seq_lens, heads)
    assert same_bits(k, ref_k) and same_bits(v, ref_v)
    # something did change: B' x |heads| rows (B' = sequences of non-zero length)
    changed = int((u16(k) != u16(w.k_cache)).any(axis=-1).sum())
    assert 0 < changed <= (len(lens) - 1) * len(heads)


@pytest.mark.parametrize("name", ["c1_tiny", "c3_13b_subset", "c5_70b_gqa"])
def test_append_full_size_then_attention(name):
    """The decode step at the real shapes: store the new token's rows of the selected heads,
    then Attention; cache bit-exact, Attention within tolerance of the checker on the checker's
    own appended cache (every selected row)."""
    spec = W.SPECS[name]
    w = W.make_workload(spec, device=DEV)
    heads = list(spec.head_ids)
    kn, vn = W.new_token_rows(w)
    k_host, v_host = u16(w.k_cache), u16(w.v_cache)
    ref_k, ref_v = oracle.kv_append(k_host, v_host, u16(kn), u16(vn), w.block_table, w.seq_lens,
                                    heads)
    gpu_append(w, w.k_cache, w.v_cache, kn, vn, w.seq_lens, heads)       # in place
    assert same_bits(w.k_cache, ref_k) and same_bits(w.v_cache, ref_v)
    out = Dev(w).decode(heads)        # the workload's tensors already live on the GPU: no copy
    ref = oracle.attn_decode(w.q.cpu().numpy(), ref_k.view(np.float16), ref_v.view(np.float16),
                             w.block_table, w.seq_lens, np.asarray(heads, dtype=np.int32),
                             spec.scale)
    check_rows(out, ref, selected_rows(spec, heads), TOL, f"{name}: append then decode")


def test_append_head_major_pool():
    """Strides of a pool laid out [head][block][slot][d]."""
    lens = [5, 16, 40, 130]
    Hkv, D = 4, 128
    w = W.make_custom(lens, Hkv, Hkv, D, [2, 0], seed=32, device=DEV)
    nb = w.num_blocks
    strides = (nb, Hkv, 16, D, 16 * D, nb * 16 * D)
    k = w.k_cache.permute(1, 0, 2, 3).contiguous()
    v = w.v_cache.permute(1, 0, 2, 3).contiguous()
    kn, vn = W.new_token_rows(w)
    ref_k, ref_v = oracle.kv_append(u16(k).reshape(-1), u16(v).reshape(-1), u16(kn), u16(vn),
                                    w.block_table, w.seq_lens, [2, 0], strides=strides)
    shape = kv_shape(w, kv_stride_block=16 * D, kv_stride_head=nb * 16 * D)
    gpu_append(w, k, v, kn, vn, w.seq_lens, [2, 0], shape=shape)
    assert same_bits(k, ref_k) and same_bits(v, ref_v)


# ------------------------------------------------------------------ store / fetch by (seq, pos, head)

@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("implicit_seq", [False, True])
def test_store_entries(D, implicit_seq):
    lens = [3, 16, 17, 48, 300, 1, 77]
    Hkv = 4
    heads = [3, 1, 2]
    w = W.make_custom(lens, Hkv, Hkv, D, heads, seed=33, device=DEV)
    if implicit_seq:
        seq, pos, n = None, np.array([L - 1 for L in lens], dtype=np.int32), len(lens)
    else:
        seq, pos = W.token_entries(w, seed=34)
        n = len(pos)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(35)
    kn = torch.randn((n, Hkv, D), generator=gen, device=DEV).half()
    vn = torch.randn((n, Hkv, D), generator=gen, device=DEV).half()
    ref_k, ref_v = oracle.kv_store(u16(w.k_cache), u16(w.v_cache), u16(kn), u16(vn), seq, pos,
                                   w.block_table, heads)
    k, v = w.k_cache.clone(), w.v_cache.clone()
    H.check(H.hetis_kv_store(kv_shape(w), kn, vn, None if seq is None else i32(seq), i32(pos), n,
                             i32(w.block_table), i32(heads), len(heads), w.num_blocks, k, v),
            "hetis_kv_store")
    torch.cuda.synchronize()
    assert same_bits(k, ref_k) and same_bits(v, ref_v)


def test_store_every_token_of_c2_then_fetch_back():
    """Prefill-sized store (all tokens of a 64-sequence batch, half the heads) into a
    sentinel-filled pool, then fetch of every stored entry: both bit-exact against the checker."""
    spec = W.SPECS["c2_7b_half"]
    w = W.make_workload(spec, device=DEV)
    heads = list(spec.head_ids)
    seq, pos = W.token_entries(w, seed=36)
    n = len(pos)
    Hkv, D = spec.n_kv_heads, spec.head_dim
    gen = torch.Generator(device=DEV)
    gen.manual_seed(37)
    kn = torch.randn((n, Hkv, D), generator=gen, device=DEV).half()
    vn = torch.randn((n, Hkv, D), generator=gen, device=DEV).half()
    k = torch.empty_like(w.k_cache)
    v = torch.empty_like(w.v_cache)
    k.view(torch.int16).fill_(np.int16(SENTINEL))
    v.view(torch.int16).fill_(np.int16(SENTINEL))
    ref_k, ref_v = oracle.kv_store(u16(k), u16(v), u16(kn), u16(vn), seq, pos, w.block_table,
                                   heads)
    bt, hid = i32(w.block_table), i32(heads)
    H.check(H.hetis_kv_store(kv_shape(w), kn, vn, i32(seq), i32(pos), n, bt, hid, len(heads),
                             w.num_blocks, k, v), "hetis_kv_store")
    torch.cuda.synchronize()
    assert same_bits(k, ref_k) and same_bits(v, ref_v)
    # fetch every entry back
    m = n
    ko = torch.empty((m, Hkv, D), dtype=torch.float16, device=DEV)
    vo = torch.empty_like(ko)
    ko.view(torch.int16).fill_(np.int16(SENTINEL))
    vo.view(torch.int16).fill_(np.int16(SENTINEL))
    H.check(H.hetis_kv_fetch(kv_shape(w), k, v, i32(seq[:m]), i32(pos[:m]), m, bt, hid, len(heads),
                             w.num_blocks, ko, vo), "hetis_kv_fetch")
    torch.cuda.synchronize()
    ref_ko, ref_vo = oracle.kv_fetch(ref_k, ref_v, seq[:m], pos[:m], w.block_table, heads,
                                     fill=SENTINEL)
    assert same_bits(ko, ref_ko) and same_bits(vo, ref_vo)
    # and the fetched rows are the rows that were stored
    assert torch.equal(ko[:, heads], kn[:m][:, heads]) and torch.equal(vo[:, heads], vn[:m][:, heads])


def test_entries_outside_the_tables_are_skipped():
    lens = [20, 7, 64]
    Hkv, D = 2, 64
    w = W.make_custom(lens, Hkv, Hkv, D, [0, 1], seed=38, device=DEV)
    bt = w.block_table.copy()
    bt[1, 0] = w.num_blocks                       # block id past the pool
    mb = bt.shape[1]
    seq = np.array([-1, 3, 0, 0, 0, 1, 2, 0], dtype=np.int32)
    pos = np.array([0, 0, -1, 16 * mb, 40, 3, 63, 19], dtype=np.int32)
    #               seq<0 seq>=B pos<0 past row  id -1 id=nb  ok   ok
    n = len(seq)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(39)
    kn = torch.randn((n, Hkv, D), generator=gen, device=DEV).half()
    vn = torch.randn((n, Hkv, D), generator=gen, device=DEV).half()
    ref_k, ref_v = oracle.kv_store(u16(w.k_cache), u16(w.v_cache), u16(kn), u16(vn), seq, pos, bt,
                                   [1, 0])
    k, v = w.k_cache.clone(), w.v_cache.clone()
    H.check(H.hetis_kv_store(kv_shape(w), kn, vn, i32(seq), i32(pos), n, i32(bt), i32([1, 0]), 2,
                             w.num_blocks, k, v), "hetis_kv_store")
    torch.cuda.synchronize()
    assert same_bits(k, ref_k) and same_bits(v, ref_v)
    assert int((u16(k) != u16(w.k_cache)).any(axis=-1).sum()) == 2 * 2
    # head ids outside the pool are skipped as well
    k2, v2 = w.k_cache.clone(), w.v_cache.clone()
    H.check(H.hetis_kv_store(kv_shape(w), kn, vn, i32(seq), i32(pos), n, i32(bt), i32([5, -2]), 2,
                             w.num_blocks, k2, v2), "hetis_kv_store")
    torch.cuda.synchronize()
    assert torch.equal(k2.view(torch.int16), w.k_cache.view(torch.int16))
    assert torch.equal(v2.view(torch.int16), w.v_cache.view(torch.int16))
    # fetch with the same entries
    ko = torch.empty((n, Hkv, D), dtype=torch.float16, device=DEV)
    vo = torch.empty_like(ko)
    ko.view(torch.int16).fill_(np.int16(SENTINEL))
    vo.view(torch.int16).fill_(np.int16(SENTINEL))
    H.check(H.hetis_kv_fetch(kv_shape(w), k, v, i32(seq), i32(pos), n, i32(bt), i32([1, 0]), 2,
                             w.num_blocks, ko, vo), "hetis_kv_fetch")
    torch.cuda.synchronize()
    ref_ko, ref_vo = oracle.kv_fetch(ref_k, ref_v, seq, pos, bt, [1, 0], fill=SENTINEL)
    assert same_bits(ko, ref_ko) and same_bits(vo, ref_vo)
    assert (u16(ko)[:6] == SENTINEL).all()


# ------------------------------------------------------------------ tile copy (migration)

def compact_copy(w, moved, head_major, seed):
    """Move the tiles of heads `moved` of every used block into a pool that holds only those
    heads.  Returns (dst_k, dst_v, dst_table, ref_k_bits, ref_v_bits, dst_num_blocks)."""
    s = w.spec
    D = s.head_dim
    n_mv = len(moved)
    src_b, dst_b, dnb, table = W.migration_plan(w, seed)
    dst_heads = list(range(n_mv))
    if head_major:
        strides = (dnb, n_mv, 16, D, 16 * D, dnb * 16 * D)
        dk = torch.empty((n_mv, dnb, 16, D), dtype=torch.float16, device=DEV)
        dpool = H.make_pool(n_mv, D, dnb, kv_stride_block=16 * D, kv_stride_head=dnb * 16 * D)
    else:
        strides = None
        dk = torch.empty((dnb, n_mv, 16, D), dtype=torch.float16, device=DEV)
        dpool = H.make_pool(n_mv, D, dnb)
    dk.view(torch.int16).fill_(np.int16(SENTINEL))
    dv = dk.clone()
    d0 = u16(dk) if not head_major else u16(dk).reshape(-1)
    ref_k, ref_v = oracle.kv_copy_tiles(u16(w.k_cache), u16(w.v_cache), d0, d0, src_b, dst_b,
                                        moved, dst_heads, dst_strides=strides)
    spool = H.make_pool(s.n_kv_heads, D, w.num_blocks)
    H.check(H.hetis_kv_copy_tiles(spool, w.k_cache, w.v_cache, dpool, dk, dv, i32(src_b),
                                  i32(dst_b), len(src_b), i32(moved), i32(dst_heads), n_mv),
            "hetis_kv_copy_tiles")
    torch.cuda.synchronize()
    return dk, dv, table, ref_k, ref_v, dnb


@pytest.mark.parametrize("head_major", [False, True])
@pytest.mark.parametrize("D,Hkv,moved", [(64, 8, [6, 1, 3]), (128, 4, [2])])
def test_copy_tiles_small(D, Hkv, moved, head_major):
    lens = [1, 16, 17, 100, 255, 40]
    w = W.make_custom(lens, Hkv, Hkv, D, moved, seed=40, device=DEV)
    dk, dv, _, ref_k, ref_v, _ = compact_copy(w, moved, head_major, seed=41)
    assert same_bits(dk, ref_k) and same_bits(dv, ref_v)


@pytest.mark.parametrize("name,head_major", [("c3_13b_subset", False), ("c3_13b_subset", True),
                                             ("c5_70b_gqa", False)])
def test_copy_tiles_full_size_and_attention_invariance(name, head_major):
    """Migration of one device's head share at its real shape into a compact pool: tiles
    bit-exact against the checker, and Attention over the destination pool (remapped block
    table, heads renumbered 0..S-1) returns bit for bit the rows of Attention over the source."""
    spec = W.SPECS[name]
    w = W.make_workload(spec, device=DEV)
    moved = list(spec.head_ids)
    dk, dv, table, ref_k, ref_v, dnb = compact_copy(w, moved, head_major, seed=42)
    assert same_bits(dk, ref_k) and same_bits(dv, ref_v)
    src = Dev(w)
    out_src = src.decode(moved)
    r, S, D = spec.group_size, len(moved), spec.head_dim
    rows = selected_rows(spec, moved)
    q2 = w.q[:, rows].contiguous()                      # [B, S*r, D]: heads renumbered
    shape2 = H.make_shape(spec.batch, S * r, S, D, table.shape[1],
                          kv_stride_block=16 * D if head_major else 0,
                          kv_stride_head=dnb * 16 * D if head_major else 0)
    out2 = torch.zeros_like(q2)
    H.check(H.hetis_attn_decode(shape2, q2, dk, dv, i32(table), i32(w.seq_lens),
                                i32(list(range(S))), S, spec.scale, out2), "hetis_attn_decode")
    torch.cuda.synchronize()
    assert torch.equal(out2.view(torch.int16), out_src[:, rows].contiguous().view(torch.int16))


def test_copy_tiles_skips_and_same_pool():
    lens = [64, 64, 64]
    Hkv, D = 4, 128
    w = W.make_custom(lens, Hkv, Hkv, D, [0], seed=43, device=DEV, permute=False)
    nb = w.num_blocks                                    # 12 blocks
    # inside one pool: blocks 0..3 -> 8..11 (disjoint), plus pairs that must be skipped
    src_b = [0, 1, 2, 3, -1, nb, 4, 5]
    dst_b = [8, 9, 10, 11, 0, 1, nb, -7]
    sh, dh = [1, 3], [3, 0]
    ref_k, ref_v = oracle.kv_copy_tiles(u16(w.k_cache), u16(w.v_cache), u16(w.k_cache),
                                        u16(w.v_cache), src_b, dst_b, sh, dh)
    pool = H.make_pool(Hkv, D, nb)
    k, v = w.k_cache.clone(), w.v_cache.clone()
    H.check(H.hetis_kv_copy_tiles(pool, k, v, pool, k, v, i32(src_b), i32(dst_b), len(src_b),
                                  i32(sh), i32(dh), 2), "hetis_kv_copy_tiles")
    torch.cuda.synchronize()
    assert same_bits(k, ref_k) and same_bits(v, ref_v)
    assert torch.equal(k[8, 3], w.k_cache[0, 1]) and torch.equal(v[11, 0], w.v_cache[3, 3])


def test_kv_profile_events_bracket_the_launch():
    spec = W.SPECS["c3_13b_subset"]
    w = W.make_workload(spec, device=DEV)
    kn, vn = W.new_token_rows(w)
    b, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    b.record()
    e.record()
    torch.cuda.synchronize()
    assert H.hetis_kv_profile_events(b.cuda_event, e.cuda_event) == 0
    try:
        gpu_append(w, w.k_cache, w.v_cache, kn, vn, w.seq_lens, list(spec.head_ids))
    finally:
        H.hetis_kv_profile_events(None, None)
    ms = b.elapsed_time(e)
    assert 0.0 < ms < 5.0
