"""Pins of the CPU checker against facts fixed by the mathematics, not by itself.

Each test would fail for a plausible mistake in oracle/hetis_oracle.c: a wrong
block/slot/head index, a dropped scale, a softmax over the wrong axis, a wrong
group mapping, an off-by-one in the length mask, a transposed operand.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2509_08309_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def f16(a):
    return np.asarray(a, dtype=np.float16)


def dense_softmax_attention(q, k_cache, v_cache, block_table, seq_lens, head_ids, scale):
    """Independent brute force: gather to dense arrays, then numpy softmax(qK^T)V in fp64."""
    q = np.asarray(q, dtype=np.float64)
    B, Hq, D = q.shape
    Hkv = k_cache.shape[1]
    r = Hq // Hkv
    out = np.full((B, Hq, D), np.nan)
    kc = np.asarray(k_cache, dtype=np.float64)
    vc = np.asarray(v_cache, dtype=np.float64)
    for b in range(B):
        L = int(seq_lens[b])
        toks = np.arange(L)
        blks = np.asarray(block_table[b])[toks // 16]
        slots = toks % 16
        for g in head_ids:
            Kd = kc[blks, g, slots, :]          # [L, D]
            Vd = vc[blks, g, slots, :]
            for h in range(g * r, g * r + r):
                if L == 0:
                    out[b, h] = 0.0
                    continue
                logits = Kd @ q[b, h] * scale
                e = np.exp(logits - logits.max())
                out[b, h] = (e / e.sum()) @ Vd
    return out


def np_workload(lens, Hq, Hkv, D, head_ids, seed, **kw):
    w = W.make_custom(lens, Hq, Hkv, D, head_ids, seed, device="cpu", **kw)
    return w, w.q.numpy(), w.k_cache.numpy(), w.v_cache.numpy()


def run_oracle(w, q, k, v, head_ids=None, scale=None):
    hid = w.head_ids if head_ids is None else np.asarray(head_ids, dtype=np.int32)
    sc = w.spec.scale if scale is None else scale
    return oracle.attn_decode(q, k, v, w.block_table, w.seq_lens, hid, sc)


# ---------------------------------------------------------------- conversions
def test_half_to_double_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    same = (got == ref) | (np.isnan(got) & np.isnan(ref))
    assert same.all()
    assert np.array_equal(np.signbit(got[~np.isnan(ref)]), np.signbit(ref[~np.isnan(ref)]))


# ---------------------------------------------------------------- P1 length 1
def test_length_one_returns_v_exactly():
    w, q, k, v = np_workload([1, 1, 1], 4, 4, 64, [0, 2, 3], 11)
    out = run_oracle(w, q, k, v)
    for b in range(3):
        blk = w.block_table[b, 0]
        for g in (0, 2, 3):
            assert np.array_equal(out[b, g], v[blk, g, 0].astype(np.float64))
    assert np.isnan(out[:, 1]).all()          # head 1 not selected: never written


# ---------------------------------------------------------------- P2 constant keys / zero query
def test_constant_keys_give_mean_of_v():
    w, q, k, v = np_workload([37, 16, 5], 2, 2, 64, [0, 1], 12)
    k2 = k.copy()
    k2[...] = f16(0.375)                       # every key row identical
    out = run_oracle(w, q, k2, v)
    dense = dense_softmax_attention(q, k2, v, w.block_table, w.seq_lens, [0, 1], w.spec.scale)
    for b, L in enumerate(w.seq_lens):
        blks = w.block_table[b][np.arange(L) // 16]
        for g in (0, 1):
            mean = v[blks, g, np.arange(L) % 16].astype(np.float64).mean(axis=0)
            assert np.abs(out[b, g] - mean).max() < 1e-13
    assert np.abs(out - dense).max() < 1e-13
    out0 = run_oracle(w, np.zeros_like(q), k, v)     # q = 0: uniform weights as well
    for b, L in enumerate(w.seq_lens):
        blks = w.block_table[b][np.arange(L) // 16]
        mean = v[blks, 1, np.arange(L) % 16].astype(np.float64).mean(axis=0)
        assert np.abs(out0[b, 1] - mean).max() < 1e-13


# ---------------------------------------------------------------- P3 subset = slice
def test_subset_equals_slice_of_full_bitwise():
    w, q, k, v = np_workload([17, 64, 130, 255], 8, 8, 64, [1, 3, 4, 6], 1001)
    full = run_oracle(w, q, k, v, head_ids=list(range(8)))
    sub = run_oracle(w, q, k, v)
    for g in (1, 3, 4, 6):
        assert np.array_equal(sub[:, g], full[:, g])
    for g in (0, 2, 5, 7):
        assert np.isnan(sub[:, g]).all()
    # order of head_ids does not matter
    sub2 = run_oracle(w, q, k, v, head_ids=[6, 1, 4, 3])
    assert np.array_equal(np.nan_to_num(sub2), np.nan_to_num(sub))


# ---------------------------------------------------------------- P4 brute force
@pytest.mark.parametrize("lens,Hq,Hkv,D,hid", [
    ([3, 40, 16], 4, 4, 64, [0, 3]),
    ([1, 17, 33], 6, 2, 64, [1]),
    ([40, 7], 8, 2, 128, [0, 1]),
    ([31, 32, 33], 2, 1, 64, [0]),
])
def test_brute_force_agrees(lens, Hq, Hkv, D, hid):
    w, q, k, v = np_workload(lens, Hq, Hkv, D, hid, 13)
    out = run_oracle(w, q, k, v)
    ref = dense_softmax_attention(q, k, v, w.block_table, w.seq_lens, hid, w.spec.scale)
    sel = ~np.isnan(ref)
    assert np.array_equal(np.isnan(out), np.isnan(ref))
    assert np.abs(out[sel] - ref[sel]).max() < 1e-13


# ---------------------------------------------------------------- P5 closed form
def test_geometric_closed_form():
    # q = a e0, K_t = (t*delta) e0, V_t[0] = t  =>  logits c*t, c = scale*a*delta, and
    # out[0] = sum t x^t / sum x^t with x = e^c: ratio of finite geometric sums.
    L, D = 45, 64
    a, delta, scale = 2.0, 0.0625, 0.5
    w, q, k, v = np_workload([L], 1, 1, D, [0], 14, poison=False)
    q[...] = 0
    k[...] = 0
    v[...] = 0
    q[0, 0, 0] = a
    for t in range(L):
        blk, slot = w.block_table[0, t // 16], t % 16
        k[blk, 0, slot, 0] = t * delta           # exact in fp16 (multiples of 1/16 below 2048)
        v[blk, 0, slot, 0] = t
        v[blk, 0, slot, 1] = 1.0
    out = run_oracle(w, q, k, v, scale=scale)
    x = math.exp(scale * a * delta)
    n = L
    s0 = (x ** n - 1) / (x - 1)
    s1 = x * (1 - n * x ** (n - 1) + (n - 1) * x ** n) / (x - 1) ** 2
    assert abs(out[0, 0, 0] - s1 / s0) < 1e-11
    assert abs(out[0, 0, 1] - 1.0) < 1e-14
    assert np.abs(out[0, 0, 2:]).max() == 0.0
    # halving the scale changes the answer (scale is really applied)
    out2 = run_oracle(w, q, k, v, scale=scale / 2)
    assert abs(out2[0, 0, 0] - out[0, 0, 0]) > 0.1


# ---------------------------------------------------------------- P6 block permutation invariance
def test_physical_block_permutation_invariance():
    w, q, k, v = np_workload([50, 33, 16], 3, 3, 64, [0, 2], 15)
    out = run_oracle(w, q, k, v)
    rng = np.random.default_rng(5)
    perm = rng.permutation(w.num_blocks)          # new physical place of old block i
    k2 = np.empty_like(k)
    v2 = np.empty_like(v)
    k2[perm] = k
    v2[perm] = v
    bt2 = np.where(w.block_table >= 0, perm[np.maximum(w.block_table, 0)], -1).astype(np.int32)
    out2 = oracle.attn_decode(q, k2, v2, bt2, w.seq_lens, w.head_ids, w.spec.scale)
    assert np.array_equal(np.nan_to_num(out), np.nan_to_num(out2))


# ---------------------------------------------------------------- P7 shift invariance
def test_key_shift_invariance():
    rng = np.random.default_rng(16)
    w, q, k, v = np_workload([29, 64], 2, 2, 64, [0, 1], 16, poison=False)
    # dyadic values so that K + u is exact in fp16
    k[...] = f16(rng.integers(-32, 33, size=k.shape) / 16.0)
    q[...] = f16(rng.integers(-16, 17, size=q.shape) / 8.0)
    u = f16(rng.integers(-32, 33, size=(1, 1, 1, 64)) / 16.0)
    out = run_oracle(w, q, k, v)
    out2 = run_oracle(w, q, (k + u).astype(np.float16), v)
    assert np.abs(out - out2).max() < 1e-13


# ---------------------------------------------------------------- P8 linearity and convex hull
def test_linear_in_v_and_inside_hull():
    w, q, k, v = np_workload([23, 48, 100], 2, 2, 64, [0, 1], 17, poison=False)
    rng = np.random.default_rng(17)
    v1 = f16(rng.integers(-64, 65, size=v.shape) / 32.0)
    v2 = f16(rng.integers(-64, 65, size=v.shape) / 32.0)
    o1 = run_oracle(w, q, k, v1)
    o2 = run_oracle(w, q, k, v2)
    o12 = run_oracle(w, q, k, (v1 + v2).astype(np.float16))      # exact sum in fp16
    assert np.abs(o12 - (o1 + o2)).max() < 1e-13
    for b, L in enumerate(w.seq_lens):
        toks = np.arange(L)
        rows = v1[w.block_table[b][toks // 16], :, toks % 16, :].astype(np.float64)  # [L, H, D]
        assert (o1[b] <= rows.max(axis=0) + 1e-15).all()
        assert (o1[b] >= rows.min(axis=0) - 1e-15).all()


# ---------------------------------------------------------------- P9 grouped-query reductions
def test_gqa_group_mapping():
    # (a) query heads of one group with identical q give identical rows
    w, q, k, v = np_workload([35, 70], 8, 2, 64, [0, 1], 18)
    q[:, 1] = q[:, 0]
    q[:, 7] = q[:, 4]
    out = run_oracle(w, q, k, v)
    assert np.array_equal(out[:, 1], out[:, 0])
    assert np.array_equal(out[:, 7], out[:, 4])
    assert not np.array_equal(out[:, 3], out[:, 4])   # heads 3 and 4 sit in different groups
    # (b) GQA equals MHA on a cache with each KV head repeated r times
    r = 4
    k_rep = np.repeat(k, r, axis=1)
    v_rep = np.repeat(v, r, axis=1)
    mha = oracle.attn_decode(q, k_rep, v_rep, w.block_table, w.seq_lens, np.arange(8), w.spec.scale)
    assert np.array_equal(mha, out)
    # (c) selecting KV head 1 alone writes exactly query heads 4..7
    sub = run_oracle(w, q, k, v, head_ids=[1])
    assert np.isnan(sub[:, :4]).all() and np.array_equal(sub[:, 4:], out[:, 4:])


# ---------------------------------------------------------------- P10 split/merge identity
@pytest.mark.parametrize("chunk", [16, 48, 512, 4096])
def test_split_merge_identity(chunk):
    w, q, k, v = np_workload([1, 16, 49, 700], 4, 2, 64, [1, 0], 19)
    full = run_oracle(w, q, k, v)
    max_chunks = (700 + chunk - 1) // chunk
    o_p, lse_p = oracle.attn_partial(q, k, v, w.block_table, w.seq_lens, w.head_ids,
                                     w.spec.scale, chunk, max_chunks)
    merged = oracle.attn_merge(o_p, lse_p, w.seq_lens, w.head_ids, 4, 2, chunk)
    assert np.abs(merged - full).max() < 1e-13
    # chunks past the end are not written
    for b, L in enumerate(w.seq_lens):
        n = (L + chunk - 1) // chunk
        assert np.isnan(lse_p[b, :, n:]).all() and not np.isnan(lse_p[b, :, :n]).any()


def test_partial_lse_is_log_sum_exp_of_logits():
    w, q, k, v = np_workload([40], 1, 1, 64, [0], 20)
    o_p, lse_p = oracle.attn_partial(q, k, v, w.block_table, w.seq_lens, w.head_ids,
                                     w.spec.scale, 16, 3)
    kd = k.astype(np.float64)
    for c, (t0, t1) in enumerate([(0, 16), (16, 32), (32, 40)]):
        toks = np.arange(t0, t1)
        rows = kd[w.block_table[0][toks // 16], 0, toks % 16]
        logits = rows @ q[0, 0].astype(np.float64) * w.spec.scale
        assert abs(lse_p[0, 0, c] - np.log(np.exp(logits).sum())) < 1e-12


# ---------------------------------------------------------------- P11 one-hot limit
def test_one_hot_limit():
    w, q, k, v = np_workload([90], 1, 1, 64, [0], 21, poison=False)
    k[...] = 0
    q[...] = f16(1.0)
    t_star = 53
    blk, slot = w.block_table[0, t_star // 16], t_star % 16
    k[blk, 0, slot, :] = f16(8.0)               # logit 64*8*scale = 64 above the rest
    out = run_oracle(w, q, k, v, scale=0.125)
    assert np.abs(out[0, 0] - v[blk, 0, slot].astype(np.float64)).max() < 1e-6


# ---------------------------------------------------------------- length mask / poison
def test_slots_past_the_end_are_never_used():
    w, q, k, v = np_workload([17, 31], 2, 2, 64, [0, 1], 22, poison=True)
    assert np.isnan(k).any() and np.isnan(v).any()        # poison is really there
    out = run_oracle(w, q, k, v)
    assert not np.isnan(out).any()
    # and the last valid token is used: changing it changes the result
    v2 = v.copy()
    blk = w.block_table[0, 1]
    v2[blk, 0, 0, :] += f16(1.0)
    out2 = run_oracle(w, q, k, v2)
    assert np.abs(out2[0, 0] - out[0, 0]).max() > 1e-4


def test_length_zero_gives_zeros():
    w, q, k, v = np_workload([0, 5], 2, 2, 64, [0, 1], 23)
    out = run_oracle(w, q, k, v)
    assert (out[0] == 0).all() and not np.isnan(out[1]).any()


def test_strided_cache_layout():
    # head-major pool [Hkv, num_blocks, 16, D] addressed through the two strides
    w, q, k, v = np_workload([20, 45], 3, 3, 64, [0, 2], 24)
    ref = run_oracle(w, q, k, v)
    kh = np.ascontiguousarray(k.transpose(1, 0, 2, 3))
    vh = np.ascontiguousarray(v.transpose(1, 0, 2, 3))
    import ctypes as C
    lib = oracle.lib()
    shp = oracle._Shape(2, 3, 3, 64, 16, w.block_table.shape[1], 16 * 64, w.num_blocks * 16 * 64)
    out = np.full(q.shape, np.nan)
    bt = np.ascontiguousarray(w.block_table)
    rc = lib.oracle_attn_decode(C.byref(shp), oracle._ptr(q.view(np.uint16)),
                                oracle._ptr(kh.view(np.uint16)), oracle._ptr(vh.view(np.uint16)),
                                oracle._ptr(bt), oracle._ptr(w.seq_lens), oracle._ptr(w.head_ids),
                                C.c_int32(2), C.c_double(w.spec.scale), oracle._ptr(out),
                                C.c_int32(1))
    assert rc == 0
    assert np.array_equal(np.nan_to_num(out), np.nan_to_num(ref))


# ---------------------------------------------------------------- P12 byte accounting
def test_kv_footprint_matches_paper_statement():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "kv_footprint.txt"))
            if l.strip() and not l.startswith("#")]
    tokens, layers, heads, D, bpe, lower, closed = map(int, rows[0])
    per_layer = tokens * heads * 2 * D * bpe      # K and V, one layer
    assert per_layer * layers == closed
    assert closed > lower


def test_workload_kv_bytes_formula():
    w = W.make_custom([17, 64], 4, 2, 64, [1], 3)
    assert w.kv_bytes() == (17 + 64) * 1 * 2 * 64 * 2


def test_threads_do_not_change_result():
    w, q, k, v = np_workload([100, 200, 50, 17], 4, 4, 64, [0, 1, 2, 3], 25)
    a = oracle.attn_decode(q, k, v, w.block_table, w.seq_lens, w.head_ids, w.spec.scale, n_threads=1)
    b = oracle.attn_decode(q, k, v, w.block_table, w.seq_lens, w.head_ids, w.spec.scale, n_threads=4)
    assert np.array_equal(a, b)
