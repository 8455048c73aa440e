"""Pins of the cache-management checker (oracle/hetis_kv_oracle.c) against facts it does not
define itself: dense per-sequence arrays rebuilt with numpy indexing, the (pinned) Attention
checker on the stored cache versus brute-force attention on the dense data, round trips, and
invariance of Attention under a tile copy into a differently laid out pool.

Each test would fail for a plausible mistake: block and slot swapped, head stride misused, the
new token stored at seq_lens instead of seq_lens - 1, source and destination of a copy
exchanged, a skipped entry that still writes.
"""
import numpy as np
import pytest

import oracle

SENT = 0x7E00 | 0x155     # an fp16 NaN pattern no generator produces


def dense_data(lens, Hkv, D, seed):
    """Per-sequence dense K and V [L, Hkv, D] as fp16 (values are exact small dyadics)."""
    rng = np.random.default_rng(seed)
    Ks = [(rng.integers(-64, 64, size=(L, Hkv, D)) / 16.0).astype(np.float16) for L in lens]
    Vs = [(rng.integers(-64, 64, size=(L, Hkv, D)) / 16.0).astype(np.float16) for L in lens]
    return Ks, Vs


def paged_layout(lens, seed, extra_blocks=3, block_size=16, slack=0):
    """A block table with a seeded permutation of physical blocks (+ unused blocks).
    slack = blocks reserved per sequence beyond those its length needs."""
    rng = np.random.default_rng(seed)
    need = [(L + block_size - 1) // block_size + slack for L in lens]
    nb = sum(need) + extra_blocks
    perm = rng.permutation(nb)
    max_blocks = max(need) + 1
    bt = np.full((len(lens), max_blocks), -1, dtype=np.int32)
    o = 0
    for b, n in enumerate(need):
        bt[b, :n] = perm[o:o + n]
        o += n
    return bt, nb


def empty_cache(nb, Hkv, D):
    return np.full((nb, Hkv, 16, D), SENT, dtype=np.uint16)


def all_tokens(lens):
    seq = np.concatenate([np.full(L, b, dtype=np.int32) for b, L in enumerate(lens)])
    pos = np.concatenate([np.arange(L, dtype=np.int32) for L in lens])
    return seq, pos


def store_all(lens, Ks, Vs, bt, nb, head_ids, Hkv, D):
    seq, pos = all_tokens(lens)
    kn = np.concatenate(Ks).view(np.uint16)
    vn = np.concatenate(Vs).view(np.uint16)
    return oracle.kv_store(empty_cache(nb, Hkv, D), empty_cache(nb, Hkv, D), kn, vn, seq, pos, bt,
                           head_ids)


def brute_attention(q, Kd, Vd, scale):
    """softmax(q K^T scale) V for one head, dense fp64."""
    s = Kd.astype(np.float64) @ q.astype(np.float64) * scale
    e = np.exp(s - s.max())
    return (e / e.sum()) @ Vd.astype(np.float64)


LENS = [1, 16, 17, 40, 95]


def test_store_places_every_row_where_numpy_indexing_finds_it():
    Hkv, D = 3, 8
    Ks, Vs = dense_data(LENS, Hkv, D, 1)
    bt, nb = paged_layout(LENS, 2)
    k, v = store_all(LENS, Ks, Vs, bt, nb, [0, 1, 2], Hkv, D)
    touched = np.zeros((nb, 16), dtype=bool)
    for b, L in enumerate(LENS):
        t = np.arange(L)
        assert np.array_equal(k[bt[b, t // 16], :, t % 16, :], Ks[b].view(np.uint16))
        assert np.array_equal(v[bt[b, t // 16], :, t % 16, :], Vs[b].view(np.uint16))
        touched[bt[b, t // 16], t % 16] = True
    # every slot no token maps to is still the sentinel, for K and for V
    for c in (k, v):
        rest = np.moveaxis(c, 2, 1)[~touched]          # [slots, Hkv, D]
        assert np.all(rest == SENT)


def test_store_only_selected_heads():
    Hkv, D = 4, 8
    Ks, Vs = dense_data(LENS, Hkv, D, 3)
    bt, nb = paged_layout(LENS, 4)
    k, v = store_all(LENS, Ks, Vs, bt, nb, [3, 1], Hkv, D)
    assert np.all(k[:, [0, 2]] == SENT) and np.all(v[:, [0, 2]] == SENT)
    b, t = 4, 77
    assert np.array_equal(k[bt[b, t // 16], 3, t % 16], Ks[b][t, 3].view(np.uint16))
    assert np.array_equal(v[bt[b, t // 16], 1, t % 16], Vs[b][t, 1].view(np.uint16))


def test_attention_on_stored_cache_equals_dense_attention():
    """Links the store to the Attention checker: a wrong slot, head or block index in the
    store shows up as a different attention result."""
    Hkv, D = 2, 16
    Ks, Vs = dense_data(LENS, Hkv, D, 5)
    bt, nb = paged_layout(LENS, 6)
    k, v = store_all(LENS, Ks, Vs, bt, nb, [0, 1], Hkv, D)
    rng = np.random.default_rng(7)
    q = (rng.integers(-32, 32, size=(len(LENS), Hkv, D)) / 16.0).astype(np.float16)
    out = oracle.attn_decode(q, k, v, bt, np.array(LENS), [0, 1], 0.25)
    for b in range(len(LENS)):
        for g in range(Hkv):
            ref = brute_attention(q[b, g], Ks[b][:, g], Vs[b][:, g], 0.25)
            assert np.max(np.abs(out[b, g] - ref)) < 1e-12


def test_append_is_the_last_position_and_changes_nothing_else():
    Hkv, D = 3, 8
    lens = [1, 16, 17, 33, 48]                # after the append; 17 and 33 open a new block
    old = [L - 1 for L in lens]
    Ks, Vs = dense_data(lens, Hkv, D, 8)
    bt, nb = paged_layout(lens, 9)
    sel = [2, 0]
    k0, v0 = store_all(old, [K[:-1] for K in Ks], [V[:-1] for V in Vs], bt, nb, sel, Hkv, D)
    kn = np.stack([K[-1] for K in Ks]).view(np.uint16)
    vn = np.stack([V[-1] for V in Vs]).view(np.uint16)
    k1, v1 = oracle.kv_append(k0, v0, kn, vn, bt, np.array(lens), sel)
    # the result is what storing all tokens at once gives
    kf, vf = store_all(lens, Ks, Vs, bt, nb, sel, Hkv, D)
    assert np.array_equal(k1, kf) and np.array_equal(v1, vf)
    # exactly B * |sel| rows differ from before (new rows are never the sentinel)
    assert int((k1 != k0).any(axis=-1).sum()) == len(lens) * len(sel)
    assert int((v1 != v0).any(axis=-1).sum()) == len(lens) * len(sel)
    # length 0: nothing stored
    k2, v2 = oracle.kv_append(k0, v0, kn, vn, bt, np.zeros(len(lens), dtype=np.int32), sel)
    assert np.array_equal(k2, k0) and np.array_equal(v2, v0)


def test_attention_after_append_sees_the_new_token():
    Hkv, D = 2, 16
    lens = [5, 17, 64]
    Ks, Vs = dense_data(lens, Hkv, D, 10)
    bt, nb = paged_layout(lens, 11)
    k0, v0 = store_all([L - 1 for L in lens], [K[:-1] for K in Ks], [V[:-1] for V in Vs], bt, nb,
                       [0, 1], Hkv, D)
    kn = np.stack([K[-1] for K in Ks]).view(np.uint16)
    vn = np.stack([V[-1] for V in Vs]).view(np.uint16)
    k1, v1 = oracle.kv_append(k0, v0, kn, vn, bt, np.array(lens), [0, 1])
    rng = np.random.default_rng(12)
    q = (rng.integers(-32, 32, size=(len(lens), Hkv, D)) / 16.0).astype(np.float16)
    out = oracle.attn_decode(q, k1, v1, bt, np.array(lens), [0, 1], 0.25)
    for b in range(len(lens)):
        for g in range(Hkv):
            ref = brute_attention(q[b, g], Ks[b][:, g], Vs[b][:, g], 0.25)
            assert np.max(np.abs(out[b, g] - ref)) < 1e-12


def test_fetch_inverts_store_and_leaves_other_rows():
    Hkv, D = 4, 8
    Ks, Vs = dense_data(LENS, Hkv, D, 13)
    bt, nb = paged_layout(LENS, 14)
    k, v = store_all(LENS, Ks, Vs, bt, nb, [0, 1, 2, 3], Hkv, D)
    seq, pos = all_tokens(LENS)
    rng = np.random.default_rng(15)
    pick = rng.permutation(len(seq))[:60]
    ko, vo = oracle.kv_fetch(k, v, seq[pick], pos[pick], bt, [1, 3], fill=0xBEEF)
    dense_k = np.concatenate(Ks).view(np.uint16)[pick]
    dense_v = np.concatenate(Vs).view(np.uint16)[pick]
    assert np.array_equal(ko[:, [1, 3]], dense_k[:, [1, 3]])
    assert np.array_equal(vo[:, [1, 3]], dense_v[:, [1, 3]])
    assert np.all(ko[:, [0, 2]] == 0xBEEF) and np.all(vo[:, [0, 2]] == 0xBEEF)


def test_entries_outside_the_tables_are_skipped():
    Hkv, D = 2, 8
    lens = [20, 7]
    Ks, Vs = dense_data(lens, Hkv, D, 16)
    bt, nb = paged_layout(lens, 17)
    k, v = store_all(lens, Ks, Vs, bt, nb, [0, 1], Hkv, D)
    bt_bad = bt.copy()
    bt_bad[1, 0] = nb                  # physical block past the pool
    cases_seq = np.array([-1, 2, 0, 0, 0, 1], dtype=np.int32)
    cases_pos = np.array([0, 0, -1, 16 * bt.shape[1], 40, 3], dtype=np.int32)
    #                     seq<0 seq>=B pos<0 past the row   block id -1   block id == nb
    rows = np.full((6, Hkv, D), 0x3C00, dtype=np.uint16)
    k2, v2 = oracle.kv_store(k, v, rows, rows, cases_seq, cases_pos, bt_bad, [0, 1])
    assert np.array_equal(k2, k) and np.array_equal(v2, v)
    ko, vo = oracle.kv_fetch(k, v, cases_seq, cases_pos, bt_bad, [0, 1], fill=0xBEEF)
    assert np.all(ko == 0xBEEF) and np.all(vo == 0xBEEF)


def test_implicit_sequence_ids():
    Hkv, D = 2, 8
    lens = [9, 30, 16]
    Ks, Vs = dense_data(lens, Hkv, D, 18)
    bt, nb = paged_layout(lens, 19)
    pos = np.array([8, 29, 15], dtype=np.int32)
    kn = np.stack([K[-1] for K in Ks]).view(np.uint16)
    vn = np.stack([V[-1] for V in Vs]).view(np.uint16)
    e = empty_cache(nb, Hkv, D)
    a = oracle.kv_store(e, e, kn, vn, None, pos, bt, [0, 1])
    b = oracle.kv_store(e, e, kn, vn, np.arange(3, dtype=np.int32), pos, bt, [0, 1])
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert np.array_equal(a[0][bt[1, 1], 1, 13], kn[1, 1])


def test_tile_copy_matches_numpy_indexing_and_touches_nothing_else():
    rng = np.random.default_rng(20)
    sH, dH, D, snb, dnb = 5, 3, 8, 12, 9
    sk = rng.integers(0, 0x7000, size=(snb, sH, 16, D)).astype(np.uint16)
    sv = rng.integers(0, 0x7000, size=(snb, sH, 16, D)).astype(np.uint16)
    dk0, dv0 = empty_cache(dnb, dH, D), empty_cache(dnb, dH, D)
    sb = np.array([3, 11, 0, 7], dtype=np.int32)
    db = np.array([8, 2, 5, 0], dtype=np.int32)
    shd, dhd = [4, 1], [0, 2]
    dk, dv = oracle.kv_copy_tiles(sk, sv, dk0, dv0, sb, db, shd, dhd)
    for i in range(4):
        for s_, d_ in zip(shd, dhd):
            assert np.array_equal(dk[db[i], d_], sk[sb[i], s_])
            assert np.array_equal(dv[db[i], d_], sv[sb[i], s_])
    mask = np.ones((dnb, dH), dtype=bool)
    mask[np.ix_(db, dhd)] = False
    assert np.all(dk[mask] == SENT) and np.all(dv[mask] == SENT)
    # pairs with a block outside either pool are skipped
    dk2, dv2 = oracle.kv_copy_tiles(sk, sv, dk0, dv0, [snb, -1, 1, 2], [0, 1, dnb, -1], shd, dhd)
    assert np.array_equal(dk2, dk0) and np.array_equal(dv2, dv0)


@pytest.mark.parametrize("head_major", [False, True])
def test_attention_is_invariant_under_migration_to_a_compact_pool(head_major):
    """Copy the tiles of two heads of every block into a pool that holds only those heads, in
    other physical blocks (and, optionally, head-major): Attention over the new pool with the
    remapped block table gives bit-identical rows."""
    Hkv, D = 4, 16
    lens = [3, 31, 64, 100]
    Ks, Vs = dense_data(lens, Hkv, D, 21)
    bt, nb = paged_layout(lens, 22)
    k, v = store_all(lens, Ks, Vs, bt, nb, [0, 1, 2, 3], Hkv, D)
    rng = np.random.default_rng(23)
    q = (rng.integers(-32, 32, size=(len(lens), Hkv, D)) / 16.0).astype(np.float16)
    moved = [3, 1]                           # source heads -> destination heads 0, 1
    used = bt[bt >= 0]
    dnb = len(used) + 2
    new_ids = rng.permutation(dnb)[:len(used)].astype(np.int32)
    bt2 = bt.copy()
    bt2[bt >= 0] = new_ids
    if head_major:
        strides = (dnb, 2, 16, D, 16 * D, dnb * 16 * D)      # [head][block][slot][d]
        dk0 = np.full(dnb * 2 * 16 * D, SENT, dtype=np.uint16)
    else:
        strides = None
        dk0 = empty_cache(dnb, 2, D)
    dk, dv = oracle.kv_copy_tiles(k, v, dk0, dk0, used, new_ids, moved, [0, 1],
                                  dst_strides=strides)
    if head_major:
        dk = np.ascontiguousarray(dk.reshape(2, dnb, 16, D).transpose(1, 0, 2, 3))
        dv = np.ascontiguousarray(dv.reshape(2, dnb, 16, D).transpose(1, 0, 2, 3))
    ref = oracle.attn_decode(q, k, v, bt, np.array(lens), moved, 0.25)
    q2 = np.ascontiguousarray(q[:, moved])
    out = oracle.attn_decode(q2, dk, dv, bt2, np.array(lens), [0, 1], 0.25)
    assert np.array_equal(out, ref[:, moved])


# ---------------------------------------------------------------- pairs form of the decode-step store

def test_append_pairs_then_attention_sees_the_new_token():
    """Per-request head subsets over single-head tiles: after the append, the pairs Attention
    checker equals brute-force attention on the dense sequences (new token included), the rows
    written are exactly one K and one V row per pair, and pairs that point outside the tables
    are skipped."""
    from paper_2509_08309_amd import workloads as W
    lens = [5, 17, 64, 33]
    Hq = Hkv = 4
    D = 16
    subsets = [[0, 3], [1], [0, 1, 2, 3], [2]]
    spec = W.WorkloadSpec("pairs", len(lens), Hq, Hkv, D, tuple(range(Hkv)), 24, "fixed",
                          (tuple(lens),), max(lens))
    pw = W.make_pairs_workload(spec, subsets=subsets, poison=False)
    k0, v0 = pw.k_tiles.numpy().view(np.uint16), pw.v_tiles.numpy().view(np.uint16)
    rng = np.random.default_rng(25)
    kn = (rng.integers(-64, 64, size=(len(lens), Hkv, D)) / 16.0).astype(np.float16)
    vn = (rng.integers(-64, 64, size=(len(lens), Hkv, D)) / 16.0).astype(np.float16)
    k1, v1 = oracle.kv_append_pairs(k0, v0, kn, vn, pw.block_table, pw.seq_lens, pw.pair_seq,
                                    pw.pair_head)
    assert int((k1 != k0).any(axis=-1).sum()) == pw.n_pairs
    assert int((v1 != v0).any(axis=-1).sum()) == pw.n_pairs
    q = pw.q.numpy()
    out = oracle.attn_decode_pairs(q, k1.view(np.float16), v1.view(np.float16), pw.block_table,
                                   pw.seq_lens, pw.pair_seq, pw.pair_head, Hkv, 0.25)
    for p in range(pw.n_pairs):
        b, g = int(pw.pair_seq[p]), int(pw.pair_head[p])
        L = lens[b]
        t = np.arange(L)
        tiles = pw.block_table[p, t // 16]
        Kd = k0.view(np.float16)[tiles, t % 16].copy()
        Vd = v0.view(np.float16)[tiles, t % 16].copy()
        Kd[-1], Vd[-1] = kn[b, g], vn[b, g]             # the new token is the last one
        ref = brute_attention(q[b, g], Kd, Vd, 0.25)
        assert np.max(np.abs(out[b, g] - ref)) < 1e-12
    # skipped pairs: bad sequence id, bad head id, empty sequence, tile id outside the pool
    bad_seq = pw.pair_seq.copy(); bad_seq[0] = len(lens)
    bad_head = pw.pair_head.copy(); bad_head[1] = -1
    sl0 = pw.seq_lens.copy(); sl0[2] = 0
    bt_bad = pw.block_table.copy(); bt_bad[-1, (lens[3] - 1) // 16] = pw.num_tiles
    k2, v2 = oracle.kv_append_pairs(k0, v0, kn, vn, bt_bad, sl0, bad_seq, bad_head)
    changed = (k2 != k0).any(axis=-1)
    assert int(changed.sum()) == pw.n_pairs - (1 + 1 + 4 + 1)
