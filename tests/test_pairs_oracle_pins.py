"""Pins of the per-request head-subset form of the Attention checker
(oracle_attn_decode_pairs) against the pinned common-subset checker and dense brute force."""
import numpy as np
import pytest

import oracle
from paper_2509_08309_amd import workloads as W


def spec_of(lens, Hq, Hkv, D, seed):
    lens = tuple(int(x) for x in lens)
    return W.WorkloadSpec("pairs", len(lens), Hq, Hkv, D, tuple(range(Hkv)), seed, "fixed", (lens,),
                          max(max(lens), 1))


def dense_rows(pw, p):
    """K and V rows [L, D] of pair p, gathered with numpy indexing."""
    L = int(pw.seq_lens[pw.pair_seq[p]])
    t = np.arange(L)
    tiles = pw.block_table[p, t // 16]
    return pw.k_tiles.numpy()[tiles, t % 16], pw.v_tiles.numpy()[tiles, t % 16]


def run(pw, order=None):
    idx = np.arange(pw.n_pairs) if order is None else np.asarray(order)
    return oracle.attn_decode_pairs(pw.q.numpy(), pw.k_tiles.numpy(), pw.v_tiles.numpy(),
                                    pw.block_table[idx], pw.seq_lens, pw.pair_seq[idx],
                                    pw.pair_head[idx], pw.spec.n_kv_heads, pw.spec.scale)


@pytest.mark.parametrize("Hq,Hkv,D", [(6, 6, 16), (8, 2, 64)])
def test_pairs_against_dense_brute_force(Hq, Hkv, D):
    lens = [1, 16, 17, 40, 95, 0, 33]
    subsets = [[0], [Hkv - 1, 0], [], list(range(Hkv)), [1], [0, 1], [Hkv - 1]]
    pw = W.make_pairs_workload(spec_of(lens, Hq, Hkv, D, 51), subsets=subsets)
    out = run(pw)
    r = Hq // Hkv
    named = np.zeros((len(lens), Hq), dtype=bool)
    q = pw.q.numpy().astype(np.float64)
    for p in range(pw.n_pairs):
        b, g = int(pw.pair_seq[p]), int(pw.pair_head[p])
        Kd, Vd = dense_rows(pw, p)
        for h in range(g * r, g * r + r):
            named[b, h] = True
            if lens[b] == 0:
                assert np.all(out[b, h] == 0.0)
                continue
            s = Kd.astype(np.float64) @ q[b, h] * pw.spec.scale
            e = np.exp(s - s.max())
            ref = (e / e.sum()) @ Vd.astype(np.float64)
            assert np.max(np.abs(out[b, h] - ref)) < 1e-12
    assert np.isnan(out[~named]).all() and not np.isnan(out[named]).any()


def test_cross_product_of_pairs_equals_the_common_subset_form_bitwise():
    """A standard pool [nb, Hkv, 16, D] read as a pool of nb*Hkv single-head tiles, with the
    row of pair (b, g) = block_table[b] * Hkv + g: the two forms must agree bit for bit."""
    lens = [5, 64, 130, 31]
    Hq, Hkv, D = 8, 4, 32
    heads = [3, 1]
    w = W.make_custom(lens, Hq, Hkv, D, heads, seed=52)
    ref = oracle.attn_decode(w.q.numpy(), w.k_cache.numpy(), w.v_cache.numpy(), w.block_table,
                             w.seq_lens, heads, w.spec.scale)
    pair_seq = np.repeat(np.arange(len(lens)), len(heads)).astype(np.int32)
    pair_head = np.tile(np.asarray(heads, dtype=np.int32), len(lens))
    table = w.block_table[pair_seq] * Hkv + pair_head[:, None]
    table[w.block_table[pair_seq] < 0] = -1
    k_tiles = w.k_cache.numpy().reshape(-1, 16, D)
    v_tiles = w.v_cache.numpy().reshape(-1, 16, D)
    out = oracle.attn_decode_pairs(w.q.numpy(), k_tiles, v_tiles, table, w.seq_lens, pair_seq,
                                   pair_head, Hkv, w.spec.scale)
    assert np.array_equal(out, ref, equal_nan=True)


def test_pair_order_and_duplicates_do_not_matter():
    lens = [20, 7, 64, 100]
    pw = W.make_pairs_workload(spec_of(lens, 4, 4, 16, 53), mean_heads=2)
    assert pw.n_pairs > 3
    a = run(pw)
    order = np.random.default_rng(1).permutation(pw.n_pairs)
    b = run(pw, order)
    c = run(pw, np.concatenate([order, order[:2]]))
    assert np.array_equal(a, b, equal_nan=True) and np.array_equal(a, c, equal_nan=True)


def test_each_pair_uses_its_own_table_row():
    """Two heads of one sequence with different tiles: exchanging the two table rows exchanges
    what the two heads attend over."""
    lens = [48]
    pw = W.make_pairs_workload(spec_of(lens, 2, 2, 16, 54), subsets=[[0, 1]])
    out = run(pw)
    swapped = oracle.attn_decode_pairs(pw.q.numpy(), pw.k_tiles.numpy(), pw.v_tiles.numpy(),
                                       pw.block_table[::-1], pw.seq_lens, pw.pair_seq,
                                       pw.pair_head, 2, pw.spec.scale)
    assert not np.allclose(out, swapped)
    q = pw.q.numpy().astype(np.float64)
    Kd, Vd = dense_rows(pw, 1)                       # head 0 now reads pair 1's tiles
    s = Kd.astype(np.float64) @ q[0, 0] * pw.spec.scale
    e = np.exp(s - s.max())
    assert np.max(np.abs(swapped[0, 0] - (e / e.sum()) @ Vd.astype(np.float64))) < 1e-12


def test_generator_shapes():
    spec = W.SPECS["c3_13b_subset"]
    pw = W.make_pairs_workload(spec)
    assert pw.block_table.shape == (pw.n_pairs, spec.max_blocks_per_seq)
    assert 0.7 * 13 * spec.batch < pw.n_pairs < 1.3 * 13 * spec.batch
    used = pw.block_table[pw.block_table >= 0]
    assert len(np.unique(used)) == len(used) and used.max() < pw.num_tiles
    need = (pw.seq_lens[pw.pair_seq].astype(np.int64) + 15) // 16
    assert int(need.sum()) == len(used)
