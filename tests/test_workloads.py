"""The seeded input recipes: shapes, length ranges, block-table structure, poison."""
import numpy as np
import pytest

from paper_2509_08309_amd import workloads as W


@pytest.mark.parametrize("name", list(W.SPECS))
def test_lengths_and_table_structure(name):
    spec = W.SPECS[name]
    rng = np.random.default_rng(spec.seed)
    lens = W.draw_lengths(spec, rng)
    assert lens.shape == (spec.batch,) and lens.dtype == np.int32
    assert lens.min() >= 1 and lens.max() <= spec.max_seq_len
    table, nblk = W.build_block_table(lens, spec.max_blocks_per_seq, 16, rng)
    need = (lens.astype(np.int64) + 15) // 16
    assert nblk == need.sum()
    used = table[table >= 0]
    assert len(used) == nblk and len(np.unique(used)) == nblk      # a permutation, no sharing
    for b in range(spec.batch):
        assert (table[b, :need[b]] >= 0).all() and (table[b, need[b]:] == -1).all()


def test_named_length_distributions():
    s3 = W.SPECS["c3_13b_subset"]
    lens = W.draw_lengths(s3, np.random.default_rng(s3.seed))
    assert 32 <= lens.min() and lens.max() <= 4096 and 500 < np.median(lens) < 1300
    s1 = W.SPECS["c1_tiny"]
    assert list(W.draw_lengths(s1, np.random.default_rng(0))) == [17, 64, 130, 255]
    assert W.SPECS["c5_70b_gqa"].group_size == 8
    assert W.SPECS["c3_13b_subset"].head_ids == tuple(range(27, 40))


def test_tiny_workload_is_seeded_and_poisoned():
    a = W.make_workload(W.SPECS["c1_tiny"])
    b = W.make_workload(W.SPECS["c1_tiny"])
    assert np.array_equal(a.block_table, b.block_table)
    assert np.array_equal(a.k_cache.numpy().view(np.uint16), b.k_cache.numpy().view(np.uint16))
    assert a.num_blocks == 2 + 4 + 9 + 16
    k = a.k_cache.numpy()
    blk = a.block_table[0, 1]                     # L=17: slot 0 valid, slots 1..15 poisoned
    assert not np.isnan(k[blk, :, 0]).any() and np.isnan(k[blk, :, 1:]).all()
    assert a.kv_bytes() == 466 * 4 * 2 * 64 * 2


def test_same_seed_same_cache_for_the_two_7b_runs():
    a, b = W.SPECS["c2_7b_all"], W.SPECS["c2_7b_half"]
    la = W.draw_lengths(a, np.random.default_rng(a.seed))
    lb = W.draw_lengths(b, np.random.default_rng(b.seed))
    assert np.array_equal(la, lb)
