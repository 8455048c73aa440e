"""Parity of hetis_attn_decode_pairs (per-request head subsets over single-head tiles) against
the CPU checker, and bit-identity with the common-subset entry point."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_08309_amd as H
from paper_2509_08309_amd import workloads as W

from gpu_harness import SENTINEL, TOL, Dev, as_f64, bits, check_mask, no_expired_wait

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def i32(a):
    return torch.from_numpy(np.ascontiguousarray(np.asarray(a, dtype=np.int32))).to(DEV)


def spec_of(lens, Hq, Hkv, D, seed):
    lens = tuple(int(x) for x in lens)
    return W.WorkloadSpec("pairs", len(lens), Hq, Hkv, D, tuple(range(Hkv)), seed, "fixed", (lens,),
                          max(max(lens), 1))


def run_pairs(pw, order=None, out=None):
    s = pw.spec
    idx = np.arange(pw.n_pairs) if order is None else np.asarray(order)
    shape = H.make_shape(s.batch, s.n_q_heads, s.n_kv_heads, s.head_dim, pw.block_table.shape[1])
    bt, sl = i32(pw.block_table[idx]), i32(pw.seq_lens)
    ps, ph = i32(pw.pair_seq[idx]), i32(pw.pair_head[idx])
    H.check(H.hetis_attn_validate_pairs(shape, bt, sl, ps, ph, len(idx), pw.num_tiles),
            "validate_pairs")
    if out is None:
        out = torch.empty_like(pw.q)
        out.view(torch.int16).fill_(np.int16(SENTINEL))
    H.check(H.hetis_attn_decode_pairs(shape, pw.q, pw.k_tiles, pw.v_tiles, bt, sl, ps, ph,
                                      len(idx), s.scale, out), "hetis_attn_decode_pairs")
    torch.cuda.synchronize()
    no_expired_wait()
    return out


def named_rows(pw):
    r = pw.spec.group_size
    m = np.zeros((pw.spec.batch, pw.spec.n_q_heads), dtype=bool)
    for b, g in zip(pw.pair_seq, pw.pair_head):
        m[b, g * r:(g + 1) * r] = True
    return m


def oracle_pairs(pw, pick=None):
    idx = np.arange(pw.n_pairs) if pick is None else np.asarray(pick)
    return oracle.attn_decode_pairs(pw.q.cpu().numpy(), pw.k_tiles.cpu().numpy(),
                                    pw.v_tiles.cpu().numpy(), pw.block_table[idx], pw.seq_lens,
                                    pw.pair_seq[idx], pw.pair_head[idx], pw.spec.n_kv_heads,
                                    pw.spec.scale)


@pytest.mark.parametrize("Hq,Hkv,D", [(8, 8, 64), (6, 6, 128), (16, 8, 128), (16, 4, 64),
                                      (32, 4, 128)])
def test_pairs_small(Hq, Hkv, D):
    lens = [1, 15, 16, 17, 100, 255, 256, 257, 0, 600, 1025, 31]
    rng = np.random.default_rng(61)
    subsets = W.draw_head_subsets(len(lens), Hkv, Hkv / 2, rng)
    subsets[0] = np.arange(Hkv, dtype=np.int32)          # one request with every head
    subsets[3] = np.zeros(0, dtype=np.int32)             # one with none on this device
    subsets[8] = np.array([Hkv - 1], dtype=np.int32)     # the empty sequence has a pair
    pw = W.make_pairs_workload(spec_of(lens, Hq, Hkv, D, 62), device=DEV, subsets=subsets)
    out = run_pairs(pw)
    ref = oracle_pairs(pw)
    m = named_rows(pw)
    check_mask(out, ref, m, TOL, "pairs small")
    # order of the pairs does not matter, bit for bit; run to run deterministic
    order = rng.permutation(pw.n_pairs)
    assert torch.equal(run_pairs(pw, order).view(torch.int16), out.view(torch.int16))
    assert torch.equal(run_pairs(pw).view(torch.int16), out.view(torch.int16))


@pytest.mark.parametrize("Hq,Hkv,D", [(8, 8, 128), (16, 2, 128)])
def test_pairs_rows_equal_the_common_subset_rows_bitwise(Hq, Hkv, D):
    """A standard pool read as single-head tiles (tile = block * Hkv + head): every pair's rows
    must be the rows hetis_attn_decode computes for all heads."""
    lens = [40, 256, 257, 700, 1500, 16, 3]
    w = W.make_custom(lens, Hq, Hkv, D, list(range(Hkv)), seed=63, device=DEV)
    full = Dev(w).decode(list(range(Hkv)))
    rng = np.random.default_rng(64)
    subsets = W.draw_head_subsets(len(lens), Hkv, Hkv / 2, rng)
    subsets[1] = np.arange(Hkv, dtype=np.int32)
    pair_seq = np.concatenate([np.full(len(h), b, dtype=np.int32) for b, h in enumerate(subsets)])
    pair_head = np.concatenate(subsets).astype(np.int32)
    table = w.block_table[pair_seq] * Hkv + pair_head[:, None]
    table[w.block_table[pair_seq] < 0] = -1
    pw = W.PairsWorkload(w.spec, w.seq_lens, pair_seq, pair_head, table.astype(np.int32),
                         w.num_blocks * Hkv, w.q, w.k_cache.view(-1, 16, D),
                         w.v_cache.view(-1, 16, D))
    out = run_pairs(pw)
    m = named_rows(pw)
    assert (bits(out)[m] == bits(full)[m]).all()
    assert (bits(out)[~m] == SENTINEL).all()


@pytest.mark.parametrize("name", ["c3_13b_subset", "c5_70b_gqa"])
def test_pairs_full_size(name):
    """The device's share when every request has its own head subset (13 of 40 heads on
    average for the 13B shape; 3 of 8 groups for the grouped-query shape): every named row
    against the checker, every other row untouched."""
    spec = W.SPECS[name]
    pw = W.make_pairs_workload(spec, device=DEV)
    out = run_pairs(pw)
    check_mask(out, oracle_pairs(pw), named_rows(pw), TOL, name)


def test_more_pairs_than_the_persistent_kernel_holds():
    """2500 pairs: more than one launch holds; they run as two launches over slices of the pairs."""
    rng = np.random.default_rng(66)
    B, Hkv, D = 250, 10, 64
    lens = rng.integers(1, 400, size=B)
    subsets = [np.arange(Hkv, dtype=np.int32) for _ in range(B)]
    pw = W.make_pairs_workload(spec_of(lens, Hkv, Hkv, D, 67), device=DEV, subsets=subsets)
    assert pw.n_pairs == 2500
    out = run_pairs(pw)
    check_mask(out, oracle_pairs(pw), named_rows(pw), TOL, "2500 pairs")


def test_no_pairs_and_bad_content():
    lens = [20, 7]
    pw = W.make_pairs_workload(spec_of(lens, 4, 4, 64, 68), device=DEV, subsets=[[0, 2], [1]])
    s = pw.spec
    shape = H.make_shape(s.batch, s.n_q_heads, s.n_kv_heads, s.head_dim, pw.block_table.shape[1])
    out = torch.empty_like(pw.q)
    out.view(torch.int16).fill_(np.int16(SENTINEL))
    assert H.hetis_attn_decode_pairs(shape, pw.q, pw.k_tiles, pw.v_tiles, i32(pw.block_table),
                                     i32(pw.seq_lens), i32(pw.pair_seq), i32(pw.pair_head), 0,
                                     s.scale, out) == 0
    torch.cuda.synchronize()
    assert (bits(out) == SENTINEL).all()
    bad = H.binding.HETIS_ERR_BAD_CONTENT
    v = lambda bt, ps, ph, nt=pw.num_tiles: H.hetis_attn_validate_pairs(
        shape, i32(bt), i32(pw.seq_lens), i32(ps), i32(ph), pw.n_pairs, nt)
    assert v(pw.block_table, pw.pair_seq, pw.pair_head) == 0
    assert v(pw.block_table, [0, 0, 2], pw.pair_head) == bad
    assert v(pw.block_table, pw.pair_seq, [0, 4, 1]) == bad
    assert v(pw.block_table, pw.pair_seq, pw.pair_head, nt=int(pw.block_table.max())) == bad
    t = pw.block_table.copy()
    t[2, 0] = -1
    assert v(t, pw.pair_seq, pw.pair_head) == bad


def test_pairs_at_the_persistent_kernel_limit_grouped_query():
    """2048 pairs of a grouped-query shape (r = 8, D = 128): the largest LDS footprint the
    persistent kernel can ask for (tables of 2048 rows, mailboxes of 8 rows, MFMA staging)."""
    rng = np.random.default_rng(69)
    B, Hq, Hkv, D = 256, 64, 8, 128
    lens = rng.integers(1, 900, size=B)
    subsets = [np.arange(Hkv, dtype=np.int32) for _ in range(B)]
    pw = W.make_pairs_workload(spec_of(lens, Hq, Hkv, D, 70), device=DEV, subsets=subsets)
    assert pw.n_pairs == 2048
    out = run_pairs(pw)
    check_mask(out, oracle_pairs(pw), named_rows(pw), TOL, "2048 grouped-query pairs")


@pytest.mark.parametrize("name", [None, "c3_13b_subset"])
def test_append_pairs_then_decode_pairs(name):
    """The decode step of the pairs form: the new rows go into the single-head tiles through
    the per-pair tables (bit-exact against the checker, whole pools compared), then Attention
    over the appended pools matches the checker on the checker's own appended pools."""
    if name is None:
        lens = [1, 16, 17, 255, 256, 300, 0, 1025]
        rng = np.random.default_rng(71)
        subsets = W.draw_head_subsets(len(lens), 8, 3, rng)
        subsets[0] = np.arange(8, dtype=np.int32)
        subsets[6] = np.array([2], dtype=np.int32)
        pw = W.make_pairs_workload(spec_of(lens, 16, 8, 128, 72), device=DEV, subsets=subsets)
    else:
        pw = W.make_pairs_workload(W.SPECS[name], device=DEV)
    s = pw.spec
    gen = torch.Generator(device=DEV)
    gen.manual_seed(73)
    kn = torch.randn((s.batch, s.n_kv_heads, s.head_dim), generator=gen, device=DEV).half()
    vn = torch.randn((s.batch, s.n_kv_heads, s.head_dim), generator=gen, device=DEV).half()
    ref_k, ref_v = oracle.kv_append_pairs(bits(pw.k_tiles), bits(pw.v_tiles), bits(kn), bits(vn),
                                          pw.block_table, pw.seq_lens, pw.pair_seq, pw.pair_head)
    shape = H.make_shape(s.batch, s.n_q_heads, s.n_kv_heads, s.head_dim, pw.block_table.shape[1])
    H.check(H.hetis_kv_append_pairs(shape, kn, vn, i32(pw.block_table), i32(pw.seq_lens),
                                    i32(pw.pair_seq), i32(pw.pair_head), pw.n_pairs, pw.num_tiles,
                                    pw.k_tiles, pw.v_tiles), "hetis_kv_append_pairs")
    torch.cuda.synchronize()
    same = lambda t, ref: bool(torch.equal(t.view(torch.int16).reshape(-1),
                                           torch.from_numpy(ref.view(np.int16)).to(DEV).reshape(-1)))
    assert same(pw.k_tiles, ref_k) and same(pw.v_tiles, ref_v)
    out = run_pairs(pw)
    ref = oracle.attn_decode_pairs(pw.q.cpu().numpy(), ref_k.view(np.float16), ref_v.view(np.float16),
                                   pw.block_table, pw.seq_lens, pw.pair_seq, pw.pair_head,
                                   s.n_kv_heads, s.scale)
    check_mask(out, ref, named_rows(pw), TOL, "append_pairs then decode_pairs")


def test_append_pairs_skips_what_points_outside():
    lens = [20, 7, 64, 0]
    pw = W.make_pairs_workload(spec_of(lens, 4, 4, 64, 75), device=DEV,
                               subsets=[[0, 2], [1], [3], [0]])
    s = pw.spec
    kn = torch.ones((4, 4, 64), dtype=torch.float16, device=DEV)
    ps, ph, bt = pw.pair_seq.copy(), pw.pair_head.copy(), pw.block_table.copy()
    ps[0] = 4                  # sequence id past the batch
    ph[1] = -1                 # head id out of range
    bt[2, 0] = pw.num_tiles    # tile id past the pool
    ref_k, ref_v = oracle.kv_append_pairs(bits(pw.k_tiles), bits(pw.v_tiles), bits(kn), bits(kn), bt,
                                          pw.seq_lens, ps, ph)
    k, v = pw.k_tiles.clone(), pw.v_tiles.clone()
    shape = H.make_shape(4, 4, 4, 64, bt.shape[1])
    H.check(H.hetis_kv_append_pairs(shape, kn, kn, i32(bt), i32(pw.seq_lens), i32(ps), i32(ph),
                                    pw.n_pairs, pw.num_tiles, k, v), "hetis_kv_append_pairs")
    torch.cuda.synchronize()
    assert np.array_equal(bits(k), ref_k) and np.array_equal(bits(v), ref_v)
    # only the pair of sequence 2 was stored (sequence 3 is empty)
    assert int((bits(k) != bits(pw.k_tiles)).any(axis=-1).sum()) == 1


@pytest.mark.parametrize("name", ["few", "many", "c3_13b_subset", "c5_70b_gqa"])
def test_decode_pairs_step_equals_append_pairs_then_decode_pairs(name):
    """One call for the decode step of the pairs form: pools and outputs bit-identical to
    hetis_kv_append_pairs + hetis_attn_decode_pairs, and within tolerance of the checker on the
    checker's appended pools.  `few`: a handful of pairs (the store runs as a launch of its own);
    `many` and the named shapes: the store inside the Attention kernel."""
    if name in ("few", "many"):
        lens = [1, 16, 17, 255, 256, 300, 0, 1025, 4095, 4096, 4097, 5000]
        if name == "many":
            lens = lens * 12
        rng = np.random.default_rng(76)
        subsets = W.draw_head_subsets(len(lens), 8, 4, rng)
        subsets[0] = np.arange(8, dtype=np.int32)
        subsets[6] = np.array([2], dtype=np.int32)
        pw = W.make_pairs_workload(spec_of(lens, 16, 8, 128, 77), device=DEV, subsets=subsets)
        assert (pw.n_pairs >= 512) == (name == "many")
    else:
        pw = W.make_pairs_workload(W.SPECS[name], device=DEV)
    s = pw.spec
    gen = torch.Generator(device=DEV)
    gen.manual_seed(78)
    kn = torch.randn((s.batch, s.n_kv_heads, s.head_dim), generator=gen, device=DEV).half()
    vn = torch.randn((s.batch, s.n_kv_heads, s.head_dim), generator=gen, device=DEV).half()
    shape = H.make_shape(s.batch, s.n_q_heads, s.n_kv_heads, s.head_dim, pw.block_table.shape[1])
    bt, sl, ps, ph = i32(pw.block_table), i32(pw.seq_lens), i32(pw.pair_seq), i32(pw.pair_head)
    new_out = lambda: torch.full_like(pw.q, 0).view(torch.int16).fill_(np.int16(SENTINEL)).view(torch.float16)
    # two calls on copies of the pools
    k2, v2, out2 = pw.k_tiles.clone(), pw.v_tiles.clone(), new_out()
    H.check(H.hetis_kv_append_pairs(shape, kn, vn, bt, sl, ps, ph, pw.n_pairs, pw.num_tiles, k2, v2),
            "hetis_kv_append_pairs")
    H.check(H.hetis_attn_decode_pairs(shape, pw.q, k2, v2, bt, sl, ps, ph, pw.n_pairs, s.scale, out2),
            "hetis_attn_decode_pairs")
    # one call, once on the library's workspace and once on the caller's
    for use_ws in (False, True):
        k1, v1, out1 = pw.k_tiles.clone(), pw.v_tiles.clone(), new_out()
        if use_ws:
            rc, nbytes = H.hetis_attn_decode_pairs_workspace_bytes(shape, pw.n_pairs)
            H.check(rc, "pairs_workspace_bytes")
            ws = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
            H.check(H.hetis_attn_decode_pairs_step_ws(shape, pw.q, kn, vn, k1, v1, bt, sl, ps, ph,
                                                      pw.n_pairs, s.scale, out1, ws, nbytes),
                    "hetis_attn_decode_pairs_step_ws")
        else:
            ws = None
            H.check(H.hetis_attn_decode_pairs_step(shape, pw.q, kn, vn, k1, v1, bt, sl, ps, ph,
                                                   pw.n_pairs, s.scale, out1),
                    "hetis_attn_decode_pairs_step")
        torch.cuda.synchronize()
        no_expired_wait(ws)
        assert torch.equal(k1.view(torch.int16), k2.view(torch.int16))
        assert torch.equal(v1.view(torch.int16), v2.view(torch.int16))
        assert torch.equal(out1.view(torch.int16), out2.view(torch.int16))
    ref_k, ref_v = oracle.kv_append_pairs(bits(pw.k_tiles), bits(pw.v_tiles), bits(kn), bits(vn),
                                          pw.block_table, pw.seq_lens, pw.pair_seq, pw.pair_head)
    same = lambda t, ref: bool(torch.equal(t.view(torch.int16).reshape(-1),
                                           torch.from_numpy(ref.view(np.int16)).to(DEV).reshape(-1)))
    assert same(k1, ref_k) and same(v1, ref_v)
    ref = oracle.attn_decode_pairs(pw.q.cpu().numpy(), ref_k.view(np.float16), ref_v.view(np.float16),
                                   pw.block_table, pw.seq_lens, pw.pair_seq, pw.pair_head,
                                   s.n_kv_heads, s.scale)
    check_mask(out1, ref, named_rows(pw), TOL, "decode_pairs_step")
