"""How a launch hands out its work must not show in the results.  Calls with few rows
(sequences x selected heads, or pairs) hand out single chunks, whose results meet in the
workspace; calls with many rows hand out whole segments, folded inside a workgroup.  Both
must give the same bits: a head subset (few rows) against the all-heads run (many rows), a
call that was given a workspace too small for single chunks against one that was not."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_08309_amd as H
from paper_2509_08309_amd import workloads as W

from gpu_harness import SENTINEL, TOL, Dev, bits, check_rows, no_expired_wait, selected_rows

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

# lengths around block, chunk, fine-chunk and segment boundaries, one to several segments
LENS = [0, 1, 17, 64, 65, 255, 256, 257, 1000, 1024, 1025, 2047, 3000, 4095, 4096, 4097, 4200,
        5000, 8192, 8193, 9000, 12288, 13001]


def last_mode(ws):
    """How the last launch on this workspace handed out its work: 1 whole segments, 3 single chunks."""
    torch.cuda.synchronize()
    return int(ws[:16].view(torch.int32)[3].item())


def segments_workspace_bytes(shape, n_rows, r, D):
    """Size of a workspace that holds one slot per segment only."""
    segs = (shape.max_blocks_per_seq * 16 + 4095) // 4096
    if segs <= 1:
        return 256
    rows = n_rows * segs * r
    return 256 + 4 * (1 << 18) + rows * D * 4 + (rows * 4 + 255) // 256 * 256


@pytest.mark.parametrize("Hq,Hkv,D,sub", [
    (24, 24, 128, [0, 5, 6, 23]),       # 23 x 24 = 552 rows against 92
    (48, 24, 64, [1, 2, 22]),           # r = 2
    (96, 24, 128, [3, 11]),             # r = 4
    (192, 24, 128, [7]),                # r = 8
])
def test_subset_in_single_chunks_equals_all_heads_in_segments(Hq, Hkv, D, sub):
    w = W.make_custom(LENS, Hq, Hkv, D, sub, seed=901, device=DEV)
    assert len(LENS) * Hkv >= 512 > len(LENS) * len(sub)
    d = Dev(w)
    full = d.decode(list(range(Hkv)))
    part = d.decode(sub)
    rows = selected_rows(w.spec, sub)
    assert np.array_equal(bits(part)[:, rows], bits(full)[:, rows])
    rest = [h for h in range(Hq) if h not in rows]
    assert (bits(part)[:, rest] == SENTINEL).all()
    ref = oracle.attn_decode(w.q.cpu().numpy(), w.k_cache.cpu().numpy(), w.v_cache.cpu().numpy(),
                             w.block_table, w.seq_lens, np.asarray(sub, dtype=np.int32), w.spec.scale)
    check_rows(part, ref, rows, TOL, "single chunks")
    assert np.array_equal(bits(d.decode(sub)), bits(part))          # deterministic
    # the two runs really were handed out differently
    ws = d.workspace(len(sub))
    assert np.array_equal(bits(d.decode_ws(sub, ws)), bits(part)) and last_mode(ws) == 3
    ws = d.workspace(Hkv)
    assert np.array_equal(bits(d.decode_ws(list(range(Hkv)), ws)), bits(full)) and last_mode(ws) == 1


@pytest.mark.parametrize("Hq,Hkv,D,heads", [(8, 8, 128, [0, 2, 5, 7]), (16, 2, 128, [1])])
def test_a_workspace_for_segments_only_gives_the_same_bits(Hq, Hkv, D, heads):
    w = W.make_custom(LENS, Hq, Hkv, D, heads, seed=902, device=DEV)
    d = Dev(w)
    big = d.workspace(len(heads))
    ref = d.decode_ws(heads, big)
    n_small = segments_workspace_bytes(d.shape, len(LENS) * len(heads), Hq // Hkv, D)
    assert n_small < big.numel()
    small = torch.empty(n_small, dtype=torch.uint8, device=DEV)
    H.check(H.hetis_attn_workspace_init(small, n_small), "workspace_init")
    assert last_mode(big) == 3
    for _ in range(2):
        out = d.decode_ws(heads, small)
        assert np.array_equal(bits(out), bits(ref))
    assert last_mode(small) == 1
    # one byte less is not enough for anything
    hid, n = d.heads(heads)
    rc = H.hetis_attn_decode_ws(d.shape, d.q, d.k, d.v, d.bt, d.sl, hid, n, d.scale, d.new_out(),
                                small, n_small - 1)
    assert rc == H.binding.HETIS_ERR_WORKSPACE
    torch.cuda.synchronize()


def test_pairs_in_single_chunks_equal_pairs_in_segments():
    """The pairs of a few requests alone (few rows) against the same pairs among those of many
    requests (many rows)."""
    Hkv, D = 8, 128
    rng = np.random.default_rng(903)
    lens = list(LENS) + [int(x) for x in rng.integers(1, 1500, size=120)]
    w = W.make_custom(lens, Hkv, Hkv, D, list(range(Hkv)), seed=904, device=DEV)
    subsets = W.draw_head_subsets(len(lens), Hkv, Hkv / 2, rng)
    pair_seq = np.concatenate([np.full(len(h), b, dtype=np.int32) for b, h in enumerate(subsets)])
    pair_head = np.concatenate(subsets).astype(np.int32)
    table = (w.block_table[pair_seq] * Hkv + pair_head[:, None]).astype(np.int32)
    table[w.block_table[pair_seq] < 0] = -1
    assert len(pair_seq) >= 512
    few = np.flatnonzero(pair_seq < len(LENS))              # the pairs of the first requests
    assert 0 < len(few) < 512
    k_tiles, v_tiles = w.k_cache.view(-1, 16, D), w.v_cache.view(-1, 16, D)
    shape = H.make_shape(len(lens), Hkv, Hkv, D, w.block_table.shape[1])

    def run(idx):
        out = torch.empty((len(lens), Hkv, D), dtype=torch.float16, device=DEV)
        out.view(torch.int16).fill_(np.int16(SENTINEL))
        bt = torch.from_numpy(np.ascontiguousarray(table[idx])).to(DEV)
        sl = torch.from_numpy(w.seq_lens).to(DEV)
        ps = torch.from_numpy(np.ascontiguousarray(pair_seq[idx])).to(DEV)
        ph = torch.from_numpy(np.ascontiguousarray(pair_head[idx])).to(DEV)
        H.check(H.hetis_attn_decode_pairs(shape, w.q, k_tiles, v_tiles, bt, sl, ps, ph, len(idx),
                                          w.spec.scale, out), "hetis_attn_decode_pairs")
        torch.cuda.synchronize()
        no_expired_wait()
        return out

    many = run(np.arange(len(pair_seq)))
    alone = run(few)
    m = np.zeros((len(lens), Hkv), dtype=bool)
    m[pair_seq[few], pair_head[few]] = True
    assert (bits(alone)[m] == bits(many)[m]).all()
    assert (bits(alone)[~m] == SENTINEL).all()


def test_long_rows_few_heads_against_the_checker():
    """Rows of several segments handed out as single chunks: every piece of the combination
    (chunks of a segment in order, then the segments) against the fp64 checker."""
    lens = [32768, 20000, 4097, 16384, 1, 0, 12289, 31000]
    heads = [1, 2]
    w = W.make_custom(lens, 4, 4, 128, heads, seed=905, device=DEV)
    d = Dev(w)
    out = d.decode(heads)
    ref = oracle.attn_decode(w.q.cpu().numpy(), w.k_cache.cpu().numpy(), w.v_cache.cpu().numpy(),
                             w.block_table, w.seq_lens, np.asarray(heads, dtype=np.int32), w.spec.scale)
    check_rows(out, ref, selected_rows(w.spec, heads), TOL, "long rows")
    for _ in range(3):
        assert np.array_equal(bits(d.decode(heads)), bits(out))


def test_few_rows_of_many_segments_are_handed_out_as_segments():
    """Fewer than 512 rows, so the host lays the workspace out for single chunks, but more
    segments than workgroups: the kernel hands out whole segments inside that layout, and the
    partial results of the rows' segments are merged inside the launch."""
    lens = [32768] * 20 + [20000] * 19 + [4097, 300, 0]
    w = W.make_custom(lens, 2, 1, 64, [0], seed=906, device=DEV)           # r = 2
    d = Dev(w)
    ws = d.workspace(1)
    out = d.decode_ws([0], ws)
    assert last_mode(ws) == 1
    ref = oracle.attn_decode(w.q.cpu().numpy(), w.k_cache.cpu().numpy(), w.v_cache.cpu().numpy(),
                             w.block_table, w.seq_lens, np.asarray([0], dtype=np.int32), w.spec.scale)
    check_rows(out, ref, selected_rows(w.spec, [0]), TOL, "segments inside the chunk layout")
    # the first sequences alone: few segments, single chunks, same bits
    k = 12
    w2 = W.Workload(W.WorkloadSpec("custom", k, 2, 1, 64, (0,), 906, "fixed", (tuple(lens[:k]),), max(lens)),
                    w.seq_lens[:k], w.block_table[:k], w.num_blocks, w.q[:k], w.k_cache, w.v_cache,
                    np.asarray([0], dtype=np.int32))
    d2 = Dev(w2)
    ws2 = d2.workspace(1)
    out2 = d2.decode_ws([0], ws2)
    assert last_mode(ws2) == 3
    assert np.array_equal(bits(out2), bits(out)[:k])


@pytest.mark.parametrize("Hq,Hkv,D", [(2, 2, 64), (8, 2, 128), (16, 2, 64)])
def test_one_or_two_very_long_rows(Hq, Hkv, D):
    """A launch of a handful of rows of tens of segments each: single chunks all over the device,
    per-segment folds, one merge per row."""
    lens = [100000, 70001]
    w = W.make_custom(lens, Hq, Hkv, D, [0, 1], seed=907, device=DEV)
    d = Dev(w)
    ws = d.workspace(2)
    out = d.decode_ws([0, 1], ws)
    assert last_mode(ws) == 3
    ref = oracle.attn_decode(w.q.cpu().numpy(), w.k_cache.cpu().numpy(), w.v_cache.cpu().numpy(),
                             w.block_table, w.seq_lens, np.asarray([0, 1], dtype=np.int32), w.spec.scale)
    check_rows(out, ref, selected_rows(w.spec, [0, 1]), TOL, "very long rows")
    one = d.decode([1])
    rows = selected_rows(w.spec, [1])
    assert np.array_equal(bits(one)[:, rows], bits(out)[:, rows])


@pytest.mark.parametrize("Hq,Hkv,D", [(8, 8, 128), (16, 8, 64), (32, 8, 128), (64, 8, 128)])
def test_a_wider_block_table_changes_nothing(Hq, Hkv, D):
    """The same rows described by a block table that would allow rows of several segments: the
    launch then runs the kernel's other instantiation (the one that can combine partial results
    inside the launch) on a workspace with arrival counters, and must give the same bits."""
    lens = [4096, 4095, 3000, 2049, 2048, 1025, 1024, 513, 300, 256, 255, 100, 17, 16, 1, 0] * 20
    heads = list(range(Hkv))
    narrow = W.make_custom(lens, Hq, Hkv, D, heads, seed=908, device=DEV)
    wide = W.make_custom(lens, Hq, Hkv, D, heads, seed=908, device=DEV, max_seq_len=3 * 4096)
    assert narrow.block_table.shape[1] == 256 and wide.block_table.shape[1] == 768
    assert np.array_equal(wide.block_table[:, :256], narrow.block_table)
    assert torch.equal(wide.k_cache.view(torch.int16), narrow.k_cache.view(torch.int16))     # (NaN in unused slots)
    assert torch.equal(wide.v_cache.view(torch.int16), narrow.v_cache.view(torch.int16))
    assert torch.equal(wide.q, narrow.q)
    dn, dw = Dev(narrow), Dev(wide)
    rc, n_narrow = H.hetis_attn_decode_workspace_bytes(dn.shape, Hkv)
    rc2, n_wide = H.hetis_attn_decode_workspace_bytes(dw.shape, Hkv)
    assert rc == 0 and rc2 == 0 and n_narrow == 256 < n_wide       # control words only / counters and slots
    a, b = dn.decode(heads), dw.decode(heads)
    assert np.array_equal(bits(a), bits(b))
    sub = [1, 6]
    assert np.array_equal(bits(dn.decode(sub)), bits(dw.decode(sub)))
    rows = selected_rows(narrow.spec, sub)
    assert np.array_equal(bits(dw.decode(sub))[:, rows], bits(a)[:, rows])
