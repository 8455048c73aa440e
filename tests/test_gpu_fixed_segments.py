"""Launches around the numbers of segments at which the hand-out changes: up to one segment a
workgroup (no tickets), up to two (every workgroup's second segment is fixed as well: some have
one, some none), up to three (a fixed third for some), up to four (three fixed, the rest drawn),
more (one fixed, the rest drawn).
Every row against the fp64 checker, the decode step against append + decode bit for bit, and
a head subset against the all-heads run bit for bit (the two launches are on different sides of
such a boundary)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_08309_amd as H
from paper_2509_08309_amd import workloads as W

from gpu_harness import SENTINEL, TOL, Dev, bits, check_rows, selected_rows
from test_gpu_step import check_step

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def workgroups():
    return torch.cuda.get_device_properties(0).multi_processor_count


def lengths(n, seed, longest):
    rng = np.random.default_rng(seed)
    # (no row much longer than the rest: the kernel fixes second and third segments only when
    # the longest row is well below a workgroup's share of the tokens)
    lens = rng.integers(longest // 2, longest + 1, size=n)
    lens[rng.integers(0, n, size=max(1, n // 50))] = 0          # a few empty sequences
    lens[:4] = [longest, 1, 16, 17]
    return [int(x) for x in lens]


@pytest.mark.parametrize("delta", [-1, 0, 1])
@pytest.mark.parametrize("per_wg", [1, 2, 3, 4])
@pytest.mark.parametrize("Hq,Hkv,D", [(2, 2, 128), (16, 2, 64)])
def test_rows_around_the_boundaries(per_wg, delta, Hq, Hkv, D):
    G = workgroups()
    n_sel = 2
    batch = (per_wg * G) // n_sel + delta           # rows = batch x 2: per_wg x G - 2, + 0, + 2
    # rows of up to 1000 tokens: also below the number of rows at which single chunks are offered
    # the kernel hands out whole segments (no row is longer than one turn of a workgroup)
    w = W.make_custom(lengths(batch, 1100 + per_wg, 1000), Hq, Hkv, D, [0, 1], seed=1200 + per_wg,
                      device=DEV)
    d = Dev(w)
    out = d.decode([0, 1])
    ref = oracle.attn_decode(w.q.cpu().numpy(), w.k_cache.cpu().numpy(), w.v_cache.cpu().numpy(),
                             w.block_table, w.seq_lens, np.asarray([0, 1], dtype=np.int32), w.spec.scale)
    check_rows(out, ref, selected_rows(w.spec, [0, 1]), TOL, f"{per_wg} segments a workgroup")
    assert np.array_equal(bits(d.decode([0, 1])), bits(out))
    # half the rows: the other side of a boundary, same bits
    one = d.decode([1])
    rows = selected_rows(w.spec, [1])
    assert np.array_equal(bits(one)[:, rows], bits(out)[:, rows])
    rest = [h for h in range(Hq) if h not in rows]
    assert (bits(one)[:, rest] == SENTINEL).all()


@pytest.mark.parametrize("per_wg,Hq,Hkv,D", [(2, 4, 4, 128), (3, 32, 4, 128), (4, 8, 4, 64), (5, 4, 4, 128)])
def test_step_with_fixed_second_segments(per_wg, Hq, Hkv, D):
    """The store of the new token inside a launch whose second segments are fixed (and, with five
    segments a workgroup, one that draws them): rows of up to one segment, many of them ending in
    the chunk that the writer wave holds back until the new rows are stored."""
    G = workgroups()
    heads = list(range(Hkv))
    batch = per_wg * G // Hkv - 1
    w = W.make_custom(lengths(batch, 1300 + per_wg, 4096), Hq, Hkv, D, heads, seed=1400 + per_wg,
                      device=DEV)
    check_step(w, heads)
