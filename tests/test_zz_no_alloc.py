"""hetis_attn_decode_static (the entry point that allocates nothing: its workspace is a static
device array inside the library) against hetis_attn_decode, through the C ABI: two calls in a
row, the second on a smaller input, both bit-identical to the allocating entry point."""
import numpy as np
import pytest
import torch

import paper_2509_08309_amd as H
from paper_2509_08309_amd import workloads as W

from gpu_harness import SENTINEL, Dev, bits, selected_rows

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def decode_static(d, heads):
    hid, n = d.heads(heads)
    out = d.new_out()
    H.check(H.hetis_attn_decode_static(d.shape, d.q, d.k, d.v, d.bt, d.sl, hid, n, d.scale, out),
            "hetis_attn_decode_static")
    torch.cuda.synchronize()
    return out


def test_static_scratch_matches_decode_on_two_calls_in_a_row():
    rng = np.random.default_rng(301)
    big_lens = np.clip(np.rint(rng.lognormal(np.log(900), 0.8, size=64)), 1, 4096).astype(int)
    big_lens[:4] = [4096, 0, 1, 257]
    big = W.make_custom(big_lens, 16, 16, 128, [0, 3, 4, 9, 15], seed=302, device=DEV)
    small = W.make_custom([700, 16, 300, 1300, 5], 8, 2, 128, [1], seed=303, device=DEV)
    for w, heads in ((big, [0, 3, 4, 9, 15]), (small, [1]), (big, [9, 3])):
        d = Dev(w)
        ref = d.decode(heads)                     # the allocating entry point
        got = decode_static(d, heads)
        rows = selected_rows(w.spec, heads)
        assert (bits(got)[:, rows] != SENTINEL).all()
        assert torch.equal(got.view(torch.int16), ref.view(torch.int16))


def test_static_scratch_refuses_what_does_not_fit():
    # 2048 sequences x 40 heads x 8 segments of partial rows need far more than the static array
    s = H.make_shape(2048, 40, 40, 128, 2048)
    rc, need = H.hetis_attn_decode_workspace_bytes(s, 40)
    assert rc == 0 and need > H.binding.HETIS_ATTN_STATIC_SCRATCH_BYTES
    P = 0x1000                                    # never touched: the call fails before any launch
    assert H.hetis_attn_decode_static(s, P, P, P, P, P, P, 40, 0.1, P, 0) == H.binding.HETIS_ERR_WORKSPACE
