"""The entry points that run from a caller-owned workspace (names ending in _ws): same bits
as the library-owned forms, safe on several streams at once and under stream capture, plus
the rules of the library-owned workspace around HIP graphs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_08309_amd as H
from paper_2509_08309_amd import workloads as W

from gpu_harness import (SENTINEL, TOL, Dev, bits, check_rows, host_copy, no_expired_wait,
                         selected_rows)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def i32(a):
    return torch.from_numpy(np.ascontiguousarray(np.asarray(a, dtype=np.int32))).to(DEV)


def test_decode_ws_equals_decode_bitwise_and_reuses_its_workspace():
    lens = [0, 1, 300, 257, 1500, 4000, 16, 777]
    heads = [0, 2, 5]
    w = W.make_custom(lens, 8, 8, 128, heads, seed=201, device=DEV)
    d = Dev(w)
    ref = d.decode(heads)
    ws = d.workspace(len(heads))
    for _ in range(3):                                   # the control words re-arm themselves
        out = d.decode_ws(heads, ws)
        assert torch.equal(out.view(torch.int16), ref.view(torch.int16))
    orc = oracle.attn_decode(w.q.cpu().numpy(), w.k_cache.cpu().numpy(), w.v_cache.cpu().numpy(),
                             w.block_table, w.seq_lens, np.asarray(heads, dtype=np.int32), w.spec.scale)
    check_rows(out, orc, selected_rows(w.spec, heads), TOL, "decode_ws")
    # a workspace too small even for whole segments (here: for the control words), or
    # misaligned, is refused before anything is launched
    hid, n = d.heads(heads)
    out2 = d.new_out()
    args = (d.shape, d.q, d.k, d.v, d.bt, d.sl, hid, n, d.scale, out2)
    assert H.hetis_attn_decode_ws(*args, ws, 255) == H.binding.HETIS_ERR_WORKSPACE
    assert H.hetis_attn_decode_ws(*args, ws.data_ptr() + 16, ws.numel()) == H.binding.HETIS_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert (bits(out2) == SENTINEL).all()
    # one byte short of the size asked for: the call hands out whole segments instead of single
    # chunks, which needs less, and gives the same bits
    assert H.hetis_attn_decode_ws(*args, ws, ws.numel() - 1) == H.binding.HETIS_OK
    torch.cuda.synchronize()
    assert torch.equal(out2.view(torch.int16), ref.view(torch.int16))


def test_concurrent_decode_ws_on_two_streams():
    """Two hetis_attn_decode_ws calls in flight at once, each with its own workspace and
    output, give the bits of the same calls run one after the other."""
    w1 = W.make_custom([2000, 900, 3000, 64, 1200, 4096], 8, 8, 128, [0, 3, 5, 7], seed=202, device=DEV)
    w2 = W.make_custom([1200, 2500, 300, 3333], 16, 2, 128, [1, 0], seed=203, device=DEV)
    devs, heads = [Dev(w1), Dev(w2)], [[0, 3, 5, 7], [1, 0]]
    serial = [d.decode(h) for d, h in zip(devs, heads)]
    wss = [d.workspace(len(h)) for d, h in zip(devs, heads)]
    outs = [d.new_out() for d in devs]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    hids = [d.heads(h) for d, h in zip(devs, heads)]     # alive until the final synchronize
    torch.cuda.synchronize()
    for rep in range(8):
        for d, h, ws, out, st, hid in zip(devs, heads, wss, outs, streams, hids):
            d.decode_ws(h, ws, out=out, stream=st, sync=False, hid=hid)
    torch.cuda.synchronize()
    for ws, out, ref in zip(wss, outs, serial):
        no_expired_wait(ws)
        assert torch.equal(out.view(torch.int16), ref.view(torch.int16))


def test_decode_ws_captured_with_no_eager_call_before():
    """The _ws form allocates nothing and never synchronises: its very first call may be made
    under stream capture."""
    w = W.make_custom([40, 300, 1500, 17, 700, 2049], 8, 8, 128, [1, 4, 6], seed=204, device=DEV)
    d = Dev(w)
    heads = [1, 4, 6]
    ws = d.workspace(len(heads))
    out = d.new_out()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    torch.cuda.synchronize()
    hid = d.heads(heads)                                 # the graph holds its address
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        d.decode_ws(heads, ws, out=out, stream=side, sync=False, hid=hid)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(205)
    for it in range(3):
        d.q.copy_(torch.randn(d.q.shape, generator=gen, device=DEV).half())
        out.view(torch.int16).fill_(np.int16(SENTINEL))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        no_expired_wait(ws)
        ref = d.decode(heads)
        assert torch.equal(out.view(torch.int16), ref.view(torch.int16)), f"replay {it}"


def test_library_workspace_and_graphs():
    """Library-owned workspace: a call on a capturing stream never allocates (it reports
    HETIS_ERR_WORKSPACE when the workspace is missing or too small); after
    hetis_attn_reserve_workspace it can be captured; a later, larger eager call gets a new
    buffer while the captured graph keeps replaying correctly from the old one."""
    small = W.make_custom([300, 700, 64, 1025], 4, 4, 128, [0, 1, 3], seed=206, device=DEV)
    large = W.make_custom(np.full(96, 2000), 16, 16, 128, list(range(16)), seed=207, device=DEV)
    ds, dl = Dev(small), Dev(large)
    heads = [0, 1, 3]
    hid, n = ds.heads(heads)
    H.check(H.hetis_attn_release_workspace(), "release")
    out = ds.new_out()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    torch.cuda.synchronize()
    g0 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g0, stream=side):
        out.view(torch.int16).fill_(np.int16(SENTINEL))        # something to capture
        rc = H.hetis_attn_decode(ds.shape, ds.q, ds.k, ds.v, ds.bt, ds.sl, hid, n, ds.scale, out, side)
    assert rc == H.binding.HETIS_ERR_WORKSPACE
    rc, need = H.hetis_attn_decode_workspace_bytes(ds.shape, n)
    H.check(rc, "workspace_bytes")
    H.check(H.hetis_attn_reserve_workspace(need), "reserve")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        H.check(H.hetis_attn_decode(ds.shape, ds.q, ds.k, ds.v, ds.bt, ds.sl, hid, n, ds.scale, out, side))
    g.replay()
    torch.cuda.synchronize()
    first = out.clone()
    ref = oracle.attn_decode(small.q.cpu().numpy(), small.k_cache.cpu().numpy(),
                             small.v_cache.cpu().numpy(), small.block_table, small.seq_lens,
                             np.asarray(heads, dtype=np.int32), small.spec.scale)
    check_rows(first, ref, selected_rows(small.spec, heads), TOL, "captured decode")
    # a much larger eager call: the library takes a new buffer, the old one stays alive
    big = dl.decode(list(range(16)))
    assert not torch.isnan(big.float()).any()
    for it in range(3):
        out.view(torch.int16).fill_(np.int16(SENTINEL))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), first.view(torch.int16)), f"replay {it}"
        dl.decode([3, 9])
    no_expired_wait()


def test_decode_pairs_ws_and_split_ws():
    lens = [1, 17, 300, 1025, 0, 2500, 256]
    rng = np.random.default_rng(208)
    subsets = W.draw_head_subsets(len(lens), 8, 3, rng)
    subsets[0] = np.arange(8, dtype=np.int32)
    spec = W.WorkloadSpec("pairs", len(lens), 16, 8, 128, tuple(range(8)), 209, "fixed",
                          (tuple(lens),), max(lens))
    pw = W.make_pairs_workload(spec, device=DEV, subsets=subsets)
    shape = H.make_shape(spec.batch, 16, 8, 128, pw.block_table.shape[1])
    bt, sl, ps, ph = i32(pw.block_table), i32(pw.seq_lens), i32(pw.pair_seq), i32(pw.pair_head)
    new_out = lambda: torch.full_like(pw.q, 0).view(torch.int16).fill_(np.int16(SENTINEL)).view(torch.float16)
    ref = new_out()
    H.check(H.hetis_attn_decode_pairs(shape, pw.q, pw.k_tiles, pw.v_tiles, bt, sl, ps, ph, pw.n_pairs,
                                      spec.scale, ref), "decode_pairs")
    rc, nbytes = H.hetis_attn_decode_pairs_workspace_bytes(shape, pw.n_pairs)
    H.check(rc, "pairs_workspace_bytes")
    ws = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    out = new_out()
    for _ in range(2):
        H.check(H.hetis_attn_decode_pairs_ws(shape, pw.q, pw.k_tiles, pw.v_tiles, bt, sl, ps, ph,
                                             pw.n_pairs, spec.scale, out, ws, nbytes), "decode_pairs_ws")
    torch.cuda.synchronize()
    no_expired_wait(ws)
    assert torch.equal(out.view(torch.int16), ref.view(torch.int16))
    assert H.hetis_attn_decode_pairs_ws(shape, pw.q, pw.k_tiles, pw.v_tiles, bt, sl, ps, ph,
                                        pw.n_pairs, spec.scale, out, ws, 128) \
        == H.binding.HETIS_ERR_WORKSPACE
    # split form with the caller's control words
    w = W.make_custom([700, 64, 1300, 2000], 8, 8, 128, [2, 6], seed=210, device=DEV)
    d = Dev(w)
    o_ref, lse_ref = d.split([2, 6], 512, 2000)
    hid, n = d.heads([2, 6])
    control = torch.zeros(H.binding.HETIS_ATTN_CONTROL_BYTES, dtype=torch.uint8, device=DEV)
    o_p, lse_p = torch.full_like(o_ref, float("nan")), torch.full_like(lse_ref, float("nan"))
    H.check(H.hetis_attn_decode_split_ws(d.shape, d.q, d.k, d.v, d.bt, d.sl, hid, n, d.scale, 512,
                                         2000, o_p, lse_p, control), "decode_split_ws")
    torch.cuda.synchronize()
    no_expired_wait(control)
    same = lambda a, b: torch.equal(a.view(torch.int32), b.view(torch.int32))
    assert same(o_p, o_ref) and same(lse_p, lse_ref)
