"""hetis_attn_decode_step: the decode-step store of the new token's K/V rows folded into the
Attention call (Section 5.1: store, then attend to all stored keys and values, the new one
included).  The cache must end up bit for bit as hetis_kv_append / the checker's append leave
it, and the output as hetis_attn_decode computes it on the appended cache."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_08309_amd as H
from paper_2509_08309_amd import workloads as W

from gpu_harness import SENTINEL, TOL, Dev, bits, check_rows, no_expired_wait, selected_rows

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_step(d, heads, kn, vn, ws=None):
    hid, n = d.heads(heads)
    out = d.new_out()
    if ws is None:
        H.check(H.hetis_attn_decode_step(d.shape, d.q, kn, vn, d.k, d.v, d.bt, d.sl, hid, n, d.scale,
                                         out), "hetis_attn_decode_step")
    else:
        H.check(H.hetis_attn_decode_step_ws(d.shape, d.q, kn, vn, d.k, d.v, d.bt, d.sl, hid, n,
                                            d.scale, out, ws, ws.numel()), "hetis_attn_decode_step_ws")
    torch.cuda.synchronize()
    no_expired_wait(ws)
    return out


def check_step(w, heads, use_ws=False):
    spec = w.spec
    kn, vn = W.new_token_rows(w)
    ref_k, ref_v = oracle.kv_append(bits(w.k_cache), bits(w.v_cache), bits(kn), bits(vn),
                                    w.block_table, w.seq_lens, heads)
    ref = oracle.attn_decode(w.q.cpu().numpy(), ref_k.view(np.float16), ref_v.view(np.float16),
                             w.block_table, w.seq_lens, np.asarray(heads, dtype=np.int32), spec.scale)
    # the two-call form on a copy of the cache
    two = Dev(w)
    two.k, two.v = w.k_cache.clone(), w.v_cache.clone()
    hid, n = two.heads(heads)
    H.check(H.hetis_kv_append(two.shape, kn, vn, two.bt, two.sl, hid, n, w.num_blocks, two.k, two.v),
            "hetis_kv_append")
    out_two = two.decode(heads)
    # the one-call form, in place on the workload's own cache
    one = Dev(w)
    ws = one.workspace(len(heads)) if use_ws else None
    out_one = run_step(one, heads, kn, vn, ws)
    same = lambda t, r: bool(torch.equal(t.view(torch.int16).reshape(-1),
                                         torch.from_numpy(r.view(np.int16)).to(DEV).reshape(-1)))
    assert same(one.k, ref_k) and same(one.v, ref_v), "cache differs from the checker's append"
    assert torch.equal(one.k.view(torch.int16), two.k.view(torch.int16))
    rows = selected_rows(spec, heads)
    check_rows(out_one, ref, rows, TOL, "decode_step")
    assert torch.equal(out_one.view(torch.int16), out_two.view(torch.int16)), \
        "one call differs from append + decode"
    rest = [h for h in range(spec.n_q_heads) if h not in set(rows)]
    if rest:
        assert (bits(out_one)[:, rest] == SENTINEL).all()
    return one, kn, vn, out_one


@pytest.mark.parametrize("Hq,Hkv,D,heads", [
    (4, 4, 64, [0, 2, 3]),
    (8, 8, 128, [1, 6]),
    (8, 4, 128, [0, 3]),       # r = 2
    (16, 2, 128, [1]),         # r = 8
    (8, 1, 64, [0]),           # r = 8, D = 64
    (32, 32, 128, list(range(32))),      # 576 rows: whole segments, the store inside the kernel
    (256, 32, 128, list(range(3, 32))),  # the same with r = 8
])
def test_step_edge_lengths(Hq, Hkv, D, heads):
    # lengths around block, chunk and segment boundaries; the new token is the last one counted
    lens = [0, 1, 2, 15, 16, 17, 33, 255, 256, 257, 511, 512, 513, 1000, 4095, 4096, 4097, 5000]
    w = W.make_custom(lens, Hq, Hkv, D, heads, seed=501, device=DEV)
    one, kn, vn, out = check_step(w, heads)
    # a second step on the same (already appended) cache gives the same bits
    again = run_step(one, heads, kn, vn)
    assert torch.equal(again.view(torch.int16), out.view(torch.int16))


@pytest.mark.parametrize("name", ["c1_tiny", "c3_13b_subset", "c5_70b_gqa"])
def test_step_full_size(name):
    spec = W.SPECS[name]
    w = W.make_workload(spec, device=DEV)
    check_step(w, list(spec.head_ids), use_ws=(name == "c3_13b_subset"))


def test_step_many_short_rows():
    """Thousands of one-chunk rows: the new row is stored by the wave that publishes the chunk,
    also when chunks are published in batches and when a workgroup's first chunk is the one
    that holds the new token."""
    rng = np.random.default_rng(502)
    lens = rng.integers(1, 300, size=1200)
    w = W.make_custom(lens, 4, 4, 128, [0, 1, 3], seed=503, device=DEV)
    check_step(w, [0, 1, 3])
