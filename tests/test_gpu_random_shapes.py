"""Seeded random shapes, lengths and head subsets through hetis_attn_decode, hetis_attn_decode_step and
hetis_attn_decode_pairs against the fp64 checker, all selected rows, and against each other bit for
bit (a subset equals the slice of the all-heads run; pairs equal the common form)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2509_08309_amd as H
from paper_2509_08309_amd import workloads as W

from gpu_harness import SENTINEL, TOL, Dev, bits, check_rows, no_expired_wait, selected_rows

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def draw_case(seed):
    rng = np.random.default_rng(seed)
    r = int(rng.choice([1, 1, 2, 4, 8]))
    Hkv = int(rng.choice([1, 2, 3, 5, 8, 12]))
    D = int(rng.choice([64, 128]))
    B = int(rng.choice([1, 2, 5, 17, 40, 130]))
    kind = rng.choice(["short", "mixed", "long", "edges"])
    if kind == "short":
        lens = rng.integers(0, 300, size=B)
    elif kind == "mixed":
        lens = np.exp(rng.normal(np.log(600), 1.0, size=B)).astype(np.int64).clip(0, 9000)
    elif kind == "long":
        lens = rng.integers(3000, 14000, size=B)
    else:
        lens = rng.choice([0, 1, 15, 16, 17, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 512, 513,
                           1023, 1024, 1025, 4095, 4096, 4097, 8191, 8192, 8193], size=B)
    lens = np.minimum(lens, max(1, 400000 // (B * Hkv)))        # bound the pool
    n_sel = int(rng.integers(1, Hkv + 1))
    sub = sorted(rng.choice(Hkv, size=n_sel, replace=False).tolist())
    return r, Hkv, D, [int(x) for x in lens], sub


@pytest.mark.parametrize("seed", range(3000, 3024))
def test_random_case(seed):
    r, Hkv, D, lens, sub = draw_case(seed)
    w = W.make_custom(lens, Hkv * r, Hkv, D, sub, seed=seed, device=DEV)
    d = Dev(w)
    full = d.decode(list(range(Hkv)))
    part = d.decode(sub)
    rows = selected_rows(w.spec, sub)
    assert np.array_equal(bits(part)[:, rows], bits(full)[:, rows]), (r, Hkv, D, len(lens), sub)
    rest = [h for h in range(Hkv * r) if h not in set(rows)]
    if rest:
        assert (bits(part)[:, rest] == SENTINEL).all()
    ref = oracle.attn_decode(w.q.cpu().numpy(), w.k_cache.cpu().numpy(), w.v_cache.cpu().numpy(),
                             w.block_table, w.seq_lens, np.asarray(sub, dtype=np.int32), w.spec.scale)
    check_rows(part, ref, rows, TOL, f"seed {seed}")
    # the same (sequence, head) combinations as pairs over the same tiles
    ps = np.repeat(np.arange(len(lens), dtype=np.int32), len(sub))
    ph = np.tile(np.asarray(sub, dtype=np.int32), len(lens))
    perm = np.random.default_rng(seed + 1).permutation(len(ps))
    ps, ph = ps[perm], ph[perm]
    table = (w.block_table[ps].astype(np.int64) * Hkv + ph[:, None]).astype(np.int32)
    table[w.block_table[ps] < 0] = -1
    out = d.new_out()
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    H.check(H.hetis_attn_decode_pairs(d.shape, d.q, d.k.view(-1, 16, D), d.v.view(-1, 16, D), to(table),
                                      d.sl, to(ps), to(ph), len(ps), d.scale, out), "decode_pairs")
    torch.cuda.synchronize()
    no_expired_wait()
    assert np.array_equal(bits(out), bits(part))
    # one decode step: new rows stored by the call, then the same Attention
    kn, vn = W.new_token_rows(w)
    two_k, two_v = d.k.clone(), d.v.clone()
    hid, n = d.heads(sub)
    H.check(H.hetis_kv_append(d.shape, kn, vn, d.bt, d.sl, hid, n, w.num_blocks, two_k, two_v), "append")
    out_two = d.new_out()
    H.check(H.hetis_attn_decode(d.shape, d.q, two_k, two_v, d.bt, d.sl, hid, n, d.scale, out_two), "decode")
    one_k, one_v, out_one = d.k.clone(), d.v.clone(), d.new_out()
    H.check(H.hetis_attn_decode_step(d.shape, d.q, kn, vn, one_k, one_v, d.bt, d.sl, hid, n, d.scale,
                                     out_one), "decode_step")
    torch.cuda.synchronize()
    no_expired_wait()
    assert torch.equal(one_k.view(torch.int16), two_k.view(torch.int16))
    assert torch.equal(one_v.view(torch.int16), two_v.view(torch.int16))
    assert torch.equal(out_one.view(torch.int16), out_two.view(torch.int16))
