"""Profiler -> Dispatcher -> head-wise decode step, end to end on one GPU.

The coefficients fitted on this GPU (Section 5.1, Eq. (3)) describe three simulated devices;
hetis_dispatch_solve divides the heads of newly arrived requests among them (Section 5.2,
Eq. (5)-(7)); every device then holds single-head tiles of exactly its (request, head) pairs
(moved there with hetis_kv_copy_tiles), stores the new token's rows (hetis_kv_append_pairs) and
computes its share (hetis_attn_decode_pairs); the shares concatenated by head (Eq. (2a)) must be
the Attention of all heads: within tolerance of the checker, and bit-identical to one
hetis_attn_decode call over the undivided cache."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
import paper_2509_08309_amd as H
from oracle import dispatch_oracle as DO
from paper_2509_08309_amd import profiler
from paper_2509_08309_amd import workloads as W

from gpu_harness import SENTINEL, TOL, Dev, bits, check_rows, no_expired_wait

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def i32(a):
    return torch.from_numpy(np.ascontiguousarray(np.asarray(a, dtype=np.int32))).to(DEV)


@pytest.fixture(scope="module")
def fitted():
    rec = profiler.run("13b", reps=3, h_values=(128, 512, 1536),
                       g_values=(256 * 1024, 1024 * 1024, 2048 * 1024))
    a, b, c = rec["dispatcher_abc"]
    assert a >= 0 and b > 0 and c > 0
    return a, b, c


@pytest.mark.parametrize("Hq,Hkv", [(40, 40), (32, 8)])
def test_profiler_dispatcher_pairs_end_to_end(fitted, Hq, Hkv):
    a, b, c = fitted
    r, D, J, N = Hq // Hkv, 128, 16, 3
    rng = np.random.default_rng(401)
    lens = np.clip(np.rint(rng.lognormal(np.log(700), 0.9, size=J)), 2, 4096).astype(np.int32)
    lens[:3] = [4096, 2, 513]
    # three devices: this GPU as the Primary worker with some load already on it, and two slower
    # Attention workers behind links (Eq. (4)); the third cannot hold much cache
    unit = 2.0 / r                                       # cache units per query head and token
    devices = [dict(a=a, b=b, c=c, h=256.0, g=3.0e5, capacity=1e9, primary=True),
               dict(a=1.5 * a + 1e-4, b=2 * b, c=c, h=0.0, g=0.0, capacity=1e9, primary=False,
                    gamma=0.02, beta=5.0),
               dict(a=2 * a + 1e-4, b=3 * b, c=1.2 * c, h=64.0, g=1.0e4,
                    capacity=1.0e4 + unit * float(lens.sum()) * r * 2, primary=False,
                    gamma=0.05, beta=8.0)]
    cdev = (H.hetis_dispatch_device * N)()
    for i, d in enumerate(devices):
        cdev[i] = H.hetis_dispatch_device(d["a"], d["b"], d["c"], d.get("gamma", 0.0),
                                          d.get("beta", 0.0), d["h"], d["g"], d["capacity"],
                                          1 if d["primary"] else 0, 0)
    l = lens.astype(np.float64)
    x_frac, x_heads = np.zeros((J, N)), np.zeros((J, N), dtype=np.int32)
    z_lp, z_r = C.c_double(0), C.c_double(0)
    H.check(H.hetis_dispatch_solve(cdev, N, l, J, Hq, r, x_frac, x_heads, z_lp, z_r), "dispatch_solve")
    # Eq. (5): every request's heads are all placed, in whole groups of r
    assert (x_heads.sum(axis=1) == Hq).all() and (x_heads % r == 0).all() and (x_heads >= 0).all()
    ref = DO.dispatch(devices, l, Hq, r)
    assert ref is not None and abs(z_lp.value - ref[0]) <= 1e-7 * abs(ref[0])
    assert np.array_equal(x_heads, DO.round_to_groups(devices, l, Hq, r, x_frac))
    assert DO.times(devices, l, r, x_heads).max() == pytest.approx(z_r.value, rel=1e-9)
    assert (x_heads.sum(axis=0) > 0).all(), "the instance is meant to use every device"
    # capacity (Eq. (7b)) holds for the whole-group division
    used = unit * (l[:, None] * x_heads).sum(axis=0)
    assert all(used[i] <= devices[i]["capacity"] - devices[i]["g"] + 1e-6 for i in range(N))

    # ---- the undivided cache (the model's view) and the new token's rows
    w = W.make_custom(lens, Hq, Hkv, D, list(range(Hkv)), seed=402, device=DEV)
    kn, vn = W.new_token_rows(w)
    groups = x_heads // r                                  # KV heads of request j on device i
    first = np.concatenate([np.zeros((J, 1), dtype=np.int64), np.cumsum(groups, axis=1)], axis=1)
    shape_pool = H.make_pool(Hkv, D, w.num_blocks)
    nblk = (lens.astype(np.int64) + 15) // 16
    outs, owner = [], np.full((J, Hkv), -1)
    for i in range(N):
        pair_seq = np.concatenate([np.full(groups[j, i], j) for j in range(J)]).astype(np.int32)
        pair_head = np.concatenate([np.arange(first[j, i], first[j, i + 1]) for j in range(J)]).astype(np.int32)
        owner[pair_seq, pair_head] = i
        P = len(pair_seq)
        # the device's own pool of single-head tiles, handed out in a seeded random order
        table, num_tiles = W.build_block_table(lens[pair_seq], w.block_table.shape[1], 16,
                                               np.random.default_rng(403 + i), extra_blocks=2)
        k_t = torch.full((num_tiles, 16, D), float("nan"), dtype=torch.float16, device=DEV)
        v_t = torch.full_like(k_t, float("nan"))
        dst_pool = H.make_pool(1, D, num_tiles)
        # migration of the heads' tiles into the device's pool, one call per KV head
        for g in np.unique(pair_head):
            rows = np.nonzero(pair_head == g)[0]
            src = np.concatenate([w.block_table[pair_seq[p], :nblk[pair_seq[p]]] for p in rows])
            dst = np.concatenate([table[p, :nblk[pair_seq[p]]] for p in rows])
            H.check(H.hetis_kv_copy_tiles(shape_pool, w.k_cache, w.v_cache, dst_pool, k_t, v_t,
                                          i32(src), i32(dst), len(src), i32([g]), i32([0]), 1),
                    "kv_copy_tiles")
        shape = H.make_shape(J, Hq, Hkv, D, table.shape[1])
        bt, sl, ps, ph = i32(table), i32(lens), i32(pair_seq), i32(pair_head)
        H.check(H.hetis_attn_validate_pairs(shape, bt, sl, ps, ph, P, num_tiles), "validate_pairs")
        H.check(H.hetis_kv_append_pairs(shape, kn, vn, bt, sl, ps, ph, P, num_tiles, k_t, v_t),
                "kv_append_pairs")
        out = torch.empty_like(w.q)
        out.view(torch.int16).fill_(np.int16(SENTINEL))
        H.check(H.hetis_attn_decode_pairs(shape, w.q, k_t, v_t, bt, sl, ps, ph, P, w.spec.scale, out),
                "decode_pairs")
        torch.cuda.synchronize()
        no_expired_wait()
        outs.append(bits(out))
    assert (owner >= 0).all()
    # ---- Concat over devices (Eq. (2a)): every row was written by its owner and by nobody else
    own_rows = np.repeat(owner, r, axis=1)                  # [J, Hq]
    cat = np.full_like(outs[0], SENTINEL)
    for i in range(N):
        mine = own_rows == i
        assert (outs[i][~mine] == SENTINEL).all(), f"device {i} wrote rows it does not own"
        cat[mine] = outs[i][mine]
    out_cat = torch.from_numpy(cat.view(np.int16)).to(DEV).view(torch.float16)
    # ---- against the checker: append on the undivided cache, Attention of all heads
    u16 = lambda t: bits(t)
    ref_k, ref_v = oracle.kv_append(u16(w.k_cache), u16(w.v_cache), u16(kn), u16(vn), w.block_table,
                                    lens, np.arange(Hkv))
    ref_out = oracle.attn_decode(w.q.cpu().numpy(), ref_k.view(np.float16), ref_v.view(np.float16),
                                 w.block_table, lens, np.arange(Hkv, dtype=np.int32), w.spec.scale)
    check_rows(out_cat, ref_out, range(Hq), TOL, "concatenated shares")
    # ---- and bit for bit against one call over the undivided cache
    d = Dev(w)
    hid, n = d.heads(list(range(Hkv)))
    H.check(H.hetis_kv_append(d.shape, kn, vn, d.bt, d.sl, hid, n, w.num_blocks, d.k, d.v), "kv_append")
    whole = d.decode(list(range(Hkv)))
    assert np.array_equal(bits(whole), cat), "head sharding changed the result"
