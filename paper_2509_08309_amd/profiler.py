"""The Profiler's offline run on one device (Section 5.1, Eq. (3); Section 7.4, "Modeling
accuracy"): time head-wise decode Attention over a grid of eight head counts h and eight
cache amounts g, fit tau = a*h + b*g + c, and check the three properties the model rests on
(Fig. 7: time independent of the number of requests at fixed (h, g); linear in g; linear in h).
The grid is laid over (request, KV head) pairs, 64 to 2048 of them, i.e. h = r times that.

Measurements go through hetis_attn_decode_pairs (the per-request head-subset entry point: h
query heads spread over some requests, g cached tokens x KV heads in single-head tiles); the
fit is hetis_profiler_fit.  Units: tau in microseconds of device time per call (chunk kernel +
merge kernel, back-to-back calls), h in query heads, g in cached tokens x KV heads (one unit
= 2 * head_dim * 2 bytes of K and V).

Run:  python -m paper_2509_08309_amd.profiler [--model 13b|70b] [--reps 7]
Prints one JSON object.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json

import numpy as np

H_VALUES = (64, 128, 256, 512, 768, 1024, 1536, 2048)            # (request, KV head) pairs; h = r times that
G_VALUES = tuple(k * 1024 for k in (32, 64, 128, 256, 512, 1024, 1536, 2048))   # tokens x heads
MODELS = {"13b": (40, 40, 128), "70b": (64, 8, 128)}             # Hq, Hkv, D


class Bench:
    """One tile pool, reused by every configuration (contents do not matter for time)."""

    def __init__(self, model: str, max_units: int, seed: int = 2025):
        import torch
        from . import binding
        binding.load()
        self.torch = torch
        self.Hq, self.Hkv, self.D = MODELS[model]
        self.r = self.Hq // self.Hkv
        self.dev = torch.device("cuda:0")
        self.rng = np.random.default_rng(seed)
        self.num_tiles = max_units // 16 + 4096
        gen = torch.Generator(device=self.dev)
        gen.manual_seed(seed)
        shape = (self.num_tiles, 16, self.D)
        self.k_tiles = torch.randn(shape, generator=gen, device=self.dev, dtype=torch.float16)
        self.v_tiles = torch.randn(shape, generator=gen, device=self.dev, dtype=torch.float16)
        self.stream = torch.cuda.current_stream()

    def time_config(self, n_requests: int, heads_per_request: int, lengths, reps: int) -> float:
        """Device microseconds per hetis_attn_decode_pairs call for n_requests requests that
        each hold heads_per_request KV heads on this device; lengths: int array [n_requests]."""
        import paper_2509_08309_amd as H
        torch = self.torch
        lens = np.asarray(lengths, dtype=np.int32)
        assert len(lens) == n_requests and heads_per_request <= self.Hkv
        pair_seq = np.repeat(np.arange(n_requests, dtype=np.int32), heads_per_request)
        pair_head = np.concatenate([np.sort(self.rng.choice(self.Hkv, heads_per_request, replace=False))
                                    for _ in range(n_requests)]).astype(np.int32)
        nblk = (lens[pair_seq].astype(np.int64) + 15) // 16
        max_blocks = int(nblk.max())
        need = int(nblk.sum())
        assert need <= self.num_tiles
        # Successive calls read different tiles, as successive layers of a model do: the block
        # tables rotate over disjoint slices of one permutation of the pool until about 1 GB
        # has been touched, so that no call finds its tiles in the 256 MB last-level cache.
        tile_bytes = 2 * 16 * self.D * 2
        n_tables = int(min(64, self.num_tiles // need, max(1, -(-(1 << 30) // (need * tile_bytes)))))
        perm = self.rng.permutation(self.num_tiles).astype(np.int32)
        mask = np.arange(max_blocks)[None, :] < nblk[:, None]
        to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)
        tables = []
        for v in range(n_tables):
            table = np.full((len(pair_seq), max_blocks), -1, dtype=np.int32)
            table[mask] = perm[v * need:(v + 1) * need]
            tables.append(to_dev(table))
        bt = tables[0]
        sl, ps, ph = to_dev(lens), to_dev(pair_seq), to_dev(pair_head)
        q = torch.randn((n_requests, self.Hq, self.D), device=self.dev, dtype=torch.float16)
        out = torch.empty_like(q)
        shape = H.make_shape(n_requests, self.Hq, self.Hkv, self.D, max_blocks)
        H.check(H.hetis_attn_validate_pairs(shape, bt, sl, ps, ph, len(pair_seq), self.num_tiles),
                "validate_pairs")

        turn = [0]

        def call():
            t = tables[turn[0] % n_tables]
            turn[0] += 1
            H.check(H.hetis_attn_decode_pairs(shape, q, self.k_tiles, self.v_tiles, t, sl, ps, ph,
                                              len(pair_seq), 1.0 / np.sqrt(self.D), out,
                                              self.stream), "hetis_attn_decode_pairs")
        for _ in range(2):
            call()
        torch.cuda.synchronize()
        times = []
        inner = 4
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(self.stream)
            for _ in range(inner):
                call()
            b.record(self.stream)
            torch.cuda.synchronize()
            times.append(a.elapsed_time(b) * 1e3 / inner)
        return float(np.median(times))

    def time_hg(self, h: int, g: int, reps: int, n_requests: int | None = None) -> float:
        """h query heads and g cached tokens x KV heads, spread evenly: every (request, head)
        has the same length."""
        pairs = h // self.r
        if n_requests is None:
            per = min(16, self.Hkv)                       # KV heads of a request on this device
            while pairs % per:
                per //= 2
            n_requests = pairs // per
        per = pairs // n_requests
        assert per * n_requests == pairs and 1 <= per <= self.Hkv
        length = max(1, g // pairs)
        return self.time_config(n_requests, per, np.full(n_requests, length), reps)


def fit(h, g, tau):
    import paper_2509_08309_amd as H
    arr = lambda x: np.ascontiguousarray(x, dtype=np.float64)
    h, g, tau = arr(h), arr(g), arr(tau)
    abc, acc = np.zeros(3), C.c_double(0)
    H.check(H.hetis_profiler_fit(h, g, tau, len(h), abc, acc), "hetis_profiler_fit")
    return abc, acc.value


def fit_nonneg(h, g, tau):
    """The fit under a >= 0, b >= 0: the coefficients in the form the Dispatcher accepts."""
    import paper_2509_08309_amd as H
    arr = lambda x: np.ascontiguousarray(x, dtype=np.float64)
    h, g, tau = arr(h), arr(g), arr(tau)
    abc, acc = np.zeros(3), C.c_double(0)
    H.check(H.hetis_profiler_fit_nonneg(h, g, tau, len(h), abc, acc), "hetis_profiler_fit_nonneg")
    return abc, acc.value


def predict(abc, h, g):
    import paper_2509_08309_amd as H
    arr = lambda x: np.ascontiguousarray(x, dtype=np.float64)
    h, g = arr(h), arr(g)
    out = np.zeros_like(h)
    H.check(H.hetis_profiler_predict(arr(abc), h, g, len(h), out), "hetis_profiler_predict")
    return out


def r_squared(x, y):
    x, y = np.asarray(x, dtype=np.float64), np.asarray(y, dtype=np.float64)
    A = np.stack([x, np.ones_like(x)], axis=1)
    coef = np.linalg.lstsq(A, y, rcond=None)[0]
    res = y - A @ coef
    return 1.0 - float(res @ res) / float(((y - y.mean()) ** 2).sum())


def run(model: str = "13b", reps: int = 7, h_values=None, g_values=G_VALUES) -> dict:
    r = MODELS[model][0] // MODELS[model][1]
    if h_values is None:
        h_values = tuple(v * r for v in H_VALUES)       # query heads: r per (request, KV head)
    bench = Bench(model, max(g_values) + 16 * max(h_values) // r)
    hs, gs, taus = [], [], []
    for h in h_values:
        for g in g_values:
            if g // (h // r) > 32768:
                continue
            taus.append(bench.time_hg(h, g, reps))
            hs.append(h)
            gs.append((g // (h // r)) * (h // r))           # what was actually cached
    abc, acc = fit(hs, gs, taus)
    abc_nn, acc_nn = fit_nonneg(hs, gs, taus)
    pred = predict(abc, hs, gs)
    rel = np.abs(pred - np.asarray(taus)) / np.asarray(taus)
    rec = {"model": model, "n_points": len(taus), "a_us_per_query_head": abc[0],
           "b_us_per_token_head": abc[1], "c_us": abc[2], "accuracy": acc,
           "worst_point_accuracy": 1.0 - float(rel.max()),
           "b_as_GBps": 2 * bench.D * 2 / abc[1] / 1e3 if abc[1] > 0 else None,
           "dispatcher_abc": [float(v) for v in abc_nn], "dispatcher_abc_accuracy": acc_nn,
           "points": [{"h": int(a), "g": int(b), "tau_us": round(c, 2), "pred_us": round(float(d), 2)}
                      for a, b, c, d in zip(hs, gs, taus, pred)]}
    # Fig. 7 (a): the number of requests does not matter at fixed (h, g)
    h0, g0 = 512 * r, 512 * 1024
    by_requests = {}
    for n in (16, 32, 64, 128, 256, 512):
        if (h0 // r) % n == 0 and (h0 // r) // n <= bench.Hkv:
            by_requests[n] = bench.time_hg(h0, g0, reps, n_requests=n)
    v = np.array(list(by_requests.values()))
    rec["fig7a_requests"] = {"h": h0, "g": g0, "tau_us_by_n_requests": by_requests,
                             "spread": float(v.max() / v.min() - 1.0)}
    # (b) linear in g at fixed h, (c) linear in h at fixed g
    hs_a, gs_a, ta = np.asarray(hs), np.asarray(gs), np.asarray(taus)
    mh = hs_a == 512 * r if 512 * r in hs_a else hs_a == hs_a[len(hs_a) // 2]
    rec["fig7b_r2_linear_in_g"] = r_squared(gs_a[mh], ta[mh])
    g_mid = sorted(set(g_values))[len(set(g_values)) // 2]
    mg = np.abs(gs_a - g_mid) <= 16 * max(h_values) // r
    # a straight line in h may well be flat here (a close to 0): report slope and spread too
    A = np.stack([hs_a[mg], np.ones(int(mg.sum()))], axis=1)
    slope_h = float(np.linalg.lstsq(A, ta[mg], rcond=None)[0][0])
    rec["fig7c_h_at_fixed_g"] = {"g": int(g_mid), "r2_linear_in_h": r_squared(hs_a[mg], ta[mg]),
                                 "slope_us_per_query_head": slope_h,
                                 "spread": float(ta[mg].max() / ta[mg].min() - 1.0)}
    # held out: a ragged batch (lengths of the 13B workload, 13 KV heads per request)
    from . import workloads as W
    spec = W.SPECS["c3_13b_subset" if model == "13b" else "c5_70b_gqa"]
    lens = W.draw_lengths(spec, np.random.default_rng(spec.seed))
    per = len(spec.head_ids)
    t = bench.time_config(spec.batch, per, lens, reps)
    h_r, g_r = spec.batch * per * r, int(lens.astype(np.int64).sum()) * per
    p = float(predict(abc, [h_r], [g_r])[0])
    rec["held_out_ragged"] = {"workload_lengths": spec.name, "h": h_r, "g": g_r, "tau_us": t,
                              "pred_us": p, "accuracy": 1.0 - abs(p - t) / t}
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--model", default="13b", choices=sorted(MODELS))
    ap.add_argument("--reps", type=int, default=7)
    args = ap.parse_args()
    print(json.dumps(run(args.model, args.reps)))


if __name__ == "__main__":
    main()
