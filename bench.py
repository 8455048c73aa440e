#!/usr/bin/env python3
"""Benchmark of head-subset paged decode Attention on one MI355X.

Default (--op decode) is the headline measurement described below.  --op kv_append,
kv_store and kv_copy time the cache-management kernels on the same workload shapes and
print a line of the same form (value = bytes moved per second of step time).

A step is one pass of the whole hot path (hetis_attn_decode through the C ABI:
work enumeration, block-table gather, q.K^T, online softmax, p.V, chunk merge,
fp16 store) over one batch of seeded synthetic input that is already resident
in HBM.  Prints ONE JSON line:
  value       decode tokens/s of this device's head share (batch / step time)
  roofline    KV bytes the step must read / average duration of the chunk kernel (the
              kernel that streams the KV cache), measured with an event pair that the library
              attaches to that kernel's dispatch on the launch stream, against the 8 TB/s peak
  cpu_baseline  the fp64 CPU checker timed on a bounded sample of the same workload
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
PROFILE_DIR = os.path.join(ROOT, "profiles")


def read_traffic(workload: str):
    """HBM bytes per step from the committed counter summary, or None.  The counters cannot be
    read from inside this process: the figure is the one a rocprofv3 --pmc run of this same
    command produced (see traffic_source in the output)."""
    path = traffic_file(workload)
    if not os.path.exists(path):
        return None
    m = re.search(r"^traffic_bytes_per_step\s*=\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
    return float(m.group(1)) if m else None


def traffic_file(key: str) -> str:
    """key = <op>_<workload>, e.g. decode_c3_13b_subset."""
    return os.path.join(PROFILE_DIR, f"{key}.txt")


def traffic_source(workload: str):
    path = traffic_file(workload)
    if not os.path.exists(path):
        return None
    return ("stored figure, not measured in this run: profiles/" + os.path.basename(path) +
            " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command)")


def cpu_baseline(w_host, budget_s: float):
    """Time the CPU checker on the first n sequences of the workload (all selected heads)."""
    import numpy as np
    import oracle
    spec = w_host.spec
    q, k, v = w_host.q.numpy(), w_host.k_cache.numpy(), w_host.v_cache.numpy()
    threads = oracle.max_threads()
    # one short probe to size the sample, then the timed sample itself
    n = min(spec.batch, 2)
    t0 = time.perf_counter()
    oracle.attn_decode(q[:n], k, v, w_host.block_table[:n], w_host.seq_lens[:n], w_host.head_ids,
                       spec.scale)
    probe = time.perf_counter() - t0
    tok_probe = int(w_host.seq_lens[:n].sum())
    rate = tok_probe / max(probe, 1e-6)                      # cached tokens per wall second
    lens = w_host.seq_lens.astype(np.int64)
    csum = np.cumsum(lens)
    n = int(np.searchsorted(csum, rate * budget_s, side="right"))
    n = max(1, min(spec.batch, n))
    t0 = time.perf_counter()
    ref = oracle.attn_decode(q[:n], k, v, w_host.block_table[:n], w_host.seq_lens[:n],
                             w_host.head_ids, spec.scale)
    dt = time.perf_counter() - t0
    kv_bytes = int(lens[:n].sum()) * len(w_host.head_ids) * 4 * spec.head_dim
    return ref, {
        "value": n / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
        "sample": f"first {n} of {spec.batch} sequences of {spec.name}, all {len(w_host.head_ids)} "
                  f"selected heads, {int(lens[:n].sum())} cached tokens, {dt:.2f} s wall",
        "kv_gbps": kv_bytes / dt / 1e9,
    }


def timed_steps(step, set_events, stream, steps, warmup):
    """W untimed steps, then K timed ones between synchronisations: that is the step time.  The
    duration of the main kernel alone comes from a second pass of K steps whose dispatches carry
    event pairs that the library attaches to them; those steps are not part of the step time,
    because a dispatch that carries events costs a few microseconds more.  Returns (wall seconds
    of the K timed steps, device ms per step from one event pair around them, per-step kernel ms
    of the second pass)."""
    import numpy as np
    import torch
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()

    def new_event():
        e = torch.cuda.Event(enable_timing=True)
        e.record(stream)                 # creates the underlying hipEvent_t
        return e
    ev_region = (new_event(), new_event())
    ev_kernel = [(new_event(), new_event()) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev_region[0].record(stream)
    for _ in range(steps):
        step()
    ev_region[1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dev_ms = ev_region[0].elapsed_time(ev_region[1]) / steps
    for kb, ke in ev_kernel:
        set_events(kb.cuda_event, ke.cuda_event)
        step()
    torch.cuda.synchronize()
    set_events(None, None)
    return wall, dev_ms, np.array([a.elapsed_time(b) for a, b in ev_kernel])


def calibrate_copy():
    """A plain elementwise kernel of known traffic (1 GiB read, 1 GiB written) for scaling the
    FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this command."""
    import torch
    src = torch.zeros(1 << 28, dtype=torch.int32, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(3):
        torch.add(src, 1, out=dst)
    torch.cuda.synchronize()


def bench_pairs(args):
    """hetis_attn_decode_pairs on the workload's shape when every request has its own head
    subset (drawn around the workload's number of selected heads) over single-head tiles."""
    import numpy as np
    import torch
    import paper_2509_08309_amd as H
    from paper_2509_08309_amd import workloads as W

    spec = W.SPECS[args.workload]
    dev = torch.device("cuda:0")
    pw = W.make_pairs_workload(spec, device=dev)
    stream = torch.cuda.current_stream()
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    bt, sl = to_dev(pw.block_table), to_dev(pw.seq_lens)
    ps, ph = to_dev(pw.pair_seq), to_dev(pw.pair_head)
    shape = H.make_shape(spec.batch, spec.n_q_heads, spec.n_kv_heads, spec.head_dim,
                         pw.block_table.shape[1])
    H.check(H.hetis_attn_validate_pairs(shape, bt, sl, ps, ph, pw.n_pairs, pw.num_tiles), "validate")
    out = torch.zeros_like(pw.q)

    def step():
        H.check(H.hetis_attn_decode_pairs(shape, pw.q, pw.k_tiles, pw.v_tiles, bt, sl, ps, ph,
                                          pw.n_pairs, spec.scale, out, stream), "decode_pairs")

    wall, dev_ms, kern_ms = timed_steps(step, H.hetis_attn_profile_events, stream, args.steps,
                                        args.warmup)
    ms_per_step = wall * 1e3 / args.steps
    kv_bytes = pw.kv_bytes()
    achieved = kv_bytes / (float(kern_ms.mean()) * 1e-3) / 1e9
    rec = {
        "metric": "decode-attention tokens/s with per-request head subsets "
                  "(KV-read HBM GB/s in roofline), 1 GPU",
        "value": spec.batch / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 in, f32 accumulate", "data": "synthetic",
        "config": {"workload": spec.name, "op": "decode_pairs", "batch": spec.batch,
                   "n_q_heads": spec.n_q_heads, "n_kv_heads": spec.n_kv_heads,
                   "head_dim": spec.head_dim, "n_pairs": pw.n_pairs,
                   "mean_heads_per_request": pw.n_pairs / spec.batch, "seed": spec.seed,
                   "entry_point": "hetis_attn_decode_pairs"},
        "kv_gbps_step": kv_bytes / (ms_per_step * 1e-3) / 1e9,
        "device_us_per_step": dev_ms * 1e3,
        "chunk_kernel_us": {"mean": float(kern_ms.mean() * 1e3),
                            "median": float(np.median(kern_ms) * 1e3),
                            "min": float(kern_ms.min() * 1e3)},
        "roofline": {"bound": "hbm", "kernel": "attn_chunk_persistent_kernel<..., pairs>",
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": read_traffic(f"decode_pairs_{spec.name}"),
                     "traffic_source": traffic_source(f"decode_pairs_{spec.name}"),
                     "algorithmic_bytes": kv_bytes},
    }
    if not args.no_cpu_baseline:
        import oracle
        lens_p = pw.seq_lens[pw.pair_seq].astype(np.int64)
        n = max(1, min(pw.n_pairs, int(np.searchsorted(np.cumsum(lens_p), 40000))))
        q, k, v = pw.q.cpu().numpy(), pw.k_tiles.cpu().numpy(), pw.v_tiles.cpu().numpy()
        t0 = time.perf_counter()
        oracle.attn_decode_pairs(q, k, v, pw.block_table[:n], pw.seq_lens, pw.pair_seq[:n],
                                 pw.pair_head[:n], spec.n_kv_heads, spec.scale)
        dt = time.perf_counter() - t0
        seqs = len(np.unique(pw.pair_seq[:n]))
        rec["cpu_baseline"] = {
            "value": seqs / dt, "unit": "tokens/s", "cores": oracle.max_threads(), "kind": "oracle",
            "sample": f"first {n} of {pw.n_pairs} pairs ({seqs} sequences, {int(lens_p[:n].sum())} "
                      f"cached tokens x heads), {dt:.2f} s wall"}
    print(json.dumps(rec))


def bench_kv(args):
    """Cache-management kernels on the workload's shapes: the decode-step store of the new
    token (kv_append), a store of every cached token as after prefill (kv_store), and the move
    of the selected heads' tiles into a compact pool (kv_copy)."""
    import numpy as np
    import torch
    import paper_2509_08309_amd as H
    from paper_2509_08309_amd import workloads as W

    spec = W.SPECS[args.workload]
    dev = torch.device("cuda:0")
    w = W.make_workload(spec, device=dev)
    stream = torch.cuda.current_stream()
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    bt, sl, hid = to_dev(w.block_table), to_dev(w.seq_lens), to_dev(w.head_ids)
    n_sel, D, Hkv = len(w.head_ids), spec.head_dim, spec.n_kv_heads
    shape = H.make_shape(spec.batch, spec.n_q_heads, Hkv, D, w.block_table.shape[1])
    row_bytes = 2 * D * 2                                   # one K row + one V row
    if args.op == "kv_append":
        kn, vn = W.new_token_rows(w)
        units, unit_name = spec.batch * n_sel, "rows"
        moved = units * row_bytes                           # read once, written once
        kernel = "kv_rows_kernel<D, false>"

        def step():
            H.check(H.hetis_kv_append(shape, kn, vn, bt, sl, hid, n_sel, w.num_blocks, w.k_cache,
                                      w.v_cache, stream), "kv_append")

    elif args.op == "kv_store":
        seq, pos = W.token_entries(w, seed=spec.seed)
        n = len(pos)
        gen = torch.Generator(device=dev)
        gen.manual_seed(spec.seed)
        kn = torch.randn((n, Hkv, D), generator=gen, device=dev).half()
        vn = torch.randn((n, Hkv, D), generator=gen, device=dev).half()
        tseq, tpos = to_dev(seq), to_dev(pos)
        units, unit_name = n * n_sel, "rows"
        moved = units * row_bytes
        kernel = "kv_rows_kernel<D, false>"

        def step():
            H.check(H.hetis_kv_store(shape, kn, vn, tseq, tpos, n, bt, hid, n_sel, w.num_blocks,
                                     w.k_cache, w.v_cache, stream), "kv_store")
    else:
        src_b, dst_b, dnb, _ = W.migration_plan(w, seed=spec.seed)
        dk = torch.empty((dnb, n_sel, 16, D), dtype=torch.float16, device=dev)
        dv = torch.empty_like(dk)
        spool, dpool = H.make_pool(Hkv, D, w.num_blocks), H.make_pool(n_sel, D, dnb)
        tsb, tdb, dh = to_dev(src_b), to_dev(dst_b), to_dev(np.arange(n_sel))
        units, unit_name = len(src_b) * n_sel, "(block, head) tile pairs"
        moved = units * 16 * row_bytes
        kernel = "kv_copy_tiles_kernel<D>"

        def step():
            H.check(H.hetis_kv_copy_tiles(spool, w.k_cache, w.v_cache, dpool, dk, dv, tsb, tdb,
                                          len(src_b), hid, dh, n_sel, stream), "kv_copy_tiles")

    wall, dev_ms, kern_ms = timed_steps(step, H.hetis_kv_profile_events, stream, args.steps,
                                        args.warmup)
    ms_per_step = wall * 1e3 / args.steps
    traffic_alg = 2 * moved                                  # every byte is read and written
    achieved = traffic_alg / (float(kern_ms.mean()) * 1e-3) / 1e9
    rec = {
        "metric": f"{args.op}: HBM bytes moved per second (read + written), 1 GPU",
        "value": traffic_alg / (ms_per_step * 1e-3) / 1e9, "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8 (byte copy)", "data": "synthetic",
        "config": {"workload": spec.name, "op": args.op, "units": units, "unit": unit_name,
                   "selected_kv_heads": [int(x) for x in w.head_ids], "head_dim": D,
                   "seed": spec.seed},
        "device_us_per_step": dev_ms * 1e3,
        "kernel_us": {"mean": float(kern_ms.mean() * 1e3), "median": float(np.median(kern_ms) * 1e3),
                      "min": float(kern_ms.min() * 1e3)},
        "roofline": {"bound": "hbm", "kernel": kernel, "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": read_traffic(f"{args.op}_{spec.name}"),
                     "traffic_source": traffic_source(f"{args.op}_{spec.name}"),
                     "algorithmic_bytes": traffic_alg},
    }
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = kv_cpu_baseline(args.op, w, spec)
    print(json.dumps(rec))


def kv_cpu_baseline(op, w, spec):
    """The CPU checker's version of the same operation on the whole workload, timed."""
    import numpy as np
    import torch
    import oracle
    from paper_2509_08309_amd import workloads as W
    u16 = lambda t: t.cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
    k, v = u16(w.k_cache), u16(w.v_cache)
    heads = w.head_ids
    row_bytes = 2 * spec.head_dim * 2
    if op == "kv_append":
        kn, vn = W.new_token_rows(w)
        kn, vn = u16(kn), u16(vn)
        t0 = time.perf_counter()
        oracle.kv_append(k, v, kn, vn, w.block_table, w.seq_lens, heads)
        dt = time.perf_counter() - t0
        moved = spec.batch * len(heads) * row_bytes
        sample = (f"one append of {spec.batch} x {len(heads)} rows; the timed call includes the "
                  f"checker's copy of both caches ({k.nbytes * 2 / 1e9:.2f} GB)")
    elif op == "kv_store":
        seq, pos = W.token_entries(w, seed=spec.seed)
        n = min(len(pos), 20000)
        rng = np.random.default_rng(spec.seed)
        kn = rng.integers(0, 0x7000, size=(n, spec.n_kv_heads, spec.head_dim)).astype(np.uint16)
        t0 = time.perf_counter()
        oracle.kv_store(k, v, kn, kn, seq[:n], pos[:n], w.block_table, heads)
        dt = time.perf_counter() - t0
        moved = n * len(heads) * row_bytes
        sample = (f"{n} of {len(pos)} entries x {len(heads)} heads; includes the checker's copy of "
                  f"both caches ({k.nbytes * 2 / 1e9:.2f} GB)")
    else:
        src_b, dst_b, dnb, _ = W.migration_plan(w, seed=spec.seed)
        d0 = np.zeros((dnb, len(heads), 16, spec.head_dim), dtype=np.uint16)
        t0 = time.perf_counter()
        oracle.kv_copy_tiles(k, v, d0, d0, src_b, dst_b, heads, np.arange(len(heads)))
        dt = time.perf_counter() - t0
        moved = len(src_b) * len(heads) * 16 * row_bytes
        sample = (f"all {len(src_b)} blocks x {len(heads)} heads; includes the checker's copy of "
                  f"the destination pools ({d0.nbytes * 2 / 1e9:.2f} GB)")
    return {"value": 2 * moved / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": sample + f", {dt:.3f} s wall"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c3_13b_subset")
    ap.add_argument("--op", default="decode", choices=["decode", "decode_step", "decode_pairs", "kv_append", "kv_store", "kv_copy"])
    ap.add_argument("--cpu-seconds", type=float, default=1.5,
                    help="wall-clock budget of the CPU checker sample (x cores = CPU work)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (known traffic) for counter scaling")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (the head share of one device); "
                 "--gpus N with N > 1 is not supported.")

    import numpy as np
    import torch
    import paper_2509_08309_amd as H
    from paper_2509_08309_amd import workloads as W

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    H.binding.load()                       # the HIP library must be built; no fallback exists
    # everything runs on one stream of its own (not the null stream)
    torch.cuda.set_stream(torch.cuda.Stream())
    if args.op == "decode_pairs":
        bench_pairs(args)
    elif args.op not in ("decode", "decode_step"):
        bench_kv(args)
    if args.op not in ("decode", "decode_step"):
        if args.calibrate_copy:
            calibrate_copy()
        return
    spec = W.SPECS[args.workload]
    dev = torch.device("cuda:0")
    w = W.make_workload(spec, device=dev)
    bt = torch.from_numpy(w.block_table).to(dev)
    sl = torch.from_numpy(w.seq_lens).to(dev)
    hid = torch.from_numpy(w.head_ids).to(dev)
    n_sel = len(w.head_ids)
    shape = H.make_shape(spec.batch, spec.n_q_heads, spec.n_kv_heads, spec.head_dim,
                         w.block_table.shape[1])
    H.check(H.hetis_attn_validate(shape, bt, sl, hid, n_sel, w.num_blocks), "validate")
    out = torch.zeros_like(w.q)
    stream = torch.cuda.current_stream()

    if spec.chunk_tokens and args.op == "decode":
        C = H.hetis_attn_split_num_chunks(spec.max_seq_len, spec.chunk_tokens)
        r = spec.group_size
        o_p = torch.empty((spec.batch, n_sel, C, r, spec.head_dim), dtype=torch.float32, device=dev)
        lse_p = torch.empty((spec.batch, n_sel, C, r), dtype=torch.float32, device=dev)

        merge_events = []

        def step():
            H.check(H.hetis_attn_decode_split(shape, w.q, w.k_cache, w.v_cache, bt, sl, hid, n_sel,
                                              spec.scale, spec.chunk_tokens, spec.max_seq_len,
                                              o_p, lse_p, stream), "decode_split")
            if merge_events:                # second pass only: time the merge kernel as well
                H.hetis_attn_profile_events(merge_events[-1][0].cuda_event,
                                            merge_events[-1][1].cuda_event)
            H.check(H.hetis_attn_merge(shape, o_p, lse_p, sl, hid, n_sel, spec.chunk_tokens,
                                       spec.max_seq_len, out, stream), "merge")
        path = f"hetis_attn_decode_split(chunk={spec.chunk_tokens}) + hetis_attn_merge"
    elif args.op == "decode_step":
        # the whole decode step of the layer: store of the new token's rows + Attention, one call
        kn, vn = W.new_token_rows(w)

        def step():
            H.check(H.hetis_attn_decode_step(shape, w.q, kn, vn, w.k_cache, w.v_cache, bt, sl, hid,
                                             n_sel, spec.scale, out, stream), "decode_step")
        path = "hetis_attn_decode_step"
    else:
        def step():
            H.check(H.hetis_attn_decode(shape, w.q, w.k_cache, w.v_cache, bt, sl, hid, n_sel,
                                        spec.scale, out, stream), "decode")
        path = "hetis_attn_decode"

    # Events: one pair brackets the whole timed region on the launch stream; one pair per
    # step is handed to the library, which attaches it to the dispatch of the chunk kernel
    # (the kernel that streams the KV cache) inside the call.
    split = bool(spec.chunk_tokens) and args.op == "decode"

    def set_events(b, e):
        if split and b is not None:
            pair = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
            for ev in pair:
                ev.record(stream)
            merge_events.append(pair)
        return H.hetis_attn_profile_events(b, e)

    wall, dev_ms_per_step, kern_ms = timed_steps(step, set_events, stream, args.steps, args.warmup)
    ms_per_step = wall * 1e3 / args.steps
    merge_ms = np.array([a.elapsed_time(b) for a, b in merge_events]) if split else None

    if args.calibrate_copy:
        calibrate_copy()

    kv_bytes = w.kv_bytes()
    # every kernel of a step counts: the decode entry point is one kernel; the split-KV form
    # adds its merge kernel
    avg_kernel_s = float(kern_ms.mean()) * 1e-3
    if merge_ms is not None:
        avg_kernel_s += float(merge_ms.mean()) * 1e-3
    achieved = kv_bytes / avg_kernel_s / 1e9
    rec = {
        "metric": "decode-attention tokens/s (KV-read HBM GB/s in roofline), 1 GPU",
        "value": spec.batch / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 in, f32 accumulate", "data": "synthetic",
        "config": {"workload": spec.name, "batch": spec.batch, "n_q_heads": spec.n_q_heads,
                   "n_kv_heads": spec.n_kv_heads, "head_dim": spec.head_dim,
                   "selected_kv_heads": [int(x) for x in w.head_ids],
                   "total_cached_tokens": w.total_tokens, "block_size": spec.block_size,
                   "seed": spec.seed, "op": args.op, "entry_point": path},
        "kv_gbps_step": kv_bytes / (ms_per_step * 1e-3) / 1e9,
        "device_us_per_step": dev_ms_per_step * 1e3,
        "chunk_kernel_us": {"mean": float(kern_ms.mean() * 1e3),
                            "median": float(np.median(kern_ms) * 1e3),
                            "min": float(kern_ms.min() * 1e3)},
        "kernels_per_step": 1 if merge_ms is None else 2,
        "roofline": {"bound": "hbm",
                     "kernel": "attn_chunk_persistent_kernel" + ("" if merge_ms is None
                                                                 else " + attn_merge_kernel"),
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": read_traffic(f"{args.op}_{spec.name}"),
                     "traffic_source": traffic_source(f"{args.op}_{spec.name}"),
                     "algorithmic_bytes": kv_bytes},
    }
    if merge_ms is not None:
        rec["merge_kernel_us"] = {"mean": float(merge_ms.mean() * 1e3),
                                  "median": float(np.median(merge_ms) * 1e3),
                                  "min": float(merge_ms.min() * 1e3)}
        rec["roofline"]["frac_chunk_kernel_only"] = kv_bytes / (float(kern_ms.mean()) * 1e-3) / 1e9 / HBM_PEAK_GBPS
    if not args.no_cpu_baseline:
        w_host = W.Workload(spec, w.seq_lens, w.block_table, w.num_blocks, w.q.cpu(),
                            w.k_cache.cpu(), w.v_cache.cpu(), w.head_ids)
        ref, rec["cpu_baseline"] = cpu_baseline(w_host, args.cpu_seconds)
        # the checker's result is not thrown away: every selected row of the sequences it
        # covered is compared with what the timed GPU steps left in `out`
        r = spec.group_size
        rows = sorted(int(g) * r + i for g in w.head_ids for i in range(r))
        n = ref.shape[0]
        got = out[:n].cpu().numpy().astype(np.float64)[:, rows]
        rec["parity"] = {"max_abs_err": float(np.abs(got - ref[:, rows]).max()),
                         "tolerance": 4e-3, "sequences_checked": n, "sequences": spec.batch,
                         "rows_checked": n * len(rows), "against": "oracle (fp64 CPU checker)"}
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
