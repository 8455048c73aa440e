#!/usr/bin/env python3
"""Benchmark of head-subset paged decode Attention on one MI355X.

A step is one pass of the whole hot path (hetis_attn_decode through the C ABI:
work enumeration, block-table gather, q.K^T, online softmax, p.V, chunk merge,
fp16 store) over one batch of seeded synthetic input that is already resident
in HBM.  Prints ONE JSON line:
  value       decode tokens/s of this device's head share (batch / step time)
  roofline    KV bytes the step must read / average duration of the chunk kernel (the
              kernel that streams the KV cache), measured with events that the library
              records around that launch on the launch stream, against the 8 TB/s peak
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
    """HBM bytes per step from the committed counter summary, or None."""
    path = os.path.join(PROFILE_DIR, f"pmc_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    m = re.search(r"^traffic_bytes_per_step\s*=\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
    return float(m.group(1)) if m else None


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
    oracle.attn_decode(q[:n], k, v, w_host.block_table[:n], w_host.seq_lens[:n], w_host.head_ids,
                       spec.scale)
    dt = time.perf_counter() - t0
    kv_bytes = int(lens[:n].sum()) * len(w_host.head_ids) * 4 * spec.head_dim
    return {
        "value": n / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
        "sample": f"first {n} of {spec.batch} sequences of {spec.name}, all {len(w_host.head_ids)} "
                  f"selected heads, {int(lens[:n].sum())} cached tokens, {dt:.2f} s wall",
        "kv_gbps": kv_bytes / dt / 1e9,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c3_13b_subset")
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

    if spec.chunk_tokens:
        C = H.hetis_attn_split_num_chunks(spec.max_seq_len, spec.chunk_tokens)
        r = spec.group_size
        o_p = torch.empty((spec.batch, n_sel, C, r, spec.head_dim), dtype=torch.float32, device=dev)
        lse_p = torch.empty((spec.batch, n_sel, C, r), dtype=torch.float32, device=dev)

        def step():
            H.check(H.hetis_attn_decode_split(shape, w.q, w.k_cache, w.v_cache, bt, sl, hid, n_sel,
                                              spec.scale, spec.chunk_tokens, spec.max_seq_len,
                                              o_p, lse_p, stream), "decode_split")
            H.check(H.hetis_attn_merge(shape, o_p, lse_p, sl, hid, n_sel, spec.chunk_tokens,
                                       spec.max_seq_len, out, stream), "merge")
        path = f"hetis_attn_decode_split(chunk={spec.chunk_tokens}) + hetis_attn_merge"
    else:
        def step():
            H.check(H.hetis_attn_decode(shape, w.q, w.k_cache, w.v_cache, bt, sl, hid, n_sel,
                                        spec.scale, out, stream), "decode")
        path = "hetis_attn_decode"

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # Events: one pair brackets the whole timed region on the launch stream; one pair per
    # step is handed to the library, which records it around the launch of the chunk kernel
    # (the kernel that streams the KV cache) inside the call.
    def new_event():
        e = torch.cuda.Event(enable_timing=True)
        e.record(stream)                 # creates the underlying hipEvent_t
        return e
    ev_region = (new_event(), new_event())
    ev_kernel = [(new_event(), new_event()) for _ in range(args.steps)]
    torch.cuda.synchronize()

    # timed region: exactly K steps, synchronised on both sides
    t0 = time.perf_counter()
    ev_region[0].record(stream)
    for kb, ke in ev_kernel:
        H.hetis_attn_profile_events(kb.cuda_event, ke.cuda_event)
        step()
    ev_region[1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    H.hetis_attn_profile_events(None, None)
    ms_per_step = wall * 1e3 / args.steps
    dev_ms_per_step = ev_region[0].elapsed_time(ev_region[1]) / args.steps
    kern_ms = np.array([a.elapsed_time(b) for a, b in ev_kernel])

    if args.calibrate_copy:
        # a plain elementwise kernel of known traffic (1 GiB read, 1 GiB written) for scaling
        # the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run
        src = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)
        torch.cuda.synchronize()

    kv_bytes = w.kv_bytes()
    avg_kernel_s = float(kern_ms.mean()) * 1e-3
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
                   "seed": spec.seed, "entry_point": path},
        "kv_gbps_step": kv_bytes / (ms_per_step * 1e-3) / 1e9,
        "device_us_per_step": dev_ms_per_step * 1e3,
        "chunk_kernel_us": {"mean": float(kern_ms.mean() * 1e3),
                            "median": float(np.median(kern_ms) * 1e3),
                            "min": float(kern_ms.min() * 1e3)},
        "roofline": {"bound": "hbm", "kernel": "attn_chunk_*_persistent_kernel",
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": read_traffic(spec.name),
                     "algorithmic_bytes": kv_bytes},
    }
    if not args.no_cpu_baseline:
        w_host = W.Workload(spec, w.seq_lens, w.block_table, w.num_blocks, w.q.cpu(),
                            w.k_cache.cpu(), w.v_cache.cpu(), w.head_ids)
        rec["cpu_baseline"] = cpu_baseline(w_host, args.cpu_seconds)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
