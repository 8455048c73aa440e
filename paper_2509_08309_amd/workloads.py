"""Seeded synthetic inputs for head-subset paged decode Attention.

This module only draws shapes, lengths, block tables and random fp16 data.  It
holds none of the method's arithmetic (no dot products, no softmax), so both
the HIP path and the CPU checker can be fed from it without sharing any
computation.  Nothing here touches the HIP library.

The five named workloads stand in for the request mixes of the paper's
evaluation (Section 7.1: chat, code-completion and long-context traces on
Llama-13B / OPT-30B / Llama-70B head shapes); they are synthetic length
distributions with the same head shapes, not items of those datasets.

Cache layout (Section 6, "KV cache management": fixed-size blocks split again
on the head dimension, addressed by sequence, position and head):
    k_cache, v_cache : fp16 [num_blocks, n_kv_heads, block_size, head_dim]
    block_table      : int32 [batch, max_blocks_per_seq], unused entries = -1
Token t of sequence b lives in physical block block_table[b, t // block_size]
at slot t % block_size.  Slots past the end of a sequence hold fp16 NaN so that
a masking mistake shows up as NaN rather than as a small error.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, Optional, Sequence

import numpy as np
import torch

BLOCK_SIZE = 16


@dataclass
class WorkloadSpec:
    """Shape and distribution of one workload; no data."""
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    head_ids: Sequence[int]            # selected KV-head ids
    seed: int
    length_kind: str                   # "fixed" | "uniform" | "lognormal"
    length_args: tuple
    max_seq_len: int                   # upper bound of the length distribution
    chunk_tokens: int = 0              # >0: the workload is run through split-KV
    block_size: int = BLOCK_SIZE

    @property
    def group_size(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def max_blocks_per_seq(self) -> int:
        return (self.max_seq_len + self.block_size - 1) // self.block_size

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)


SPECS: Dict[str, WorkloadSpec] = {
    # tiny MHA case, finishes instantly on the CPU
    "c1_tiny": WorkloadSpec("c1_tiny", 4, 8, 8, 64, (1, 3, 4, 6), 1001,
                            "fixed", ((17, 64, 130, 255),), 256),
    # 7B-shaped, all heads
    "c2_7b_all": WorkloadSpec("c2_7b_all", 64, 32, 32, 128, tuple(range(32)), 1002,
                              "uniform", (128, 2048), 2048),
    # 7B-shaped, first half of the heads (same seed: same cache as c2_7b_all)
    "c2_7b_half": WorkloadSpec("c2_7b_half", 64, 32, 32, 128, tuple(range(16)), 1002,
                               "uniform", (128, 2048), 2048),
    # 13B-shaped, one device's head share (the metric's workload)
    "c3_13b_subset": WorkloadSpec("c3_13b_subset", 128, 40, 40, 128, tuple(range(27, 40)), 1003,
                                  "lognormal", (800.0, 0.8, 32, 4096), 4096),
    # long context, split-KV with 512-token chunks
    "c4_13b_long": WorkloadSpec("c4_13b_long", 8, 40, 40, 128, tuple(range(40)), 1004,
                                "uniform", (10000, 32768), 32768, chunk_tokens=512),
    # 70B-shaped GQA, three KV groups
    "c5_70b_gqa": WorkloadSpec("c5_70b_gqa", 256, 64, 8, 128, (2, 5, 7), 1005,
                               "uniform", (256, 4096), 4096),
}


def draw_lengths(spec: WorkloadSpec, rng: np.random.Generator) -> np.ndarray:
    """KV lengths (current token included) for every sequence of the batch."""
    if spec.length_kind == "fixed":
        lens = np.asarray(spec.length_args[0], dtype=np.int64)
        assert lens.shape[0] == spec.batch
    elif spec.length_kind == "uniform":
        lo, hi = spec.length_args
        lens = rng.integers(lo, hi + 1, size=spec.batch)
    elif spec.length_kind == "lognormal":
        median, sigma, lo, hi = spec.length_args
        lens = np.rint(rng.lognormal(math.log(median), sigma, size=spec.batch))
        lens = np.clip(lens, lo, hi)
    else:
        raise ValueError(spec.length_kind)
    return lens.astype(np.int32)


def build_block_table(seq_lens: np.ndarray, max_blocks_per_seq: int, block_size: int,
                      rng: Optional[np.random.Generator], extra_blocks: int = 0):
    """One global random permutation of the physical blocks.

    num_blocks = sum_b ceil(L_b / block_size) + extra_blocks; logical block j of
    sequence b maps to perm[offset_b + j].  Distinct sequences never share a
    block.  With rng=None the mapping is the identity.
    """
    nblk = (seq_lens.astype(np.int64) + block_size - 1) // block_size
    assert int(nblk.max(initial=0)) <= max_blocks_per_seq
    total = int(nblk.sum()) + int(extra_blocks)
    perm = rng.permutation(total) if rng is not None else np.arange(total)
    table = np.full((len(seq_lens), max_blocks_per_seq), -1, dtype=np.int32)
    off = 0
    for b, n in enumerate(nblk):
        table[b, :n] = perm[off:off + n]
        off += int(n)
    return table, total


@dataclass
class Workload:
    spec: WorkloadSpec
    seq_lens: np.ndarray                # int32 [B]          (host)
    block_table: np.ndarray             # int32 [B, max_blk] (host)
    num_blocks: int
    q: torch.Tensor                     # fp16 [B, Hq, D]
    k_cache: torch.Tensor               # fp16 [num_blocks, Hkv, 16, D]
    v_cache: torch.Tensor
    head_ids: np.ndarray = field(default=None)  # int32 [S]

    @property
    def total_tokens(self) -> int:
        return int(self.seq_lens.astype(np.int64).sum())

    def kv_bytes(self, n_sel_heads: Optional[int] = None) -> int:
        """K+V bytes of the selected heads over all cached tokens."""
        s = len(self.head_ids) if n_sel_heads is None else n_sel_heads
        return self.total_tokens * s * 2 * self.spec.head_dim * 2


def _randn_fp16(shape, gen: torch.Generator, device) -> torch.Tensor:
    """N(0,1) drawn in fp32 and rounded to fp16, in pieces to bound memory."""
    n = int(np.prod(shape))
    out = torch.empty(n, dtype=torch.float16, device=device)
    step = 1 << 26
    for s in range(0, n, step):
        e = min(n, s + step)
        out[s:e] = torch.randn(e - s, generator=gen, dtype=torch.float32, device=device).half()
    return out.view(*shape)


def poison_unused_slots(cache: torch.Tensor, seq_lens: np.ndarray, block_table: np.ndarray,
                        block_size: int) -> None:
    """Write NaN into the slots of every last block that lie past the sequence end."""
    for b, L in enumerate(seq_lens):
        L = int(L)
        rem = L % block_size
        if L > 0 and rem:
            blk = int(block_table[b, (L - 1) // block_size])
            cache[blk, :, rem:, :] = float("nan")


def make_workload(spec: WorkloadSpec, device="cpu", poison: bool = True) -> Workload:
    """Draw every input of `spec` from its seed on `device`."""
    rng = np.random.default_rng(spec.seed)
    seq_lens = draw_lengths(spec, rng)
    block_table, num_blocks = build_block_table(seq_lens, spec.max_blocks_per_seq,
                                                spec.block_size, rng)
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(spec.seed)
    q = _randn_fp16((spec.batch, spec.n_q_heads, spec.head_dim), gen, dev)
    cshape = (num_blocks, spec.n_kv_heads, spec.block_size, spec.head_dim)
    k_cache = _randn_fp16(cshape, gen, dev)
    v_cache = _randn_fp16(cshape, gen, dev)
    if poison:
        poison_unused_slots(k_cache, seq_lens, block_table, spec.block_size)
        poison_unused_slots(v_cache, seq_lens, block_table, spec.block_size)
    return Workload(spec, seq_lens, block_table, num_blocks, q, k_cache, v_cache,
                    np.asarray(spec.head_ids, dtype=np.int32))


def make_custom(batch_lens: Sequence[int], n_q_heads: int, n_kv_heads: int, head_dim: int,
                head_ids: Sequence[int], seed: int, device="cpu", max_seq_len: Optional[int] = None,
                permute: bool = True, poison: bool = True, name: str = "custom") -> Workload:
    """A workload with explicitly given lengths (edge-case and sweep inputs)."""
    lens = tuple(int(x) for x in batch_lens)
    msl = max_seq_len if max_seq_len is not None else max(max(lens, default=1), 1)
    spec = WorkloadSpec(name, len(lens), n_q_heads, n_kv_heads, head_dim, tuple(head_ids), seed,
                        "fixed", (lens,), msl)
    rng = np.random.default_rng(seed)
    seq_lens = draw_lengths(spec, rng)
    block_table, num_blocks = build_block_table(seq_lens, spec.max_blocks_per_seq, spec.block_size,
                                                rng if permute else None)
    num_blocks = max(num_blocks, 1)
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    q = _randn_fp16((spec.batch, n_q_heads, head_dim), gen, dev)
    cshape = (num_blocks, n_kv_heads, spec.block_size, head_dim)
    k_cache = _randn_fp16(cshape, gen, dev)
    v_cache = _randn_fp16(cshape, gen, dev)
    if poison:
        poison_unused_slots(k_cache, seq_lens, block_table, spec.block_size)
        poison_unused_slots(v_cache, seq_lens, block_table, spec.block_size)
    return Workload(spec, seq_lens, block_table, num_blocks, q, k_cache, v_cache,
                    np.asarray(spec.head_ids, dtype=np.int32))


# ---------------------------------------------------------------- cache-management inputs

def new_token_rows(w: Workload, seed: Optional[int] = None):
    """K and V rows of the token each sequence has just produced: fp16 [B, Hkv, D] each, on the
    device of the workload."""
    s = w.spec
    gen = torch.Generator(device=w.q.device)
    gen.manual_seed((s.seed if seed is None else seed) + 7919)
    shape = (s.batch, s.n_kv_heads, s.head_dim)
    return _randn_fp16(shape, gen, w.q.device), _randn_fp16(shape, gen, w.q.device)


def token_entries(w: Workload, seed: int, n: Optional[int] = None):
    """(token_seq, token_pos) int32 arrays naming cached tokens of the workload: all of them in
    a seeded random order, or a seeded sample of n distinct ones."""
    lens = w.seq_lens.astype(np.int64)
    seq = np.repeat(np.arange(len(lens), dtype=np.int32), lens)
    pos = (np.arange(int(lens.sum()), dtype=np.int64) - np.repeat(np.cumsum(lens) - lens, lens))
    order = np.random.default_rng(seed).permutation(len(seq))
    if n is not None:
        order = order[:n]
    return seq[order], pos[order].astype(np.int32)


def migration_plan(w: Workload, seed: int, extra_blocks: int = 5):
    """A move of every used block of the workload into another pool: (src_blocks, dst_blocks,
    dst_num_blocks, dst_block_table).  Destination blocks are a seeded random choice among
    dst_num_blocks = used + extra_blocks."""
    used_mask = np.zeros_like(w.block_table, dtype=bool)
    nblk = (w.seq_lens.astype(np.int64) + w.spec.block_size - 1) // w.spec.block_size
    for b, n in enumerate(nblk):
        used_mask[b, :n] = True
    src = w.block_table[used_mask].astype(np.int32)
    dst_num = len(src) + extra_blocks
    dst = np.random.default_rng(seed).permutation(dst_num)[:len(src)].astype(np.int32)
    table = np.full_like(w.block_table, -1)
    table[used_mask] = dst
    return src, dst, dst_num, table


# ---------------------------------------------------------------- per-request head subsets

@dataclass
class PairsWorkload:
    """A list of (sequence, KV head) pairs over a pool of single-head tiles, one block-table
    row per pair (the form in which a device sees requests whose head subsets differ)."""
    spec: WorkloadSpec
    seq_lens: np.ndarray                # int32 [B]
    pair_seq: np.ndarray                # int32 [P]
    pair_head: np.ndarray               # int32 [P]
    block_table: np.ndarray             # int32 [P, max_blocks_per_seq] tile ids, -1 past the end
    num_tiles: int
    q: torch.Tensor                     # fp16 [B, Hq, D]
    k_tiles: torch.Tensor               # fp16 [num_tiles, 16, D]
    v_tiles: torch.Tensor

    @property
    def n_pairs(self) -> int:
        return len(self.pair_seq)

    def kv_bytes(self) -> int:
        lens = self.seq_lens.astype(np.int64)[self.pair_seq]
        return int(lens.sum()) * 2 * self.spec.head_dim * 2


def draw_head_subsets(batch: int, n_kv_heads: int, mean_heads: float, rng: np.random.Generator):
    """Per request: a count drawn uniformly from [0, 2 * mean_heads] (clipped to the head count)
    and that many distinct KV heads, ascending.  Returns a list of int arrays."""
    hi = int(min(n_kv_heads, round(2 * mean_heads)))
    counts = rng.integers(0, hi + 1, size=batch)
    return [np.sort(rng.choice(n_kv_heads, size=int(c), replace=False)).astype(np.int32)
            for c in counts]


def make_pairs_workload(spec: WorkloadSpec, device="cpu", mean_heads: Optional[float] = None,
                        subsets=None, seq_lens=None, poison: bool = True,
                        extra_tiles: int = 3) -> PairsWorkload:
    """Lengths as in `spec`; every request gets its own head subset (drawn around
    mean_heads = len(spec.head_ids) unless `subsets` is given); tiles are handed out by one
    seeded permutation of the pool, data ~ N(0,1) rounded to fp16."""
    rng = np.random.default_rng(spec.seed)
    lens = draw_lengths(spec, rng) if seq_lens is None else np.asarray(seq_lens, dtype=np.int32)
    if subsets is None:
        mh = len(spec.head_ids) if mean_heads is None else mean_heads
        subsets = draw_head_subsets(spec.batch, spec.n_kv_heads, mh, rng)
    pair_seq = np.concatenate([np.full(len(h), b, dtype=np.int32) for b, h in enumerate(subsets)]
                              + [np.zeros(0, dtype=np.int32)])
    pair_head = np.concatenate([np.asarray(h, dtype=np.int32) for h in subsets]
                               + [np.zeros(0, dtype=np.int32)])
    table, num_tiles = build_block_table(lens[pair_seq], spec.max_blocks_per_seq, spec.block_size,
                                         rng, extra_blocks=extra_tiles)
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(spec.seed)
    q = _randn_fp16((spec.batch, spec.n_q_heads, spec.head_dim), gen, dev)
    tshape = (num_tiles, spec.block_size, spec.head_dim)
    k_tiles = _randn_fp16(tshape, gen, dev)
    v_tiles = _randn_fp16(tshape, gen, dev)
    if poison:
        for p, b in enumerate(pair_seq):
            L = int(lens[b])
            rem = L % spec.block_size
            if L > 0 and rem:
                t = int(table[p, (L - 1) // spec.block_size])
                k_tiles[t, rem:, :] = float("nan")
                v_tiles[t, rem:, :] = float("nan")
    return PairsWorkload(spec, lens, pair_seq, pair_head, table, num_tiles, q, k_tiles, v_tiles)
