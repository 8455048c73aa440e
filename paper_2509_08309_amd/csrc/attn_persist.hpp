// Persistent chunk kernel: work enumeration, tile streaming and chunk results for Eq. (2b),
// independent of how a tile is turned into scores and sums (that is the Policy: vector ALU
// arithmetic for small query groups, MFMA for grouped-query attention).
//
// Work enumeration: every workgroup scans the sequence lengths into a table of first-chunk
// indices (LDS), which turns a flat item number into (sequence, chunk, selected head)
// without launching a workgroup per possible chunk.  Workgroup k takes items k, k + G, ...
//
// A workgroup is NW streaming waves plus one writer wave.
//   - Streaming waves: wave w owns blocks w, w + NW, ... of the chunk and streams their
//     tiles through a two-slot register ring; a slot is refilled right after it has been
//     consumed, so one to two tile pairs (8-16 KB per wave) are always in flight, and the
//     ring runs on into the first pair of the next item before the current item's merge.
//     Every global load is issued unconditionally (indices clamped, tiles that do not
//     exist turned into zero-length buffer descriptors), so the in-order load counter is
//     known exactly at every wait.  These waves never store to global memory: on
//     gfx9-class hardware loads and stores share one counter that is in order only among
//     loads, so a single pending store would force every later wait to drain all loads.
//   - Writer wave: after the barrier that ends an item it combines the NW wave results
//     from LDS (ascending wave order) and stores the fp16 row or the fp32 partial.
// Dynamic LDS: int lens[batch], int first[batch + 1], int hids[n_sel]; two WaveMergeLds
// areas used alternately; NW per-wave staging areas of Policy::kWaveLdsBytes.
// Nothing depends on how many heads were selected or on the grid size: the result for one
// (sequence, head) is a function of that sequence's length alone.
#pragma once
#include "attn_common.hpp"

namespace hetis {

// LDS area through which the waves of a workgroup are merged (ascending wave order).
template <int D, int R, int NW>
struct WaveMergeLds {
    float o[NW][R][D];
    float m[NW][R];
    float l[NW][R];
};

// After a barrier: final result of the chunk, to `out` (fp16) or to the partial buffers.
template <int D, int R, int NW, int NTHREADS>
__device__ __forceinline__ void lds_finish(const WaveMergeLds<D, R, NW> &sm, const AttnParams &p,
                                           int tid, int b, int g, int si, int c, bool to_out)
{
    const int rows = p.n_sel * R;
    for (int idx = tid; idx < R * D; idx += NTHREADS) {
        const int r = idx / D, d = idx % D;
        float M = sm.m[0][r];
#pragma unroll
        for (int w = 1; w < NW; ++w) M = fmaxf(M, sm.m[w][r]);
        float acc = 0.f, lsum = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float a = fast_exp2(sm.m[w][r] - M);
            acc += sm.o[w][r][d] * a;
            lsum += sm.l[w][r] * a;
        }
        const float res = acc / lsum;
        if (to_out) {
            p.out[((int64_t)b * p.n_q_heads + g * R + r) * D + d] = __float2half_rn(res);
        } else {
            const int64_t row = ((int64_t)b * rows + si * R + r) * p.max_chunks + c;
            p.o_partial[row * D + d] = res;
            if (d == 0) p.lse_partial[row] = (M + fast_log2(lsum)) * kLn2;
        }
    }
}

template <int D, int R, int NTHREADS>
__device__ __forceinline__ void write_zero_rows(const AttnParams &p, int tid, int b, int g)
{
    for (int idx = tid; idx < R * D; idx += NTHREADS) {
        const int r = idx / D, d = idx % D;
        p.out[((int64_t)b * p.n_q_heads + g * R + r) * D + d] = __float2half_rn(0.f);
    }
}

struct ItemHdr {
    int b, si, c, g;
    int nblk;       // blocks of this chunk
    int rem;        // tokens in the ragged last block (0: none)
    int t0;         // first token of the chunk
    bool to_out;    // result goes to `out` (fp16), not to the partial buffers
    bool zero;      // length-0 sequence whose zeros this pass writes
};

__host__ __device__ constexpr size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

template <class Policy, int NW>
__host__ __device__ constexpr size_t persist_lds_bytes(int batch, int n_sel)
{
    return align16((size_t)(2 * batch + 1 + n_sel) * sizeof(int)) +
           2 * sizeof(WaveMergeLds<Policy::D, Policy::R, NW>) +
           (size_t)NW * Policy::kWaveLdsBytes;
}

__device__ __forceinline__ void workgroup_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

template <class Policy, int NW>
__global__ __launch_bounds__((NW + 1) * 64) void attn_chunk_persistent_kernel(const AttnParams p,
                                                                              const int batch)
{
    constexpr int D = Policy::D;
    constexpr int R = Policy::R;
    constexpr int NT = (NW + 1) * 64;
    constexpr int kTileBytes = kBlockTokens * D * 2;
    using Lds = WaveMergeLds<D, R, NW>;
    using Tile = typename Policy::Tile;
    extern __shared__ __align__(16) unsigned char smem[];
    int *lens = reinterpret_cast<int *>(smem);
    int *first = lens + batch;
    int *hids = first + batch + 1;
    unsigned char *after_tables = smem + align16((size_t)(2 * batch + 1 + p.n_sel) * sizeof(int));
    Lds *sm = reinterpret_cast<Lds *>(after_tables);
    unsigned char *staging = after_tables + 2 * sizeof(Lds);
    __shared__ int scan[NT];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- work enumeration: exclusive scan of items per sequence
    for (int i = tid; i < p.n_sel; i += NT) hids[i] = p.head_ids[i];
    {
        const int seg = (batch + NT - 1) / NT;
        const int lo = min(batch, tid * seg), hi = min(batch, lo + seg);
        int sum = 0;
        for (int b = lo; b < hi; ++b) {
            const int L = p.seq_lens[b];
            lens[b] = L;
            int n = (L + p.chunk_tokens - 1) / p.chunk_tokens;
            if (L <= 0) n = p.direct_single ? 1 : 0;      // the item that writes the zeros
            sum += n;
        }
        scan[tid] = sum;
        __syncthreads();
        for (int off = 1; off < NT; off <<= 1) {
            const int v = (tid >= off) ? scan[tid - off] : 0;
            __syncthreads();
            scan[tid] += v;
            __syncthreads();
        }
        int run = scan[tid] - sum;
        for (int b = lo; b < hi; ++b) {
            first[b] = run;
            const int L = lens[b];
            int n = (L + p.chunk_tokens - 1) / p.chunk_tokens;
            if (L <= 0) n = p.direct_single ? 1 : 0;
            run += n;
        }
        if (tid == NT - 1) first[batch] = scan[NT - 1];
        __syncthreads();
    }
    const int total = first[batch] * p.n_sel;
    const int G = gridDim.x;

    int b_scan = 0;   // sequences are visited in ascending order: resume the search where it ended
    auto decode = [&](int w, ItemHdr &h) {
        const int cg = w / p.n_sel;
        h.si = w - cg * p.n_sel;
        while (first[b_scan + 1] <= cg) ++b_scan;
        b_scan = __builtin_amdgcn_readfirstlane(b_scan);
        h.b = b_scan;
        h.c = __builtin_amdgcn_readfirstlane(cg - first[h.b]);
        const int L = __builtin_amdgcn_readfirstlane(lens[h.b]);
        h.g = __builtin_amdgcn_readfirstlane(hids[h.si]);
        const int n_chunks = (L + p.chunk_tokens - 1) / p.chunk_tokens;
        h.to_out = p.direct_single && n_chunks <= 1;
        h.zero = L <= 0;
        h.t0 = h.c * p.chunk_tokens;
        const int n_tok = h.zero ? 0 : min(L, h.t0 + p.chunk_tokens) - h.t0;
        h.nblk = (n_tok + kBlockTokens - 1) / kBlockTokens;
        h.rem = n_tok & (kBlockTokens - 1);
    };

    int w = blockIdx.x;
    if (w >= total) return;

    if (wave == NW) {
        // ------------------------------------------------------------ writer wave
        int parity = 0;
        for (; w < total; w += G) {
            ItemHdr h;
            decode(w, h);
            if (h.zero) {
                write_zero_rows<D, R, 64>(p, lane, h.b, h.g);
                continue;
            }
            workgroup_barrier();
            lds_finish<D, R, NW, 64>(sm[parity], p, lane, h.b, h.g, h.si, h.c, h.to_out);
            parity ^= 1;
        }
        return;
    }

    // ---------------------------------------------------------------- streaming waves
    struct Slot {
        ItemHdr h;
        int n_my;           // tiles this wave owns: blocks wave, wave+NW, ...
        int ids;            // lane i: physical block of this wave's i-th tile
        int64_t head_off;
        bool exists;
    };
    auto fill = [&](int wi, Slot &s) {
        s.exists = wi < total;
        decode(min(wi, total - 1), s.h);
        s.n_my = (s.exists && s.h.nblk > wave) ? (s.h.nblk - wave + NW - 1) / NW : 0;
        s.head_off = (int64_t)s.h.g * p.stride_head;
        const int32_t *bt =
            p.block_table + (int64_t)s.h.b * p.max_blocks_per_seq + s.h.t0 / kBlockTokens;
        s.ids = bt[min(wave + NW * lane, max(s.h.nblk - 1, 0))];
    };
    auto load_q = [&](const Slot &s, typename Policy::Query &q) {
        Policy::load_q(q, p.q + ((int64_t)s.h.b * p.n_q_heads + s.h.g * R) * D, lane);
    };
    auto issue = [&](Tile &t, int ids, int idx, int64_t head_off, bool valid) {
        const int blk = __builtin_amdgcn_readlane(ids, idx & 63);
        const int64_t base = (int64_t)blk * p.stride_block + head_off;
        Policy::issue(t, tile_rsrc(p.k_cache + base, kTileBytes, valid),
                      tile_rsrc(p.v_cache + base, kTileBytes, valid), lane);
    };

    Slot cur, nxt, nn;
    typename Policy::Query q, q_nxt;
    Tile A, B;
    unsigned char *my_staging = staging + (size_t)wave * Policy::kWaveLdsBytes;
    fill(w, cur);
    fill(w + G, nxt);
    load_q(cur, q);
    issue(A, cur.ids, 0, cur.head_off, 0 < cur.n_my);
    issue(B, cur.ids, 1, cur.head_off, 1 < cur.n_my);
    int parity = 0;
    for (;;) {
        fill(w + 2 * G, nn);        // header and block ids two items ahead
        load_q(nxt, q_nxt);         // query rows one item ahead

        typename Policy::State st;
        Policy::reset(st);
        const int n_my = cur.n_my;
        const int lim = 2 * max(1, (n_my + 1) >> 1);     // tiles of this item, as whole pairs
        // refill with tile j of the pair stream: tiles of `cur`, then the first pair of `nxt`
        auto refill = [&](Tile &t, int j) {
            const bool in_cur = j < lim;
            issue(t, in_cur ? cur.ids : nxt.ids, in_cur ? j : j - lim,
                  in_cur ? cur.head_off : nxt.head_off, in_cur ? j < n_my : j - lim < nxt.n_my);
        };
        // the ragged block, if any, is the chunk's last block: the last tile of one wave
        const bool mine_ragged = cur.h.rem != 0 && ((cur.h.nblk - 1) % NW) == wave;
        auto consume = [&](const Tile &t, int i) {
            if (mine_ragged && i == n_my - 1)
                Policy::template update<true>(st, t, q, p.scale_log2, lane, cur.h.rem, my_staging);
            else
                Policy::template update<false>(st, t, q, p.scale_log2, lane, kBlockTokens, my_staging);
        };
        // The scheduling fences keep "consume a slot, refill it at once" in program order;
        // without them the compiler batches both tiles' arithmetic ahead of both refills
        // and the wave ends up waiting with nothing in flight.
        for (int i = 0; i < lim; i += 2) {
            if (i < n_my) consume(A, i);
            __builtin_amdgcn_sched_barrier(0);
            refill(A, i + 2);
            __builtin_amdgcn_sched_barrier(0);
            if (i + 1 < n_my) consume(B, i + 1);
            __builtin_amdgcn_sched_barrier(0);
            refill(B, i + 3);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (cur.exists && !cur.h.zero) {
            Policy::template put<NW>(st, sm[parity], wave, lane);
            workgroup_barrier();
            parity ^= 1;
        }
        if (!nxt.exists) break;
        cur = nxt;
        nxt = nn;
        q = q_nxt;
        w += G;
    }
}

}  // namespace hetis
