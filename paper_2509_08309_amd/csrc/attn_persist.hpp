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
//     After the barrier that ends an item the streaming waves also combine the NW wave
//     results (ascending wave order), a quarter of the rows each, into an LDS result area.
//     They also keep the query rows flowing: each wave loads its share of the rows of item
//     n + 2 while item n streams and puts them into LDS one item later, from where all
//     waves take their query operand.
//   - Writer wave: one item behind, it copies the finished result area to global memory
//     (fp16 row or fp32 partial).  It never loads from global memory, so it never has to
//     wait for its stores.
// Every item ends with exactly one workgroup barrier; one more follows the last item.
// Dynamic LDS: int lens[batch], int first[batch + 1], int hids[n_sel]; two WaveMergeLds
// areas, two result areas and two query areas used alternately; NW per-wave staging areas
// of Policy::kWaveLdsBytes.
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

// Finished rows of one item, before they leave for global memory.
template <int D, int R>
struct ResultLds {
    float o[R][D];      // normalised output rows
    float lse[R];       // natural-log log-sum-exp of each row (used by partial results only)
};

// After the barrier that ends an item: combine the NW wave results into the result area.
// Called by the NTHREADS streaming threads; thread `tid` takes elements tid, tid + NTHREADS, ...
template <int D, int R, int NW, int NTHREADS>
__device__ __forceinline__ void lds_combine(const WaveMergeLds<D, R, NW> &sm, ResultLds<D, R> &res,
                                            int tid)
{
#pragma unroll
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
        res.o[r][d] = acc * __builtin_amdgcn_rcpf(lsum);
        if (d == 0) res.lse[r] = (M + fast_log2(lsum)) * kLn2;
    }
}

// Result area -> `out` (fp16) or the partial buffers (fp32); one wave, four elements a lane.
template <int D, int R>
__device__ __forceinline__ void flush_result(const ResultLds<D, R> &res, const AttnParams &p,
                                             int lane, int b, int g, int si, int c, bool to_out)
{
    const int rows = p.n_sel * R;
#pragma unroll
    for (int idx = lane * 4; idx < R * D; idx += 256) {
        const int r = idx / D, d = idx % D;
        const float4 v = *reinterpret_cast<const float4 *>(&res.o[r][d]);
        if (to_out) {
            union {
                __half2 h[2];
                uint2 u;
            } pk;
            pk.h[0] = __floats2half2_rn(v.x, v.y);
            pk.h[1] = __floats2half2_rn(v.z, v.w);
            *reinterpret_cast<uint2 *>(p.out + ((int64_t)b * p.n_q_heads + g * R + r) * D + d) = pk.u;
        } else {
            const int64_t row = ((int64_t)b * rows + si * R + r) * p.max_chunks + c;
            *reinterpret_cast<float4 *>(p.o_partial + row * D + d) = v;
            if (d == 0) p.lse_partial[row] = res.lse[r];
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
           2 * sizeof(ResultLds<Policy::D, Policy::R>) +
           2 * (size_t)Policy::R * Policy::D * sizeof(__half) +
           (size_t)NW * Policy::kWaveLdsBytes;
}

__device__ __forceinline__ void workgroup_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

template <class Policy, int NW>
__global__ __launch_bounds__((NW + 1) * 64) __attribute__((amdgpu_waves_per_eu(Policy::kWavesPerEu))) void attn_chunk_persistent_kernel(const AttnParams p,
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
    using Res = ResultLds<D, R>;
    Res *res = reinterpret_cast<Res *>(after_tables + 2 * sizeof(Lds));
    constexpr int kQBytes = R * D * (int)sizeof(__half);      // query rows of one item
    unsigned char *q_stage = after_tables + 2 * sizeof(Lds) + 2 * sizeof(Res);
    unsigned char *staging = q_stage + 2 * kQBytes;
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

    // sequences are visited in ascending order: `cursor` resumes the search where it ended
    auto decode = [&](int w, ItemHdr &h, int &cursor) {
        const int cg = w / p.n_sel;
        h.si = w - cg * p.n_sel;
        while (first[cursor + 1] <= cg) ++cursor;
        cursor = __builtin_amdgcn_readfirstlane(cursor);
        h.b = cursor;
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

    // ---- query rows: global -> registers -> LDS, a share per streaming wave
    static_assert(kQBytes % (NW * 16) == 0, "query rows split evenly over the streaming waves");
    constexpr int kQShare = kQBytes / NW;                     // bytes per wave
    constexpr int kQVec = (kQShare / 16 + 63) / 64;           // uint4 per lane
    int cursor_q = 0;
    auto q_fetch = [&](int wi, uint4 (&qv)[kQVec]) {          // unconditional, indices clamped
        ItemHdr h;
        decode(min(wi, total - 1), h, cursor_q);
        const uint4 *src = reinterpret_cast<const uint4 *>(
            p.q + ((int64_t)h.b * p.n_q_heads + h.g * R) * D) + wave * (kQShare / 16);
#pragma unroll
        for (int i = 0; i < kQVec; ++i) qv[i] = src[min(lane + 64 * i, kQShare / 16 - 1)];
    };
    auto q_store = [&](const uint4 (&qv)[kQVec], int par) {
        uint4 *dst = reinterpret_cast<uint4 *>(q_stage + par * kQBytes) + wave * (kQShare / 16);
#pragma unroll
        for (int i = 0; i < kQVec; ++i)
            if (lane + 64 * i < kQShare / 16) dst[lane + 64 * i] = qv[i];
    };
    uint4 qv[kQVec];
    if (wave < NW) {
        q_fetch(w, qv);
        q_store(qv, 0);
        q_fetch(w + G, qv);           // stays in registers until the first item's barrier
    }
    __syncthreads();

    if (wave == NW) {
        // ------------------------------------------------------------ writer wave
        int n = 0, cursor = 0;
        ItemHdr prev;
        bool have_prev = false;
        for (; w < total; w += G, ++n) {
            ItemHdr h;
            decode(w, h, cursor);
            workgroup_barrier();                  // ends item n; item n - 1 is now combined
            if (have_prev)
                flush_result<D, R>(res[(n - 1) & 1], p, lane, prev.b, prev.g, prev.si, prev.c,
                                   prev.to_out);
            have_prev = !h.zero;
            prev = h;
            if (h.zero) write_zero_rows<D, R, 64>(p, lane, h.b, h.g);
        }
        workgroup_barrier();                      // the last item is combined
        if (have_prev)
            flush_result<D, R>(res[(n - 1) & 1], p, lane, prev.b, prev.g, prev.si, prev.c,
                               prev.to_out);
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
    int cursor = 0;
    auto fill = [&](int wi, Slot &s) {
        s.exists = wi < total;
        decode(min(wi, total - 1), s.h, cursor);
        s.n_my = (s.exists && s.h.nblk > wave) ? (s.h.nblk - wave + NW - 1) / NW : 0;
        s.head_off = (int64_t)s.h.g * p.stride_head;
        const int32_t *bt =
            p.block_table + (int64_t)s.h.b * p.max_blocks_per_seq + s.h.t0 / kBlockTokens;
        s.ids = bt[min(wave + NW * lane, max(s.h.nblk - 1, 0))];
    };
    auto issue = [&](Tile &t, int ids, int idx, int64_t head_off, bool valid) {
        const int blk = __builtin_amdgcn_readlane(ids, idx & 63);
        const int64_t base = (int64_t)blk * p.stride_block + head_off;
        Policy::issue(t, tile_rsrc(p.k_cache + base, kTileBytes, valid),
                      tile_rsrc(p.v_cache + base, kTileBytes, valid), lane);
    };

    Slot cur, nxt, nn;
    typename Policy::Query q;
    Tile A, B;
    unsigned char *my_staging = staging + (size_t)wave * Policy::kWaveLdsBytes;
    fill(w, cur);
    fill(w + G, nxt);
    issue(A, cur.ids, 0, cur.head_off, 0 < cur.n_my);
    issue(B, cur.ids, 1, cur.head_off, 1 < cur.n_my);
    int n = 0;
    for (;; ++n) {
        fill(w + 2 * G, nn);        // header and block ids two items ahead
        Policy::load_q(q, reinterpret_cast<const __half *>(q_stage + (n & 1) * kQBytes), lane);
        q_store(qv, (n + 1) & 1);   // rows of item n + 1, loaded one item ago
        q_fetch(w + 2 * G, qv);     // rows of item n + 2

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
            const int n_valid = (mine_ragged && i == n_my - 1) ? cur.h.rem : kBlockTokens;
            Policy::update(st, t, q, p.scale_log2, lane, n_valid, my_staging);
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
        if (!cur.h.zero) Policy::template put<NW>(st, sm[n & 1], wave, lane);
        workgroup_barrier();                      // ends item n
        if (!cur.h.zero) lds_combine<D, R, NW, NW * 64>(sm[n & 1], res[n & 1], tid);
        if (!nxt.exists) break;
        cur = nxt;
        nxt = nn;
        w += G;
    }
    workgroup_barrier();                          // lets the writer see the last combined item
}

}  // namespace hetis
