// Persistent chunk kernel: work enumeration, tile streaming and chunk results for Eq. (2b),
// independent of how a tile is turned into scores and sums (that is the Policy: vector ALU
// arithmetic for small query groups, MFMA for grouped-query attention).
//
// Work enumeration: every workgroup scans the sequence lengths into a table of first-chunk
// indices (LDS), which turns a flat item number into (sequence, chunk, selected head)
// without launching a workgroup per possible chunk.  An item is one chunk of one
// (sequence, selected head) and is processed by ONE wave; streaming wave number
// blockIdx * NW + wave takes items of that number, that number + (waves in the grid), ...
//
// A workgroup is NW streaming waves plus one writer wave; after the prologue they never
// meet at a barrier.
//   - Streaming waves stream the tiles of their item through a two-slot register ring; a
//     slot is refilled right after it has been consumed, so one to two tile pairs (8-16 KB
//     per wave) are always in flight, and the ring runs on into the first pair of the next
//     item before the current item is finished off.  Every global load is issued
//     unconditionally (indices clamped, tiles that do not exist turned into zero-length
//     buffer descriptors), so the in-order load counter is known exactly at every wait.
//     These waves never store to global memory: on gfx9-class hardware loads and stores
//     share one counter that is in order only among loads, so a single pending store would
//     force every later wait to drain all loads.  A finished item (normalised rows and
//     their log-sum-exp) is handed over through one of the wave's two LDS mailboxes.
//   - The writer wave polls the mailboxes and copies full ones to global memory (fp16 row,
//     fp32 partial, or zeros for an empty sequence).  It never loads from global memory,
//     so it never waits for its stores.
// Mailbox protocol (flag is a workgroup-scope atomic in LDS): EMPTY -> the producer fills
// data and header -> FULL -> the writer copies it out -> EMPTY.  A producer that has no more
// items marks its next mailbox DONE; the writer leaves when all NW are DONE.  All waits are
// polling loops with an iteration bound, so every wave reaches its end whatever happens.
// Dynamic LDS: int lens[batch], int first[batch + 1], int hids[n_sel]; NW x 2 mailboxes; NW
// per-wave staging areas of Policy::kWaveLdsBytes.
// Nothing depends on how many heads were selected or on the grid size: the result for one
// (sequence, head) is a function of that sequence's length alone.
#pragma once
#include "attn_common.hpp"

namespace hetis {

enum : int { kMailEmpty = 0, kMailFull = 1, kMailDone = 2 };
enum : int { kKindOut = 0, kKindPartial = 1, kKindZero = 2 };
constexpr int kSpinLimit = 1 << 22;     // polls before a wait gives up (far beyond any real wait)

// One finished item on its way to global memory.
template <int D, int R>
struct Mailbox {
    float o[R][D];      // normalised output rows
    float lse[R];       // natural-log log-sum-exp of each row (partial results only)
    int b, g, si, c;    // sequence, KV head, position in head_ids, chunk
    int kind;           // kKindOut / kKindPartial / kKindZero
    int flag;           // kMailEmpty / kMailFull / kMailDone
    int pad[2];
};

// Mailbox -> `out` (fp16) or the partial buffers (fp32); one wave, four elements a lane.
template <int D, int R>
__device__ __forceinline__ void flush_mailbox(const Mailbox<D, R> &mb, const AttnParams &p, int lane)
{
    const int b = __builtin_amdgcn_readfirstlane(mb.b);
    const int g = __builtin_amdgcn_readfirstlane(mb.g);
    const int si = __builtin_amdgcn_readfirstlane(mb.si);
    const int c = __builtin_amdgcn_readfirstlane(mb.c);
    const int kind = __builtin_amdgcn_readfirstlane(mb.kind);
    const int rows = p.n_sel * R;
#pragma unroll
    for (int idx = lane * 4; idx < R * D; idx += 256) {
        const int r = idx / D, d = idx % D;
        float4 v = *reinterpret_cast<const float4 *>(&mb.o[r][d]);
        if (kind == kKindPartial) {
            const int64_t row = ((int64_t)b * rows + si * R + r) * p.max_chunks + c;
            *reinterpret_cast<float4 *>(p.o_partial + row * D + d) = v;
            if (d == 0) p.lse_partial[row] = mb.lse[r];
        } else {
            if (kind == kKindZero) v = make_float4(0.f, 0.f, 0.f, 0.f);
            union {
                __half2 h[2];
                uint2 u;
            } pk;
            pk.h[0] = __floats2half2_rn(v.x, v.y);
            pk.h[1] = __floats2half2_rn(v.z, v.w);
            *reinterpret_cast<uint2 *>(p.out + ((int64_t)b * p.n_q_heads + g * R + r) * D + d) = pk.u;
        }
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
           2 * NW * sizeof(Mailbox<Policy::D, Policy::R>) + (size_t)NW * Policy::kWaveLdsBytes;
}

__device__ __forceinline__ int mail_load(const int *flag)
{
    return __hip_atomic_load(flag, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void mail_store(int *flag, int v)
{
    __hip_atomic_store(flag, v, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
}

template <class Policy, int NW>
__global__ __launch_bounds__((NW + 1) * 64)
    __attribute__((amdgpu_waves_per_eu(Policy::kWavesPerEu))) void attn_chunk_persistent_kernel(
        const AttnParams p, const int batch)
{
    constexpr int D = Policy::D;
    constexpr int R = Policy::R;
    constexpr int NT = (NW + 1) * 64;
    constexpr int kTileBytes = kBlockTokens * D * 2;
    using Mail = Mailbox<D, R>;
    using Tile = typename Policy::Tile;
    extern __shared__ __align__(16) unsigned char smem[];
    int *lens = reinterpret_cast<int *>(smem);
    int *first = lens + batch;
    int *hids = first + batch + 1;
    unsigned char *after_tables = smem + align16((size_t)(2 * batch + 1 + p.n_sel) * sizeof(int));
    Mail *mail = reinterpret_cast<Mail *>(after_tables);             // [NW][2]
    unsigned char *staging = after_tables + 2 * NW * sizeof(Mail);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- work enumeration: exclusive scan of items per sequence, done by wave 0 alone
    // (64 sequences per step: per-lane count, in-wave inclusive scan, running carry)
    for (int i = tid; i < p.n_sel; i += NT) hids[i] = p.head_ids[i];
    if (tid < 2 * NW) mail[tid].flag = kMailEmpty;
    if (wave == 0) {
        int carry = 0;
        for (int b0 = 0; b0 < batch; b0 += 64) {
            const int b = b0 + lane;
            const int L = b < batch ? p.seq_lens[b] : 0;
            int n = (L + p.chunk_tokens - 1) / p.chunk_tokens;
            if (L <= 0) n = (p.direct_single && b < batch) ? 1 : 0;   // the item that writes the zeros
            int incl = n;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int up = __shfl_up(incl, off, 64);
                if (lane >= off) incl += up;
            }
            if (b < batch) {
                lens[b] = L;
                first[b] = carry + incl - n;
            }
            carry += __shfl(incl, 63, 64);
        }
        if (lane == 0) first[batch] = carry;
    }
    __syncthreads();
    const int total = first[batch] * p.n_sel;

    if (wave == NW) {
        // ------------------------------------------------------------ writer wave
        int next_box[NW];
#pragma unroll
        for (int v = 0; v < NW; ++v) next_box[v] = 0;
        int done_mask = 0;
        int idle = 0;
        while (done_mask != (1 << NW) - 1 && idle < kSpinLimit) {
            bool progressed = false;
#pragma unroll
            for (int v = 0; v < NW; ++v) {
                if (done_mask & (1 << v)) continue;
                Mail &mb = mail[v * 2 + next_box[v]];
                const int f = __builtin_amdgcn_readfirstlane(mail_load(&mb.flag));
                if (f == kMailFull) {
                    flush_mailbox<D, R>(mb, p, lane);
                    mail_store(&mb.flag, kMailEmpty);
                    next_box[v] ^= 1;
                    progressed = true;
                } else if (f == kMailDone) {
                    done_mask |= 1 << v;
                    progressed = true;
                }
            }
            if (progressed) {
                idle = 0;
            } else {
                ++idle;
                __builtin_amdgcn_s_sleep(8);
            }
        }
        return;
    }

    // ---------------------------------------------------------------- streaming waves
    // item number -> sequence: binary search in the first-chunk table; sequences are visited
    // in ascending order, so `cursor` (the last answer) is the lower end of the search
    auto decode = [&](int w, ItemHdr &h, int &cursor) {
        const int cg = w / p.n_sel;
        h.si = w - cg * p.n_sel;
        int lo = cursor, hi = batch - 1;          // answer: the last b with first[b] <= cg
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (first[mid] <= cg)
                lo = mid;
            else
                hi = mid - 1;
        }
        cursor = __builtin_amdgcn_readfirstlane(lo);
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
    struct Slot {
        ItemHdr h;
        int ids;            // lane i: physical block of the item's i-th tile
        int64_t head_off;
        bool exists;
    };
    int cursor = 0;
    auto fill = [&](int wi, Slot &s) {
        s.exists = wi < total;
        decode(min(wi, max(total - 1, 0)), s.h, cursor);
        if (!s.exists) s.h.nblk = 0;
        s.head_off = (int64_t)s.h.g * p.stride_head;
        const int32_t *bt =
            p.block_table + (int64_t)s.h.b * p.max_blocks_per_seq + s.h.t0 / kBlockTokens;
        s.ids = bt[min(lane, max(s.h.nblk - 1, 0))];
    };
    auto q_rows = [&](const Slot &s) {
        return p.q + ((int64_t)s.h.b * p.n_q_heads + s.h.g * R) * D;
    };
    auto issue = [&](Tile &t, int ids, int idx, int64_t head_off, bool valid) {
        const int blk = __builtin_amdgcn_readlane(ids, idx & 63);
        const int64_t base = (int64_t)blk * p.stride_block + head_off;
        Policy::issue(t, tile_rsrc(p.k_cache + base, kTileBytes, valid),
                      tile_rsrc(p.v_cache + base, kTileBytes, valid), lane);
    };
    // bounded wait for a mailbox of this wave to be empty
    auto wait_empty = [&](Mail &mb) {
        for (int spin = 0; spin < kSpinLimit; ++spin) {
            if (__builtin_amdgcn_readfirstlane(mail_load(&mb.flag)) == kMailEmpty) break;
            __builtin_amdgcn_s_sleep(2);
        }
    };

    const int stride = gridDim.x * NW;
    int w = blockIdx.x * NW + wave;
    unsigned char *my_staging = staging + (size_t)wave * Policy::kWaveLdsBytes;
    Mail *my_mail = mail + wave * 2;
    if (total <= 0 || w >= total) {
        mail_store(&my_mail[0].flag, kMailDone);
        return;
    }

    Slot cur, nxt, nn;
    typename Policy::Query q;
    typename Policy::QueryPrefetch q_pre;
    Tile A, B;
    fill(w, cur);
    fill(w + stride, nxt);
    Policy::q_prefetch(q_pre, q_rows(cur), lane);
    issue(A, cur.ids, 0, cur.head_off, 0 < cur.h.nblk);
    issue(B, cur.ids, 1, cur.head_off, 1 < cur.h.nblk);
    int n = 0;
    for (;; ++n) {
        fill(w + 2 * stride, nn);                       // header and block ids two items ahead
        Policy::q_commit(q, q_pre, my_staging, lane);   // this item's query operand
        Policy::q_prefetch(q_pre, q_rows(nxt), lane);   // next item's query rows

        typename Policy::State st;
        Policy::reset(st);
        const int n_my = cur.h.nblk;
        const int lim = 2 * max(1, (n_my + 1) >> 1);    // tiles of this item, as whole pairs
        // refill with tile j of the pair stream: tiles of `cur`, then the first pair of `nxt`
        auto refill = [&](Tile &t, int j) {
            const bool in_cur = j < lim;
            issue(t, in_cur ? cur.ids : nxt.ids, in_cur ? j : j - lim,
                  in_cur ? cur.head_off : nxt.head_off, in_cur ? j < n_my : j - lim < nxt.h.nblk);
        };
        auto consume = [&](const Tile &t, int i) {
            const int n_valid = (cur.h.rem != 0 && i == n_my - 1) ? cur.h.rem : kBlockTokens;
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
        // hand the finished item to the writer
        Mail &mb = my_mail[n & 1];
        wait_empty(mb);
        if (!cur.h.zero) Policy::finish(st, mb.o, mb.lse, lane);
        if (lane == 0) {
            mb.b = cur.h.b;
            mb.g = cur.h.g;
            mb.si = cur.h.si;
            mb.c = cur.h.c;
            mb.kind = cur.h.zero ? kKindZero : (cur.h.to_out ? kKindOut : kKindPartial);
        }
        mail_store(&mb.flag, kMailFull);
        if (!nxt.exists) break;
        cur = nxt;
        nxt = nn;
        w += stride;
    }
    Mail &last = my_mail[(n + 1) & 1];
    wait_empty(last);
    mail_store(&last.flag, kMailDone);
}

}  // namespace hetis
