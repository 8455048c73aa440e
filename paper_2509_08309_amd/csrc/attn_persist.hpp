// Persistent chunk kernel: work enumeration, tile streaming and chunk results for Eq. (2b),
// independent of how a tile is turned into scores and sums (that is the Policy: vector ALU
// arithmetic for small query groups, MFMA for grouped-query attention).
//
// Work enumeration: every workgroup loads the sequence lengths and scans them into tables of
// running counts (LDS): whole chunks per sequence, and ragged last chunks per sequence in four
// classes by size.  A flat item number then decodes into (sequence, chunk, selected head) by binary
// search, whole chunks first, then the ragged ones from the longest class to the shortest,
// without launching a workgroup per possible chunk; the items handed out last are the
// shortest, which keeps the tail of the launch short.  An item is one chunk of one
// (sequence, selected head) and is processed by ONE wave.
// Work distribution: the first two items of a streaming wave are fixed by its number; the
// rest come from a global ticket counter, so that waves which drew short chunks simply take
// more of them.  Tickets are drawn by the workgroup's writer wave, eight per device atomic
// while plenty of work is left and fewer towards the end, decoded there (one ticket per
// lane), and put into a small LDS pool from which the streaming waves take them, ready to
// use, with an LDS atomic shortly before they finish an item.  Which wave computes an item has no
// influence on the item's arithmetic.  The ticket counter and a counter of finished
// workgroups are control words of the call's workspace (AttnParams::control); the workgroup
// that finishes last sets both back to zero for the next launch.
//
// A workgroup is NW streaming waves plus one writer wave; after the prologue they never
// meet at a barrier.
//   - Streaming waves stream the tiles of their item through a register ring of
//     Policy::kRing slots; a slot is refilled right after it has been consumed, so up to
//     kRing tile pairs (8 KB each) per wave are in flight, and the ring runs on into the
//     first tiles of the next item before the current item is finished off.  Every global load is issued
//     unconditionally (indices clamped, tiles that do not exist turned into zero-length
//     buffer descriptors), so the in-order load counter is known exactly at every wait.
//     These waves never store to global memory: on gfx9-class hardware loads and stores
//     share one counter that is in order only among loads, so a single pending store would
//     force every later wait to drain all loads.  A finished item (normalised rows and
//     their log-sum-exp) is handed over through one of the wave's two LDS mailboxes.
//   - The writer wave polls the mailboxes and copies full ones to global memory (fp16 row,
//     fp32 partial, or zeros for an empty sequence), and keeps the ticket pool filled.
// Mailbox protocol (flag is a workgroup-scope atomic in LDS): EMPTY -> the producer fills
// data and header -> FULL -> the writer copies it out -> EMPTY.  A producer that has no more
// items marks its next mailbox DONE; the writer leaves when all NW are DONE.  All waits are
// polling loops with an iteration bound, so every wave reaches its end whatever happens; a
// wait that runs into its bound sets a flag in the workspace's error word, which the host
// reads with hetis_attn_workspace_status (the launch may then have lost a result).
// Dynamic LDS: int lens[batch], int firstF[batch + 1], int firstT[4][batch + 1], int
// hids[n_sel] (pairs mode: hids[batch], pseq[batch]); NW x 2 mailboxes; NW per-wave staging
// areas of Policy::kWaveLdsBytes.
// Pairs mode (per-request head subsets, Section 4.2 / 5.2.1): the rows of the enumeration are
// (sequence, KV head) pairs instead of sequences, each with its own block-table row over a
// pool of single-head tiles; everything else, the arithmetic of an item included, is shared.
// Nothing depends on how many heads were selected or on the grid size: the result for one
// (sequence, head) is a function of that sequence's length alone.
#pragma once
#include "attn_common.hpp"

namespace hetis {

enum : int { kMailEmpty = 0, kMailFull = 1, kMailDone = 2 };
enum : int { kKindOut = 0, kKindPartial = 1, kKindZero = 2 };
constexpr int kSpinLimit = 1 << 22;     // polls before a wait gives up (far beyond any real wait)
constexpr int kPoolSize = 32;           // item numbers the LDS ticket pool can hold
constexpr int kTicketBatch = 8;         // tickets per device atomic

// An item, decoded: what a streaming wave needs to start on it.
struct ItemDesc {
    int b, c, si, g;    // enumeration row (sequence, or pair), chunk, position in head_ids, KV head
    int seq;            // sequence whose query rows and output rows the item uses
    int n_tok;          // tokens of the chunk
    int flags;          // kItemExists | kItemToOut | kItemZero
    int pad;
};
enum : int { kItemExists = 1, kItemToOut = 2, kItemZero = 4 };

// Items waiting to be taken by the streaming waves of one workgroup, already decoded by the
// writer wave.
struct TicketPool {
    int next;                   // entries taken so far  (LDS atomic, streaming waves)
    int end;                    // entries published so far (written by the writer wave)
    ItemDesc desc[kPoolSize];   // ring: entry i lives in desc[i % kPoolSize]
};

// One finished item on its way to global memory.
template <int D, int R>
struct Mailbox {
    float o[R][D];      // normalised output rows
    float lse[R];       // natural-log log-sum-exp of each row (partial results only)
    int out_row;        // first of the item's R rows in `out`: sequence * n_q_heads + KV head * R
    int item;           // index of the item's slot in the partial buffers
    int kind;           // kKindOut / kKindPartial / kKindZero
    int flag;           // kMailEmpty / kMailFull / kMailDone
};

// Mailbox -> `out` (fp16) or the partial buffers (fp32); one wave, four elements a lane.
template <int D, int R>
__device__ __forceinline__ void flush_mailbox(const Mailbox<D, R> &mb, const AttnParams &p, int lane)
{
    const int64_t out_row = __builtin_amdgcn_readfirstlane(mb.out_row);
    const int kind = __builtin_amdgcn_readfirstlane(mb.kind);
    // the r rows of one (sequence, head, chunk) are contiguous in the partial buffers, so an
    // item leaves as one run of r*D floats plus one run of r floats
    const int64_t item = __builtin_amdgcn_readfirstlane(mb.item);
#pragma unroll
    for (int idx = lane * 4; idx < R * D; idx += 256) {
        const int r = idx / D, d = idx % D;
        float4 v = *reinterpret_cast<const float4 *>(&mb.o[r][d]);
        if (kind == kKindPartial) {
            *reinterpret_cast<float4 *>(p.o_partial + item * (R * D) + idx) = v;
        } else {
            if (kind == kKindZero) v = make_float4(0.f, 0.f, 0.f, 0.f);
            union {
                __half2 h[2];
                uint2 u;
            } pk;
            pk.h[0] = __floats2half2_rn(v.x, v.y);
            pk.h[1] = __floats2half2_rn(v.z, v.w);
            *reinterpret_cast<uint2 *>(p.out + (out_row + r) * D + d) = pk.u;
        }
    }
    if (kind == kKindPartial && lane < R) p.lse_partial[item * R + lane] = mb.lse[lane];
}

struct ItemHdr {
    int b, si, c, g;    // enumeration row (sequence, or pair), position in head_ids, chunk, KV head
    int seq;            // sequence whose query rows and output rows the item uses
    int nblk;       // blocks of this chunk
    int rem;        // tokens in the ragged last block (0: none)
    int t0;         // first token of the chunk
    bool to_out;    // result goes to `out` (fp16), not to the partial buffers
    bool zero;      // length-0 sequence whose zeros this pass writes
};

__host__ __device__ constexpr size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

// Table words after the six per-row tables: the selected heads, or in pairs mode the head and
// the sequence of every pair.
__host__ __device__ constexpr int persist_id_words(int batch, int n_sel, bool pairs)
{
    return pairs ? 2 * batch : n_sel;
}

template <class Policy, int NW>
__host__ __device__ constexpr size_t persist_lds_bytes(int batch, int n_sel, bool pairs)
{
    return align16((size_t)(6 * batch + 5 + persist_id_words(batch, n_sel, pairs)) * sizeof(int)) +
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

template <class Policy, int NW, bool PAIRS>
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
    int *firstF = lens + batch;               // whole chunks before sequence b
    int *firstT = firstF + batch + 1;         // [4][batch + 1]: ragged last chunks of size class
                                              // k before sequence b (class 3 also holds the
                                              // items that write zeros)
    int *hids = firstT + 4 * (batch + 1);     // KV head of position si in head_ids / of pair b
    int *pseq = hids + batch;                 // pairs mode: sequence of pair b
    const int n_sel = PAIRS ? 1 : p.n_sel;    // items per (row, chunk)
    const int n_ids = PAIRS ? batch : p.n_sel;
    unsigned char *after_tables =
        smem + align16((size_t)(6 * batch + 5 + persist_id_words(batch, p.n_sel, PAIRS)) * sizeof(int));
    __shared__ TicketPool pool;
    Mail *mail = reinterpret_cast<Mail *>(after_tables);             // [NW][2]
    unsigned char *staging = after_tables + 2 * NW * sizeof(Mail);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- work enumeration.  All threads fetch the lengths and work out the counts of their
    // rows (whole chunks; size class of the ragged last chunk), four rows a thread and round
    // so that the loads of a round are in flight together.  Wave 0 then turns the counts into
    // running counts in place: lane l owns `per` consecutive rows, adds up their counts, the
    // 64 lane totals go through one in-wave scan, and a second pass over the lane's rows
    // writes the tables.  `per` is odd so that the lanes' LDS accesses (stride `per` words)
    // fall into different banks.
    for (int i = tid; i < n_ids; i += NT) {
        hids[i] = PAIRS ? p.pair_head[i] : p.head_ids[i];
        if (PAIRS) pseq[i] = p.pair_seq[i];
    }
    // size class of a ragged last chunk of `rt` tokens: 0 = longest quarter ... 3 = shortest
    auto ragged_class = [&](int rt) { return 3 - min(3, (4 * rt - 1) / p.chunk_tokens); };
    for (int i0 = tid; i0 < batch; i0 += 4 * NT) {
        int row[4], L[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = min(i0 + u * NT, batch - 1);
            row[u] = PAIRS ? p.pair_seq[i] : i;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) L[u] = p.seq_lens[row[u]];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + u * NT;
            if (i >= batch) continue;
            const int nF = L[u] > 0 ? L[u] / p.chunk_tokens : 0;
            const int rt = L[u] > 0 ? L[u] - nF * p.chunk_tokens : 0;
            int cls = -1;
            if (rt > 0) cls = ragged_class(rt);
            if (L[u] <= 0 && p.direct_single) cls = 3;      // the item that writes the zeros
            lens[i] = L[u];
            firstF[i] = nF;                 // counts for now; running counts after the scan
            firstT[i] = cls;
        }
    }
    if (tid < 2 * NW) mail[tid].flag = kMailEmpty;
    if (tid == 0) {
        pool.next = 0;
        pool.end = 0;
    }
    __syncthreads();
    if (wave == 0) {
        // classes 0,1 and 2,3 travel packed in 16-bit halves (batch < 65536)
        auto class_counts = [&](int cls, int &n01, int &n23) {
            n01 = cls == 0 ? 1 : (cls == 1 ? 1 << 16 : 0);
            n23 = cls == 2 ? 1 : (cls == 3 ? 1 << 16 : 0);
        };
        const int per = ((batch + 63) / 64) | 1;
        const int lo = min(lane * per, batch), hi = min(lo + per, batch);
        int sumF = 0, sum01 = 0, sum23 = 0;
        for (int b = lo; b < hi; ++b) {
            int n01, n23;
            class_counts(firstT[b], n01, n23);
            sumF += firstF[b];
            sum01 += n01;
            sum23 += n23;
        }
        int inclF = sumF, incl01 = sum01, incl23 = sum23;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int upF = __shfl_up(inclF, off, 64);
            const int up01 = __shfl_up(incl01, off, 64);
            const int up23 = __shfl_up(incl23, off, 64);
            if (lane >= off) {
                inclF += upF;
                incl01 += up01;
                incl23 += up23;
            }
        }
        int runF = inclF - sumF, run01 = incl01 - sum01, run23 = incl23 - sum23;
        for (int b = lo; b < hi; ++b) {
            int n01, n23;
            class_counts(firstT[b], n01, n23);
            const int nF = firstF[b];
            firstF[b] = runF;
            firstT[0 * (batch + 1) + b] = run01 & 0xffff;
            firstT[1 * (batch + 1) + b] = run01 >> 16;
            firstT[2 * (batch + 1) + b] = run23 & 0xffff;
            firstT[3 * (batch + 1) + b] = run23 >> 16;
            runF += nF;
            run01 += n01;
            run23 += n23;
        }
        if (lane == 63) {
            firstF[batch] = inclF;
            firstT[0 * (batch + 1) + batch] = incl01 & 0xffff;
            firstT[1 * (batch + 1) + batch] = incl01 >> 16;
            firstT[2 * (batch + 1) + batch] = incl23 & 0xffff;
            firstT[3 * (batch + 1) + batch] = incl23 >> 16;
        }
    }
    __syncthreads();
    const int totalF = firstF[batch];                         // whole chunks of all sequences
    int class_end[4];                                         // running ends of the ragged classes
    {
        int run = totalF;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            run += firstT[k * (batch + 1) + batch];
            class_end[k] = run;
        }
    }
    const int total = class_end[3] * n_sel;
    const int stride = gridDim.x * NW;                        // streaming waves in the grid

    // item number -> (row, chunk, head): whole chunks come first, ragged last chunks after
    // them by size class; binary search in the matching running-count table.  Works per lane
    // (the writer wave decodes a batch of tickets at once, one per lane).
    auto upper = [&](const int *tab, int key) {               // last b with tab[b] <= key
        int lo = 0, hi = batch - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (tab[mid] <= key)
                lo = mid;
            else
                hi = mid - 1;
        }
        return lo;
    };
    auto decode = [&](int item) {
        ItemDesc d;
        d.flags = item < total ? kItemExists : 0;
        const int w = min(item, max(total - 1, 0));
        const int cg = PAIRS ? w : w / n_sel;
        d.si = PAIRS ? 0 : w - cg * n_sel;
        int L;
        if (cg < totalF) {
            d.b = upper(firstF, cg);
            d.c = cg - firstF[d.b];
            L = lens[d.b];
            d.n_tok = p.chunk_tokens;
        } else {
            int k = 0, begin = totalF;
#pragma unroll
            for (int j = 0; j < 3; ++j)
                if (cg >= class_end[j]) {
                    k = j + 1;
                    begin = class_end[j];
                }
            d.b = upper(firstT + k * (batch + 1), cg - begin);
            L = lens[d.b];
            d.c = L > 0 ? L / p.chunk_tokens : 0;
            d.n_tok = L > 0 ? L - d.c * p.chunk_tokens : 0;
        }
        d.g = hids[PAIRS ? d.b : d.si];
        d.seq = PAIRS ? pseq[d.b] : d.b;
        const int n_chunks = (L + p.chunk_tokens - 1) / p.chunk_tokens;
        if (p.direct_single && n_chunks <= 1) d.flags |= kItemToOut;
        if (L <= 0) d.flags |= kItemZero;
        d.pad = 0;
        return d;
    };

    if (wave == NW) {
        // ------------------------------------------------------------ writer wave
        int next_box[NW];
#pragma unroll
        for (int v = 0; v < NW; ++v) next_box[v] = 0;
        int done_mask = 0;
        int idle = 0;
        int pool_end = 0;                 // entries published so far
        long long last_base = 2ll * stride;   // item number of the last ticket drawn here
        bool exhausted = total <= 2 * stride;    // no item left beyond the fixed ones
        while (done_mask != (1 << NW) - 1 && idle < kSpinLimit) {
            bool progressed = false;
            // keep the ticket pool ahead of the streaming waves
            const int taken = __builtin_amdgcn_readfirstlane(
                __hip_atomic_load(&pool.next, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
            // batch size shrinks as the work runs out (judged by the last ticket seen), so
            // that the last items are not parked in one workgroup's pool
            const long long left = (long long)total - last_base;
            const int n_draw = left > 8ll * stride ? kTicketBatch : (left > 2ll * stride ? 2 : 1);
            if (pool_end - taken < n_draw) {
                long long base = total;   // past the last item: "no more work"
                if (!exhausted) {
                    unsigned t = 0;
                    if (lane == 0)
                        t = __hip_atomic_fetch_add(p.control + kCtlTickets, (unsigned)n_draw,
                                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    base = 2ll * stride + __builtin_amdgcn_readfirstlane(t);
                    last_base = base;
                    if (base + n_draw >= total) exhausted = true;
                }
                if (lane < n_draw)
                    pool.desc[(pool_end + lane) % kPoolSize] =
                        decode((int)min(base + lane, (long long)total));
                pool_end += n_draw;
                __hip_atomic_store(&pool.end, pool_end, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                progressed = true;
            }
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
                __builtin_amdgcn_s_sleep(4);
            }
        }
        // every streaming wave of this workgroup is done, so no more tickets will be drawn
        // here: count the workgroup out; the last one to leave rearms both counters
        if (lane == 0) {
            if (done_mask != (1 << NW) - 1) report_error(p.control, kErrWriterWait);
            const unsigned gone = __hip_atomic_fetch_add(p.control + kCtlGone, 1u, __ATOMIC_RELAXED,
                                                         __HIP_MEMORY_SCOPE_AGENT);
            if (gone == gridDim.x - 1) {
                __hip_atomic_store(p.control + kCtlTickets, 0u, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(p.control + kCtlGone, 0u, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        return;
    }

    // ---------------------------------------------------------------- streaming waves
    struct Slot {
        ItemHdr h;
        int ids;            // lane i: physical block of the item's i-th tile
        int64_t head_off;
        bool exists;
    };
    // decoded item -> the wave's (uniform) bookkeeping, and the load of its block ids
    auto fill = [&](const ItemDesc &d, Slot &s) {
        const int flags = __builtin_amdgcn_readfirstlane(d.flags);
        const int n_tok = __builtin_amdgcn_readfirstlane(d.n_tok);
        s.h.b = __builtin_amdgcn_readfirstlane(d.b);
        s.h.c = __builtin_amdgcn_readfirstlane(d.c);
        s.h.si = __builtin_amdgcn_readfirstlane(d.si);
        s.h.g = __builtin_amdgcn_readfirstlane(d.g);
        s.h.seq = __builtin_amdgcn_readfirstlane(d.seq);
        s.exists = (flags & kItemExists) != 0;
        s.h.to_out = (flags & kItemToOut) != 0;
        s.h.zero = (flags & kItemZero) != 0;
        s.h.t0 = s.h.c * p.chunk_tokens;
        s.h.nblk = s.exists ? (n_tok + kBlockTokens - 1) / kBlockTokens : 0;
        s.h.rem = n_tok & (kBlockTokens - 1);
        s.head_off = PAIRS ? 0 : (int64_t)s.h.g * p.stride_head;   // pairs: single-head tiles
        const int32_t *bt =
            p.block_table + (int64_t)s.h.b * p.max_blocks_per_seq + s.h.t0 / kBlockTokens;
        s.ids = bt[min(lane, max(s.h.nblk - 1, 0))];
    };
    auto q_rows = [&](const Slot &s) {
        return p.q + ((int64_t)s.h.seq * p.n_q_heads + s.h.g * R) * D;
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
            if (__builtin_amdgcn_readfirstlane(mail_load(&mb.flag)) == kMailEmpty) return;
            __builtin_amdgcn_s_sleep(2);
        }
        if (lane == 0) report_error(p.control, kErrMailboxWait);
    };
    // next item from the workgroup's pool, decoded by the writer wave (flags 0 = none left)
    auto take_ticket = [&]() {
        int i = 0;
        if (lane == 0)
            i = __hip_atomic_fetch_add(&pool.next, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        i = __builtin_amdgcn_readfirstlane(i);
        for (int spin = 0; spin < kSpinLimit; ++spin) {
            const int end = __builtin_amdgcn_readfirstlane(
                __hip_atomic_load(&pool.end, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP));
            if (end > i) return pool.desc[i % kPoolSize];
            __builtin_amdgcn_s_sleep(2);
        }
        if (lane == 0) report_error(p.control, kErrTicketWait);
        ItemDesc none{};
        return none;
    };

    const int w = blockIdx.x * NW + wave;
    unsigned char *my_staging = staging + (size_t)wave * Policy::kWaveLdsBytes;
    Mail *my_mail = mail + wave * 2;
    if (total <= 0 || w >= total) {
        mail_store(&my_mail[0].flag, kMailDone);
        return;
    }

    constexpr int RING = Policy::kRing;             // tile pairs a wave keeps in flight, at most
    Slot cur, nxt;
    typename Policy::Query q;
    typename Policy::QueryPrefetch q_pre;
    Tile ring[RING];
    fill(decode(w), cur);           // items w and w + stride are this wave's without a ticket
    nxt = cur;
    Policy::q_prefetch(q_pre, q_rows(cur), lane);
#pragma unroll
    for (int s = 0; s < RING; ++s) issue(ring[s], cur.ids, s, cur.head_off, s < cur.h.nblk);
    int n = 0;
    for (;; ++n) {
        Policy::q_commit(q, q_pre, my_staging, lane);   // this item's query operand

        typename Policy::State st;
        Policy::reset(st);
        const int n_my = cur.h.nblk;
        const int lim = RING * max(1, (n_my + RING - 1) / RING);   // tiles, as whole ring turns
        // The scheduling fences keep "consume a slot, refill it at once" in program order;
        // without them the compiler batches the tiles' arithmetic ahead of the refills and
        // the wave ends up waiting with nothing in flight.
        auto steady_turn = [&](int i) {                 // whole tiles; refills stay in this item
#pragma unroll
            for (int s = 0; s < RING; ++s) {
                Policy::template update<false>(st, ring[s], q, p.scale_log2, lane, kBlockTokens,
                                               my_staging);
                __builtin_amdgcn_sched_barrier(0);
                issue(ring[s], cur.ids, i + RING + s, cur.head_off, i + RING + s < n_my);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // The next item is chosen as late as its block ids allow (three ring turns before
        // the end of this one), so that little undone work is held back when the tickets run
        // out.
        int i = 0;
        for (; i + 4 * RING < lim; i += RING) steady_turn(i);
        fill(n == 0 ? decode(w + stride) : take_ticket(), nxt);
        Policy::q_prefetch(q_pre, q_rows(nxt), lane);   // next item's query rows
        for (; i + RING < lim; i += RING) steady_turn(i);
        // last turn of this item (the only place a ragged block can be): its refills are the
        // first tiles of the next item
#pragma unroll
        for (int s = 0; s < RING; ++s) {
            if (i + s < n_my) {
                const int n_valid = (cur.h.rem != 0 && i + s == n_my - 1) ? cur.h.rem : kBlockTokens;
                Policy::template update<true>(st, ring[s], q, p.scale_log2, lane, n_valid, my_staging);
            }
            __builtin_amdgcn_sched_barrier(0);
            issue(ring[s], nxt.ids, s, nxt.head_off, s < nxt.h.nblk);
            __builtin_amdgcn_sched_barrier(0);
        }

        // hand the finished item to the writer
        Mail &mb = my_mail[n & 1];
        wait_empty(mb);
        if (!cur.h.zero) Policy::finish(st, mb.o, mb.lse, lane);
        if (lane == 0) {
            mb.out_row = cur.h.seq * p.n_q_heads + cur.h.g * R;
            mb.item = (cur.h.b * n_sel + cur.h.si) * p.max_chunks + cur.h.c;
            mb.kind = cur.h.zero ? kKindZero : (cur.h.to_out ? kKindOut : kKindPartial);
        }
        mail_store(&mb.flag, kMailFull);
        if (!nxt.exists) break;
        cur = nxt;
    }
    Mail &last = my_mail[(n + 1) & 1];
    wait_empty(last);
    mail_store(&last.flag, kMailDone);
}

}  // namespace hetis
