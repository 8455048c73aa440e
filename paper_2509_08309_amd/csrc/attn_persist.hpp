// Persistent kernel of head-subset decode Attention: work enumeration, tile streaming and
// the combination of chunk results for Eq. (2b), independent of how a tile is turned into
// scores and sums (that is the Policy: vector ALU arithmetic for small query groups, MFMA
// for grouped-query attention).
//
// Units of work.  A ROW is one (enumeration row, selected KV head): a sequence (or, in pairs
// mode, a (sequence, head) pair) and one of the heads computed for it.  The tokens of a row
// are cut into SEGMENTS of seg_tokens tokens from token 0; a segment is cut into CHUNKS of
// chunk_tokens tokens.  A chunk is processed by ONE wave; a segment is processed by ONE
// workgroup, whose waves take its chunks and whose writer wave folds the chunk results
// together in LDS, in ascending chunk order, so a segment leaves the workgroup as a single
// result: the finished fp16 row when the segment is the whole row, an fp32 partial result
// (normalised sum and log-sum-exp) otherwise.  With seg_tokens = chunk_tokens every chunk is
// its own segment (the split-KV entry points); with seg_tokens = 4096 a row of up to 4096
// tokens never touches global memory between its first tile and its output row.
//
// Work enumeration: every workgroup loads the row lengths and builds two tables in LDS: the
// running count of whole segments per row, and the list of the rows that end in a shorter
// segment, sorted by the size class of that segment (kClasses classes, a counting sort done by
// the whole workgroup: see the prologue).  A flat segment number then decodes into (row,
// segment, head): whole segments first (binary search in the running counts), then the shorter
// ones from the largest class to the smallest (a look-up in the sorted list), so the segments
// handed out last are the short ones, which keeps the end of the launch short.
// Work distribution: segment number blockIdx.x belongs to the workgroup without asking (when
// every segment is a single chunk: two such segments per streaming wave); the rest are tickets
// from a device counter, drawn by the workgroup's writer wave, which decodes a segment,
// reserves a fold slot for it and puts its chunks, ready to use, into an LDS pool; the
// streaming waves take chunks from the pool with an LDS atomic shortly before they finish the
// chunk at hand.  Which wave or workgroup computes a chunk has no influence on the arithmetic:
// a row's result is a function of its length and the compile-time constants alone.
// The ticket counter and a counter of workgroups that will draw no more are control words of
// the call's workspace (AttnParams::control); the last workgroup to count itself out sets both
// back to zero for the next launch.
// Scheduling modes (AttnParams::mode).  kModeSegments is the above.  kModeSplit: seg_tokens =
// chunk_tokens, every chunk leaves as a partial result for a separate merge launch.
// kModeSpread, for launches with few rows, where whole segments would leave most workgroups
// without work: the unit handed out is the chunk (the enumeration counts chunks per row, in
// row order, no sorting), chunk results go through the partial buffers in global memory, and
// the wave that stores the last chunk result of a segment folds that segment's chunks with the
// operations and in the order of the in-LDS fold (fold_coef / fold_weight / fold_elem are
// shared), so that the mode never shows in a result.  The kernel takes kModeSpread only when
// some row is longer than two turns of a workgroup's waves.
//
// A workgroup is NW streaming waves plus one writer wave; after the prologue they never
// meet at a barrier.
//   - Streaming waves stream the tiles of their chunk through a register ring of
//     Policy::kRing slots; a slot is refilled right after it has been consumed, so up to
//     kRing tile pairs per wave are in flight, and the ring runs on into the first tiles of
//     the next chunk before the current one is finished off.  Every global load is issued
//     unconditionally (indices clamped, tiles that do not exist turned into zero-length
//     buffer descriptors), so the in-order load counter is known exactly at every wait.
//     These waves never store to global memory: on gfx9-class hardware loads and stores
//     share one counter that is in order only among loads, so a single pending store would
//     force every later wait to drain all loads.  A finished chunk (normalised rows and
//     their base-2 log-sum-exp) is handed over through one of the wave's two LDS mailboxes.
//   - The writer wave polls the mailboxes.  A chunk that is a whole segment goes straight to
//     global memory (fp16 row, fp32 partial, or zeros for an empty sequence).  A chunk of a
//     longer segment is folded into the segment's slot: running maximum M, weight sum W and
//     weighted sum A with  M' = max(M, lse_c), A' = A 2^(M-M') + o_c 2^(lse_c-M'), W likewise;
//     chunk c is folded only after chunks 0..c-1 (a mailbox whose turn has not come stays
//     full), so the order of the floating-point operations is fixed.  After the last chunk
//     A / W leaves as the segment's result.
// Mailbox protocol (flag is a workgroup-scope atomic in LDS): EMPTY -> the producer fills
// data and header -> FULL -> the writer consumes it -> EMPTY.  A producer that has no more
// chunks marks its next mailbox DONE; the writer leaves when all NW are DONE.
// No wait can last for ever: chunks enter the pool in order, a wave's two mailboxes hold
// only chunks it took earlier, so the earliest chunk not yet folded can always be deposited
// and is always next in its segment.  All the same every wait is a polling loop with an
// iteration bound, so that every wave reaches its end whatever happens; a wait that runs
// into its bound sets a flag in the workspace's error word, which the host reads with
// hetis_attn_workspace_status (the launch may then have lost a result).
// Dynamic LDS: int lens[rows], int firstF[rows + 1] (and two spare words), uint16 order[rows],
// int hids[n_sel] (pairs mode: hids[rows], pseq[rows]); NW x 2 mailboxes; fold slots; NW
// per-wave staging areas of Policy::kWaveLdsBytes.  Static LDS: the chunk pool and the scan
// array of the enumeration.
// Decode step with the store folded in (AttnParams::k_new): the new token's K and V rows go
// to position L - 1 of the cache inside this launch.  The writer wave stores the rows of a
// (sequence, head) right before it puts the chunk that contains position L - 1 into the pool,
// and waits for the stores to complete; the wave that takes the chunk runs on the same
// compute unit and takes it with an acquire, so it reads the new rows.  That chunk is never
// one of those taken without the pool.  (kModeSegments only: the host runs the store as a
// launch of its own when it offers kModeSpread.)
// Pairs mode (per-request head subsets, Section 4.2 / 5.2.1): the rows of the enumeration are
// (sequence, KV head) pairs instead of sequences, each with its own block-table row over a
// pool of single-head tiles; everything else, the arithmetic included, is shared.
#pragma once
#include "attn_common.hpp"

namespace hetis {

enum : int { kMailEmpty = 0, kMailFull = 1, kMailDone = 2 };
enum : int { kKindOut = 0, kKindPartial = 1, kKindZero = 2, kKindFold = 3 };
constexpr int kSpinLimit = 1 << 22;     // polls before a wait gives up (far beyond any real wait)
// Size classes of a row's last, shorter segment, largest first: fifteen of one sixteenth of a
// whole segment each, then the last sixteenth split at 1/32, 1/64 and 1/128 of a segment.
constexpr int kLinClasses = 15;
constexpr int kClasses = kLinClasses + 4;
static_assert(kClasses + 1 <= 32, "class number + 1 is packed into five bits");
constexpr int kMaxSegChunks = 32;       // chunks of a segment, at most (one writer lane each)
constexpr int kPoolSize = 2 * kMaxSegChunks;   // chunk descriptors the LDS pool can hold
constexpr int kTicketBatch = 8;         // tickets per device atomic while segments are single chunks
// Segments of at most 1/HETIS_FINE_CHUNK_BELOW of a whole one are cut into chunks of half the
// size, those of at most a quarter of that into chunks of a quarter of the size.
#ifndef HETIS_FINE_CHUNK_BELOW
#define HETIS_FINE_CHUNK_BELOW 4
#endif
// Chunks of multi-chunk segments a workgroup keeps waiting in its pool before it draws the
// next segment.
#ifndef HETIS_POOL_AHEAD
#define HETIS_POOL_AHEAD 2
#endif
// ... until so many segments are left to draw, in quarters of the number of workgroups.
#ifndef HETIS_LATE_SEGMENTS_X4
#define HETIS_LATE_SEGMENTS_X4 2
#endif
// Launches of up to this many segments a workgroup give every workgroup up to three segments
// without a ticket (0: one, always).
#ifndef HETIS_STATIC_SECOND_UPTO
#define HETIS_STATIC_SECOND_UPTO 4
#endif
// ... and only when the longest segment holds at most this many sixteenths of the tokens a
// workgroup gets on average.
#ifndef HETIS_STATIC_FLAT_X16
#define HETIS_STATIC_FLAT_X16 14
#endif
enum : int { kItemExists = 1 };

// x / d for x >= 0, d > 0 the same in all lanes: integer division has no instruction of its
// own and costs about forty; the divisors of the enumeration are powers of two unless a caller
// of the split entry points chooses otherwise.
__device__ __forceinline__ int udiv(int x, int d)
{
    if ((d & (d - 1)) == 0) return x >> __builtin_ctz(d);
    return x / d;
}

// Tokens per chunk of a segment of n_tok tokens: the shorter the segment, the later it is
// handed out and the finer it is cut, so that the chunks still running when the work runs out
// are short ones.  A function of the row's length and of constants only, like everything that
// shapes the arithmetic.
__device__ __forceinline__ int chunk_tokens_of(int n_tok, int chunk_tokens, int seg_tokens)
{
    int ct = chunk_tokens;
    if (seg_tokens > chunk_tokens) {
        if (n_tok <= seg_tokens / HETIS_FINE_CHUNK_BELOW) ct = chunk_tokens / 2;
        if (n_tok <= seg_tokens / (4 * HETIS_FINE_CHUNK_BELOW)) ct = chunk_tokens / 4;
        ct = max(ct, 2 * kBlockTokens);
    }
    return ct;
}

// One step of the running combination of chunk results (o_c normalised, lse_c base 2) into
// (A, M, W): M' = max(M, lse_c), A' = A 2^(M-M') + o_c 2^(lse_c-M'), W' = W 2^(M-M') + 2^(lse_c-M').
// Written once, with explicit fused multiply-adds, because two code paths (the fold in LDS and
// the fold from the partial buffers) must produce the same bits.
struct FoldCoef {
    float Mn, so, sc;
};
__device__ __forceinline__ FoldCoef fold_coef(float Mo, float lc)
{
    FoldCoef f;
    f.Mn = fmaxf(Mo, lc);
    f.so = fast_exp2(Mo - f.Mn);
    f.sc = fast_exp2(lc - f.Mn);
    return f;
}
__device__ __forceinline__ float fold_weight(float Wo, const FoldCoef &f)
{
    return __builtin_fmaf(Wo, f.so, f.sc);
}
__device__ __forceinline__ float fold_elem(float y, float x, const FoldCoef &f)
{
    return __builtin_fmaf(y, f.so, x * f.sc);
}

// A chunk, decoded: what a streaming wave needs to start on it and to label its result.
struct ChunkDesc {
    int b, g, seq;      // enumeration row (sequence, or pair), KV head, sequence of q / out rows
    int t0;             // first token of the chunk in its sequence
    int n_tok;          // tokens of the chunk
    int flags;          // kItemExists, or 0: no work is left, the wave may finish
    int kind;           // kKindOut / kKindPartial / kKindZero (whole segment) or kKindFold
    int dest;           // Out / Zero: first of the R rows in `out`; Partial: slot in the partial
                        // buffers; Fold: the segment's fold slot
    int cs;             // Fold: index of the chunk in its segment
    int nseg;           // segments of the chunk's row
    int out_row;        // first of the R rows of the chunk's (sequence, head) in `out`
    int len;            // tokens of the chunk's row
};

// Chunks waiting to be taken by the streaming waves of one workgroup, in order.
struct ChunkPool {
    int next;                   // entries taken so far  (LDS atomic, streaming waves)
    int end;                    // entries published so far (written by the writer wave)
    ChunkDesc desc[kPoolSize];  // ring: entry i lives in desc[i % kPoolSize]
};

// One finished chunk on its way to the writer wave.
template <int D, int R>
struct alignas(16) Mailbox {
    float o[R][D];      // normalised output rows
    float lse[R];       // base-2 log-sum-exp of each row: m + log2(sum_t 2^(s_t - m))
    int kind, dest, cs; // as in the chunk's descriptor
    int nseg, out_row, len;
    int flag;           // kMailEmpty / kMailFull / kMailDone
};

// Running combination of the chunks of one segment (writer wave only).
template <int D, int R>
struct alignas(16) FoldSlot {
    float acc[R][D];    // sum over folded chunks of o_c 2^(lse_c - M)
    float M[R];         // running maximum of lse_c (base 2); at the end M + log2 W
    float W[R];         // sum over folded chunks of 2^(lse_c - M)
    int next;           // chunk to fold next
    int ns;             // chunks of the segment
    int kind, dest;     // where the finished segment goes: kKindOut / kKindPartial
    int nseg, out_row;  // of the segment's row
};

template <int R>
__host__ __device__ constexpr int fold_slots() { return R >= 4 ? 5 : 8; }

// Result rows in LDS -> `out` (fp16) or the partial buffers (fp32); one wave, four elements a
// lane.  `lse2`: base-2 log-sum-exp per row; `w`: when not null, row r is divided by w[r] on
// the way out (the weight sum of a fold slot).
template <int D, int R>
__device__ __forceinline__ void store_result(const float (&o)[R][D], const float *lse2,
                                             const float *w, int kind, int64_t dest,
                                             const AttnParams &p, int lane)
{
#pragma unroll
    for (int idx = lane * 4; idx < R * D; idx += 256) {
        const int r = idx / D, d = idx % D;
        float4 v = *reinterpret_cast<const float4 *>(&o[r][d]);
        if (w) {
            const float s = __builtin_amdgcn_rcpf(w[r]);
            v = make_float4(v.x * s, v.y * s, v.z * s, v.w * s);
        }
        if (kind == kKindPartial) {
            // the r rows of one (row, head, segment) are contiguous in the partial buffers
            *reinterpret_cast<float4 *>(p.o_partial + dest * (R * D) + idx) = v;
        } else {
            if (kind == kKindZero) v = make_float4(0.f, 0.f, 0.f, 0.f);
            union {
                __half2 h[2];
                uint2 u;
            } pk;
            pk.h[0] = __floats2half2_rn(v.x, v.y);
            pk.h[1] = __floats2half2_rn(v.z, v.w);
            *reinterpret_cast<uint2 *>(p.out + (dest + r) * D + d) = pk.u;
        }
    }
    // partial results carry the natural-log log-sum-exp
    if (kind == kKindPartial && lane < R) p.lse_partial[dest * R + lane] = lse2[lane] * kLn2;
}

// Partial result of a segment that is merged inside this launch (AttnParams::arrivals): by
// whichever wave stores the row's last segment, possibly on another XCD, so the words are
// stored device-coherently, one per lane and step.
// `base2`: the log-sum-exp is stored as it is (chunk results of kModeSpread), otherwise as a
// natural logarithm (segment results).
template <int D, int R>
__device__ __forceinline__ void store_partial_coherent(const float (&o)[R][D], const float *lse2,
                                                       const float *w, int64_t dest,
                                                       const AttnParams &p, int lane, bool base2)
{
    static_assert(R * D % 64 == 0, "whole steps of one word a lane");
#pragma unroll
    for (int k = 0; k < R * D / 64; ++k) {
        const int idx = k * 64 + lane;
        float v = (&o[0][0])[idx];
        if (w) v *= __builtin_amdgcn_rcpf(w[idx / D]);
        coherent_store(p.o_partial + dest * (R * D) + idx, v);
    }
    if (lane < R)
        coherent_store(p.lse_partial + dest * R + lane, base2 ? lse2[lane] : lse2[lane] * kLn2);
}

// Log-sum-exp merge of the n_segs partial results of one row, ascending segment order, by one
// wave: M = max_c lse_c, w_c = exp(lse_c - M), out = fp16(sum_c w_c o_c / sum_c w_c).  Lane l
// owns dims l and l + 64 (D = 128) of each of the R query rows.  `first` is the index of
// segment 0 of the row in the partial buffers, segment c sits `stride` * c slots further.  The
// partial results may come from other XCDs: they are read with device-coherent loads.
template <int D, int R>
__device__ __forceinline__ void merge_partials(const AttnParams &p, int64_t first, int n_segs,
                                               int stride, int64_t out_row, int lane)
{
    constexpr int V = D / 64;                        // words per lane and row: 1 or 2
    const int64_t step = (int64_t)stride * R;        // rows of the buffers per segment
    const float *lse = p.lse_partial + first * R;    // [segment][r]
    const float *op = p.o_partial + first * (R * D) + lane;
    float M[R];
#pragma unroll
    for (int r = 0; r < R; ++r) M[r] = coherent_load(lse + r);
    for (int c = 1; c < n_segs; ++c) {
#pragma unroll
        for (int r = 0; r < R; ++r) M[r] = fmaxf(M[r], coherent_load(lse + c * step + r));
    }
    float W[R], acc[R][V];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        W[r] = 0.f;
#pragma unroll
        for (int v = 0; v < V; ++v) acc[r][v] = 0.f;
    }
    for (int c = 0; c < n_segs; ++c) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float w = fast_exp2((coherent_load(lse + c * step + r) - M[r]) * kLog2e);
            W[r] += w;
            const float *src = op + (c * step + r) * D;
#pragma unroll
            for (int v = 0; v < V; ++v) acc[r][v] = fmaf(w, coherent_load(src + v * 64), acc[r][v]);
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        __half *dst = p.out + (out_row + r) * D + lane;
#pragma unroll
        for (int v = 0; v < V; ++v) dst[v * 64] = __float2half_rn(acc[r][v] / W[r]);
    }
}

// kModeSpread: the ns chunk results of one segment lie in the partial buffers (chunk c in slot
// slot0 + c, log-sum-exp base 2).  One wave combines them with the operations a workgroup
// applies to the chunks of a segment in kModeSegments, in the same order: folded in ascending
// order, then normalised.  `whole_row`: the segment is the whole row and the result goes to
// `out`; otherwise it replaces the first chunk result in the buffers, as the partial result of
// the segment (natural-log log-sum-exp) that merge_partials expects.  Lane l owns dims l, l + 64.
template <int D, int R>
__device__ __forceinline__ void fold_segment_from_chunks(const AttnParams &p, int64_t slot0, int ns,
                                                         bool whole_row, int64_t out_row, int lane)
{
    constexpr int V = D / 64;
    constexpr int U = 16 / R;                         // chunk results loaded together
    float a[R][V], M[R], W[R];
    for (int c0 = 0; c0 < ns; c0 += U) {
        float x[U][R][V], lc[U][R];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t slot = slot0 + min(c0 + u, ns - 1);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                lc[u][r] = coherent_load(p.lse_partial + slot * R + r);
#pragma unroll
                for (int v = 0; v < V; ++v)
                    x[u][r][v] = coherent_load(p.o_partial + (slot * R + r) * D + v * 64 + lane);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (c0 + u >= ns) continue;
                if (c0 + u == 0) {
                    M[r] = lc[u][r];
                    W[r] = 1.f;
#pragma unroll
                    for (int v = 0; v < V; ++v) a[r][v] = x[u][r][v];
                } else {
                    const FoldCoef f = fold_coef(M[r], lc[u][r]);
                    W[r] = fold_weight(W[r], f);
                    M[r] = f.Mn;
#pragma unroll
                    for (int v = 0; v < V; ++v) a[r][v] = fold_elem(a[r][v], x[u][r][v], f);
                }
            }
        }
    }
    if (ns > 1) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float s = __builtin_amdgcn_rcpf(W[r]);
            M[r] = M[r] + fast_log2(W[r]);
#pragma unroll
            for (int v = 0; v < V; ++v) a[r][v] *= s;
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (whole_row) {
            __half *dst = p.out + (out_row + r) * D + lane;
#pragma unroll
            for (int v = 0; v < V; ++v) dst[v * 64] = __float2half_rn(a[r][v]);
        } else {
#pragma unroll
            for (int v = 0; v < V; ++v)
                coherent_store(p.o_partial + (slot0 * R + r) * D + v * 64 + lane, a[r][v]);
            if (lane == 0) coherent_store(p.lse_partial + slot0 * R + r, M[r] * kLn2);
        }
    }
}

// Partial results (of segments, or in kModeSpread of chunks) that a writer wave has stored in
// one pass over its mailboxes and that still have to be counted in.  Ordering across waves and
// XCDs without cache-wide write-backs or invalidations (which were measured to cost several
// times the merge launch they replace): the partial results are written with device-coherent
// stores; the wave waits once until all its stores have completed, then bumps the counters of
// the rows concerned with device-scope atomics, one lane per result; the wave whose atomic
// completes a row reads the partial results with device-coherent loads issued after that
// atomic has returned, combines them into `out` and rearms the counter.  Waiting once per pass
// instead of once per result matters: a store takes a few microseconds to complete, about as
// long as the streaming waves of a workgroup need to produce the next results.
template <int NW>
struct Arrivals {
    int dest[NW], parts[NW], out_row[NW], len[NW];     // lives in LDS, used by the writer wave only
};

// Counters (AttnParams::arrivals), n_rows = (enumeration rows) x (selected heads) of the launch:
// entry row counts the stored segment results of that row; in kModeSpread entry
// n_rows + row * (segments per row the buffers provide for) + j counts the stored chunk results
// of segment j of that row.  There the wave that completes a segment folds its chunks, which
// spreads the folding of a long row over as many waves as it has segments, stores the segment
// result and counts it in for the row in turn.
template <int D, int R, int NW>
__device__ __forceinline__ void count_in_and_combine(const AttnParams &p, const Arrivals<NW> &arr,
                                                     int n_arr, bool spread, int n_rows, int lane)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);                   // every store of this wave has completed
    const int seg_slots = p.max_segs / p.part_stride;   // segments per row (kModeSpread)
    unsigned old = 0;
    if (lane < n_arr) {
        const int d = arr.dest[lane];
        const int64_t row = d / p.max_segs;          // (enumeration row, head)
        const int64_t counter = spread ? n_rows + row * seg_slots + (d % p.max_segs) / p.part_stride : row;
        old = __hip_atomic_fetch_add(p.arrivals + counter, 1u, __ATOMIC_RELAXED,
                                     __HIP_MEMORY_SCOPE_AGENT);
    }
    for (int i = 0; i < n_arr; ++i) {
        const int before = __builtin_amdgcn_readlane((int)old, i);
        const int d = __builtin_amdgcn_readfirstlane(arr.dest[i]);
        const int64_t row = d / p.max_segs;
        const int64_t out_row = __builtin_amdgcn_readfirstlane(arr.out_row[i]);
        int n_segs = __builtin_amdgcn_readfirstlane(arr.parts[i]);
        if (spread) {
            const int L = __builtin_amdgcn_readfirstlane(arr.len[i]);
            const int j = (d % p.max_segs) / p.part_stride;
            const int n_tok = min(p.seg_tokens, L - j * p.seg_tokens);
            const int ct = chunk_tokens_of(n_tok, p.chunk_tokens, p.seg_tokens);
            const int ns = (n_tok + ct - 1) / ct;
            if (before + 1 != ns) continue;
            n_segs = (L + p.seg_tokens - 1) / p.seg_tokens;
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            fold_segment_from_chunks<D, R>(p, row * p.max_segs + (int64_t)j * p.part_stride, ns,
                                           n_segs == 1, out_row, lane);
            unsigned seen = 0;
            if (n_segs > 1) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                __builtin_amdgcn_s_waitcnt(0);       // the segment result is stored
            }
            if (lane == 0) {
                __hip_atomic_store(p.arrivals + n_rows + row * seg_slots + j, 0u, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
                if (n_segs > 1)
                    seen = __hip_atomic_fetch_add(p.arrivals + row, 1u, __ATOMIC_RELAXED,
                                                  __HIP_MEMORY_SCOPE_AGENT);
            }
            if (n_segs == 1 || (int)__builtin_amdgcn_readfirstlane(seen) + 1 != n_segs) continue;
        } else if (before + 1 != n_segs) {
            continue;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        merge_partials<D, R>(p, row * p.max_segs, n_segs, spread ? p.part_stride : 1, out_row, lane);
        if (lane == 0)
            __hip_atomic_store(p.arrivals + row, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

struct ItemHdr {
    int b, g, seq;  // enumeration row (sequence, or pair), KV head, sequence of q / out rows
    int nblk;       // blocks of this chunk
    int rem;        // tokens in the ragged last block (0: none)
    int t0;         // first token of the chunk
    int kind, dest, cs;
    int nseg, out_row, len;
};

__host__ __device__ constexpr size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

// Table bytes: lens, firstF (int), order (uint16), then the selected heads, or in pairs mode
// the head and the sequence of every pair.
__host__ __device__ constexpr size_t persist_table_bytes(int rows, int n_sel, bool pairs)
{
    return align16((size_t)(2 * rows + 2) * sizeof(int)) +
           align16((size_t)rows * sizeof(unsigned short)) +
           align16((size_t)(pairs ? 2 * rows : n_sel) * sizeof(int));
}
// Rows of one launch, at most: bounds the static LDS of the enumeration (groups of 64 rows).
constexpr int kMaxRows = 2048;
constexpr int kMaxRowGroups = kMaxRows / 64;

template <class Policy, int NW>
__host__ __device__ constexpr size_t persist_lds_bytes(int rows, int n_sel, bool pairs)
{
    return persist_table_bytes(rows, n_sel, pairs) +
           2 * NW * sizeof(Mailbox<Policy::D, Policy::R>) +
           fold_slots<Policy::R>() * sizeof(FoldSlot<Policy::D, Policy::R>) +
           (size_t)NW * Policy::kWaveLdsBytes;
}

__device__ __forceinline__ int mail_load(const int *flag)
{
    return __hip_atomic_load(flag, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void mail_store(int *flag, int v)
{
    __hip_atomic_store(flag, v, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
}
// Orders the LDS accesses of one wave around a point where lanes read what other lanes of
// the same wave wrote (the hardware keeps a wave's LDS operations in order; this keeps the
// compiler from moving them).
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// The new token's K row and V row of (sequence, KV head g) -> slot pos % 16 of the tile
// (block, g); lanes [0, D/8) move the K row, the next D/8 lanes the V row, 16 bytes each.
template <int D>
__device__ __forceinline__ void store_new_rows(const AttnParams &p, int seq, int g, int64_t tile_off,
                                               int slot, int n_kv_heads, int lane)
{
    constexpr int LR = D / 8;
    if (lane < 2 * LR) {
        const bool is_v = lane >= LR;
        const int c = lane % LR;
        const __half *src = (is_v ? p.v_new : p.k_new) + ((int64_t)seq * n_kv_heads + g) * D + c * 8;
        __half *dst = const_cast<__half *>(is_v ? p.v_cache : p.k_cache) + tile_off + slot * D + c * 8;
        *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(src);
    }
}

// VARIANT selects what is compiled in besides the common path; code that a launch cannot reach
// still costs it (launches measured 0.5 to 1.5 % faster without each of the two parts):
//   kVariantPlain  many rows, none of which can leave partial results
//   kVariantFew    also the fixed second and third segments of launches with few segments a
//                  workgroup
//   kVariantMerge  also partial results that are combined inside the launch
//                  (AttnParams::arrivals is set), and single-chunk scheduling
enum : int { kVariantPlain = 0, kVariantFew = 1, kVariantMerge = 2 };
template <class Policy, int NW, bool PAIRS, int VARIANT>
__global__ __launch_bounds__((NW + 1) * 64)
    __attribute__((amdgpu_waves_per_eu(Policy::kWavesPerEu))) void attn_chunk_persistent_kernel(
        const AttnParams p, const int batch)
{
    constexpr int D = Policy::D;
    constexpr int R = Policy::R;
    constexpr bool MERGE = VARIANT == kVariantMerge;
    constexpr bool FEW = VARIANT >= kVariantFew;
    constexpr int NT = (NW + 1) * 64;
    constexpr int kTileBytes = kBlockTokens * D * 2;
    constexpr int NS = fold_slots<R>();
    using Mail = Mailbox<D, R>;
    using Fold = FoldSlot<D, R>;
    using Tile = typename Policy::Tile;
    extern __shared__ __align__(16) unsigned char smem[];
    int *lens = reinterpret_cast<int *>(smem);
    int *firstF = lens + batch;               // whole segments before row b; one spare word after
    // rows that end in a shorter segment (or, empty, in the segment that writes zeros), sorted
    // by the size class of that segment, largest first
    unsigned short *order =
        reinterpret_cast<unsigned short *>(smem + align16((size_t)(2 * batch + 2) * sizeof(int)));
    // KV head of position si in head_ids / of pair b; pairs mode: then the sequence of pair b
    int *hids = reinterpret_cast<int *>(reinterpret_cast<unsigned char *>(order) +
                                        align16((size_t)batch * sizeof(unsigned short)));
    int *pseq = hids + batch;
    const int n_sel = PAIRS ? 1 : p.n_sel;    // heads per enumeration row
    const int n_ids = PAIRS ? batch : p.n_sel;
    unsigned char *after_tables = smem + persist_table_bytes(batch, p.n_sel, PAIRS);
    __shared__ ChunkPool pool;
    __shared__ Arrivals<NW> arrivals;       // writer wave only
    Mail *mail = reinterpret_cast<Mail *>(after_tables);             // [NW][2]
    Fold *fold = reinterpret_cast<Fold *>(after_tables + 2 * NW * sizeof(Mail));
    unsigned char *staging = reinterpret_cast<unsigned char *>(fold + NS);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int seg_tokens = p.seg_tokens;
    const int chunk_tokens = p.chunk_tokens;
    // kModeSpread is an offer: it is taken up only when some row is long enough to gain from
    // being worked on by several workgroups (decided below, once the lengths are known)
    bool spread = MERGE && p.mode == kModeSpread;
    const bool merging = MERGE && p.arrivals != nullptr;
    // kModeSpread: chunks of a row of L tokens (a row without tokens has one, which writes zeros)
    auto row_chunks = [&](int L) {
        if (L <= 0) return 1;
        const int nF = udiv(L, seg_tokens), rt = L - nF * seg_tokens;
        const int ct = chunk_tokens_of(rt, chunk_tokens, seg_tokens);
        return nF * p.part_stride + udiv(rt + ct - 1, ct);
    };

    // ---- work enumeration.  Rows are handled in groups of 64 consecutive rows, one row a lane:
    // group u * (NW + 1) + wave belongs to round u of that wave, so a thread holds up to UR rows
    // in registers and one round covers a whole launch.
    //  1. All threads fetch the lengths of their rows (in pairs mode first the pair's sequence
    //     and head; the loads of all rounds are in flight together) and work out, per row, the
    //     number of whole segments and the size class of the last, shorter one.  Inside each
    //     group a shuffle scan gives the running count of whole segments, and five ballots
    //     (one per bit of the class number) give every row the set of rows of its class, hence
    //     its rank among them and the class's count.
    //  2. The per-(class, group) counts, laid out class-major, and the per-group segment
    //     totals go through exclusive scans over the workgroup (three elements a thread, a
    //     shuffle scan per wave, wave totals through LDS).
    //  3. Every thread writes its rows' table entries: firstF[row] = whole segments before
    //     the row; order[position] = row, position = rows of larger classes + rows of the
    //     same class in lower groups + rank.
    // size class of a last segment of `rt` tokens (0 < rt <= seg_tokens): 0 = the largest
    auto size_class = [&](int rt) {
        const int j = udiv(16 * rt - 1, seg_tokens);    // rt in (j/16, (j+1)/16] of a segment
        if (j >= 1) return kLinClasses - j;
        return kLinClasses + (rt <= (seg_tokens >> 5) ? 1 : 0) + (rt <= (seg_tokens >> 6) ? 1 : 0) +
               (rt <= (seg_tokens >> 7) ? 1 : 0);
    };
    constexpr int UR = (kMaxRows + NT - 1) / NT;        // rounds
    constexpr int kScanElems = kClasses * kMaxRowGroups + kMaxRowGroups;
    constexpr int E = (kScanElems + NT - 1) / NT;       // scan elements per thread
    __shared__ int scan[E * NT];                        // [class][group] counts, then [group] totals
    __shared__ int wave_tot[2 * (NW + 1)];
    const int n_groups = (batch + 63) / 64;
    {
        // The lengths go to LDS at once and the later steps run as loops that are not unrolled:
        // the prologue must not need more registers than the streaming loop, or the register
        // allocation of that loop suffers (measured: 12 % of the kernel's time).
        // Every load is issued unconditionally (indices clamped) and before the first use of any
        // of them, so that all of them are in flight together: a conditional load ends up
        // behind a branch and a full wait, and the prologue then pays one memory latency per
        // round instead of one in all (two in pairs mode).
        int row[UR], L[UR], head[UR];
#pragma unroll
        for (int u = 0; u < UR; ++u) {
            const int i = min(tid + u * NT, batch - 1);
            row[u] = PAIRS ? p.pair_seq[i] : i;
            head[u] = PAIRS ? p.pair_head[i] : 0;
        }
#pragma unroll
        for (int u = 0; u < UR; ++u) L[u] = p.seq_lens[row[u]];
        constexpr int UH = 4;                           // n_sel <= 1024 < UH * NT
        int sel[UH];
#pragma unroll
        for (int u = 0; u < UH; ++u) sel[u] = PAIRS ? 0 : p.head_ids[min(tid + u * NT, n_ids - 1)];
#pragma unroll
        for (int u = 0; u < UH; ++u)
            if (!PAIRS && tid + u * NT < n_ids) hids[tid + u * NT] = sel[u];
#pragma unroll
        for (int u = 0; u < UR; ++u) {
            const int i = tid + u * NT;
            if (i >= batch) continue;
            lens[i] = L[u];
            if (PAIRS) {
                hids[i] = head[u];
                pseq[i] = row[u];
            }
        }
        if (spread) {
            // Single chunks pay a round trip through global memory per chunk result.  They are
            // worth it only when whole segments would leave workgroups without work although
            // there is work to share: when there are fewer segments than workgroups and some
            // row is longer than a workgroup's own waves finish in one turn.  Otherwise:
            // whole segments, folded in LDS, after all.
            int longest = 0, n_segments = 0;
#pragma unroll
            for (int u = 0; u < UR; ++u) {
                longest = max(longest, L[u]);
                if (tid + u * NT < batch) n_segments += max(1, udiv(max(L[u], 0) + seg_tokens - 1, seg_tokens));
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                longest = max(longest, __shfl_xor(longest, off, 64));
                n_segments += __shfl_xor(n_segments, off, 64);
            }
            if (lane == 0) {
                wave_tot[wave] = longest;
                wave_tot[NW + 1 + wave] = n_segments;
            }
            __syncthreads();
            n_segments = 0;
#pragma unroll
            for (int w = 0; w < NW + 1; ++w) {
                longest = max(longest, wave_tot[w]);
                n_segments += wave_tot[NW + 1 + w];
            }
            // (readfirstlane: the compiler must see that the decision is the same in all lanes, or
            // every branch on it, the streaming loop's included, is compiled as a divergent one;
            // wave_tot is written again only after the next barrier)
            spread = __builtin_amdgcn_readfirstlane((int)(longest > NW * chunk_tokens &&
                                                          (long long)n_segments * n_sel < (long long)gridDim.x)) != 0;
        }
    }
    // Per row, kept in the row's firstF entry until step 3:
    // (whole segments of the group's lower rows) << 11 | (rank in its class) << 5 | (class + 1)
#pragma unroll 1
    for (int u = 0; u < UR; ++u) {
        const int i = tid + u * NT;
        const int g = u * (NW + 1) + wave;              // the row's group
        if (g >= n_groups) break;                       // same in all lanes: no rows from here on
        int nF = 0, cls = -1;
        if (i < batch) {
            const int L = lens[i];                      // this thread's own write
            nF = L > 0 ? udiv(L, seg_tokens) : 0;
            const int rt = L > 0 ? L - nF * seg_tokens : 0;
            if (spread) {
                // chunks are counted instead of whole segments, and no row is listed
                nF = row_chunks(L);
            } else {
                if (rt > 0) cls = size_class(rt);
                if (L <= 0 && p.direct_single) cls = kClasses - 1;   // the segment that writes the zeros
            }
        }
        int incl = nF, rank = 0;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off, 64);
            if (lane >= off) incl += up;
        }
        // lanes of the same class, from one ballot per bit of the class number
        unsigned long long same = ~0ull;
#pragma unroll
        for (int bit = 0; bit < 5; ++bit) {
            const bool one = ((cls + 1) >> bit) & 1;
            const unsigned long long b = __builtin_amdgcn_ballot_w64(one);
            same &= one ? b : ~b;
        }
        rank = __builtin_amdgcn_mbcnt_hi((unsigned)(same >> 32),
                                         __builtin_amdgcn_mbcnt_lo((unsigned)same, 0));
        const int count = __builtin_popcountll(same);
        if (i < batch) firstF[i] = ((incl - nF) << 11) | (rank << 5) | (cls + 1);
        // class counts of the group: zero, then the last row of every class present writes its own
        if (lane < kClasses) scan[lane * n_groups + g] = 0;
        wave_lds_fence();
        if (cls >= 0 && rank == count - 1) scan[cls * n_groups + g] = count;
        if (lane == 63) scan[kClasses * n_groups + g] = incl;
    }
    if (tid < 2 * NW) mail[tid].flag = kMailEmpty;
    if (tid == 0) {
        pool.next = 0;
        pool.end = 0;
    }
    __syncthreads();
    {
        // exclusive scans of scan[0, n_cls) (class counts) and scan[n_cls, n_all) (segment totals)
        const int n_cls = kClasses * n_groups, n_all = n_cls + n_groups;
        int v[E], sumC = 0, sumF = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int idx = tid * E + e;
            v[e] = idx < n_all ? scan[idx] : 0;
            if (idx < n_cls)
                sumC += v[e];
            else
                sumF += v[e];
        }
        int inclC = sumC, inclF = sumF;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int upC = __shfl_up(inclC, off, 64), upF = __shfl_up(inclF, off, 64);
            if (lane >= off) {
                inclC += upC;
                inclF += upF;
            }
        }
        if (lane == 63) {
            wave_tot[wave] = inclC;
            wave_tot[NW + 1 + wave] = inclF;
        }
        __syncthreads();
        int baseC = inclC - sumC, baseF = inclF - sumF, allC = 0, allF = 0;
#pragma unroll
        for (int w = 0; w < NW + 1; ++w) {
            const int tc = wave_tot[w], tf = wave_tot[NW + 1 + w];
            if (w < wave) {
                baseC += tc;
                baseF += tf;
            }
            allC += tc;
            allF += tf;
        }
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int idx = tid * E + e;
            if (idx < n_cls) {
                scan[idx] = baseC;
                baseC += v[e];
            } else if (idx < n_all) {
                scan[idx] = baseF;
                baseF += v[e];
            }
        }
        if (tid == 0) {
            firstF[batch] = allF;               // whole segments of all rows
            lens[2 * batch + 1] = allC;         // number of listed rows, kept in the table's spare word
        }
    }
    __syncthreads();
#pragma unroll 1
    for (int u = 0; u < UR; ++u) {
        const int i = tid + u * NT;
        const int g = u * (NW + 1) + wave;
        if (i >= batch) break;
        const int info = firstF[i];
        const int cls = (info & 31) - 1, rank = (info >> 5) & 63;
        firstF[i] = scan[kClasses * n_groups + g] + (int)((unsigned)info >> 11);
        if (cls >= 0) order[scan[cls * n_groups + g] + rank] = (unsigned short)i;
    }
    __syncthreads();
    const int totalF = firstF[batch];                         // whole segments of all rows
    const int total = (totalF + lens[2 * batch + 1]) * n_sel; // segments of this launch

    // segment number -> (row, segment, head): whole segments come first (binary search in the
    // running counts), last segments after them by size class (sorted list).  Works per lane.
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
    struct Segment {
        int b, g, seq;      // enumeration row, KV head, sequence
        int t0, n_tok;      // first token, tokens
        int ct, ns;         // tokens per chunk, chunks
        int kind, dest;     // where the whole segment goes
        int nseg, out_row;  // segments of the row (kModeSpread: its chunks); first of its R rows in `out`
        int tail;           // 1: the segment ends with the row's last token
        int len;            // tokens of the row
    };
    auto chunk_for = [&](int n_tok) { return chunk_tokens_of(n_tok, chunk_tokens, seg_tokens); };
    // kModeSpread: item number -> (row, chunk, head); the item is returned as a segment of one chunk
    auto decode_spread = [&](int itemno) {
        Segment s;
        const int w = min(itemno, max(total - 1, 0));
        const int cg = PAIRS ? w : w / n_sel;
        const int si = PAIRS ? 0 : w - cg * n_sel;
        s.b = upper(firstF, cg);
        const int k = cg - firstF[s.b];                 // chunk of the row
        const int L = lens[s.b];
        const int gc = p.part_stride;
        const int nF = L > 0 ? udiv(L, seg_tokens) : 0;
        int j, c;
        if (k < nF * gc) {
            j = udiv(k, gc);
            c = k - j * gc;
            s.ct = chunk_tokens;
            s.n_tok = chunk_tokens;
        } else {
            j = nF;
            c = k - nF * gc;
            const int rt = max(L, 0) - nF * seg_tokens;
            s.ct = chunk_for(rt);
            s.n_tok = max(0, min(s.ct, rt - c * s.ct));
        }
        s.t0 = j * seg_tokens + c * s.ct;
        s.ns = 1;
        s.g = hids[PAIRS ? s.b : si];
        s.seq = PAIRS ? pseq[s.b] : s.b;
        s.nseg = row_chunks(L);
        s.out_row = s.seq * p.n_q_heads + s.g * R;
        s.tail = L > 0 && s.t0 + s.n_tok == L;
        s.len = L;
        if (L <= 0) {
            s.kind = kKindZero;
            s.dest = s.out_row;
        } else if (s.nseg == 1) {
            s.kind = kKindOut;
            s.dest = s.out_row;
        } else {
            s.kind = kKindPartial;
            s.dest = (s.b * n_sel + si) * p.max_segs + j * gc + c;
        }
        return s;
    };
    auto decode = [&](int segno) {
        if (spread) return decode_spread(segno);
        Segment s;
        const int w = min(segno, max(total - 1, 0));
        const int cg = PAIRS ? w : w / n_sel;
        const int si = PAIRS ? 0 : w - cg * n_sel;
        int L, j;
        if (cg < totalF) {
            s.b = upper(firstF, cg);
            j = cg - firstF[s.b];
            L = lens[s.b];
            s.n_tok = seg_tokens;
        } else {
            s.b = order[cg - totalF];
            L = lens[s.b];
            j = L > 0 ? udiv(L, seg_tokens) : 0;
            s.n_tok = L > 0 ? L - j * seg_tokens : 0;
        }
        s.t0 = j * seg_tokens;
        s.ct = chunk_for(s.n_tok);
        s.ns = max(1, udiv(s.n_tok + s.ct - 1, s.ct));
        s.g = hids[PAIRS ? s.b : si];
        s.seq = PAIRS ? pseq[s.b] : s.b;
        const int n_segs = udiv(max(L, 0) + seg_tokens - 1, seg_tokens);
        s.nseg = n_segs;
        s.out_row = s.seq * p.n_q_heads + s.g * R;
        s.tail = L > 0 && s.t0 + s.n_tok == L;
        s.len = L;
        if (L <= 0) {
            s.kind = kKindZero;
            s.dest = s.out_row;
        } else if (p.direct_single && n_segs <= 1) {
            s.kind = kKindOut;
            s.dest = s.out_row;
        } else {
            s.kind = kKindPartial;
            s.dest = (s.b * n_sel + si) * p.max_segs + j;
        }
        return s;
    };
    // chunk i of a segment; `slot`: the segment's fold slot (segments of several chunks)
    auto chunk_of = [&](const Segment &s, int i, int slot) {
        ChunkDesc d;
        d.b = s.b;
        d.g = s.g;
        d.seq = s.seq;
        d.t0 = s.t0 + i * s.ct;
        d.n_tok = max(0, min(s.ct, s.n_tok - i * s.ct));
        d.flags = kItemExists;
        d.kind = s.ns > 1 ? (int)kKindFold : s.kind;
        d.dest = s.ns > 1 ? slot : s.dest;
        d.cs = i;
        d.nseg = s.nseg;
        d.out_row = s.out_row;
        d.len = s.len;
        return d;
    };
    // Work a workgroup has without a ticket.  When segments have several chunks: segment number
    // blockIdx.x, whose first NW chunks the streaming waves take directly (wave v takes chunk
    // v) and which owns fold slot 0.  When every segment is a single chunk: segments
    // (blockIdx.x + k gridDim.x) * NW + v, k = 0, 1, two per streaming wave v (the waves of a
    // workgroup work on neighbouring heads of one chunk position).  Tickets number the segments
    // after these.
    const bool single_mode = p.mode == kModeSplit || spread;
    const bool have_first = (int)blockIdx.x < total;
    const bool step_mode = p.k_new != nullptr;      // never together with single_mode
    // chunks of the first segment that are taken without the pool: the first NW, but not the
    // one that holds the row's last position when the new token is stored in this launch
    auto direct_chunks = [&](const Segment &s0) {
        int n = min(NW, s0.ns);
        if (step_mode && s0.tail && n == s0.ns) --n;
        return n;
    };
    // store of the new token's rows of the segment's (sequence, head), done before the chunk
    // that reads them becomes visible to the streaming waves
    auto store_tail = [&](const Segment &sg) {
        const int L = sg.t0 + sg.n_tok;             // tail segment: the row's length
        const int pos = L - 1;
        const int blk = p.block_table[(int64_t)sg.b * p.max_blocks_per_seq + pos / kBlockTokens];
        const int64_t off = (int64_t)blk * p.stride_block + (PAIRS ? 0 : (int64_t)sg.g * p.stride_head);
        store_new_rows<D>(p, sg.seq, sg.g, off, pos % kBlockTokens, p.n_q_heads / R, lane);
    };
    if (wave == NW) {
        // ------------------------------------------------------------ writer wave
        // Segments a workgroup has without a ticket: its first, and, in some launches of at most
        // HETIS_STATIC_SECOND_UPTO segments a workgroup, a second and a third.  The second comes
        // from the other end of the next gridDim.x segments of the sorted list, so that the two
        // together hold about the same number of tokens in every workgroup; the third goes by
        // the rank of that sum (the largest sum takes the shortest of the following gridDim.x
        // segments).  With so few segments the draws of all workgroups come in bursts (every
        // pool runs low at the same moment) and pair long segments with long ones as often as
        // not; with many segments a workgroup the tickets even the load out by themselves, and
        // fixing more of it only takes room from them.  Three conditions besides the number of
        // segments.  The longest segment must be well below the tokens a workgroup gets on
        // average: where a few long rows stand out (their workgroups are what the launch waits
        // for), they must not be given more, and the tickets see to that.  The segments must
        // differ in length, or there is nothing to balance.  And beyond two segments a
        // workgroup the longest segment must have at least as many chunks as a workgroup has
        // streaming waves: shorter rows need no balancing, and the waves would wait for the
        // writer wave's sums and for the first draw behind them.
        // The segments that need no ticket wait in a queue of three numbers (q0 next; -1: none),
        // worked out here, before the loop, so that the loop itself carries no state for them.
        const int Gn = (int)gridDim.x;
        int n_fixed = Gn * (single_mode ? 2 * NW : 1);
        int q0 = have_first && !single_mode ? (int)blockIdx.x : -1, q1 = -1, q2 = -1;
        if (FEW && HETIS_STATIC_SECOND_UPTO > 0 && !single_mode && total > Gn &&
            (long long)total <= (long long)HETIS_STATIC_SECOND_UPTO * Gn) {
            // tokens of segment number `segno` (whole-segment scheduling): what decode() would
            // put into n_tok, without the rest of it
            auto seg_n_tok = [&](int segno) {
                const int w = min(segno, max(total - 1, 0));
                const int cg = PAIRS ? w : w / n_sel;
                if (cg < totalF) return seg_tokens;
                const int L = lens[order[cg - totalF]];
                return L > 0 ? L - udiv(L, seg_tokens) * seg_tokens : 0;
            };
            const int tok0 = seg_n_tok(0);
            const bool long_rows = udiv(tok0 + chunk_for(tok0) - 1, chunk_for(tok0)) >= NW;
            // tokens of the launch from the class counts (a class's rows taken at the middle of
            // its range; one class a lane, then a sum over the wave): the same sum of integers in
            // every workgroup
            const int listed = lens[2 * batch + 1];
            long long part = 0;
            if (lane < kClasses) {
                const int c = lane;
                const int first_c = scan[c * n_groups];
                const int next_c = c + 1 < kClasses ? scan[(c + 1) * n_groups] : listed;
                const int j = kLinClasses - c;                // classes of a sixteenth of a segment
                const int mid = c < kLinClasses ? (2 * j + 1) * seg_tokens / 32
                                                : (3 * seg_tokens) >> (c - kLinClasses + 6);
                part = (long long)(next_c - first_c) * mid;
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
            const long long mean_load = ((long long)totalF * seg_tokens + part) * n_sel / Gn;
            const bool flat = 16ll * tok0 <= (long long)HETIS_STATIC_FLAT_X16 * mean_load;
            // ... and there must be something to balance: with segments of (nearly) one size the
            // tickets do better, they give the last segments to the workgroups that run fastest
            const int tok_last = seg_n_tok(min(total, 3 * Gn) - 1);
            const bool uneven = 4ll * tok0 > 5ll * tok_last;
            if (flat && uneven && (total <= 2 * Gn || long_rows)) {
                n_fixed = 2 * Gn;
                const int second_no = 2 * Gn - 1 - (int)blockIdx.x;
                if (second_no < total) q1 = second_no;
                if (total > 2 * Gn) {
                    // The third: the workgroup whose first two hold the most tokens takes the
                    // shortest of the next Gn segments, and so on (rank among the sums, which
                    // every workgroup can work out for itself).
                    n_fixed = 3 * Gn;
                    auto two_sum = [&](int b) {
                        const int s2 = 2 * Gn - 1 - b;
                        return seg_n_tok(b) + (s2 < total ? seg_n_tok(s2) : 0);
                    };
                    const int my = __builtin_amdgcn_readfirstlane(two_sum((int)blockIdx.x));
                    int rank = 0;
                    for (int b0 = 0; b0 < Gn; b0 += 64) {
                        const int b = b0 + lane;
                        const int sum_b = two_sum(min(b, Gn - 1));
                        const bool larger =
                            b < Gn && (sum_b > my || (sum_b == my && b < (int)blockIdx.x));
                        rank += __builtin_popcountll(__builtin_amdgcn_ballot_w64(larger));
                    }
                    const int third_no = 3 * Gn - 1 - rank;
                    if (third_no < total) q2 = third_no;
                }
            }
        }
        int next_box[NW];
#pragma unroll
        for (int v = 0; v < NW; ++v) next_box[v] = 0;
        int done_mask = 0;
        int idle = 0;
        int pool_end = 0;                 // entries published so far
        unsigned busy = 0;                // fold slots in use
        bool exhausted = total <= n_fixed;            // no segment left to draw
        // A workgroup that will draw no more tickets counts itself out at once, not when it
        // ends: the answer (was it the last one?) is needed only at the end, and by then the
        // atomic's round trip, which would otherwise be the last thing the kernel waits for,
        // is long over.  The last workgroup to count itself out rearms both counters; that is
        // safe while others still compute, since none of them draws again.
        bool counted_out = false;
        unsigned gone_before = 0;                     // lane 0: workgroups counted out before this one
        auto count_out = [&]() {
            if (lane == 0)
                gone_before = __hip_atomic_fetch_add(p.control + kCtlGone, 1u, __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT);
            counted_out = true;
        };
        bool first = have_first && !single_mode;      // the next segment to publish is the workgroup's first
        bool closed = false;              // the "no work left" entries have been published
        // Segments drawn and decoded (one per lane, lanes [pend_i, pend_n) still to publish)
        Segment mine{};
        int pend_i = 0, pend_n = 0;
        long long last_base = n_fixed;    // number of the last segment drawn here
        int last_tok = seg_tokens;        // tokens of the last segment seen
        const long long wave_round = (long long)gridDim.x * NW;
        auto bcast = [&](const Segment &s, int k) {
            Segment r;
            r.b = __builtin_amdgcn_readlane(s.b, k);
            r.g = __builtin_amdgcn_readlane(s.g, k);
            r.seq = __builtin_amdgcn_readlane(s.seq, k);
            r.t0 = __builtin_amdgcn_readlane(s.t0, k);
            r.n_tok = __builtin_amdgcn_readlane(s.n_tok, k);
            r.ct = __builtin_amdgcn_readlane(s.ct, k);
            r.ns = __builtin_amdgcn_readlane(s.ns, k);
            r.kind = __builtin_amdgcn_readlane(s.kind, k);
            r.dest = __builtin_amdgcn_readlane(s.dest, k);
            r.nseg = __builtin_amdgcn_readlane(s.nseg, k);
            r.out_row = __builtin_amdgcn_readlane(s.out_row, k);
            r.tail = __builtin_amdgcn_readlane(s.tail, k);
            r.len = __builtin_amdgcn_readlane(s.len, k);
            return r;
        };
        while (done_mask != (1 << NW) - 1 && idle < kSpinLimit) {
            bool progressed = false;
            if (exhausted && !counted_out) count_out();
            // ---- keep the chunk pool ahead of the streaming waves
            const int taken = __builtin_amdgcn_readfirstlane(
                __hip_atomic_load(&pool.next, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
            // Draw.  Work parked in one workgroup's pool cannot be taken by another that has run
            // dry, so little is drawn at a time and late; but a same-address device atomic
            // costs about as much as a short chunk, so short segments are drawn several at a
            // time.  Every chunk its own segment (split-KV): batches that shrink as the work
            // runs out.  Otherwise: about one full chunk's worth of tokens per draw, judged by
            // the last segment seen (they come longest first), drawn when fewer than
            // HETIS_POOL_AHEAD chunks (one, near the end) or than a draw's worth are waiting.
            const long long left = (long long)total - last_base;
            int n_draw, ahead;
            if (single_mode) {
                n_draw = left > 8 * wave_round ? kTicketBatch : (left > 2 * wave_round ? 2 : 1);
                ahead = n_draw;
            } else {
                n_draw = max(1, min(kTicketBatch, chunk_tokens / max(last_tok, 1)));
                ahead = max(4 * left > (long long)gridDim.x * HETIS_LATE_SEGMENTS_X4 ? HETIS_POOL_AHEAD : 1, n_draw);
            }
            int want = -1;                // segment to decode in this pass (one a lane)
            if (pend_i == pend_n && q0 >= 0) {
                // the next of the workgroup's own segments
                want = q0;
                q0 = q1;
                q1 = q2;
                q2 = -1;
                pend_i = 0;
                pend_n = 1;
                progressed = true;
            } else if (pend_i == pend_n && !exhausted && pool_end - taken < ahead) {
                unsigned t = 0;
                if (lane == 0)
                    t = __hip_atomic_fetch_add(p.control + kCtlTickets, (unsigned)n_draw,
                                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const long long base = n_fixed + __builtin_amdgcn_readfirstlane(t);
                last_base = base;
                if (base + n_draw >= total) exhausted = true;
                pend_i = 0;
                pend_n = (int)max(0ll, min((long long)n_draw, (long long)total - base));
                if (pend_n > 0) want = (int)min(base + lane, (long long)total - 1);
                progressed = true;
            }
            if (want >= 0) mine = decode(want);
            if (pend_i < pend_n) {
                // all remaining drawn segments are single chunks: publish them together
                const bool single = __builtin_amdgcn_ballot_w64(lane >= pend_i && lane < pend_n &&
                                                                mine.ns != 1) == 0;
                if (single && !first) {
                    const int cnt = pend_n - pend_i;
                    if (pool_end + cnt - taken <= kPoolSize) {
                        if (step_mode) {
                            for (int e = pend_i; e < pend_n; ++e) {
                                const Segment sg = bcast(mine, e);
                                if (sg.tail) store_tail(sg);
                            }
                            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                            __builtin_amdgcn_s_waitcnt(0);
                        }
                        if (lane >= pend_i && lane < pend_n)
                            pool.desc[(pool_end + lane - pend_i) % kPoolSize] = chunk_of(mine, 0, 0);
                        pool_end += cnt;
                        __hip_atomic_store(&pool.end, pool_end, __ATOMIC_RELEASE,
                                           __HIP_MEMORY_SCOPE_WORKGROUP);
                        last_tok = __builtin_amdgcn_readlane(mine.n_tok, pend_n - 1);
                        pend_i = pend_n;
                        progressed = true;
                    }
                } else {
                    const Segment seg = bcast(mine, pend_i);
                    if (pool_end + seg.ns - taken <= kPoolSize &&
                        (seg.ns == 1 || busy != (1u << NS) - 1)) {
                        int slot = 0;
                        if (seg.ns > 1) {
                            slot = __builtin_ctz(~busy);
                            busy |= 1u << slot;
                            if (lane == 0) {
                                fold[slot].next = 0;
                                fold[slot].ns = seg.ns;
                                fold[slot].kind = seg.kind;
                                fold[slot].dest = seg.dest;
                                fold[slot].nseg = seg.nseg;
                                fold[slot].out_row = seg.out_row;
                            }
                        }
                        if (step_mode && seg.tail) {
                            store_tail(seg);
                            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                            __builtin_amdgcn_s_waitcnt(0);
                        }
                        // some chunks of the first segment are taken without the pool
                        const int skip = first ? direct_chunks(seg) : 0;
                        if (lane >= skip && lane < seg.ns)
                            pool.desc[(pool_end + lane - skip) % kPoolSize] = chunk_of(seg, lane, slot);
                        pool_end += seg.ns - skip;
                        __hip_atomic_store(&pool.end, pool_end, __ATOMIC_RELEASE,
                                           __HIP_MEMORY_SCOPE_WORKGROUP);
                        ++pend_i;
                        first = false;
                        last_tok = seg.n_tok;
                        progressed = true;
                    }
                }
            }
            if (exhausted && pend_i == pend_n && q0 < 0 && !closed &&
                pool_end + NW - taken <= kPoolSize) {
                // one "no work left" entry per streaming wave
                if (lane < NW) {
                    ChunkDesc none{};
                    pool.desc[(pool_end + lane) % kPoolSize] = none;
                }
                pool_end += NW;
                __hip_atomic_store(&pool.end, pool_end, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                closed = true;
                progressed = true;
            }
            // ---- results
            // partial results stored in this pass that are merged inside this launch: counted in
            // after the pass, when their mailboxes have been handed back
            int n_arr = 0;
#pragma unroll
            for (int v = 0; v < NW; ++v) {
                if (done_mask & (1 << v)) continue;
                Mail &mb = mail[v * 2 + next_box[v]];
                const int f = __builtin_amdgcn_readfirstlane(mail_load(&mb.flag));
                if (f == kMailDone) {
                    done_mask |= 1 << v;
                    progressed = true;
                    continue;
                }
                if (f != kMailFull) continue;
                const int kind = __builtin_amdgcn_readfirstlane(mb.kind);
                const int dest = __builtin_amdgcn_readfirstlane(mb.dest);
                if (kind != kKindFold) {
                    if (kind == kKindPartial && merging) {
                        store_partial_coherent<D, R>(mb.o, mb.lse, nullptr, dest, p, lane, spread);
                        if (lane == 0) {
                            arrivals.dest[n_arr] = dest;
                            arrivals.parts[n_arr] = mb.nseg;
                            arrivals.out_row[n_arr] = mb.out_row;
                            arrivals.len[n_arr] = mb.len;
                        }
                        ++n_arr;
                    } else {
                        store_result<D, R>(mb.o, mb.lse, nullptr, kind, dest, p, lane);
                    }
                } else {
                    Fold &fs = fold[dest];
                    const int cs = __builtin_amdgcn_readfirstlane(mb.cs);
                    if (cs != __builtin_amdgcn_readfirstlane(fs.next)) continue;   // not its turn yet
                    const bool last = cs + 1 == __builtin_amdgcn_readfirstlane(fs.ns);
                    // fold chunk cs into the slot; a lane owns the same elements every time
#pragma unroll
                    for (int idx = lane * 4; idx < R * D; idx += 256) {
                        const int r = idx / D, d = idx % D;
                        const float4 x = *reinterpret_cast<const float4 *>(&mb.o[r][d]);
                        float4 a = x;
                        if (cs > 0) {
                            const FoldCoef f = fold_coef(fs.M[r], mb.lse[r]);
                            const float4 y = *reinterpret_cast<const float4 *>(&fs.acc[r][d]);
                            a = make_float4(fold_elem(y.x, x.x, f), fold_elem(y.y, x.y, f),
                                            fold_elem(y.z, x.z, f), fold_elem(y.w, x.w, f));
                        }
                        *reinterpret_cast<float4 *>(&fs.acc[r][d]) = a;
                    }
                    wave_lds_fence();       // every lane has read M before lane r rewrites it
                    if (lane < R) {
                        const float lc = mb.lse[lane];
                        float Mn = lc, Wn = 1.f;
                        if (cs > 0) {
                            const FoldCoef f = fold_coef(fs.M[lane], lc);
                            Mn = f.Mn;
                            Wn = fold_weight(fs.W[lane], f);
                        }
                        fs.W[lane] = Wn;
                        // after the last chunk the slot holds the segment's log-sum-exp
                        fs.M[lane] = last ? Mn + fast_log2(Wn) : Mn;
                    }
                    if (lane == 0) fs.next = cs + 1;
                    wave_lds_fence();
                    if (last) {
                        const int fkind = __builtin_amdgcn_readfirstlane(fs.kind);
                        const int fdest = __builtin_amdgcn_readfirstlane(fs.dest);
                        if (fkind == kKindPartial && merging) {
                            store_partial_coherent<D, R>(fs.acc, fs.M, fs.W, fdest, p, lane, false);
                            if (lane == 0) {
                                arrivals.dest[n_arr] = fdest;
                                arrivals.parts[n_arr] = fs.nseg;
                                arrivals.out_row[n_arr] = fs.out_row;
                                arrivals.len[n_arr] = 0;
                            }
                            ++n_arr;
                        } else {
                            store_result<D, R>(fs.acc, fs.M, fs.W, fkind, fdest, p, lane);
                        }
                        busy &= ~(1u << dest);
                    }
                }
                mail_store(&mb.flag, kMailEmpty);
                next_box[v] ^= 1;
                progressed = true;
            }
            if (MERGE && n_arr > 0) {
                wave_lds_fence();           // lane 0's entries are read by all lanes
                count_in_and_combine<D, R, NW>(p, arrivals, n_arr, spread, batch * n_sel, lane);
            }
            if (progressed) {
                idle = 0;
            } else {
                ++idle;
                __builtin_amdgcn_s_sleep(4);
            }
        }
        if (!counted_out) count_out();        // (only after a wait that gave up)
        if (lane == 0) {
            if (done_mask != (1 << NW) - 1) report_error(p.control, kErrWriterWait);
            if (gone_before == gridDim.x - 1) {
                p.control[kCtlLastMode] =
                    1u + (unsigned)(spread ? kModeSpread : (p.mode == kModeSplit ? kModeSplit : kModeSegments));
                __hip_atomic_store(p.control + kCtlTickets, 0u, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(p.control + kCtlGone, 0u, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        return;
    }

    // ---------------------------------------------------------------- streaming waves
    // (no padding bytes anywhere: a struct with holes is copied through scratch memory, and a
    // scratch store in a streaming wave is a global store like any other)
    struct Slot {
        int64_t head_off;
        ItemHdr h;
        int ids;            // lane i: physical block of the chunk's i-th tile
        int exists;
    };
    static_assert(sizeof(ItemHdr) == 12 * sizeof(int) && sizeof(Slot) == 8 + sizeof(ItemHdr) + 8,
                  "Slot has no padding");
    // chunk descriptor -> the wave's (uniform) bookkeeping, and the load of its block ids
    auto fill = [&](const ChunkDesc &d, Slot &s) {
        const int flags = __builtin_amdgcn_readfirstlane(d.flags);
        const int n_tok = __builtin_amdgcn_readfirstlane(d.n_tok);
        s.h.b = __builtin_amdgcn_readfirstlane(d.b);
        s.h.g = __builtin_amdgcn_readfirstlane(d.g);
        s.h.seq = __builtin_amdgcn_readfirstlane(d.seq);
        s.h.t0 = __builtin_amdgcn_readfirstlane(d.t0);
        s.h.kind = __builtin_amdgcn_readfirstlane(d.kind);
        s.h.dest = __builtin_amdgcn_readfirstlane(d.dest);
        s.h.cs = __builtin_amdgcn_readfirstlane(d.cs);
        s.h.nseg = __builtin_amdgcn_readfirstlane(d.nseg);
        s.h.out_row = __builtin_amdgcn_readfirstlane(d.out_row);
        s.h.len = __builtin_amdgcn_readfirstlane(d.len);
        s.exists = (flags & kItemExists) != 0 ? 1 : 0;
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
    // next chunk from the workgroup's pool (flags 0 = none left)
    auto take_chunk = [&]() {
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
        ChunkDesc none{};
        return none;
    };

    unsigned char *my_staging = staging + (size_t)wave * Policy::kWaveLdsBytes;
    Mail *my_mail = mail + wave * 2;

    constexpr int RING = Policy::kRing;             // tile pairs a wave keeps in flight, at most
    Slot cur, nxt;
    typename Policy::Query q;
    typename Policy::QueryPrefetch q_pre;
    Tile ring[RING];
    {
        // first chunk: of the work the workgroup has without a ticket, else from the pool
        ChunkDesc d{};
        bool direct = false;
        if (single_mode) {
            const long long mine = (long long)blockIdx.x * NW + wave;
            if (mine < total) {
                d = chunk_of(decode((int)mine), 0, 0);
                direct = true;
            }
        } else if (have_first) {
            const Segment s0 = decode(blockIdx.x);
            if (wave < direct_chunks(s0)) {
                d = chunk_of(s0, wave, 0);
                direct = true;
            }
        }
        if (!direct) d = take_chunk();
        fill(d, cur);
    }
    if (!cur.exists) {
        mail_store(&my_mail[0].flag, kMailDone);
        return;
    }
    nxt = cur;
    Policy::q_prefetch(q_pre, q_rows(cur), lane);
#pragma unroll
    for (int s = 0; s < RING; ++s) issue(ring[s], cur.ids, s, cur.head_off, s < cur.h.nblk);
    int n = 0;
    for (;; ++n) {
        Policy::q_commit(q, q_pre, my_staging, lane);   // this chunk's query operand

        typename Policy::State st;
        Policy::reset(st);
        const int n_my = cur.h.nblk;
        const int lim = RING * max(1, (n_my + RING - 1) / RING);   // tiles, as whole ring turns
        // The scheduling fences keep "consume a slot, refill it at once" in program order;
        // without them the compiler batches the tiles' arithmetic ahead of the refills and
        // the wave ends up waiting with nothing in flight.
        auto steady_turn = [&](int i) {                 // whole tiles; refills stay in this chunk
#pragma unroll
            for (int s = 0; s < RING; ++s) {
                Policy::template update<false>(st, ring[s], q, p.scale_log2, lane, kBlockTokens,
                                               my_staging);
                __builtin_amdgcn_sched_barrier(0);
                issue(ring[s], cur.ids, i + RING + s, cur.head_off, i + RING + s < n_my);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // The next chunk is taken as late as its block ids allow (three ring turns before
        // the end of this one), so that little undone work is held back when the work runs
        // out.
        int i = 0;
        for (; i + 4 * RING < lim; i += RING) steady_turn(i);
        if (single_mode && n == 0) {
            // the wave's second segment is its own as well
            const long long mine = (long long)(gridDim.x + blockIdx.x) * NW + wave;
            if (mine < total) {
                fill(chunk_of(decode((int)mine), 0, 0), nxt);
            } else {
                ChunkDesc none{};
                fill(none, nxt);
            }
        } else {
            fill(take_chunk(), nxt);
        }
        Policy::q_prefetch(q_pre, q_rows(nxt), lane);   // next chunk's query rows
        for (; i + RING < lim; i += RING) steady_turn(i);
        // last turn of this chunk (the only place a ragged block can be): its refills are the
        // first tiles of the next chunk
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

        // hand the finished chunk to the writer
        Mail &mb = my_mail[n & 1];
        wait_empty(mb);
        if (cur.h.kind != kKindZero) Policy::finish(st, mb.o, mb.lse, lane);
        if (lane == 0) {
            mb.kind = cur.h.kind;
            mb.dest = cur.h.dest;
            mb.cs = cur.h.cs;
            mb.nseg = cur.h.nseg;
            mb.out_row = cur.h.out_row;
            mb.len = cur.h.len;
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
