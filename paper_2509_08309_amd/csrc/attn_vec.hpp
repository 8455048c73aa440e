// Vector (non-MFMA) chunk kernels: Eq. (2b) restricted to the tokens of one chunk of one
// (sequence, selected KV head).  The path is HBM-bound (r flop per KV byte), so the layout
// is chosen for the loads, not for the ALUs:
//   - a (block, head) tile is 16 rows of D fp16 = 16*D*2 contiguous bytes; a wave reads
//     it with 128-bit loads, lane l taking bytes [16 l, 16 l + 16) of each 1 KB slice, so
//     D/8 neighbouring lanes hold one token row and a slice holds 64/(D/8) tokens;
//   - q.k is a v_dot2 chain per lane followed by a DPP sum over the D/8 lanes of a row;
//   - each group of D/8 lanes runs its own online softmax over the tokens it sees
//     (exp2 domain, fp32), so p never leaves registers between q.k and p.v;
//   - the lane groups of a wave, then the waves of the workgroup, are merged once per
//     chunk, in a fixed order, through shuffles and LDS.
// Nothing depends on how many heads were selected: the result for one (sequence, head)
// is a function of that sequence's length alone.
#pragma once
#include "attn_common.hpp"

namespace hetis {

template <int D, int R>
struct VecState {
    float m[R];
    float l[R];
    float o[R][8];

    __device__ __forceinline__ void reset()
    {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            m[r] = kNegBig;
            l[r] = 0.f;
#pragma unroll
            for (int x = 0; x < 8; ++x) o[r][x] = 0.f;
        }
    }
};

template <int D>
struct TileRegs {
    static constexpr int NI = 16 / (512 / D);   // 1 KB slices per tile
    uint4 k[NI];
    uint4 v[NI];
};

// Issue the 128-bit loads of one K tile and one V tile (no wait).
template <int D>
__device__ __forceinline__ void tile_issue(TileRegs<D> &t, const __half *k_cache,
                                           const __half *v_cache, int64_t base, int lane)
{
    const uint4 *kp = reinterpret_cast<const uint4 *>(k_cache + base) + lane;
    const uint4 *vp = reinterpret_cast<const uint4 *>(v_cache + base) + lane;
#pragma unroll
    for (int i = 0; i < TileRegs<D>::NI; ++i) t.k[i] = kp[i * 64];
#pragma unroll
    for (int i = 0; i < TileRegs<D>::NI; ++i) t.v[i] = vp[i * 64];
}

// Same through buffer descriptors sized to exactly one tile.  With valid == false the
// descriptor covers 0 bytes: the hardware range check makes every lane return zeros without
// touching memory, while the instruction still takes its place in the in-order load counter.
// This lets the ring issue its refills unconditionally, which is what keeps the compiler's
// wait counts exact (a load that is only issued on some paths forces full drains).
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
template <int D>
__device__ __forceinline__ void tile_issue_checked(TileRegs<D> &t, const __half *k_cache,
                                                   const __half *v_cache, int64_t base,
                                                   bool valid, int lane)
{
    constexpr int kTileBytes = kBlockTokens * D * 2;
    const int nbytes = valid ? kTileBytes : 0;
    __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<__half *>(k_cache + base), 0, nbytes, 0x00020000);
    __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<__half *>(v_cache + base), 0, nbytes, 0x00020000);
    const int voff = lane * 16;
#pragma unroll
    for (int i = 0; i < TileRegs<D>::NI; ++i) {
        const u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(rk, voff + i * 1024, 0, 0);
        t.k[i] = make_uint4(x.x, x.y, x.z, x.w);
    }
#pragma unroll
    for (int i = 0; i < TileRegs<D>::NI; ++i) {
        const u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(rv, voff + i * 1024, 0, 0);
        t.v[i] = make_uint4(x.x, x.y, x.z, x.w);
    }
}

// One tile (16 tokens) of K and V held in registers -> update of the running state.
template <int D, int R, bool MASKED>
__device__ __forceinline__ void vec_tile_update(VecState<D, R> &st, const TileRegs<D> &t,
                                                const __half2 (&qh)[R][4], float scale_log2,
                                                int gid, int n_valid)
{
    constexpr int LPR = D / 8;        // lanes per token row
    constexpr int TPI = 64 / LPR;     // tokens per 1 KB slice
    constexpr int NI = 16 / TPI;      // slices per tile
    float s[NI][R];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        Pack16 kk;
        kk.u = t.k[i];
        const bool valid = !MASKED || (i * TPI + gid < n_valid);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float acc = 0.f;
#pragma unroll
            for (int x = 0; x < 4; ++x)
                acc = __builtin_amdgcn_fdot2(kk.h2[x], qh[r][x], acc, false);
            acc = group_sum<LPR>(acc);
            s[i][r] = valid ? acc * scale_log2 : -INFINITY;
        }
    }
    float p[NI][R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float mx = st.m[r];
#pragma unroll
        for (int i = 0; i < NI; ++i) mx = fmaxf(mx, s[i][r]);
        const float alpha = fast_exp2(st.m[r] - mx);
        st.m[r] = mx;
        float ps = 0.f;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            p[i][r] = fast_exp2(s[i][r] - mx);
            ps += p[i][r];
        }
        st.l[r] = st.l[r] * alpha + ps;
#pragma unroll
        for (int x = 0; x < 8; ++x) st.o[r][x] *= alpha;
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        Pack16 vv;
        vv.u = t.v[i];
        if (MASKED && !(i * TPI + gid < n_valid)) vv.u = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const float vf = __half2float(vv.h[x]);
#pragma unroll
            for (int r = 0; r < R; ++r) st.o[r][x] = fmaf(p[i][r], vf, st.o[r][x]);
        }
    }
}

// Tile that may be the ragged last block of a sequence (n_valid < 16).
template <int D, int R>
__device__ __forceinline__ void vec_tile_update_any(VecState<D, R> &st, const TileRegs<D> &t,
                                                    const __half2 (&qh)[R][4], float scale_log2,
                                                    int gid, int n_valid)
{
    if (n_valid < kBlockTokens)
        vec_tile_update<D, R, true>(st, t, qh, scale_log2, gid, n_valid);
    else
        vec_tile_update<D, R, false>(st, t, qh, scale_log2, gid, kBlockTokens);
}

// Merge the 64/(D/8) lane groups of a wave (xor butterfly over the group index).
template <int D, int R>
__device__ __forceinline__ void vec_wave_merge(VecState<D, R> &st)
{
#pragma unroll
    for (int mask = D / 8; mask < 64; mask <<= 1) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float m2 = __shfl_xor(st.m[r], mask, 64);
            const float l2 = __shfl_xor(st.l[r], mask, 64);
            const float M = fmaxf(st.m[r], m2);
            const float a = fast_exp2(st.m[r] - M);
            const float a2 = fast_exp2(m2 - M);
            st.m[r] = M;
            st.l[r] = st.l[r] * a + l2 * a2;
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                const float o2 = __shfl_xor(st.o[r][x], mask, 64);
                st.o[r][x] = st.o[r][x] * a + o2 * a2;
            }
        }
    }
}

// LDS area through which the waves of a workgroup are merged (ascending wave order).
template <int D, int R, int NW>
struct WaveMergeLds {
    float o[NW][R][D];
    float m[NW][R];
    float l[NW][R];
};

template <int D, int R, int NW>
__device__ __forceinline__ void vec_lds_put(WaveMergeLds<D, R, NW> &sm, const VecState<D, R> &st,
                                            int wave, int gid, int sub)
{
    if (gid == 0) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int x = 0; x < 8; ++x) sm.o[wave][r][sub * 8 + x] = st.o[r][x];
            if (sub == 0) {
                sm.m[wave][r] = st.m[r];
                sm.l[wave][r] = st.l[r];
            }
        }
    }
}

// After a barrier: final result of the chunk, to `out` (fp16) or to the partial buffers.
template <int D, int R, int NW, int NTHREADS>
__device__ __forceinline__ void vec_lds_finish(const WaveMergeLds<D, R, NW> &sm,
                                               const AttnParams &p, int tid, int b, int g, int si,
                                               int c, bool to_out)
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

template <int D, int R, int NW>
__device__ __forceinline__ void vec_write_zeros(const AttnParams &p, int tid, int b, int g)
{
    for (int idx = tid; idx < R * D; idx += NW * 64) {
        const int r = idx / D, d = idx % D;
        p.out[((int64_t)b * p.n_q_heads + g * R + r) * D + d] = __float2half_rn(0.f);
    }
}

// ---------------------------------------------------------------------------------------
// Simple form: one workgroup per (chunk slot, selected head, sequence); slots past the end
// of a sequence exit at once.  Used when the batch is too large for the persistent form.
// ---------------------------------------------------------------------------------------
template <int D, int R, int NW>
__global__ __launch_bounds__(NW * 64) void attn_chunk_vec_kernel(const AttnParams p)
{
    constexpr int LPR = D / 8;
    const int c = blockIdx.x;
    const int si = blockIdx.y;
    const int b = blockIdx.z;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int gid = lane / LPR;
    const int sub = lane % LPR;

    const int L = p.seq_lens[b];
    const int g = p.head_ids[si];
    const int n_chunks = (L + p.chunk_tokens - 1) / p.chunk_tokens;
    const bool to_out = p.direct_single && n_chunks <= 1;

    if (L <= 0) {
        if (to_out && c == 0) vec_write_zeros<D, R, NW>(p, tid, b, g);
        return;
    }
    if (c >= n_chunks) return;

    const int t0 = c * p.chunk_tokens;
    const int n_tok = min(L, t0 + p.chunk_tokens) - t0;
    const int nblk = (n_tok + kBlockTokens - 1) / kBlockTokens;
    const int rem = n_tok & (kBlockTokens - 1);
    const int32_t *bt = p.block_table + (int64_t)b * p.max_blocks_per_seq + t0 / kBlockTokens;
    const int64_t head_off = (int64_t)g * p.stride_head;

    __half2 qh[R][4];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        Pack16 t;
        t.u = *reinterpret_cast<const uint4 *>(p.q + ((int64_t)b * p.n_q_heads + g * R + r) * D + sub * 8);
#pragma unroll
        for (int x = 0; x < 4; ++x) qh[r][x] = t.h2[x];
    }

    VecState<D, R> st;
    st.reset();
    TileRegs<D> cur, nxt;
    int j = wave;
    if (j < nblk) tile_issue<D>(cur, p.k_cache, p.v_cache, (int64_t)bt[j] * p.stride_block + head_off, lane);
    while (j < nblk) {
        const int jn = j + NW;
        if (jn < nblk)
            tile_issue<D>(nxt, p.k_cache, p.v_cache, (int64_t)bt[jn] * p.stride_block + head_off, lane);
        const int n_valid = (rem != 0 && j == nblk - 1) ? rem : kBlockTokens;
        vec_tile_update_any<D, R>(st, cur, qh, p.scale_log2, gid, n_valid);
        cur = nxt;
        j = jn;
    }
    vec_wave_merge<D, R>(st);
    __shared__ WaveMergeLds<D, R, NW> sm;
    vec_lds_put<D, R, NW>(sm, st, wave, gid, sub);
    __syncthreads();
    vec_lds_finish<D, R, NW, NW * 64>(sm, p, tid, b, g, si, c, to_out);
}

// ---------------------------------------------------------------------------------------
// Persistent form.  Work enumeration: every workgroup scans the sequence lengths into a
// table of first-chunk indices (LDS), which turns a flat item number into (sequence,
// chunk, selected head) without launching a workgroup per possible chunk.  Workgroup k
// takes items k, k + G, k + 2G, ...
//
// A workgroup is NW streaming waves plus one writer wave.
//   - Streaming waves: inside an item each wave streams its tiles through a two-slot
//     register ring; a slot is refilled right after it has been consumed, so one to two
//     tile pairs (8-16 KB per wave) are always in flight, and the first two tiles of the
//     next item are requested before the current item's merge.  These waves never store
//     to global memory: on gfx9-class hardware loads and stores share one in-order counter
//     only among themselves, so a single pending store would force every later wait in the
//     loop to drain all loads.
//   - Writer wave: after the barrier that ends an item it combines the NW wave results
//     from LDS (ascending wave order) and stores the fp16 row or the fp32 partial.
// Dynamic LDS: int lens[batch], int first[batch + 1], int hids[n_sel], then two
// WaveMergeLds areas used alternately.  Lengths and head ids are read once per workgroup
// and kept in LDS, so that no per-item global load sits between the tile loads.
// ---------------------------------------------------------------------------------------
struct ItemHdr {
    int b, si, c, g;
    int nblk;       // blocks of this chunk
    int rem;        // tokens in the ragged last block (0: none)
    int t0;         // first token of the chunk
    bool to_out;    // result goes to `out` (fp16), not to the partial buffers
    bool zero;      // length-0 sequence whose zeros this pass writes
};

template <int D, int R, int NW>
__host__ __device__ constexpr size_t persist_table_bytes(int batch, int n_sel)
{
    return (((size_t)(2 * batch + 1 + n_sel) * sizeof(int)) + 15) & ~(size_t)15;
}

__device__ __forceinline__ void workgroup_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

template <int D, int R, int NW>
__global__ __launch_bounds__((NW + 1) * 64) void attn_chunk_vec_persistent_kernel(const AttnParams p,
                                                                                  const int batch)
{
    constexpr int LPR = D / 8;
    constexpr int NT = (NW + 1) * 64;
    using Lds = WaveMergeLds<D, R, NW>;
    extern __shared__ __align__(16) unsigned char smem[];
    int *lens = reinterpret_cast<int *>(smem);
    int *first = lens + batch;
    int *hids = first + batch + 1;
    Lds *sm = reinterpret_cast<Lds *>(smem + persist_table_bytes<D, R, NW>(batch, p.n_sel));
    __shared__ int scan[NT];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int gid = lane / LPR;
    const int sub = lane % LPR;

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
                for (int idx = lane; idx < R * D; idx += 64) {
                    const int r = idx / D, d = idx % D;
                    p.out[((int64_t)h.b * p.n_q_heads + h.g * R + r) * D + d] = __float2half_rn(0.f);
                }
                continue;
            }
            workgroup_barrier();
            vec_lds_finish<D, R, NW, 64>(sm[parity], p, lane, h.b, h.g, h.si, h.c, h.to_out);
            parity ^= 1;
        }
        return;
    }

    // ---------------------------------------------------------------- streaming waves
    // Every global load below is issued unconditionally (indices clamped, tiles that do
    // not exist turned into zero-length descriptors), so the in-order load counter is
    // known exactly at every wait.
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
    auto load_q = [&](const Slot &s, __half2 (&qh)[R][4]) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            Pack16 t;
            t.u = *reinterpret_cast<const uint4 *>(
                p.q + ((int64_t)s.h.b * p.n_q_heads + s.h.g * R + r) * D + sub * 8);
#pragma unroll
            for (int x = 0; x < 4; ++x) qh[r][x] = t.h2[x];
        }
    };

    Slot cur, nxt, nn;
    __half2 qh[R][4], qh_nxt[R][4];
    TileRegs<D> A, B;
    fill(w, cur);
    fill(w + G, nxt);
    load_q(cur, qh);
    // refill of a ring slot with tile j of the pair stream: tiles of `cur`, then the first
    // pair of `nxt`
    int lim = 0;     // 2 * number of tile pairs of the current item
    auto refill = [&](TileRegs<D> &t, int j) {
        const bool in_cur = j < lim;
        const int idx = in_cur ? j : j - lim;
        const int idsv = in_cur ? cur.ids : nxt.ids;
        const int n_src = in_cur ? cur.n_my : nxt.n_my;
        const int64_t hoff = in_cur ? cur.head_off : nxt.head_off;
        const int blk = __builtin_amdgcn_readlane(idsv, idx & 63);
        tile_issue_checked<D>(t, p.k_cache, p.v_cache, (int64_t)blk * p.stride_block + hoff,
                              idx < n_src, lane);
    };
    // first pair of the first item
    lim = 2;
    {
        const int blk0 = __builtin_amdgcn_readlane(cur.ids, 0);
        const int blk1 = __builtin_amdgcn_readlane(cur.ids, 1);
        tile_issue_checked<D>(A, p.k_cache, p.v_cache, (int64_t)blk0 * p.stride_block + cur.head_off,
                              0 < cur.n_my, lane);
        tile_issue_checked<D>(B, p.k_cache, p.v_cache, (int64_t)blk1 * p.stride_block + cur.head_off,
                              1 < cur.n_my, lane);
    }
    int parity = 0;
    for (;;) {
        fill(w + 2 * G, nn);        // header and block ids two items ahead
        load_q(nxt, qh_nxt);        // query rows one item ahead

        VecState<D, R> st;
        st.reset();
        const int n_my = cur.n_my;
        lim = 2 * max(1, (n_my + 1) >> 1);
        // the ragged block, if any, is the chunk's last block: the last tile of one wave
        const bool mine_ragged = cur.h.rem != 0 && ((cur.h.nblk - 1) % NW) == wave;
        // The scheduling fences keep "consume a slot, refill it at once" in program order;
        // without them the compiler batches both tiles' arithmetic ahead of both refills
        // and the wave ends up waiting with nothing in flight.
        for (int i = 0; i < lim; i += 2) {
            if (i < n_my) {
                const int nv = (mine_ragged && i == n_my - 1) ? cur.h.rem : kBlockTokens;
                vec_tile_update_any<D, R>(st, A, qh, p.scale_log2, gid, nv);
            }
            __builtin_amdgcn_sched_barrier(0);
            refill(A, i + 2);
            __builtin_amdgcn_sched_barrier(0);
            if (i + 1 < n_my) {
                const int nv = (mine_ragged && i + 1 == n_my - 1) ? cur.h.rem : kBlockTokens;
                vec_tile_update_any<D, R>(st, B, qh, p.scale_log2, gid, nv);
            }
            __builtin_amdgcn_sched_barrier(0);
            refill(B, i + 3);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (cur.exists && !cur.h.zero) {
            vec_wave_merge<D, R>(st);
            vec_lds_put<D, R, NW>(sm[parity], st, wave, gid, sub);
            workgroup_barrier();
            parity ^= 1;
        }
        if (!nxt.exists) break;
        cur = nxt;
        nxt = nn;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int x = 0; x < 4; ++x) qh[r][x] = qh_nxt[r][x];
        w += G;
    }
}

// Log-sum-exp merge of chunk partials: one workgroup of D threads per (sequence, selected row).
template <int D>
__global__ __launch_bounds__(D) void attn_merge_kernel(const AttnParams p, int group)
{
    const int j = blockIdx.x;            // selected row: i*group + rr
    const int b = blockIdx.y;
    const int d = threadIdx.x;
    const int L = p.seq_lens[b];
    const int n_chunks = (L + p.chunk_tokens - 1) / p.chunk_tokens;
    if (p.direct_single && n_chunks <= 1) return;      // already written by the partial pass
    const int h = p.head_ids[j / group] * group + j % group;
    __half *o = p.out + ((int64_t)b * p.n_q_heads + h) * D;
    if (n_chunks <= 0) {
        o[d] = __float2half_rn(0.f);
        return;
    }
    const int rows = p.n_sel * group;
    const int64_t base = ((int64_t)b * rows + j) * p.max_chunks;
    const float *lse = p.lse_partial + base;
    const float *op = p.o_partial + base * D + d;
    float M = lse[0];
    for (int c = 1; c < n_chunks; ++c) M = fmaxf(M, lse[c]);
    float W = 0.f, acc = 0.f;
#pragma unroll 4
    for (int c = 0; c < n_chunks; ++c) {
        const float w = fast_exp2((lse[c] - M) * kLog2e);
        W += w;
        acc = fmaf(w, op[(int64_t)c * D], acc);
    }
    o[d] = __float2half_rn(acc / W);
}

}  // namespace hetis
