// Vector (non-MFMA) chunk kernels: Eq. (2b) restricted to the tokens of one chunk of one
// (sequence, selected KV head).  The path is HBM-bound (r flop per KV byte), so the layout
// is chosen for the loads, not for the ALUs:
//   - a (block, head) tile is 16 rows of D fp16 = 16*D*2 contiguous bytes; a wave reads
//     it with 128-bit loads, lane l taking bytes [16 l, 16 l + 16) of each 1 KB slice, so
//     D/8 neighbouring lanes hold one token row and a slice holds 64/(D/8) tokens;
//   - q.k is a v_dot2 chain per lane followed by a DPP sum over the D/8 lanes of a row;
//   - each group of D/8 lanes runs its own online softmax over the tokens it sees
//     (exp2 domain, fp32), so p never leaves registers between q.k and p.v;
//   - the lane groups of a wave are merged once per chunk, in a fixed order, through
//     shuffles.
// Nothing depends on how many heads were selected: the result for one (sequence, head)
// is a function of that sequence's length alone.
#pragma once
#include "attn_common.hpp"
#include "attn_persist.hpp"

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

// ---------------------------------------------------------------------------------------
// Policy through which the persistent kernel (attn_persist.hpp) uses the vector arithmetic.
// ---------------------------------------------------------------------------------------
template <int D_, int R_>
struct VecPolicy {
    static constexpr int D = D_;
    static constexpr int R = R_;
    static constexpr int kWaveLdsBytes = 0;      // no per-wave staging area
    static constexpr int kWavesPerEu = 2;        // register budget: 512 / 2 per lane
    // tile pairs in flight per wave: 16 KB either way (a tile pair is 8 KB at D = 128, 4 KB at 64)
    static constexpr int kRing = D_ == 64 ? 4 : 2;
    using Tile = TileRegs<D>;
    using State = VecState<D, R>;
    struct Query {
        __half2 h[R][4];                         // this lane's 8 dims of each head of the group
    };

    // K and V: lane l takes bytes [16 l, 16 l + 16) of every 1 KB slice of the tile
    __device__ static __forceinline__ void issue(Tile &t, __amdgpu_buffer_rsrc_t rk,
                                                 __amdgpu_buffer_rsrc_t rv, int lane)
    {
        const int voff = lane * 16;
#pragma unroll
        for (int i = 0; i < Tile::NI; ++i) t.k[i] = buffer_load_u4(rk, voff + i * 1024);
#pragma unroll
        for (int i = 0; i < Tile::NI; ++i) t.v[i] = buffer_load_u4(rv, voff + i * 1024);
    }
    using QueryPrefetch = Query;                 // loaded from global in its final layout
    __device__ static __forceinline__ void q_prefetch(QueryPrefetch &q, const __half *rows, int lane)
    {
        const int sub = lane % (D / 8);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            Pack16 t;
            t.u = *reinterpret_cast<const uint4 *>(rows + r * D + sub * 8);
#pragma unroll
            for (int x = 0; x < 4; ++x) q.h[r][x] = t.h2[x];
        }
    }
    __device__ static __forceinline__ void q_commit(Query &q, const QueryPrefetch &pre,
                                                    unsigned char *, int)
    {
        q = pre;
    }
    __device__ static __forceinline__ void reset(State &st) { st.reset(); }
    // MAYBE_RAGGED: the tile may be the ragged last block of a sequence (n_valid < 16); a
    // separate masked copy of the arithmetic keeps whole tiles free of compares and selects
    template <bool MAYBE_RAGGED>
    __device__ static __forceinline__ void update(State &st, const Tile &t, const Query &q,
                                                  float scale_log2, int lane, int n_valid,
                                                  unsigned char *)
    {
        if (MAYBE_RAGGED)
            vec_tile_update_any<D, R>(st, t, q.h, scale_log2, lane / (D / 8), n_valid);
        else
            vec_tile_update<D, R, false>(st, t, q.h, scale_log2, lane / (D / 8), kBlockTokens);
    }
    // normalised rows and their base-2 log-sum-exp -> LDS (the wave's mailbox)
    __device__ static __forceinline__ void finish(State &st, float (&o)[R][D], float (&lse)[R],
                                                  int lane)
    {
        vec_wave_merge<D, R>(st);                // every lane group now holds the item's totals
        const int gid = lane / (D / 8), sub = lane % (D / 8);
        if (gid == 0) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float inv = __builtin_amdgcn_rcpf(st.l[r]);
                float4 lo = make_float4(st.o[r][0] * inv, st.o[r][1] * inv, st.o[r][2] * inv,
                                        st.o[r][3] * inv);
                float4 hi = make_float4(st.o[r][4] * inv, st.o[r][5] * inv, st.o[r][6] * inv,
                                        st.o[r][7] * inv);
                *reinterpret_cast<float4 *>(&o[r][sub * 8]) = lo;
                *reinterpret_cast<float4 *>(&o[r][sub * 8 + 4]) = hi;
                if (sub == 0) lse[r] = st.m[r] + fast_log2(st.l[r]);
            }
        }
    }
};

// Log-sum-exp merge of the partial results of a row's segments: one workgroup of D threads per
// (sequence, selected query row); in pairs mode per (pair, row of the group).
template <int D>
__global__ __launch_bounds__(D) void attn_merge_kernel(const AttnParams p, int group)
{
    const int j = blockIdx.x;            // selected row: i*group + rr
    const int b = blockIdx.y;
    const int d = threadIdx.x;
    const bool pairs = p.pair_seq != nullptr;
    const int seq = pairs ? p.pair_seq[b] : b;
    const int n_sel = pairs ? 1 : p.n_sel;
    const int L = p.seq_lens[seq];
    const int n_segs = (L + p.seg_tokens - 1) / p.seg_tokens;
    if (p.direct_single && n_segs <= 1) return;        // already written by the chunk kernel
    const int h = (pairs ? p.pair_head[b] : p.head_ids[j / group]) * group + j % group;
    __half *o = p.out + ((int64_t)seq * p.n_q_heads + h) * D;
    if (n_segs <= 0) {
        o[d] = __float2half_rn(0.f);
        return;
    }
    // partial of segment c of this row: index ((b*n_sel + i)*max_segs + c)*group + rr
    const int64_t base = ((int64_t)b * n_sel + j / group) * p.max_segs * group + j % group;
    const float *lse = p.lse_partial + base;
    const float *op = p.o_partial + base * D + d;
    // (unrolled so that the loads of 16 segments are in flight together; the sums keep their order)
    float M = lse[0];
#pragma unroll 16
    for (int c = 1; c < n_segs; ++c) M = fmaxf(M, lse[(int64_t)c * group]);
    float W = 0.f, acc = 0.f;
#pragma unroll 16
    for (int c = 0; c < n_segs; ++c) {
        const float w = fast_exp2((lse[(int64_t)c * group] - M) * kLog2e);
        W += w;
        acc = fmaf(w, op[(int64_t)c * group * D], acc);
    }
    o[d] = __float2half_rn(acc / W);
}

}  // namespace hetis
