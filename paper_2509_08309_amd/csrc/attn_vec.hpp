// Vector (non-MFMA) chunk kernel: one workgroup per (sequence, selected KV head, chunk).
//
// Eq. (2b) restricted to the tokens of one chunk.  The path is HBM-bound (r flop per
// KV byte), so the layout is chosen for the loads, not for the ALUs:
//   - a (block, head) tile is 16 rows of D fp16 = 16*D*2 contiguous bytes; a wave reads
//     it with 128-bit loads, lane l taking bytes [16 l, 16 l + 16) of each 1 KB slice, so
//     D/8 neighbouring lanes hold one token row and a slice holds 64/(D/8) tokens;
//   - q.k is a v_dot2 chain per lane followed by a DPP sum over the D/8 lanes of a row;
//   - each group of D/8 lanes runs its own online softmax over the tokens it sees
//     (exp2 domain, fp32), so p never leaves registers between q.k and p.v;
//   - the lane groups of a wave, then the waves of the workgroup, are merged once at the
//     end, in a fixed order, through shuffles and LDS.
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
};

// One tile (16 tokens) of K and V held in registers -> update of the running state.
template <int D, int R, bool MASKED>
__device__ __forceinline__ void vec_tile_update(VecState<D, R> &st, const uint4 (&kb)[16 / (512 / D)],
                                                const uint4 (&vb)[16 / (512 / D)],
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
        kk.u = kb[i];
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
        vv.u = vb[i];
        if (MASKED && !(i * TPI + gid < n_valid)) vv.u = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const float vf = __half2float(vv.h[x]);
#pragma unroll
            for (int r = 0; r < R; ++r) st.o[r][x] = fmaf(p[i][r], vf, st.o[r][x]);
        }
    }
}

template <int D, int R, int NW>
__global__ __launch_bounds__(NW * 64) void attn_chunk_vec_kernel(const AttnParams p)
{
    constexpr int LPR = D / 8;
    constexpr int TPI = 64 / LPR;
    constexpr int NI = 16 / TPI;
    constexpr int TILE = kBlockTokens * D;      // elements per tile

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
        // zero-length sequence: zeros, written once (by chunk 0) when this pass owns `out`
        if (to_out && c == 0) {
            for (int idx = tid; idx < R * D; idx += NW * 64) {
                const int r = idx / D, d = idx % D;
                p.out[((int64_t)b * p.n_q_heads + g * R + r) * D + d] = __float2half_rn(0.f);
            }
        }
        return;
    }
    if (c >= n_chunks) return;

    const int t0 = c * p.chunk_tokens;
    const int t1 = min(L, t0 + p.chunk_tokens);
    const int n_tok = t1 - t0;
    const int nblk = (n_tok + kBlockTokens - 1) / kBlockTokens;
    const int rem = n_tok & (kBlockTokens - 1);
    const int32_t *bt = p.block_table + (int64_t)b * p.max_blocks_per_seq + t0 / kBlockTokens;
    const int64_t head_off = (int64_t)g * p.stride_head;

    // this lane's 8 query dims for each of the R heads of the group
    __half2 qh[R][4];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        Pack16 t;
        t.u = *reinterpret_cast<const uint4 *>(p.q + ((int64_t)b * p.n_q_heads + g * R + r) * D + sub * 8);
#pragma unroll
        for (int x = 0; x < 4; ++x) qh[r][x] = t.h2[x];
    }

    VecState<D, R> st;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        st.m[r] = kNegBig;
        st.l[r] = 0.f;
#pragma unroll
        for (int x = 0; x < 8; ++x) st.o[r][x] = 0.f;
    }

    // wave w takes blocks w, w+NW, ...; the next tile is in flight while one is consumed
    uint4 kc[NI], vc[NI], kn[NI], vn[NI];
    int j = wave;
    if (j < nblk) {
        const int64_t base = (int64_t)bt[j] * p.stride_block + head_off;
        const uint4 *kp = reinterpret_cast<const uint4 *>(p.k_cache + base) + lane;
        const uint4 *vp = reinterpret_cast<const uint4 *>(p.v_cache + base) + lane;
#pragma unroll
        for (int i = 0; i < NI; ++i) kc[i] = kp[i * 64];
#pragma unroll
        for (int i = 0; i < NI; ++i) vc[i] = vp[i * 64];
    }
    int blk_next = (j + NW < nblk) ? bt[j + NW] : 0;
    while (j < nblk) {
        const int jn = j + NW;
        if (jn < nblk) {
            const int64_t base = (int64_t)blk_next * p.stride_block + head_off;
            const uint4 *kp = reinterpret_cast<const uint4 *>(p.k_cache + base) + lane;
            const uint4 *vp = reinterpret_cast<const uint4 *>(p.v_cache + base) + lane;
#pragma unroll
            for (int i = 0; i < NI; ++i) kn[i] = kp[i * 64];
#pragma unroll
            for (int i = 0; i < NI; ++i) vn[i] = vp[i * 64];
            blk_next = (jn + NW < nblk) ? bt[jn + NW] : 0;
        }
        if (rem != 0 && j == nblk - 1)
            vec_tile_update<D, R, true>(st, kc, vc, qh, p.scale_log2, gid, rem);
        else
            vec_tile_update<D, R, false>(st, kc, vc, qh, p.scale_log2, gid, kBlockTokens);
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            kc[i] = kn[i];
            vc[i] = vn[i];
        }
        j = jn;
    }
    (void)TILE;

    // merge the TPI lane groups of the wave (xor butterfly over the group index)
#pragma unroll
    for (int mask = LPR; mask < 64; mask <<= 1) {
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

    // merge the waves through LDS, ascending wave order
    __shared__ float sm_o[NW][R][D];
    __shared__ float sm_m[NW][R];
    __shared__ float sm_l[NW][R];
    if (gid == 0) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int x = 0; x < 8; ++x) sm_o[wave][r][sub * 8 + x] = st.o[r][x];
            if (sub == 0) {
                sm_m[wave][r] = st.m[r];
                sm_l[wave][r] = st.l[r];
            }
        }
    }
    __syncthreads();
    const int rows = p.n_sel * R;
    for (int idx = tid; idx < R * D; idx += NW * 64) {
        const int r = idx / D, d = idx % D;
        float M = sm_m[0][r];
#pragma unroll
        for (int w = 1; w < NW; ++w) M = fmaxf(M, sm_m[w][r]);
        float acc = 0.f, lsum = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float a = fast_exp2(sm_m[w][r] - M);
            acc += sm_o[w][r][d] * a;
            lsum += sm_l[w][r] * a;
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
