// MFMA arithmetic for grouped-query attention (r query heads share one KV head): here a
// tile is a real dense contraction, [16 tokens x D] against [D x r] and [D x 16 tokens]
// against [16 tokens x r], so it goes to the matrix cores with the query group padded to 16
// columns.  Both products are taken transposed so that the softmax output of the first is,
// lane for lane, the B operand of the second:
//
//   S^T = K . Q^T      v_mfma_f32_16x16x32_f16, D/32 steps
//         A = K tile : lane l holds K[token l%16][dims (l/16)*8 + 32*step .. +8]  (a 16-byte
//                      load straight from the cache tile; staging K through LDS with
//                      row-coalesced loads was measured and made no difference)
//         B = Q^T    : lane l holds Q[head l%16][same dims]; heads >= r are zero columns
//         C          : lane l, reg i = score of token (l/16)*4 + i for head l%16
//   O^T += V^T . P     v_mfma_f32_16x16x16_f16, D/16 row blocks
//         B = P      : lane l holds p[token (l/16)*4 + i][head l%16], i = 0..3: exactly the
//                      C registers above after exp2 and conversion to fp16
//         A = V^T    : lane l holds V[token (l/16)*4 + i][dim 16*mb + l%16]: four tokens of
//                      one dim.  The tile is token-major in memory, so it is staged through a
//                      wave-private LDS area (coalesced 128-bit loads -> ds_write_b128) and
//                      read back with the gfx950 transposing read ds_read_b64_tr_b16.
//         C          : lane l, reg i = O[head l%16][dim 16*mb + (l/16)*4 + i]
//
// ds_read_b64_tr_b16, as measured on gfx950: inside each group of 16 lanes, source lane s
// supplies four consecutive halves X[s][0..3] from its own address, and result lane i
// receives R[i][e] = X[4e + i/4][i%4].  With source lane s pointing at
// V[token 4*grp + s/4][dim 16*mb + 4*(s%4)] the result is the A operand above.
//
// Online softmax state per head lives in the 4 lanes {l%16 == head}: the running maximum is
// kept identical in all four (two cross-lane maxima per tile), the running sum is kept per
// lane group and added up once per chunk.
#pragma once
#include "attn_common.hpp"
#include "attn_persist.hpp"

namespace hetis {

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int D_, int R_>
struct MfmaPolicy {
    static constexpr int D = D_;
    static constexpr int R = R_;
    static_assert(D % 32 == 0 && R <= 16, "MFMA tiling");
    static constexpr int KS = D / 32;                 // contraction steps of S^T = K.Q^T
    static constexpr int MB = D / 16;                 // 16-dim row blocks of O^T
    static constexpr int NV = kBlockTokens * D * 2 / 1024;   // 1 KB slices of a V tile
    // Wave-private LDS: one V tile (token-major rows, pitch padded by 32 bytes so that the
    // 4 rows x 32 bytes a 16-lane transposing read touches fall into different banks) and
    // the query rows of the current item.
    static constexpr int kPitchV = 2 * D + 32;
    static constexpr int kStageV = kBlockTokens * kPitchV;
    static constexpr int kQBytes = R * D * 2;
    static constexpr int kWaveLdsBytes = kStageV + kQBytes;
    static constexpr int kWavesPerEu = 2;             // register budget: 512 / 2 per lane
#ifndef HETIS_MFMA_RING
#define HETIS_MFMA_RING 3
#endif
    static constexpr int kRing = D_ == 64 ? 4 : HETIS_MFMA_RING;   // tile pairs in flight per wave (a third pair at D = 128 was worth 2 % on the grouped-query workloads)

    struct Tile {
        uint4 k[KS];
        uint4 v[NV];
    };
    struct Query {
        f16x8 b[KS];
    };
    struct State {
        float m;          // running maximum (base-2 domain) of head l%16
        float l;          // running sum over the tokens this lane group has seen
        f32x4 acc[MB];
    };

    __device__ static __forceinline__ void issue(Tile &t, __amdgpu_buffer_rsrc_t rk,
                                                 __amdgpu_buffer_rsrc_t rv, int lane)
    {
        const int koff = (lane & 15) * (2 * D) + (lane >> 4) * 16;
#pragma unroll
        for (int s = 0; s < KS; ++s) t.k[s] = buffer_load_u4(rk, koff + s * 64);
        const int voff = lane * 16;
#pragma unroll
        for (int i = 0; i < NV; ++i) t.v[i] = buffer_load_u4(rv, voff + i * 1024);
    }

    // Query rows: fetched as raw bytes one item ahead (kQBytes over 64 lanes), then passed
    // through the wave's LDS area into operand layout with zero columns for heads >= r.
    // (two named members instead of an array: the array form was kept in scratch memory when it
    // had two elements, and a scratch store in a streaming wave is a global store like any other)
    static constexpr int kQVec = (kQBytes / 16 + 63) / 64;
    static_assert(kQVec <= 2, "query rows of one group: at most 2 x 64 x 16 bytes");
    struct QueryPrefetch {
        u32x4 raw0, raw1;
    };
    __device__ static __forceinline__ void q_prefetch(QueryPrefetch &pre, const __half *rows, int lane)
    {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(rows);
        pre.raw0 = src[min(lane, kQBytes / 16 - 1)];
        pre.raw1 = kQVec > 1 ? src[min(lane + 64, kQBytes / 16 - 1)] : u32x4{0u, 0u, 0u, 0u};
    }
    __device__ static __forceinline__ void q_commit(Query &q, const QueryPrefetch &pre,
                                                    unsigned char *stage, int lane)
    {
        u32x4 *dst = reinterpret_cast<u32x4 *>(stage + kStageV);
        if (lane < kQBytes / 16) dst[lane] = pre.raw0;
        if (kQVec > 1 && lane + 64 < kQBytes / 16) dst[lane + 64] = pre.raw1;
        const int j = lane & 15;
        const __half *src =
            reinterpret_cast<const __half *>(stage + kStageV) + min(j, R - 1) * D + (lane >> 4) * 8;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            union {
                uint4 u;
                f16x8 h;
            } t;
            t.u = *reinterpret_cast<const uint4 *>(src + s * 32);
            if (j >= R) t.u = make_uint4(0u, 0u, 0u, 0u);
            q.b[s] = t.h;
        }
    }

    __device__ static __forceinline__ void reset(State &st)
    {
        st.m = kNegBig;
        st.l = 0.f;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) st.acc[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // One code path for full and ragged tiles (n_valid = 16 makes every select a no-op):
    // two copies of this body would leave the accumulators in different registers on the two
    // sides of a branch and cost 32 register moves per tile to reconcile.
    template <bool MAYBE_RAGGED>
    __device__ static __forceinline__ void update(State &st, const Tile &t, const Query &q,
                                                  float scale_log2, int lane, int n_valid,
                                                  unsigned char *stage)
    {
        const int grp = lane >> 4;
        unsigned char *vstage = stage;
        // ---- V tile -> wave-private LDS, token-major rows
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int pos = i * 1024 + lane * 16;
            const int row = pos / (2 * D), colb = pos % (2 * D);
            uint4 v = t.v[i];
            if (row >= n_valid) v = make_uint4(0u, 0u, 0u, 0u);   // slots past the end may hold NaN
            *reinterpret_cast<uint4 *>(vstage + row * kPitchV + colb) = v;
        }
        // ---- scores of 16 tokens x 16 (padded) heads
        f32x4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            union {
                uint4 u;
                f16x8 h;
            } a;
            a.u = t.k[s];
            c = __builtin_amdgcn_mfma_f32_16x16x32_f16(a.h, q.b[s], c, 0, 0, 0);
        }
        float s4[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool valid = grp * 4 + i < n_valid;
            s4[i] = valid ? c[i] * scale_log2 : -INFINITY;
        }
        float mt = fmaxf(fmaxf(s4[0], s4[1]), fmaxf(s4[2], s4[3]));
        mt = fmaxf(mt, __shfl_xor(mt, 16, 64));
        mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
        const float m_new = fmaxf(st.m, mt);
        const float alpha = fast_exp2(st.m - m_new);
        st.m = m_new;
        float p4[4];
        float ps = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            p4[i] = fast_exp2(s4[i] - m_new);
            ps += p4[i];
        }
        st.l = st.l * alpha + ps;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) st.acc[mb] *= alpha;
        const f16x4 pb = {(_Float16)p4[0], (_Float16)p4[1], (_Float16)p4[2], (_Float16)p4[3]};
        // ---- O^T += V^T . P, V^T through the transposing LDS read (all reads first, so
        // that their latencies overlap)
        const int srow = grp * 4 + ((lane & 15) >> 2);
        const unsigned char *vsrc = vstage + srow * kPitchV + (lane & 3) * 8;
        union {
            i16x4 i;
            f16x4 h;
        } vt[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            vt[mb].i = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) i16x4 *)(vsrc + mb * 32));
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            st.acc[mb] = __builtin_amdgcn_mfma_f32_16x16x16f16(vt[mb].h, pb, st.acc[mb], 0, 0, 0);
    }

    // normalised rows and their base-2 log-sum-exp -> LDS (the wave's mailbox)
    __device__ static __forceinline__ void finish(State &st, float (&o)[R][D], float (&lse)[R],
                                                  int lane)
    {
        const int j = lane & 15, grp = lane >> 4;
        float l = st.l;
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        if (j < R) {
            const float inv = __builtin_amdgcn_rcpf(l);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const float4 v = make_float4(st.acc[mb][0] * inv, st.acc[mb][1] * inv,
                                             st.acc[mb][2] * inv, st.acc[mb][3] * inv);
                *reinterpret_cast<float4 *>(&o[j][mb * 16 + grp * 4]) = v;
            }
            if (grp == 0) lse[j] = st.m + fast_log2(l);
        }
    }
};

}  // namespace hetis
