// Head-wise cache management kernels (Section 6, "KV cache management"): rows addressed by
// (sequence id, position, head id) through the block table, and whole (block, head) tiles
// copied between pools.  Pure data movement in 16-byte pieces; every index read from device
// memory is range-checked and an entry that fails the check is skipped.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hetis {

typedef unsigned int kv_u32x4 __attribute__((ext_vector_type(4)));

constexpr int kKvBlockTokens = 16;
// Head rows a thread of the row kernel loads before it stores the first of them.
#ifndef HETIS_KV_ROWS_IN_FLIGHT
#define HETIS_KV_ROWS_IN_FLIGHT 8
#endif
// Workgroups of the tile-copy kernel: 256 CUs x 8 resident workgroups of 4 waves.
constexpr int kKvCopyMaxWorkgroups = 2048;

struct KvRowParams {
    uint4 *rows_k;              // STORE: source rows [n_tokens, Hkv, D]; FETCH: destination
    uint4 *rows_v;
    uint4 *cache_k;             // STORE: destination; FETCH: source
    uint4 *cache_v;
    const int32_t *token_seq;   // or nullptr: entry n belongs to sequence n
    const int32_t *token_pos;   // position = token_pos[n] + pos_bias
    const int32_t *block_table;
    const int32_t *head_ids;
    int64_t stride_block, stride_head;   // in 16-byte units
    int64_t num_blocks;
    int32_t n_tokens, n_sel, n_kv_heads, batch, max_blocks_per_seq, pos_bias;
};

// One group of 2*D/8 lanes moves the K row and the V row of one (entry, head): lane c of the
// first half moves bytes [16c, 16c+16) of the K row, the second half the V row.  blockIdx.y
// strides over the selected heads, so the per-entry index loads (the same words in all lanes
// of the group: one access) are shared by the heads a thread handles.
template <int D, bool FETCH>
__global__ void __launch_bounds__(256) kv_rows_kernel(KvRowParams p)
{
    constexpr int LR = D / 8;                   // lanes per row
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t n = t / (2 * LR);
    if (n >= p.n_tokens) return;
    const int within = (int)(t % (2 * LR));
    const bool is_v = within >= LR;
    const int c = within % LR;
    const int64_t b = p.token_seq ? (int64_t)p.token_seq[n] : n;
    const int64_t pos = (int64_t)p.token_pos[n] + p.pos_bias;
    if (b < 0 || b >= p.batch || pos < 0) return;
    const int64_t j = pos / kKvBlockTokens;
    if (j >= p.max_blocks_per_seq) return;
    const int64_t blk = p.block_table[b * p.max_blocks_per_seq + j];
    if (blk < 0 || blk >= p.num_blocks) return;
    const int slot = (int)(pos % kKvBlockTokens);
    uint4 *cache = is_v ? p.cache_v : p.cache_k;
    uint4 *rows = is_v ? p.rows_v : p.rows_k;
    const int64_t cache_row = blk * p.stride_block + (int64_t)slot * LR + c;
    const int64_t rows_row = n * p.n_kv_heads * LR + c;
    // heads in batches of U: the loads of a batch are in flight together before the
    // first store (a thread that alternates one load and one store leaves the memory system
    // with a single access per thread in flight)
    constexpr int U = HETIS_KV_ROWS_IN_FLIGHT;
    for (int s0 = blockIdx.y; s0 < p.n_sel; s0 += U * gridDim.y) {
        int g[U];
        bool ok[U];
        kv_u32x4 x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int s = s0 + u * gridDim.y;
            g[u] = s < p.n_sel ? p.head_ids[s] : -1;
            ok[u] = g[u] >= 0 && g[u] < p.n_kv_heads;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (!ok[u]) continue;
            // every byte is touched once: non-temporal both ways
            const uint4 *src = FETCH ? cache + cache_row + (int64_t)g[u] * p.stride_head
                                     : rows + rows_row + (int64_t)g[u] * LR;
            x[u] = __builtin_nontemporal_load((const kv_u32x4 *)src);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (!ok[u]) continue;
            uint4 *dst = FETCH ? rows + rows_row + (int64_t)g[u] * LR
                               : cache + cache_row + (int64_t)g[u] * p.stride_head;
            __builtin_nontemporal_store(x[u], (kv_u32x4 *)dst);
        }
    }
}

struct KvPairParams {
    const uint4 *k_new, *v_new;     // [batch, Hkv, D]
    uint4 *k_tiles, *v_tiles;       // single-head tiles
    const int32_t *block_table;     // [n_pairs, max_blocks_per_seq]
    const int32_t *seq_lens, *pair_seq, *pair_head;
    int64_t stride_tile;            // in 16-byte units
    int64_t num_tiles;
    int32_t n_pairs, n_kv_heads, batch, max_blocks_per_seq;
};

// Decode-step store for per-request head subsets: 2*D/8 lanes move the new K row and V row
// of one (sequence, KV head) pair to position seq_lens[b] - 1 through the pair's own
// block-table row.  Same checks as kv_rows_kernel; a pair that fails one is skipped.
template <int D>
__global__ void __launch_bounds__(256) kv_append_pairs_kernel(KvPairParams p)
{
    constexpr int LR = D / 8;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t pr = t / (2 * LR);
    if (pr >= p.n_pairs) return;
    const int within = (int)(t % (2 * LR));
    const bool is_v = within >= LR;
    const int c = within % LR;
    const int64_t b = p.pair_seq[pr];
    const int64_t g = p.pair_head[pr];
    if (b < 0 || b >= p.batch || g < 0 || g >= p.n_kv_heads) return;
    const int64_t pos = (int64_t)p.seq_lens[b] - 1;
    if (pos < 0) return;
    const int64_t j = pos / kKvBlockTokens;
    if (j >= p.max_blocks_per_seq) return;
    const int64_t tile = p.block_table[pr * p.max_blocks_per_seq + j];
    if (tile < 0 || tile >= p.num_tiles) return;
    const uint4 *src = (is_v ? p.v_new : p.k_new) + (b * p.n_kv_heads + g) * LR + c;
    uint4 *dst = (is_v ? p.v_tiles : p.k_tiles) + tile * p.stride_tile + (pos % kKvBlockTokens) * LR + c;
    *dst = *src;
}

struct KvCopyParams {
    const uint4 *src_k, *src_v;
    uint4 *dst_k, *dst_v;
    const int32_t *src_blocks, *dst_blocks, *src_heads, *dst_heads;
    int64_t src_stride_block, src_stride_head, dst_stride_block, dst_stride_head;   // 16-byte units
    int64_t src_num_blocks, dst_num_blocks;
    int64_t n_items;            // n_pairs * n_sel
    int32_t n_sel, src_n_heads, dst_n_heads;
};

// One wave moves the K tile and the V tile of one (pair, head) per step: all loads of the
// step are issued before the first store, so a wave keeps 2 tiles (8 KB at D = 128) in
// flight.  Items are numbered pair-major, so neighbouring waves move neighbouring heads of
// one block.  Grid-stride over items.  Loads and stores are non-temporal: every byte is
// touched once, and keeping the written lines out of the caches was worth 8 % (measured).
template <int D>
__global__ void __launch_bounds__(256) kv_copy_tiles_kernel(KvCopyParams p)
{
    constexpr int NV = kKvBlockTokens * D * 2 / 1024;     // 1 KB slices per tile
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t n_waves = (int64_t)gridDim.x * 4;
    for (int64_t item = wave; item < p.n_items; item += n_waves) {
        const int64_t i = item / p.n_sel;
        const int s = (int)(item % p.n_sel);
        const int64_t sb = p.src_blocks[i], db = p.dst_blocks[i];
        const int sg = p.src_heads[s], dg = p.dst_heads[s];
        if (sb < 0 || sb >= p.src_num_blocks || db < 0 || db >= p.dst_num_blocks) continue;
        if (sg < 0 || sg >= p.src_n_heads || dg < 0 || dg >= p.dst_n_heads) continue;
        const int64_t so = sb * p.src_stride_block + (int64_t)sg * p.src_stride_head + lane;
        const int64_t dof = db * p.dst_stride_block + (int64_t)dg * p.dst_stride_head + lane;
        kv_u32x4 k[NV], v[NV];
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            k[u] = __builtin_nontemporal_load((const kv_u32x4 *)&p.src_k[so + u * 64]);
            v[u] = __builtin_nontemporal_load((const kv_u32x4 *)&p.src_v[so + u * 64]);
        }
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            __builtin_nontemporal_store(k[u], (kv_u32x4 *)&p.dst_k[dof + u * 64]);
            __builtin_nontemporal_store(v[u], (kv_u32x4 *)&p.dst_v[dof + u * 64]);
        }
    }
}

}  // namespace hetis
