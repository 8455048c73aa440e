/*
 * hetis_kv.h - C ABI of the head-wise KV cache management kernels (MI355X, gfx950).
 *
 * The operation (Section 6, "KV cache management" of the Hetis paper): the cache
 * lives in fixed-size blocks that are split again on the head dimension, and
 * rows are stored and fetched by the combination of sequence id, position
 * within the sequence and head id.  With block table bt, the row of
 * (sequence b, position p, KV head g) is
 *     cache[ bt[b][p / 16] ][ g ][ p % 16 ][ 0 .. D )
 * in the tile layout of hetis_attn.h.  A device that holds some heads of a
 * request stores, every decode step, the new token's K and V rows of those heads
 * before Attention reads them (Section 5.1: the new token attends to all stored
 * keys and values, its own included), and moves whole (block, head) tiles when
 * heads of a request are re-dispatched (Section 5.3; Section 6, "Live cache
 * migration": the copy runs on a stream of the caller's choice, beside the
 * decode work).
 *
 * Conventions: those of hetis_attn.h (device pointers unless marked host, caller
 * owns all buffers, calls enqueue on `stream` and return, status codes, nothing
 * printed).  The kernels of this header use no memory besides their arguments:
 * no entry point here allocates, keeps state or synchronises.  In addition:
 *   - New rows and fetched rows are fp16 [n_tokens, n_kv_heads, head_dim],
 *     indexed by the model's KV head id like the query rows; only rows of
 *     heads in head_ids are read / written.  The kernels move bytes and never
 *     interpret them.
 *   - shape->n_q_heads is not used here (any positive multiple of n_kv_heads).
 *   - num_blocks (host) is the number of physical blocks of the pool.  Unlike the
 *     Attention entry points these kernels DO check what they read from device
 *     memory: an entry whose sequence id is outside [0, batch), whose position
 *     is negative or at or past 16 * max_blocks_per_seq, or whose block id is
 *     outside [0, num_blocks) is skipped (nothing is read or written for it).
 *     head_ids outside [0, n_kv_heads) are skipped the same way.
 *   - If two entries of one call name the same (sequence, position, head), which
 *     of them ends up in the cache is unspecified.
 *   - A store must have completed (stream order) before an Attention call reads
 *     the rows.
 *
 * Supported: head_dim in {64, 128}; block_size 16.
 */
#ifndef HETIS_KV_H
#define HETIS_KV_H

#include "hetis_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Decode-step store: one new row per sequence, at position seq_lens[b] - 1
 * (seq_lens already counts the new token; sequences of length 0 store nothing).
 *   shape        host; batch = B
 *   k_new, v_new fp16 [B, Hkv, D]
 *   block_table  int32 [B, max_blocks_per_seq]
 *   seq_lens     int32 [B]
 *   head_ids     int32 [n_sel_heads]
 *   k_cache, v_cache   written in place: B * n_sel_heads rows of D fp16 each
 * Errors: NULL, BAD_SHAPE, UNSUPPORTED, BAD_HEADS, LAUNCH.
 */
int hetis_kv_append(const hetis_attn_shape *shape, const void *k_new, const void *v_new,
                    const int32_t *block_table, const int32_t *seq_lens,
                    const int32_t *head_ids, int32_t n_sel_heads, int64_t num_blocks,
                    void *k_cache, void *v_cache, void *stream);

/*
 * Decode-step store for per-request head subsets (the companion of
 * hetis_attn_decode_pairs; Section 4.2 / 5.2.1: the heads a device holds differ per
 * request): pair p = (pair_seq[p], pair_head[p]) stores k_new[b, g, :] and
 * v_new[b, g, :] at position seq_lens[b] - 1 of its own block-table row,
 *   tile = block_table[p][pos / 16], element tile * kv_stride_block + (pos % 16) * D
 * in a pool of single-head tiles (kv_stride_block 0 = 16 * D; kv_stride_head unused).
 *   k_new, v_new fp16 [B, Hkv, D]     block_table int32 [n_pairs, max_blocks_per_seq]
 *   num_tiles    host, tiles in the pool; pairs that point outside the tables are skipped
 * Errors: NULL, BAD_SHAPE, UNSUPPORTED, LAUNCH.  n_pairs = 0 is a no-op.
 */
int hetis_kv_append_pairs(const hetis_attn_shape *shape, const void *k_new, const void *v_new,
                          const int32_t *block_table, const int32_t *seq_lens,
                          const int32_t *pair_seq, const int32_t *pair_head, int32_t n_pairs,
                          int64_t num_tiles, void *k_tiles, void *v_tiles, void *stream);

/*
 * General store by (sequence id, position, head id): entry n carries the rows
 * k_new[n, g, :], v_new[n, g, :] of sequence token_seq[n] at position
 * token_pos[n] (e.g. all prompt tokens after prefill).
 *   token_seq    int32 [n_tokens], or NULL: entry n belongs to sequence n
 *                (then n_tokens must not exceed batch)
 *   token_pos    int32 [n_tokens]
 *   n_tokens     host, >= 0 (0 is a no-op)
 * Errors: as hetis_kv_append.
 */
int hetis_kv_store(const hetis_attn_shape *shape, const void *k_new, const void *v_new,
                   const int32_t *token_seq, const int32_t *token_pos, int32_t n_tokens,
                   const int32_t *block_table, const int32_t *head_ids, int32_t n_sel_heads,
                   int64_t num_blocks, void *k_cache, void *v_cache, void *stream);

/*
 * Fetch by (sequence id, position, head id), the inverse gather:
 *   k_out[n, g, :] = K row of (token_seq[n], token_pos[n], g) for g in head_ids.
 *   k_out, v_out  fp16 [n_tokens, Hkv, D]; rows of skipped entries and of heads
 *                 that are not selected are left untouched.
 */
int hetis_kv_fetch(const hetis_attn_shape *shape, const void *k_cache, const void *v_cache,
                   const int32_t *token_seq, const int32_t *token_pos, int32_t n_tokens,
                   const int32_t *block_table, const int32_t *head_ids, int32_t n_sel_heads,
                   int64_t num_blocks, void *k_out, void *v_out, void *stream);

/* Geometry of one paged pool (host struct). */
typedef struct {
    int32_t n_kv_heads;         /* heads per block in this pool, > 0 */
    int32_t head_dim;           /* 64 or 128 */
    int32_t block_size;         /* 16 */
    int32_t reserved;           /* 0 */
    int64_t num_blocks;         /* > 0 */
    int64_t kv_stride_block;    /* elements between blocks; 0 = n_kv_heads * 16 * D */
    int64_t kv_stride_head;     /* elements between heads of a block; 0 = 16 * D */
} hetis_kv_pool;

/*
 * Tile copy between two pools (the device-local part of moving heads of a
 * request): for every pair i < n_pairs and every j < n_sel_heads
 *   dst[dst_blocks[i]][dst_heads[j]] = src[src_blocks[i]][src_heads[j]]
 * (all 16 x D elements), for K and for V.  The pools may differ in head count,
 * strides and size, e.g. a compact pool that holds only the moved heads; they
 * must agree in head_dim and block_size.  A pair with a block id outside its
 * pool, and a head pair with an id outside its pool, is skipped.
 *   src_blocks, dst_blocks  int32 [n_pairs]     (n_pairs >= 0; 0 is a no-op)
 *   src_heads, dst_heads    int32 [n_sel_heads] (1 .. 1024 entries)
 * Source and destination tiles must not overlap (the same pool may be both if
 * the tile sets are disjoint).  One pass over the data: 2 * n_pairs *
 * n_sel_heads * 16 * D * 2 bytes read and as many written.
 * Errors: NULL, BAD_SHAPE, UNSUPPORTED, BAD_HEADS, LAUNCH.
 */
int hetis_kv_copy_tiles(const hetis_kv_pool *src_pool, const void *src_k, const void *src_v,
                        const hetis_kv_pool *dst_pool, void *dst_k, void *dst_v,
                        const int32_t *src_blocks, const int32_t *dst_blocks, int32_t n_pairs,
                        const int32_t *src_heads, const int32_t *dst_heads, int32_t n_sel_heads,
                        void *stream);

/*
 * Measurement hook, like hetis_attn_profile_events: the two events are attached to
 * the kernel dispatch of every later hetis_kv_* call of the same host thread
 * (start when the kernel begins to execute, stop when it has finished).
 * (NULL, NULL) switches it off.
 */
int hetis_kv_profile_events(void *begin, void *end);

#ifdef __cplusplus
}
#endif
#endif /* HETIS_KV_H */
