/*
 * CPU checker for head-wise KV cache management: store, fetch and tile copy.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain loops over 16-bit cache elements; shares no
 * code with the HIP path and is never called from it.
 *
 * What is computed (Section 6, "KV cache management"): the cache is kept in
 * fixed-size blocks that are split again on the head dimension, and rows are
 * stored and fetched by the combination of sequence id, position within the
 * sequence and head id.  With a block table bt (one row of physical block ids
 * per sequence) the row of (sequence b, position p, head g) is
 *     cache[ bt[b][p / block_size] ][ g ][ p % block_size ][ 0 .. D )
 * and a (block, head) tile is the block_size x D rows of one head in one block.
 * Moving the cache of some heads of a request to another pool (the device-local
 * half of the cache migration of Section 5.3 / Section 6, "Live cache
 * migration") is a copy of such tiles from (source block, source head) to
 * (destination block, destination head).
 *
 * Readings where the paper is silent:
 *   - new rows arrive as [n_tokens, n_kv_heads, D], indexed by the model's KV
 *     head id like the query rows; only rows of selected heads are used.
 *   - in the decode step the new token is the last one of its sequence and
 *     seq_lens already counts it: its position is seq_lens[b] - 1; a sequence
 *     of length 0 stores nothing.
 *   - an entry that points outside the tables (sequence id outside [0, batch),
 *     negative position, position past the block-table row, physical block
 *     outside [0, num_blocks)) is skipped: nothing is written for it.
 *   - entries are processed in ascending order; if two entries name the same
 *     (sequence, position), the later one wins here (the GPU library leaves the
 *     winner unspecified, so tests never rely on it).
 *
 * Everything is a byte copy: results are compared bit for bit.
 */
#include <stdint.h>
#include <string.h>

typedef struct {
    int32_t batch, n_q_heads, n_kv_heads, head_dim, block_size, max_blocks_per_seq;
    int64_t kv_stride_block, kv_stride_head;       /* in elements */
} oracle_shape;

typedef struct {
    int32_t n_kv_heads, head_dim, block_size, num_blocks;
    int64_t kv_stride_block, kv_stride_head;       /* in elements */
} oracle_pool;

/* element offset of row (b, p, g), or -1 if the entry must be skipped */
static int64_t row_offset(const oracle_shape *s, const int32_t *block_table, int32_t num_blocks,
                          int64_t b, int64_t p, int g)
{
    if (b < 0 || b >= s->batch || p < 0) return -1;
    int64_t j = p / s->block_size;
    if (j >= s->max_blocks_per_seq) return -1;
    int64_t blk = block_table[b * s->max_blocks_per_seq + j];
    if (blk < 0 || blk >= num_blocks) return -1;
    return blk * s->kv_stride_block + (int64_t)g * s->kv_stride_head
           + (p % s->block_size) * s->head_dim;
}

/*
 * Store: for every entry n and every selected head g,
 *   K[row(seq[n], pos[n], g)] = k_new[n][g][:],  V likewise.
 * token_seq == NULL means entry n belongs to sequence n.
 */
int oracle_kv_store(const oracle_shape *s, const uint16_t *k_new, const uint16_t *v_new,
                    const int32_t *token_seq, const int32_t *token_pos, int32_t n_tokens,
                    const int32_t *block_table, const int32_t *head_ids, int32_t n_sel,
                    int32_t num_blocks, uint16_t *k_cache, uint16_t *v_cache)
{
    const int D = s->head_dim;
    for (int64_t n = 0; n < n_tokens; ++n) {
        int64_t b = token_seq ? token_seq[n] : n;
        for (int j = 0; j < n_sel; ++j) {
            int g = head_ids[j];
            if (g < 0 || g >= s->n_kv_heads) return -1;
            int64_t off = row_offset(s, block_table, num_blocks, b, token_pos[n], g);
            if (off < 0) continue;
            const int64_t src = (n * s->n_kv_heads + g) * D;
            memcpy(k_cache + off, k_new + src, (size_t)D * 2);
            memcpy(v_cache + off, v_new + src, (size_t)D * 2);
        }
    }
    return 0;
}

/* Decode-step store: one new row per sequence at position seq_lens[b] - 1. */
int oracle_kv_append(const oracle_shape *s, const uint16_t *k_new, const uint16_t *v_new,
                     const int32_t *block_table, const int32_t *seq_lens,
                     const int32_t *head_ids, int32_t n_sel, int32_t num_blocks,
                     uint16_t *k_cache, uint16_t *v_cache)
{
    const int D = s->head_dim;
    for (int64_t b = 0; b < s->batch; ++b) {
        int64_t p = (int64_t)seq_lens[b] - 1;
        for (int j = 0; j < n_sel; ++j) {
            int g = head_ids[j];
            if (g < 0 || g >= s->n_kv_heads) return -1;
            int64_t off = row_offset(s, block_table, num_blocks, b, p, g);
            if (off < 0) continue;
            const int64_t src = (b * s->n_kv_heads + g) * D;
            memcpy(k_cache + off, k_new + src, (size_t)D * 2);
            memcpy(v_cache + off, v_new + src, (size_t)D * 2);
        }
    }
    return 0;
}

/*
 * Decode-step store for per-request head subsets (Section 4.2 / 5.2.1): the work is a list of
 * (sequence, KV head) pairs over a pool of single-head tiles, one block-table row per pair.
 * Pair p = (b, g) stores k_new[b][g][:] and v_new[b][g][:] at position seq_lens[b] - 1:
 *   tile = block_table[p][pos / block_size], element tile * kv_stride_block + (pos % block_size) * D.
 * Pairs whose sequence or head id is out of range, whose sequence is empty, whose position is
 * past the table row or whose tile id is outside [0, num_tiles) are skipped.
 */
int oracle_kv_append_pairs(const oracle_shape *s, const uint16_t *k_new, const uint16_t *v_new,
                           const int32_t *block_table, const int32_t *seq_lens,
                           const int32_t *pair_seq, const int32_t *pair_head, int32_t n_pairs,
                           int32_t num_tiles, uint16_t *k_tiles, uint16_t *v_tiles)
{
    const int D = s->head_dim;
    for (int64_t p = 0; p < n_pairs; ++p) {
        int64_t b = pair_seq[p], g = pair_head[p];
        if (b < 0 || b >= s->batch || g < 0 || g >= s->n_kv_heads) continue;
        int64_t pos = (int64_t)seq_lens[b] - 1;
        if (pos < 0 || pos / s->block_size >= s->max_blocks_per_seq) continue;
        int64_t tile = block_table[p * s->max_blocks_per_seq + pos / s->block_size];
        if (tile < 0 || tile >= num_tiles) continue;
        const int64_t dst = tile * s->kv_stride_block + (pos % s->block_size) * D;
        const int64_t src = (b * s->n_kv_heads + g) * D;
        memcpy(k_tiles + dst, k_new + src, (size_t)D * 2);
        memcpy(v_tiles + dst, v_new + src, (size_t)D * 2);
    }
    return 0;
}

/* Fetch: the inverse gather, k_out[n][g][:] = K[row(seq[n], pos[n], g)]; skipped entries and
 * rows of heads that are not selected stay as they were. */
int oracle_kv_fetch(const oracle_shape *s, const uint16_t *k_cache, const uint16_t *v_cache,
                    const int32_t *token_seq, const int32_t *token_pos, int32_t n_tokens,
                    const int32_t *block_table, const int32_t *head_ids, int32_t n_sel,
                    int32_t num_blocks, uint16_t *k_out, uint16_t *v_out)
{
    const int D = s->head_dim;
    for (int64_t n = 0; n < n_tokens; ++n) {
        int64_t b = token_seq ? token_seq[n] : n;
        for (int j = 0; j < n_sel; ++j) {
            int g = head_ids[j];
            if (g < 0 || g >= s->n_kv_heads) return -1;
            int64_t off = row_offset(s, block_table, num_blocks, b, token_pos[n], g);
            if (off < 0) continue;
            const int64_t dst = (n * s->n_kv_heads + g) * D;
            memcpy(k_out + dst, k_cache + off, (size_t)D * 2);
            memcpy(v_out + dst, v_cache + off, (size_t)D * 2);
        }
    }
    return 0;
}

/*
 * Tile copy: for every pair i and every head pair j,
 *   dst[dst_blocks[i]][dst_heads[j]] = src[src_blocks[i]][src_heads[j]]   (block_size x D rows),
 * for K and for V.  A pair with a block outside its pool is skipped.
 */
int oracle_kv_copy_tiles(const oracle_pool *sp, const uint16_t *src_k, const uint16_t *src_v,
                         const oracle_pool *dp, uint16_t *dst_k, uint16_t *dst_v,
                         const int32_t *src_blocks, const int32_t *dst_blocks, int32_t n_pairs,
                         const int32_t *src_heads, const int32_t *dst_heads, int32_t n_sel)
{
    if (sp->head_dim != dp->head_dim || sp->block_size != dp->block_size) return -1;
    const size_t tile = (size_t)sp->block_size * sp->head_dim;
    for (int64_t i = 0; i < n_pairs; ++i) {
        int64_t sb = src_blocks[i], db = dst_blocks[i];
        if (sb < 0 || sb >= sp->num_blocks || db < 0 || db >= dp->num_blocks) continue;
        for (int j = 0; j < n_sel; ++j) {
            int sg = src_heads[j], dg = dst_heads[j];
            if (sg < 0 || sg >= sp->n_kv_heads || dg < 0 || dg >= dp->n_kv_heads) return -1;
            const int64_t so = sb * sp->kv_stride_block + (int64_t)sg * sp->kv_stride_head;
            const int64_t dof = db * dp->kv_stride_block + (int64_t)dg * dp->kv_stride_head;
            memcpy(dst_k + dof, src_k + so, tile * 2);
            memcpy(dst_v + dof, src_v + so, tile * 2);
        }
    }
    return 0;
}
