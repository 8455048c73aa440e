/*
 * CPU checker for head-subset decode Attention over a block-paged fp16 KV cache.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain fp64 statement of
 * what the GPU library must compute.  It shares no code with the HIP path and
 * must never be called from it; only the tests, the smoke check and the
 * benchmark's cpu_baseline leg load it.
 *
 * What is computed (Section 4.2, Eq. (2a)/(2b)): for every sequence b and
 * every attention head that lives on this device,
 *     result = softmax( q_h . K_h^T * scale ) . V_h
 * with one query row per sequence (decode phase, Section 5.1: only the last
 * token's query attends to the stored keys and values), heads independent of
 * each other (Section 6, "Attention computation": no softmax state crosses
 * heads), and K/V read through a block table from fixed-size blocks that are
 * split again on the head dimension (Section 6, "KV cache management").
 *
 * Readings where the paper is silent:
 *   - "d" under the square root is the head dimension; the factor is passed in
 *     as `scale`.
 *   - the current token's K/V are already in the cache and seq_lens counts it;
 *     the only mask is t < L_b.
 *   - grouped-query models: query head h reads KV head h / r, r = Hq / Hkv
 *     (contiguous groups); head_ids name KV heads, so whole groups are selected.
 *   - q and out are indexed by the global query head: [B, Hq, D].
 *   - a sequence of length 0 yields zeros.
 *
 * All arithmetic is fp64 on the exact values of the fp16 inputs.  Rows of
 * heads that are not selected are never written.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* IEEE binary16 bit pattern -> double, exact (normals, subnormals, inf, NaN). */
double oracle_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);                 /* subnormal or zero */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(f | 0x400), e - 25);    /* (1 + f/1024) * 2^(e-15) */
    return sign ? -v : v;
}

typedef struct {
    int32_t batch, n_q_heads, n_kv_heads, head_dim, block_size, max_blocks_per_seq;
    int64_t kv_stride_block, kv_stride_head;       /* in elements */
} oracle_shape;

static const uint16_t *tile_row(const uint16_t *cache, const oracle_shape *s,
                                const int32_t *bt_row, int g, int t)
{
    int64_t blk = bt_row[t / s->block_size];
    int slot = t % s->block_size;
    return cache + blk * s->kv_stride_block + (int64_t)g * s->kv_stride_head
                 + (int64_t)slot * s->head_dim;
}

/*
 * Eq. (2b) for one (sequence, query head) over tokens [t0, t1).
 * Writes sum_t p_t V_t / Z into o[D] and, if lse != NULL, m + ln Z into *lse,
 * where m = max_t s_t, p_t = exp(s_t - m), Z = sum_t p_t.  Needs t1 > t0.
 */
static void attend_range(const oracle_shape *s, const uint16_t *qrow, const uint16_t *k,
                         const uint16_t *v, const int32_t *bt_row, int g, int t0, int t1,
                         double scale, double *o, double *lse, double *score)
{
    int D = s->head_dim;
    double m = -INFINITY;
    for (int t = t0; t < t1; ++t) {
        const uint16_t *kr = tile_row(k, s, bt_row, g, t);
        double acc = 0.0;
        for (int d = 0; d < D; ++d)
            acc += oracle_half_to_double(qrow[d]) * oracle_half_to_double(kr[d]);
        score[t - t0] = acc * scale;
        if (score[t - t0] > m) m = score[t - t0];
    }
    double Z = 0.0;
    for (int d = 0; d < D; ++d) o[d] = 0.0;
    for (int t = t0; t < t1; ++t) {
        double p = exp(score[t - t0] - m);
        Z += p;
        const uint16_t *vr = tile_row(v, s, bt_row, g, t);
        for (int d = 0; d < D; ++d)
            o[d] += p * oracle_half_to_double(vr[d]);
    }
    for (int d = 0; d < D; ++d) o[d] /= Z;
    if (lse) *lse = m + log(Z);
}

/*
 * Decode Attention for the selected KV heads of every sequence (Eq. (2b)).
 *   q        : fp16 bits [B, Hq, D]
 *   k, v     : fp16 bits, tile (block, head) at block*stride_block + head*stride_head,
 *              rows of D contiguous elements, block_size rows per tile
 *   out      : double [B, Hq, D]; only rows of selected heads are written
 * Returns 0, or -1 on allocation failure.
 */
int oracle_attn_decode(const oracle_shape *s, const uint16_t *q, const uint16_t *k,
                       const uint16_t *v, const int32_t *block_table, const int32_t *seq_lens,
                       const int32_t *head_ids, int32_t n_sel_heads, double scale, double *out,
                       int32_t n_threads)
{
    int r = s->n_q_heads / s->n_kv_heads;
    int D = s->head_dim;
    int64_t n_items = (int64_t)s->batch * n_sel_heads;
    int fail = 0;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#endif
    (void)n_threads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t it = 0; it < n_items; ++it) {
        int b = (int)(it / n_sel_heads);
        int g = head_ids[it % n_sel_heads];
        int L = seq_lens[b];
        const int32_t *bt_row = block_table + (int64_t)b * s->max_blocks_per_seq;
        double *score = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
        if (!score) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        for (int h = g * r; h < g * r + r; ++h) {
            double *o = out + ((int64_t)b * s->n_q_heads + h) * D;
            if (L <= 0) {
                for (int d = 0; d < D; ++d) o[d] = 0.0;
                continue;
            }
            const uint16_t *qrow = q + ((int64_t)b * s->n_q_heads + h) * D;
            attend_range(s, qrow, k, v, bt_row, g, 0, L, scale, o, NULL, score);
        }
        free(score);
    }
    return fail ? -1 : 0;
}

/*
 * Per-request head subsets (Section 4.2: the heads h_j^i of request j on device i are chosen
 * per request; Section 5.2.1 dispatches x_i^j heads of request j to device i).  The work is a
 * list of (sequence, KV head) pairs; the cache is a pool of single-head tiles (Section 6:
 * blocks split on the head dimension) and every pair has its own block-table row:
 *   pair p = (b, g) = (pair_seq[p], pair_head[p]);
 *   token t of the pair lives in tile block_table[p][t / block_size], row t % block_size,
 *   at element tile * kv_stride_block + (t % block_size) * D   (kv_stride_head is not used).
 * For every pair, the r query heads of group g of sequence b get Eq. (2b) over the L_b
 * tokens; rows no pair names are not written.
 */
int oracle_attn_decode_pairs(const oracle_shape *s, const uint16_t *q, const uint16_t *k_tiles,
                             const uint16_t *v_tiles, const int32_t *block_table,
                             const int32_t *seq_lens, const int32_t *pair_seq,
                             const int32_t *pair_head, int32_t n_pairs, double scale,
                             double *out)
{
    int r = s->n_q_heads / s->n_kv_heads;
    int D = s->head_dim;
    int fail = 0;
    oracle_shape tiles = *s;
    tiles.kv_stride_head = 0;               /* a tile holds one head: no head term in the address */
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t p = 0; p < n_pairs; ++p) {
        int b = pair_seq[p];
        int g = pair_head[p];
        int L = seq_lens[b];
        const int32_t *bt_row = block_table + p * s->max_blocks_per_seq;
        /* scores, then one result row: a row is finished in private memory and copied out
         * whole, so that a pair listed twice never exposes a half-written row */
        double *score = (double *)malloc(sizeof(double) * (size_t)((L > 0 ? L : 1) + D));
        if (!score) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        for (int h = g * r; h < g * r + r; ++h) {
            double *o = out + ((int64_t)b * s->n_q_heads + h) * D;
            double *row = score + (L > 0 ? L : 1);
            if (L <= 0) {
                for (int d = 0; d < D; ++d) row[d] = 0.0;
            } else {
                const uint16_t *qrow = q + ((int64_t)b * s->n_q_heads + h) * D;
                attend_range(&tiles, qrow, k_tiles, v_tiles, bt_row, g, 0, L, scale, row, NULL,
                             score);
            }
#pragma omp critical(oracle_pairs_row)
            memcpy(o, row, sizeof(double) * (size_t)D);
        }
        free(score);
    }
    return fail ? -1 : 0;
}

/*
 * Split-KV partials (an exact intra-device decomposition of Eq. (2b) along the
 * token axis; not part of the paper, which only splits on heads).  Chunk c of
 * sequence b covers tokens [c*chunk, min((c+1)*chunk, L_b)).  For every
 * selected row j = i*r + (h - g*r) (i = position of g in head_ids):
 *   o_partial  : double [B, n_sel*r, max_chunks, D]  = sum p v / Z_c   (normalised)
 *   lse_partial: double [B, n_sel*r, max_chunks]     = m_c + ln Z_c    (natural log)
 * Chunks with c >= ceil(L_b / chunk) are not written.
 */
int oracle_attn_partial(const oracle_shape *s, const uint16_t *q, const uint16_t *k,
                        const uint16_t *v, const int32_t *block_table, const int32_t *seq_lens,
                        const int32_t *head_ids, int32_t n_sel_heads, double scale,
                        int32_t chunk_tokens, int32_t max_chunks, double *o_partial,
                        double *lse_partial)
{
    int r = s->n_q_heads / s->n_kv_heads;
    int D = s->head_dim;
    int rows = n_sel_heads * r;
    double *score = (double *)malloc(sizeof(double) * (size_t)chunk_tokens);
    if (!score) return -1;
    for (int b = 0; b < s->batch; ++b) {
        int L = seq_lens[b];
        const int32_t *bt_row = block_table + (int64_t)b * s->max_blocks_per_seq;
        int n_chunks = (L + chunk_tokens - 1) / chunk_tokens;
        for (int i = 0; i < n_sel_heads; ++i) {
            int g = head_ids[i];
            for (int rr = 0; rr < r; ++rr) {
                int h = g * r + rr;
                int j = i * r + rr;
                const uint16_t *qrow = q + ((int64_t)b * s->n_q_heads + h) * D;
                for (int c = 0; c < n_chunks && c < max_chunks; ++c) {
                    int t0 = c * chunk_tokens;
                    int t1 = t0 + chunk_tokens < L ? t0 + chunk_tokens : L;
                    int64_t idx = ((int64_t)b * rows + j) * max_chunks + c;
                    attend_range(s, qrow, k, v, bt_row, g, t0, t1, scale,
                                 o_partial + idx * D, lse_partial + idx, score);
                }
            }
        }
    }
    free(score);
    return 0;
}

/*
 * Log-sum-exp merge of the partials above, ascending chunk order:
 *   M = max_c lse_c,  w_c = exp(lse_c - M),  out = sum_c w_c o_c / sum_c w_c.
 * out: double [B, Hq, D], selected rows only; L_b = 0 gives zeros.
 */
int oracle_attn_merge(const oracle_shape *s, const double *o_partial, const double *lse_partial,
                      const int32_t *seq_lens, const int32_t *head_ids, int32_t n_sel_heads,
                      int32_t chunk_tokens, int32_t max_chunks, double *out)
{
    int r = s->n_q_heads / s->n_kv_heads;
    int D = s->head_dim;
    int rows = n_sel_heads * r;
    for (int b = 0; b < s->batch; ++b) {
        int L = seq_lens[b];
        int n_chunks = (L + chunk_tokens - 1) / chunk_tokens;
        if (n_chunks > max_chunks) return -2;
        for (int i = 0; i < n_sel_heads; ++i) {
            for (int rr = 0; rr < r; ++rr) {
                int h = head_ids[i] * r + rr;
                int j = i * r + rr;
                double *o = out + ((int64_t)b * s->n_q_heads + h) * D;
                for (int d = 0; d < D; ++d) o[d] = 0.0;
                if (n_chunks == 0) continue;
                int64_t base = ((int64_t)b * rows + j) * max_chunks;
                double M = -INFINITY, W = 0.0;
                for (int c = 0; c < n_chunks; ++c)
                    if (lse_partial[base + c] > M) M = lse_partial[base + c];
                for (int c = 0; c < n_chunks; ++c) {
                    double w = exp(lse_partial[base + c] - M);
                    W += w;
                    for (int d = 0; d < D; ++d)
                        o[d] += w * o_partial[(base + c) * D + d];
                }
                for (int d = 0; d < D; ++d) o[d] /= W;
            }
        }
    }
    return 0;
}

/* Number of threads the OpenMP runtime will use for oracle_attn_decode. */
int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
