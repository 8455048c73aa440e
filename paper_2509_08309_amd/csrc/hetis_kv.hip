// C ABI of the head-wise cache management kernels: argument checks and launches.
// Argument errors are reported before the first HIP call.
#include "../../include/hetis_kv.h"

#include <hip/hip_ext.h>

#include "kv_cache.hpp"

namespace hetis {

struct KvChecked {
    int64_t stride_block, stride_head;      // elements
};

static int check_kv_shape(const hetis_attn_shape *s, int32_t n_sel, KvChecked *c)
{
    if (!s) return HETIS_ERR_NULL;
    if (s->batch <= 0 || s->n_q_heads <= 0 || s->n_kv_heads <= 0 || s->head_dim <= 0 ||
        s->block_size <= 0 || s->max_blocks_per_seq <= 0)
        return HETIS_ERR_BAD_SHAPE;
    if (s->n_q_heads % s->n_kv_heads != 0) return HETIS_ERR_BAD_SHAPE;
    if (s->kv_stride_block < 0 || s->kv_stride_head < 0) return HETIS_ERR_BAD_SHAPE;
    if (s->head_dim != 64 && s->head_dim != 128) return HETIS_ERR_UNSUPPORTED;
    if (s->block_size != kKvBlockTokens) return HETIS_ERR_UNSUPPORTED;
    const int64_t tile = (int64_t)s->block_size * s->head_dim;
    c->stride_head = s->kv_stride_head ? s->kv_stride_head : tile;
    c->stride_block = s->kv_stride_block ? s->kv_stride_block : tile * s->n_kv_heads;
    if (c->stride_head % 8 != 0 || c->stride_block % 8 != 0) return HETIS_ERR_BAD_SHAPE;
    if (c->stride_head < tile) return HETIS_ERR_BAD_SHAPE;
    if (n_sel < 1 || n_sel > s->n_kv_heads) return HETIS_ERR_BAD_HEADS;
    return HETIS_OK;
}

static int check_pool(const hetis_kv_pool *pl, KvChecked *c)
{
    if (!pl) return HETIS_ERR_NULL;
    if (pl->n_kv_heads <= 0 || pl->head_dim <= 0 || pl->block_size <= 0 || pl->num_blocks <= 0)
        return HETIS_ERR_BAD_SHAPE;
    if (pl->kv_stride_block < 0 || pl->kv_stride_head < 0) return HETIS_ERR_BAD_SHAPE;
    if (pl->head_dim != 64 && pl->head_dim != 128) return HETIS_ERR_UNSUPPORTED;
    if (pl->block_size != kKvBlockTokens) return HETIS_ERR_UNSUPPORTED;
    const int64_t tile = (int64_t)pl->block_size * pl->head_dim;
    c->stride_head = pl->kv_stride_head ? pl->kv_stride_head : tile;
    c->stride_block = pl->kv_stride_block ? pl->kv_stride_block : tile * pl->n_kv_heads;
    if (c->stride_head % 8 != 0 || c->stride_block % 8 != 0) return HETIS_ERR_BAD_SHAPE;
    if (c->stride_head < tile) return HETIS_ERR_BAD_SHAPE;
    return HETIS_OK;
}

// Optional events attached to the kernel's dispatch (measurement hook, per host thread):
// start is stamped when the kernel begins to execute, stop when it has finished.
static thread_local hipEvent_t t_kv_begin = nullptr;
static thread_local hipEvent_t t_kv_end = nullptr;

template <class Kernel, class Params>
static int launch_kv(Kernel kernel, dim3 grid, hipStream_t st, const Params &p)
{
    if (t_kv_begin)
        hipExtLaunchKernelGGL(kernel, grid, dim3(256), 0, st, t_kv_begin, t_kv_end, 0, p);
    else
        kernel<<<grid, 256, 0, st>>>(p);
    return hipGetLastError() == hipSuccess ? HETIS_OK : HETIS_ERR_LAUNCH;
}

// Threads of one launch of the row kernel are spread over entries (x) and, while the grid
// is small, over the selected heads (y), so that a decode-step store of a few thousand rows
// still fills the device.
static int launch_rows(bool fetch, const hetis_attn_shape *s, const KvChecked &c, KvRowParams p,
                       hipStream_t st)
{
    const int D = s->head_dim;
    const int lanes_per_entry = 2 * D / 8;
    const int64_t threads = (int64_t)p.n_tokens * lanes_per_entry;
    const int64_t gx = (threads + 255) / 256;
    if (gx > 0x7fffffff) return HETIS_ERR_UNSUPPORTED;
    int64_t gy = (262144 + threads - 1) / threads;
    if (gy > p.n_sel) gy = p.n_sel;
    if (gy < 1) gy = 1;
    p.stride_block = c.stride_block / 8;
    p.stride_head = c.stride_head / 8;
    const dim3 grid((unsigned)gx, (unsigned)gy);
    if (D == 128)
        return fetch ? launch_kv(kv_rows_kernel<128, true>, grid, st, p)
                     : launch_kv(kv_rows_kernel<128, false>, grid, st, p);
    return fetch ? launch_kv(kv_rows_kernel<64, true>, grid, st, p)
                 : launch_kv(kv_rows_kernel<64, false>, grid, st, p);
}

static int rows_call(bool fetch, const hetis_attn_shape *shape, const void *rows_k,
                     const void *rows_v, const int32_t *token_seq, const int32_t *token_pos,
                     int32_t pos_bias, int64_t n_tokens, const int32_t *block_table,
                     const int32_t *head_ids, int32_t n_sel, int64_t num_blocks,
                     const void *cache_k, const void *cache_v, void *stream)
{
    KvChecked c;
    const int rc = check_kv_shape(shape, n_sel, &c);
    if (rc != HETIS_OK) return rc;
    if (n_tokens < 0 || n_tokens > 0x7fffffff || num_blocks <= 0) return HETIS_ERR_BAD_SHAPE;
    if (!token_seq && n_tokens > shape->batch) return HETIS_ERR_BAD_SHAPE;
    if (!rows_k || !rows_v || !token_pos || !block_table || !head_ids || !cache_k || !cache_v)
        return HETIS_ERR_NULL;
    if (n_tokens == 0) return HETIS_OK;
    KvRowParams p{};
    p.rows_k = (uint4 *)rows_k;
    p.rows_v = (uint4 *)rows_v;
    p.cache_k = (uint4 *)cache_k;
    p.cache_v = (uint4 *)cache_v;
    p.token_seq = token_seq;
    p.token_pos = token_pos;
    p.block_table = block_table;
    p.head_ids = head_ids;
    p.num_blocks = num_blocks;
    p.n_tokens = (int32_t)n_tokens;
    p.n_sel = n_sel;
    p.n_kv_heads = shape->n_kv_heads;
    p.batch = shape->batch;
    p.max_blocks_per_seq = shape->max_blocks_per_seq;
    p.pos_bias = pos_bias;
    return launch_rows(fetch, shape, c, p, (hipStream_t)stream);
}

}  // namespace hetis

using namespace hetis;

extern "C" {

int hetis_kv_append(const hetis_attn_shape *shape, const void *k_new, const void *v_new,
                    const int32_t *block_table, const int32_t *seq_lens,
                    const int32_t *head_ids, int32_t n_sel_heads, int64_t num_blocks,
                    void *k_cache, void *v_cache, void *stream)
{
    // position of the new row = seq_lens[b] - 1; a length of 0 gives -1 and is skipped
    return rows_call(false, shape, k_new, v_new, nullptr, seq_lens, -1,
                     shape ? shape->batch : 0, block_table, head_ids, n_sel_heads, num_blocks,
                     k_cache, v_cache, stream);
}

int hetis_kv_append_pairs(const hetis_attn_shape *shape, const void *k_new, const void *v_new,
                          const int32_t *block_table, const int32_t *seq_lens,
                          const int32_t *pair_seq, const int32_t *pair_head, int32_t n_pairs,
                          int64_t num_tiles, void *k_tiles, void *v_tiles, void *stream)
{
    KvChecked c;
    const int rc = check_kv_shape(shape, 1, &c);
    if (rc != HETIS_OK) return rc;
    if (n_pairs < 0 || num_tiles <= 0) return HETIS_ERR_BAD_SHAPE;
    // the pool holds single-head tiles: one stride, no head term
    const int64_t tile = (int64_t)shape->block_size * shape->head_dim;
    const int64_t stride = shape->kv_stride_block ? shape->kv_stride_block : tile;
    if (stride % 8 != 0 || stride < tile) return HETIS_ERR_BAD_SHAPE;
    if (!k_new || !v_new || !block_table || !seq_lens || !pair_seq || !pair_head || !k_tiles ||
        !v_tiles)
        return HETIS_ERR_NULL;
    if (n_pairs == 0) return HETIS_OK;
    KvPairParams p{};
    p.k_new = (const uint4 *)k_new;
    p.v_new = (const uint4 *)v_new;
    p.k_tiles = (uint4 *)k_tiles;
    p.v_tiles = (uint4 *)v_tiles;
    p.block_table = block_table;
    p.seq_lens = seq_lens;
    p.pair_seq = pair_seq;
    p.pair_head = pair_head;
    p.stride_tile = stride / 8;
    p.num_tiles = num_tiles;
    p.n_pairs = n_pairs;
    p.n_kv_heads = shape->n_kv_heads;
    p.batch = shape->batch;
    p.max_blocks_per_seq = shape->max_blocks_per_seq;
    const int64_t threads = (int64_t)n_pairs * (2 * shape->head_dim / 8);
    const dim3 grid((unsigned)((threads + 255) / 256));
    const hipStream_t st = (hipStream_t)stream;
    if (shape->head_dim == 128) return launch_kv(kv_append_pairs_kernel<128>, grid, st, p);
    return launch_kv(kv_append_pairs_kernel<64>, grid, st, p);
}

int hetis_kv_store(const hetis_attn_shape *shape, const void *k_new, const void *v_new,
                   const int32_t *token_seq, const int32_t *token_pos, int32_t n_tokens,
                   const int32_t *block_table, const int32_t *head_ids, int32_t n_sel_heads,
                   int64_t num_blocks, void *k_cache, void *v_cache, void *stream)
{
    return rows_call(false, shape, k_new, v_new, token_seq, token_pos, 0, n_tokens, block_table,
                     head_ids, n_sel_heads, num_blocks, k_cache, v_cache, stream);
}

int hetis_kv_fetch(const hetis_attn_shape *shape, const void *k_cache, const void *v_cache,
                   const int32_t *token_seq, const int32_t *token_pos, int32_t n_tokens,
                   const int32_t *block_table, const int32_t *head_ids, int32_t n_sel_heads,
                   int64_t num_blocks, void *k_out, void *v_out, void *stream)
{
    return rows_call(true, shape, k_out, v_out, token_seq, token_pos, 0, n_tokens, block_table,
                     head_ids, n_sel_heads, num_blocks, k_cache, v_cache, stream);
}

int hetis_kv_copy_tiles(const hetis_kv_pool *src_pool, const void *src_k, const void *src_v,
                        const hetis_kv_pool *dst_pool, void *dst_k, void *dst_v,
                        const int32_t *src_blocks, const int32_t *dst_blocks, int32_t n_pairs,
                        const int32_t *src_heads, const int32_t *dst_heads, int32_t n_sel_heads,
                        void *stream)
{
    KvChecked sc, dc;
    int rc = check_pool(src_pool, &sc);
    if (rc != HETIS_OK) return rc;
    rc = check_pool(dst_pool, &dc);
    if (rc != HETIS_OK) return rc;
    if (src_pool->head_dim != dst_pool->head_dim || src_pool->block_size != dst_pool->block_size)
        return HETIS_ERR_BAD_SHAPE;
    if (n_pairs < 0) return HETIS_ERR_BAD_SHAPE;
    if (n_sel_heads < 1 || n_sel_heads > 1024) return HETIS_ERR_BAD_HEADS;
    if (!src_k || !src_v || !dst_k || !dst_v || !src_blocks || !dst_blocks || !src_heads ||
        !dst_heads)
        return HETIS_ERR_NULL;
    if (n_pairs == 0) return HETIS_OK;
    KvCopyParams p{};
    p.src_k = (const uint4 *)src_k;
    p.src_v = (const uint4 *)src_v;
    p.dst_k = (uint4 *)dst_k;
    p.dst_v = (uint4 *)dst_v;
    p.src_blocks = src_blocks;
    p.dst_blocks = dst_blocks;
    p.src_heads = src_heads;
    p.dst_heads = dst_heads;
    p.src_stride_block = sc.stride_block / 8;
    p.src_stride_head = sc.stride_head / 8;
    p.dst_stride_block = dc.stride_block / 8;
    p.dst_stride_head = dc.stride_head / 8;
    p.src_num_blocks = src_pool->num_blocks;
    p.dst_num_blocks = dst_pool->num_blocks;
    p.n_items = (int64_t)n_pairs * n_sel_heads;
    p.n_sel = n_sel_heads;
    p.src_n_heads = src_pool->n_kv_heads;
    p.dst_n_heads = dst_pool->n_kv_heads;
    // 4 waves per workgroup, one item per wave and step; enough workgroups to fill every
    // wave slot of the device, no more than there are items
    int64_t wgs = (p.n_items + 3) / 4;
    if (wgs > kKvCopyMaxWorkgroups) wgs = kKvCopyMaxWorkgroups;
    const hipStream_t st = (hipStream_t)stream;
    if (src_pool->head_dim == 128)
        return launch_kv(kv_copy_tiles_kernel<128>, dim3((unsigned)wgs), st, p);
    return launch_kv(kv_copy_tiles_kernel<64>, dim3((unsigned)wgs), st, p);
}

int hetis_kv_profile_events(void *begin, void *end)
{
    if ((begin == nullptr) != (end == nullptr)) return HETIS_ERR_NULL;
    t_kv_begin = (hipEvent_t)begin;
    t_kv_end = (hipEvent_t)end;
    return HETIS_OK;
}

}  // extern "C"
