/*
 * hetis_attn.h - C ABI of the MI355X (gfx950) head-subset decode-Attention library.
 *
 * The operation (Section 4.2, Eq. (2a)/(2b) of the Hetis paper): a device that
 * holds the KV cache of some attention heads computes, for every running
 * sequence b and every such head h,
 *         out[b, h, :] = softmax( scale * q[b, h, :] . K[b, :, kv(h), :]^T ) . V[b, :, kv(h), :]
 * over the L_b tokens stored so far (decode phase: one query row per sequence,
 * Section 5.1), and the per-device results are concatenated along the head
 * axis (Eq. (2a)); heads are independent, so no softmax state ever crosses
 * devices (Section 6, "Attention computation").  K and V live in fixed-size
 * blocks that are split again on the head dimension and are addressed by
 * (sequence, position, head) through a block table (Section 6, "KV cache
 * management").
 *
 * Conventions shared by every entry point
 *   - All data pointers are DEVICE pointers on the current HIP device unless
 *     marked "host".  The caller owns every buffer and keeps it alive until
 *     `stream` has passed the enqueued work.  Calls enqueue on `stream`
 *     (a hipStream_t passed as void*; NULL = the null stream) and return
 *     without synchronising.
 *   - fp16 = IEEE binary16.  q/out: [batch, n_q_heads, head_dim], indexed by the
 *     GLOBAL query head.  Only rows of selected heads are read / written.
 *   - Cache: the (block, kv head) tile starts at element
 *     block * kv_stride_block + head * kv_stride_head and holds block_size rows
 *     of head_dim contiguous fp16 (token-major inside the tile).  K and V use the
 *     same strides.  Tiles must be 16-byte aligned (strides multiples of 8).
 *   - block_table: int32 [batch, max_blocks_per_seq]; entry j of row b is the
 *     physical block of tokens [16 j, 16 j + 16).  Entries at or beyond
 *     ceil(seq_lens[b] / 16) are never read.  Slots past the end of a sequence
 *     inside its last block are loaded but never enter a result (they may hold
 *     NaN).
 *   - seq_lens: int32 [batch], number of cached tokens including the current
 *     one; 0 <= seq_lens[b] <= 16 * max_blocks_per_seq.  Length 0 gives zeros.
 *   - head_ids: int32 [n_sel_heads] KV-head ids in [0, n_kv_heads).  Selecting
 *     KV head g computes query heads g*r .. g*r + r - 1, r = n_q_heads /
 *     n_kv_heads (grouped-query models move whole groups, Section 5.2.1; for
 *     r = 1 these are plain head ids).  Duplicates are allowed and wasteful.
 *   - The work done for one (sequence, KV head) depends only on that sequence's
 *     length and on compile-time constants, never on n_sel_heads or on the grid:
 *     a head-subset call returns, bit for bit, the matching rows of the
 *     all-heads call.  No floating-point atomics are used; results are
 *     deterministic run to run.
 *   - Device-side contents (lengths, block ids, head ids) are NOT checked on the
 *     hot path; out-of-range values are undefined behaviour.  Use
 *     hetis_attn_validate in debug builds and tests.
 *   - Every function returns a status (0 = HETIS_OK, negative = error) and
 *     never throws, aborts or prints.  Argument errors are detected before any
 *     HIP call is made.
 *   - Memory.  The entry points whose names end in _ws take every byte of device
 *     memory they use from the caller: they allocate nothing, keep no state
 *     between calls and never synchronise, so they may be called under stream
 *     capture and on several streams at once (one workspace per stream).  The
 *     entry points without the suffix are the same calls run from a workspace
 *     that the library owns (see hetis_attn_decode).
 *   - Workspace.  A workspace is a 256-byte aligned device buffer whose first
 *     HETIS_ATTN_CONTROL_BYTES are control words (work tickets and an error
 *     word); the rest holds fp32 partial results whose contents mean nothing
 *     between calls.  The control words must be zero before the first call
 *     (hetis_attn_workspace_init, or any zero fill); every launch leaves them at
 *     zero again, so one workspace serves any number of calls in stream order.
 *     (32-bit word 3 of a workspace records how the last launch handed out its
 *     work: 1 whole segments, 2 chunks of a split call, 3 single chunks; a
 *     statistic for tests and tuning.)
 *     Two launches that may run at the same time must not share a workspace.
 *
 * Supported: head_dim in {64, 128}; block_size 16; r in {1, 2, 4, 8}.
 */
#ifndef HETIS_ATTN_H
#define HETIS_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    HETIS_OK = 0,
    HETIS_ERR_NULL = -1,        /* a required pointer is NULL */
    HETIS_ERR_BAD_SHAPE = -2,   /* non-positive size, n_q_heads % n_kv_heads != 0, bad strides */
    HETIS_ERR_UNSUPPORTED = -3, /* head_dim, block_size, group size or chunk_tokens not supported */
    HETIS_ERR_BAD_HEADS = -4,   /* n_sel_heads outside [1, n_kv_heads] */
    HETIS_ERR_WORKSPACE = -5,   /* max_seq_len inconsistent with the shape / chunking; workspace too
                                   small, misaligned, or in need of growth during stream capture */
    HETIS_ERR_LAUNCH = -6,      /* HIP reported an error when launching */
    HETIS_ERR_ALLOC = -7,       /* the internal workspace could not be allocated */
    HETIS_ERR_BAD_CONTENT = -8, /* hetis_attn_validate found an out-of-range value */
    HETIS_ERR_INFEASIBLE = -9,  /* hetis_dispatch_solve: the capacities cannot hold the requests */
    HETIS_ERR_DEVICE_WAIT = -10 /* hetis_attn_workspace_status: a bounded wait inside a kernel
                                   expired, results of that workspace's launches are suspect */
};

/* Bytes at the start of every workspace that hold control words. */
#define HETIS_ATTN_CONTROL_BYTES 256

typedef struct {
    int32_t batch;              /* B  > 0 */
    int32_t n_q_heads;          /* Hq > 0 */
    int32_t n_kv_heads;         /* Hkv > 0, Hq % Hkv == 0 */
    int32_t head_dim;           /* D: 64 or 128 */
    int32_t block_size;         /* 16 */
    int32_t max_blocks_per_seq; /* row stride of block_table, > 0 */
    int64_t kv_stride_block;    /* elements between blocks; 0 = Hkv * block_size * D */
    int64_t kv_stride_head;     /* elements between heads of a block; 0 = block_size * D */
} hetis_attn_shape;

/* Library version, major * 100 + minor. */
int hetis_attn_version(void);

/* Static, human-readable name of a status code (host pointer, never NULL). */
const char *hetis_attn_status_string(int status);

/*
 * Decode Attention for the selected heads (Eq. (2b)), one call = one layer of
 * one decode step for this device's head share.
 *   shape        host
 *   q            fp16 [B, Hq, D]
 *   k_cache      fp16 tiles as described above
 *   v_cache      fp16, same layout
 *   block_table  int32 [B, max_blocks_per_seq]
 *   seq_lens     int32 [B]
 *   head_ids     int32 [n_sel_heads]
 *   n_sel_heads  host, 1 .. Hkv
 *   scale        host, normally 1/sqrt(D)
 *   out          fp16 [B, Hq, D]; rows of unselected heads are left untouched
 * The tokens of a (sequence, head) are cut, from token 0, into segments of 4096
 * tokens and these into chunks (256 tokens for r < 4, 512 for r >= 4; a
 * sequence's last, shorter segment into finer ones); chunk results are
 * combined in ascending order into segment results, segment results into the
 * row.  The cut and the order depend on the sequence's length and these
 * constants only.  How the pieces are handed to the hardware does not change a
 * bit of the result: a call with 512 or more (sequence, selected head)
 * combinations hands out whole segments, whose chunks are combined on chip, so
 * that only segment results of sequences longer than 4096 tokens pass through
 * the workspace; a call with fewer hands out single chunks, whose results all
 * pass through the workspace, so that a few long sequences still occupy the
 * whole device.
 *
 * hetis_attn_decode_ws: the caller's workspace.  hetis_attn_decode_workspace_bytes(shape,
 *   n_sel_heads) is the size with which the call runs as described (it depends on batch,
 *   n_sel_heads, the group size, head_dim and max_blocks_per_seq only, and is NOT monotonic
 *   in n_sel_heads: size a workspace shared by calls with different head counts for each of
 *   them).  A call with few combinations that is given less hands out whole segments
 *   instead.  For that the control words (256 bytes) are enough when max_blocks_per_seq
 *   <= 256; otherwise it takes 256 + 4 * 2^18 bytes of counters plus, per (sequence,
 *   selected head), query head of the group and segment of the longest sequence the block
 *   table allows, head_dim + 1 floats (the head_dim part and the 1 part are separate areas,
 *   each rounded up to 256 bytes).  With less than that the call fails.
 *   Errors: NULL, BAD_SHAPE, UNSUPPORTED, BAD_HEADS, WORKSPACE (too small or not 256-byte
 *   aligned), LAUNCH.
 * hetis_attn_decode: convenience form of the same call on a workspace that the library
 *   owns, one per device.  It is allocated (hipMalloc) by the first call that needs it, by
 *   a later call that needs a larger one, or ahead of time by
 *   hetis_attn_reserve_workspace; a buffer that has been outgrown is kept until
 *   hetis_attn_release_workspace, so that a HIP graph captured earlier can still be
 *   replayed.  A call on a capturing stream never allocates: if the workspace is missing
 *   or too small it returns HETIS_ERR_WORKSPACE (reserve first, or use the _ws form).
 *   All calls on one device share the workspace: calls that may overlap (different
 *   streams, graphs replayed side by side) must use the _ws form with one workspace each.
 *   Errors: NULL, BAD_SHAPE, UNSUPPORTED, BAD_HEADS, WORKSPACE, ALLOC, LAUNCH.
 */
int hetis_attn_decode(const hetis_attn_shape *shape, const void *q, const void *k_cache,
                      const void *v_cache, const int32_t *block_table, const int32_t *seq_lens,
                      const int32_t *head_ids, int32_t n_sel_heads, float scale, void *out,
                      void *stream);
int hetis_attn_decode_ws(const hetis_attn_shape *shape, const void *q, const void *k_cache,
                         const void *v_cache, const int32_t *block_table,
                         const int32_t *seq_lens, const int32_t *head_ids, int32_t n_sel_heads,
                         float scale, void *out, void *workspace, size_t workspace_bytes,
                         void *stream);

/*
 * One decode step of this device's head share in one call (Section 5.1: the new token's key
 * and value are stored, then its query attends to all stored keys and values, its own
 * included): hetis_kv_append (hetis_kv.h) followed by hetis_attn_decode, in a single kernel.
 *   k_new, v_new  fp16 [B, Hkv, D]: the new token's rows, indexed by the model's KV head; the
 *                 rows of the heads in head_ids are written to position seq_lens[b] - 1 of
 *                 sequence b through the block table (seq_lens already counts the new token;
 *                 length 0 stores nothing); rows of other heads are not read
 *   k_cache, v_cache  read and written
 * The cache ends up as hetis_kv_append leaves it and `out` as hetis_attn_decode computes it on
 * that cache, bit for bit; unlike hetis_kv_append this call does not range-check what it reads
 * from device memory (use hetis_attn_validate).  A call that hands out whole segments stores
 * the rows inside the Attention kernel; one that hands out single chunks enqueues the store as
 * a launch of its own ahead of it.  Workspace rules as for hetis_attn_decode /
 * hetis_attn_decode_ws (same size).  Errors: those of hetis_attn_decode.
 */
int hetis_attn_decode_step(const hetis_attn_shape *shape, const void *q, const void *k_new,
                           const void *v_new, void *k_cache, void *v_cache,
                           const int32_t *block_table, const int32_t *seq_lens,
                           const int32_t *head_ids, int32_t n_sel_heads, float scale, void *out,
                           void *stream);
int hetis_attn_decode_step_ws(const hetis_attn_shape *shape, const void *q, const void *k_new,
                              const void *v_new, void *k_cache, void *v_cache,
                              const int32_t *block_table, const int32_t *seq_lens,
                              const int32_t *head_ids, int32_t n_sel_heads, float scale,
                              void *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * hetis_attn_decode for callers that cannot allocate device memory and have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same kernels and bit-identical results; the workspace is a static device
 * array of HETIS_ATTN_STATIC_SCRATCH_BYTES inside the library (each GPU the library runs on
 * holds it from the first use until the process ends).  The call makes no hipMalloc / hipFree
 * and uses no allocating routine; it enqueues one small clearing kernel and the Attention
 * kernels on `stream`.  The array plays the part of the caller's workspace of
 * hetis_attn_decode_ws: a call for which it is too small even when whole segments are handed
 * out is refused with HETIS_ERR_WORKSPACE before anything is launched.  All calls on one GPU
 * share that GPU's array: calls that may overlap (different streams) race; serialise them, or
 * use hetis_attn_decode_ws.  Errors: NULL, BAD_SHAPE, UNSUPPORTED, BAD_HEADS, WORKSPACE, LAUNCH.
 */
#define HETIS_ATTN_STATIC_SCRATCH_BYTES (32u << 20)
int hetis_attn_decode_static(const hetis_attn_shape *shape, const void *q, const void *k_cache,
                             const void *v_cache, const int32_t *block_table,
                             const int32_t *seq_lens, const int32_t *head_ids,
                             int32_t n_sel_heads, float scale, void *out, void *stream);

/* Workspace size in bytes (host out-pointer) of hetis_attn_decode_ws for this shape and
 * head count, and of hetis_attn_decode_pairs_ws for this shape and pair count (n_pairs >= 0). */
int hetis_attn_decode_workspace_bytes(const hetis_attn_shape *shape, int32_t n_sel_heads,
                                      size_t *bytes);
int hetis_attn_decode_pairs_workspace_bytes(const hetis_attn_shape *shape, int32_t n_pairs,
                                            size_t *bytes);

/* Zero-fills a workspace on `stream` with a kernel (no memset node, so the call can be
 * captured): needed once after allocation and after hetis_attn_workspace_status reported an
 * expired wait.  `bytes` a multiple of 16, at least HETIS_ATTN_CONTROL_BYTES; 256-byte
 * aligned.  Errors: NULL, WORKSPACE, LAUNCH. */
int hetis_attn_workspace_init(void *workspace, size_t bytes, void *stream);

/* Debug helper: synchronises `stream`, reads the workspace's error word into *flags (host,
 * may be NULL) and clears it on the device.  workspace == NULL means the library-owned
 * workspace of the current device (flags 0 if there is none).  Every wait inside the kernels
 * is a polling loop with an iteration bound, so that a wave always reaches its end; a wait
 * that ran into its bound sets a bit here (1: writer wave, 2: a result mailbox stayed full,
 * 4: the ticket pool stayed empty).  Returns HETIS_OK when the word is zero,
 * HETIS_ERR_DEVICE_WAIT otherwise (results written through this workspace since the last
 * check are suspect), or NULL / LAUNCH. */
int hetis_attn_workspace_status(void *workspace, void *stream, uint32_t *flags);

/* Library-owned workspace of the current device: make it at least `bytes` large now (so that
 * later calls, also under stream capture, find it), and free the workspaces of every device,
 * outgrown ones included (synchronises each device).  Both optional. */
int hetis_attn_reserve_workspace(size_t bytes);
int hetis_attn_release_workspace(void);

/*
 * Split-KV variant: the token axis of every sequence is cut into chunks of
 * chunk_tokens tokens starting at token 0 (an exact decomposition of Eq. (2b)
 * inside one device; the paper itself only splits on heads).  Chunk c of
 * sequence b covers tokens [c*chunk_tokens, min((c+1)*chunk_tokens, L_b)).
 *
 * hetis_attn_split_num_chunks: C_max = ceil(max_seq_len / chunk_tokens), or a
 *   negative status.  chunk_tokens must be a positive multiple of 16, at most 1024.
 * hetis_attn_split_workspace_bytes: sizes in bytes of the two partial buffers
 *   (host out-pointers; a status is returned, so that a bad argument is not mistaken for
 *   a size).
 */
int hetis_attn_split_num_chunks(int32_t max_seq_len, int32_t chunk_tokens);
int hetis_attn_split_workspace_bytes(const hetis_attn_shape *shape, int32_t n_sel_heads,
                                     int32_t max_seq_len, int32_t chunk_tokens,
                                     size_t *o_partial_bytes, size_t *lse_partial_bytes);

/*
 * Partial pass.  For the i-th selected KV head, chunk c and query head j = 0..r-1 of the
 * group (h = head_ids[i]*r + j), with m_c = max_t s_t, Z_c = sum_t exp(s_t - m_c):
 *   o_partial   fp32 [B, n_sel_heads, C_max, r, D]  = sum_t exp(s_t - m_c) V_t / Z_c
 *   lse_partial fp32 [B, n_sel_heads, C_max, r]     = m_c + ln Z_c   (natural log)
 * (the r rows of one chunk are adjacent, so a chunk's result is one contiguous run).
 * Entries of chunks c >= ceil(L_b / chunk_tokens) are not written.
 * max_seq_len (host) bounds every seq_lens[b]; it fixes C_max and the grid.
 * hetis_attn_decode_split_ws takes its control words from the caller: `control` is a
 * 256-byte aligned device buffer of HETIS_ATTN_CONTROL_BYTES, zeroed once (it is a
 * workspace with no partial area); hetis_attn_decode_split uses the control words of the
 * library-owned workspace (rules as for hetis_attn_decode).
 * Errors: as hetis_attn_decode, plus WORKSPACE when max_seq_len is not in
 * [1, 16 * max_blocks_per_seq].
 */
int hetis_attn_decode_split(const hetis_attn_shape *shape, const void *q, const void *k_cache,
                            const void *v_cache, const int32_t *block_table,
                            const int32_t *seq_lens, const int32_t *head_ids, int32_t n_sel_heads,
                            float scale, int32_t chunk_tokens, int32_t max_seq_len,
                            float *o_partial, float *lse_partial, void *stream);
int hetis_attn_decode_split_ws(const hetis_attn_shape *shape, const void *q, const void *k_cache,
                               const void *v_cache, const int32_t *block_table,
                               const int32_t *seq_lens, const int32_t *head_ids,
                               int32_t n_sel_heads, float scale, int32_t chunk_tokens,
                               int32_t max_seq_len, float *o_partial, float *lse_partial,
                               void *control, void *stream);

/*
 * Log-sum-exp merge of the partials, ascending chunk order, in fp32:
 *   M = max_c lse_c, w_c = exp(lse_c - M), out = fp16( sum_c w_c o_c / sum_c w_c ).
 * Only chunks c < ceil(L_b / chunk_tokens) are read; L_b = 0 writes zeros.
 *   out fp16 [B, Hq, D], selected rows only.
 */
int hetis_attn_merge(const hetis_attn_shape *shape, const float *o_partial,
                     const float *lse_partial, const int32_t *seq_lens, const int32_t *head_ids,
                     int32_t n_sel_heads, int32_t chunk_tokens, int32_t max_seq_len, void *out,
                     void *stream);

/*
 * Measurement hook.  After hetis_attn_profile_events(begin, end) with two hipEvent_t
 * (passed as void*, created by the caller with timing enabled), the next kernel that an
 * Attention entry point of this header dispatches on behalf of the SAME host thread (the
 * kernel that streams the KV cache in the decode calls, the merge kernel in hetis_attn_merge)
 * carries the pair: `begin` is stamped when that kernel begins to execute, `end` when it has
 * finished, so their difference is the kernel's duration as a profiler's kernel trace sees it.
 * The pair is used once; set it again before the next call.  A dispatch that carries events
 * costs a few microseconds more than a plain one, so time whole steps without the hook.  Pass
 * (NULL, NULL) to drop a pair that has not been used.  The state is per host thread.  Returns
 * HETIS_OK, or HETIS_ERR_NULL if exactly one is NULL.
 */
int hetis_attn_profile_events(void *begin, void *end);

/*
 * Debug helper, not for the hot path: copies seq_lens, head_ids and the used
 * part of block_table to the host (synchronises `stream`) and checks
 * 0 <= seq_lens[b] <= 16*max_blocks_per_seq, 0 <= head_ids[i] < Hkv and
 * 0 <= block id < num_blocks for every entry a call would read.
 * Returns HETIS_OK or HETIS_ERR_BAD_CONTENT (or an argument error).
 */
int hetis_attn_validate(const hetis_attn_shape *shape, const int32_t *block_table,
                        const int32_t *seq_lens, const int32_t *head_ids, int32_t n_sel_heads,
                        int64_t num_blocks, void *stream);

/*
 * Per-request head subsets (Section 4.2: the heads of request j that live on device i are
 * chosen per request; Section 5.2.1 dispatches x_i^j heads of request j to device i).  The
 * work is a list of (sequence, KV head) pairs, and the cache is a pool of single-head tiles
 * (Section 6: cache blocks split on the head dimension) with one block-table row per pair:
 *   pair_seq     int32 [n_pairs]  sequence of pair p, in [0, B)
 *   pair_head    int32 [n_pairs]  KV head of pair p, in [0, Hkv)
 *   block_table  int32 [n_pairs, max_blocks_per_seq]: entry j of row p is the tile that holds
 *                tokens [16 j, 16 j + 16) of (pair_seq[p], pair_head[p])
 *   k_tiles, v_tiles  fp16: tile t starts at element t * kv_stride_block (0 = 16 * D) and holds
 *                16 rows of D contiguous fp16; shape->kv_stride_head must be 0
 *   seq_lens     int32 [B]; q, out: fp16 [B, Hq, D] as in hetis_attn_decode
 * For every pair the r query heads of its group get Eq. (2b) over the sequence's tokens; rows
 * of `out` that no pair names are left untouched.  A (sequence, head) listed twice is computed
 * twice (same bytes written).  n_pairs = 0 is a no-op; at most 65535 pairs per call.
 * The arithmetic of a pair is that of hetis_attn_decode for the same sequence length: the
 * rows agree bit for bit with an all-heads run over the same tile contents.
 * hetis_attn_decode_pairs_ws runs from the caller's workspace
 * (hetis_attn_decode_pairs_workspace_bytes), hetis_attn_decode_pairs from the library-owned
 * one; the rules are those of hetis_attn_decode_ws / hetis_attn_decode.
 * Errors: NULL, BAD_SHAPE, UNSUPPORTED, WORKSPACE, ALLOC, LAUNCH.
 */
int hetis_attn_decode_pairs(const hetis_attn_shape *shape, const void *q, const void *k_tiles,
                            const void *v_tiles, const int32_t *block_table,
                            const int32_t *seq_lens, const int32_t *pair_seq,
                            const int32_t *pair_head, int32_t n_pairs, float scale, void *out,
                            void *stream);
int hetis_attn_decode_pairs_ws(const hetis_attn_shape *shape, const void *q, const void *k_tiles,
                               const void *v_tiles, const int32_t *block_table,
                               const int32_t *seq_lens, const int32_t *pair_seq,
                               const int32_t *pair_head, int32_t n_pairs, float scale, void *out,
                               void *workspace, size_t workspace_bytes, void *stream);

/*
 * One decode step of the pairs form in one call (Section 5.1): hetis_kv_append_pairs
 * (hetis_kv.h) followed by hetis_attn_decode_pairs.  k_new, v_new fp16 [B, Hkv, D]: pair p
 * stores the rows of (pair_seq[p], pair_head[p]) at position seq_lens[b] - 1 of its own
 * block-table row (length 0 stores nothing); k_tiles, v_tiles are read and written.  Pools
 * and `out` end up as the two calls leave them, bit for bit; what is read from device
 * memory is not range-checked (use hetis_attn_validate_pairs).  A (sequence, head) listed
 * twice with different block-table rows stores the rows through both.  Workspace rules,
 * sizes and errors as for hetis_attn_decode_pairs / hetis_attn_decode_pairs_ws.
 */
int hetis_attn_decode_pairs_step(const hetis_attn_shape *shape, const void *q, const void *k_new,
                                 const void *v_new, void *k_tiles, void *v_tiles,
                                 const int32_t *block_table, const int32_t *seq_lens,
                                 const int32_t *pair_seq, const int32_t *pair_head,
                                 int32_t n_pairs, float scale, void *out, void *stream);
int hetis_attn_decode_pairs_step_ws(const hetis_attn_shape *shape, const void *q, const void *k_new,
                                    const void *v_new, void *k_tiles, void *v_tiles,
                                    const int32_t *block_table, const int32_t *seq_lens,
                                    const int32_t *pair_seq, const int32_t *pair_head,
                                    int32_t n_pairs, float scale, void *out, void *workspace,
                                    size_t workspace_bytes, void *stream);

/* Debug helper like hetis_attn_validate for the pairs form: sequence ids, head ids, lengths
 * and every tile id a call would read (0 <= id < num_tiles). */
int hetis_attn_validate_pairs(const hetis_attn_shape *shape, const int32_t *block_table,
                              const int32_t *seq_lens, const int32_t *pair_seq,
                              const int32_t *pair_head, int32_t n_pairs, int64_t num_tiles,
                              void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HETIS_ATTN_H */
