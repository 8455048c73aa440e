// Shared device helpers and launch parameters of the decode-Attention kernels (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace hetis {

constexpr int kBlockTokens = 16;          // tokens per cache block
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kLog2e = 1.4426950408889634f;
// Finite stand-in for "no token seen yet": keeps exp2(m_old - m_new) free of inf - inf.
constexpr float kNegBig = -1.0e30f;

struct AttnParams {
    const __half *q;            // [B, Hq, D]
    const __half *k_cache;
    const __half *v_cache;
    const int32_t *block_table; // [B, max_blocks_per_seq]
    const int32_t *seq_lens;    // [B]
    const int32_t *head_ids;    // [n_sel]
    // Per-request head subsets: row b of the enumeration is the pair (pair_seq[b], pair_head[b])
    // with its own block-table row b over a pool of single-head tiles; n_sel is 1 and head_ids
    // is unused.  Both null: every sequence uses the common head_ids.
    const int32_t *pair_seq;    // [batch] or nullptr
    const int32_t *pair_head;   // [batch] or nullptr
    // Decode step with the store folded in: the new token's K and V rows [B, Hkv, D] of the
    // selected heads are written to position seq_lens[b] - 1 of the cache by the kernel itself
    // before it reads that position.  Both null: the cache is only read.
    const __half *k_new;
    const __half *v_new;
    __half *out;                // [B, Hq, D]
    float *o_partial;           // [rows, n_sel, max_segs, r, D]
    float *lse_partial;         // [rows, n_sel, max_segs, r]
    int64_t stride_block;       // elements
    int64_t stride_head;        // elements
    int32_t n_q_heads;
    int32_t n_sel;
    int32_t max_blocks_per_seq;
    int32_t chunk_tokens;       // tokens one wave processes at a time: multiple of 16, <= 1024
    int32_t seg_tokens;         // tokens whose result leaves a workgroup as one (partial) result:
                                // a multiple of chunk_tokens, at most 32 chunks
    int32_t max_segs;           // partial-result slots per row in the partial buffers
    int32_t direct_single;      // 1: a row of <= 1 segment is written to `out` by the chunk kernel
    int32_t mode;               // kModeSegments / kModeSplit / kModeSpread
    int32_t part_stride;        // kModeSpread: slots per segment (chunk c of segment j of a row
                                // uses slot j * part_stride + c); otherwise 1
    unsigned int *control;      // device words of the call's workspace (see kCtl* below)
    unsigned int *arrivals;     // [rows * n_sel] segments of a row whose partial results are stored,
                                // zero between launches; nullptr: partial results are left for a
                                // separate merge (the split-KV entry points)
    float scale_log2;           // scale * log2(e): scores are kept in the base-2 domain
};

// How the work of a launch is cut for scheduling.  The arithmetic of a row is the same in
// kModeSegments and kModeSpread.
//   kModeSegments: a workgroup takes whole segments and folds their chunks in LDS.
//   kModeSplit:    seg_tokens == chunk_tokens; every chunk leaves as a partial result in the
//                  caller's buffers (natural-log log-sum-exp), merged by a separate launch.
//   kModeSpread:   for launches with few rows: a wave takes single chunks wherever they are,
//                  so the chunks of one segment run on many workgroups; chunk results go
//                  through the partial buffers and the wave that stores a row's last one
//                  folds them in the order and with the operations of kModeSegments.
enum : int { kModeSegments = 0, kModeSplit = 1, kModeSpread = 2 };

// Control words at the start of a call's workspace.  All are zero between launches: the last
// workgroup to leave a launch sets the first two back; kCtlError is sticky (only the host
// clears it) and records that a bounded wait inside a kernel expired, which means that the
// launch may have dropped or overwritten a result.  kCtlLastMode: 1 + the scheduling mode the
// last launch ran in (a statistic for tests and tuning; nothing reads it on the device).
enum : int { kCtlTickets = 0, kCtlGone = 1, kCtlError = 2, kCtlLastMode = 3 };
enum : unsigned { kErrWriterWait = 1u, kErrMailboxWait = 2u, kErrTicketWait = 4u };
constexpr int kControlBytes = 256;

__device__ __forceinline__ void report_error(unsigned int *control, unsigned flag)
{
    __hip_atomic_fetch_or(control + kCtlError, flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// Cross-lane move inside a row of 16 lanes (DPP), no LDS traffic.
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}

// Sum over aligned groups of LANES lanes (LANES = 8 or 16); every lane gets the total.
template <int LANES>
__device__ __forceinline__ float group_sum(float x)
{
    x += dpp_mov<0xB1>(x);    // quad_perm [1,0,3,2]
    x += dpp_mov<0x4E>(x);    // quad_perm [2,3,0,1]
    x += dpp_mov<0x141>(x);   // row_half_mirror: pairs the two quads of each 8 lanes
    if (LANES == 16) x += dpp_mov<0x140>(x);  // row_mirror: pairs the two halves of the row
    return x;
}

// Buffer descriptor covering exactly one (block, head) tile, or nothing.  With valid == false
// the descriptor spans 0 bytes: the hardware range check then makes every lane of a load
// return zeros without touching memory, while the instruction still takes its place in the
// in-order load counter.  This lets the tile ring issue every refill unconditionally, which
// keeps the compiler's wait counts exact (a load that is issued only on some paths forces
// full drains).
// The tile address and the validity flag are the same in every lane; they are passed through
// readfirstlane so that the descriptor provably sits in scalar registers (a descriptor the
// compiler believes to be lane-dependent is handled with a loop around every load).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_rsrc(const __half *tile, int tile_bytes,
                                                            bool valid)
{
    const uint64_t a = reinterpret_cast<uint64_t>(tile);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    const int nbytes = __builtin_amdgcn_readfirstlane(valid ? tile_bytes : 0);
    return __builtin_amdgcn_make_buffer_rsrc(
        reinterpret_cast<void *>(((uint64_t)hi << 32) | lo), 0, nbytes, 0x00020000);
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
// 16 bytes of a KV tile.  The load is marked non-temporal (cache-policy bit 1): every tile is
// read exactly once per call, and telling the caches so was worth 9 % of the kernel's time on
// this chip (measured with the cache rotated over three physical copies, so it is not reuse
// in the last-level cache).
constexpr int kStreamingLoad = 2;
__device__ __forceinline__ uint4 buffer_load_u4(__amdgpu_buffer_rsrc_t r, int byte_offset)
{
    const u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(r, byte_offset, 0, kStreamingLoad);
    return make_uint4(x.x, x.y, x.z, x.w);
}

// One word to / from device memory, coherent across the whole device (all XCDs): these
// accesses go past the per-XCD L2, so a word stored by one wave can be read by any other wave
// once the store has completed, without invalidating or writing back whole caches.
__device__ __forceinline__ void coherent_store(float *ptr, float v)
{
    __hip_atomic_store(ptr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float coherent_load(const float *ptr)
{
    return __hip_atomic_load(ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

union Pack16 {
    uint4 u;
    __half2 h2[4];
    __half h[8];
};

}  // namespace hetis
