// C ABI of the head-subset decode-Attention library: argument checks, kernel choice, launches.
// Every argument error is reported before the first HIP call, so the checks can be
// exercised on a machine without a GPU.
#include "../../include/hetis_attn.h"
#include "../../include/hetis_kv.h"

#include <hip/hip_ext.h>

#include <algorithm>
#include <cstdlib>
#include <mutex>
#include <type_traits>
#include <vector>

#include "attn_mfma.hpp"
#include "attn_vec.hpp"

namespace hetis {

// Cut of the token axis in hetis_attn_decode.  Compile-time constants chosen by the query-group
// size only: how a row is cut must depend on its length and the model shape alone, or a
// head-subset call could not reproduce the all-heads call bit for bit.  A chunk is what one
// wave processes at a time; a segment is what leaves a workgroup as one result (rows of up to
// one segment never produce partial results in global memory).
#ifndef HETIS_DECODE_CHUNK_TOKENS
#define HETIS_DECODE_CHUNK_TOKENS 256
#endif
#ifndef HETIS_DECODE_CHUNK_TOKENS_GQA
#define HETIS_DECODE_CHUNK_TOKENS_GQA 512
#endif
#ifndef HETIS_DECODE_SEG_TOKENS
#define HETIS_DECODE_SEG_TOKENS 4096
#endif
#ifndef HETIS_DECODE_SEG_TOKENS_GQA
#define HETIS_DECODE_SEG_TOKENS_GQA 4096
#endif
constexpr int decode_chunk_tokens(int group)
{
    return group >= 4 ? HETIS_DECODE_CHUNK_TOKENS_GQA : HETIS_DECODE_CHUNK_TOKENS;
}
constexpr int decode_seg_tokens(int group)
{
    return group >= 4 ? HETIS_DECODE_SEG_TOKENS_GQA : HETIS_DECODE_SEG_TOKENS;
}
static_assert(HETIS_DECODE_SEG_TOKENS % HETIS_DECODE_CHUNK_TOKENS == 0 &&
              HETIS_DECODE_SEG_TOKENS_GQA % HETIS_DECODE_CHUNK_TOKENS_GQA == 0 &&
              HETIS_DECODE_SEG_TOKENS / HETIS_DECODE_CHUNK_TOKENS <= kMaxSegChunks &&
              HETIS_DECODE_SEG_TOKENS_GQA / HETIS_DECODE_CHUNK_TOKENS_GQA <= kMaxSegChunks,
              "a segment is a whole number of chunks, at most kMaxSegChunks");
static_assert(HETIS_DECODE_SEG_TOKENS > HETIS_DECODE_CHUNK_TOKENS &&
              HETIS_DECODE_SEG_TOKENS_GQA > HETIS_DECODE_CHUNK_TOKENS_GQA,
              "the decode path folds chunks inside a workgroup (the folded-in store relies on it)");
#ifndef HETIS_STREAM_WAVES
#define HETIS_STREAM_WAVES 4
#endif
constexpr int kVecWaves = HETIS_STREAM_WAVES;
constexpr int kWgsPerCu = 1;    // persistent workgroups per compute unit
// Rows (sequences, or pairs) per launch: what the persistent kernel's LDS tables hold.  Larger
// batches run as several launches over slices of the rows.
constexpr int kMaxPersistBatch = 2048;
static_assert(kMaxPersistBatch == kMaxRows, "the kernel's enumeration is laid out for this many rows");
// Arrival counters of a decode workspace (see the workspace layout below).
constexpr size_t kArrivalSlots = (size_t)1 << 18;
constexpr size_t kArrivalBytes = kArrivalSlots * sizeof(unsigned int);
constexpr int kMaxPersistHeads = 1024;
// A wave keeps the block ids of one chunk in one register (64 lanes).
constexpr int kMaxChunkTokens = 64 * kBlockTokens;

struct Checked {
    int group;          // r
    int64_t stride_block, stride_head;
};

static int check_shape(const hetis_attn_shape *s, int32_t n_sel, Checked *c)
{
    if (!s) return HETIS_ERR_NULL;
    if (s->batch <= 0 || s->n_q_heads <= 0 || s->n_kv_heads <= 0 || s->head_dim <= 0 ||
        s->block_size <= 0 || s->max_blocks_per_seq <= 0)
        return HETIS_ERR_BAD_SHAPE;
    if (s->n_q_heads % s->n_kv_heads != 0) return HETIS_ERR_BAD_SHAPE;
    if (s->kv_stride_block < 0 || s->kv_stride_head < 0) return HETIS_ERR_BAD_SHAPE;
    if (s->head_dim != 64 && s->head_dim != 128) return HETIS_ERR_UNSUPPORTED;
    if (s->block_size != kBlockTokens) return HETIS_ERR_UNSUPPORTED;
    const int r = s->n_q_heads / s->n_kv_heads;
    if (r != 1 && r != 2 && r != 4 && r != 8) return HETIS_ERR_UNSUPPORTED;
    if (s->batch > 65535 || s->n_kv_heads > kMaxPersistHeads) return HETIS_ERR_UNSUPPORTED;
    const int64_t tile = (int64_t)s->block_size * s->head_dim;
    c->group = r;
    c->stride_head = s->kv_stride_head ? s->kv_stride_head : tile;
    c->stride_block = s->kv_stride_block ? s->kv_stride_block : tile * s->n_kv_heads;
    if (c->stride_head % 8 != 0 || c->stride_block % 8 != 0) return HETIS_ERR_BAD_SHAPE;
    if (c->stride_head < tile) return HETIS_ERR_BAD_SHAPE;
    if (n_sel < 1 || n_sel > s->n_kv_heads) return HETIS_ERR_BAD_HEADS;
    if ((int64_t)n_sel > 65535) return HETIS_ERR_UNSUPPORTED;
    return HETIS_OK;
}

static int check_chunking(const hetis_attn_shape *s, int32_t chunk_tokens, int32_t max_seq_len)
{
    if (chunk_tokens <= 0 || chunk_tokens % kBlockTokens != 0 || chunk_tokens > kMaxChunkTokens)
        return HETIS_ERR_UNSUPPORTED;
    if (max_seq_len < 1 || (int64_t)max_seq_len > (int64_t)s->max_blocks_per_seq * kBlockTokens)
        return HETIS_ERR_WORKSPACE;
    return HETIS_OK;
}

// Number of compute units of the current device (cached per device).
static int device_cu_count()
{
    static std::mutex mu;
    static std::vector<int> cus;
    std::lock_guard<std::mutex> lock(mu);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if ((size_t)dev >= cus.size()) cus.resize(dev + 1, 0);
    if (cus[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return 0;
        cus[dev] = n;
    }
    return cus[dev];
}

// Resident workgroups per compute unit of a persistent-kernel instantiation, cached per
// (kernel, dynamic LDS bytes, device): the LDS size follows the batch, so a serving loop with
// a few recurring batch sizes asks the runtime once per size.
template <class Kernel>
static int resident_per_cu(Kernel kernel, int threads, size_t lds)
{
    struct Entry {
        const void *kernel;
        size_t lds;
        int dev, occ;
    };
    static std::mutex mu;
    static std::vector<Entry> cache;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    const void *key = reinterpret_cast<const void *>(kernel);
    std::lock_guard<std::mutex> lock(mu);
    for (const Entry &e : cache)
        if (e.kernel == key && e.lds == lds && e.dev == dev) return e.occ;
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, threads, lds) != hipSuccess || n < 1)
        return 0;
    if (cache.size() >= 256) cache.clear();
    cache.push_back(Entry{key, lds, dev, n});
    return n;
}

// Optional events attached to the dispatch of the chunk kernel (measurement hook, per host
// thread): start is stamped when the kernel begins to execute, stop when it has finished.
static thread_local hipEvent_t t_prof_begin = nullptr;
static thread_local hipEvent_t t_prof_end = nullptr;

template <class Kernel, class... Args>
static void launch_timed(Kernel kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st,
                         Args... args)
{
    if (t_prof_begin) {
        // one shot: the pair goes with the first dispatch after it was set
        hipEvent_t begin = t_prof_begin, end = t_prof_end;
        t_prof_begin = t_prof_end = nullptr;
        hipExtLaunchKernelGGL(kernel, grid, block, (std::uint32_t)lds, st, begin, end, 0, args...);
    } else {
        kernel<<<grid, block, lds, st>>>(args...);
    }
}

// One workgroup (NW streaming waves) per compute unit already keeps enough bytes in flight to
// saturate HBM; more only lengthens the tail.  HETIS_ATTN_WGS_PER_CU (optional, read once)
// overrides this, up to what fits.  It changes how items are spread over workgroups, never the
// arithmetic of an item.
static int wgs_per_cu_cap()
{
    static const int cap = [] {
        const char *e = std::getenv("HETIS_ATTN_WGS_PER_CU");
        const int v = e ? std::atoi(e) : 0;
        return v > 0 ? v : kWgsPerCu;
    }();
    return cap;
}

template <class Policy, bool PAIRS, int VARIANT>
static int launch_persistent(AttnParams p, int batch, hipStream_t st)
{
    constexpr int NW = kVecWaves;
    auto kernel = attn_chunk_persistent_kernel<Policy, NW, PAIRS, VARIANT>;
    const size_t lds = persist_lds_bytes<Policy, NW>(batch, p.n_sel, PAIRS);
    int occ = resident_per_cu(kernel, (NW + 1) * 64, lds);
    if (occ < 1) return HETIS_ERR_LAUNCH;
    const int cus = device_cu_count();
    if (cus <= 0) return HETIS_ERR_LAUNCH;
    if (occ > wgs_per_cu_cap()) occ = wgs_per_cu_cap();
    int64_t G = (int64_t)cus * occ;
    const int64_t most = (int64_t)batch * p.max_segs * p.n_sel;    // segments, at most
    if (G > most) G = most;
    launch_timed(kernel, dim3((unsigned)G), dim3((NW + 1) * 64), lds, st, p, batch);
    return HETIS_OK;
}

// Kernel choice depends on the shape only (never on the head subset): vector arithmetic for
// query groups of 1 or 2, MFMA for groups of 4 or 8.  `rows` is the number of rows of the
// enumeration: sequences, or (sequence, head) pairs in pairs mode.  More rows than one launch's
// tables hold run as several launches over slices of the rows, one after the other on the
// stream (they share the control words, which every launch leaves at zero); a row's arithmetic
// is the same wherever it runs.
template <int D, int R>
static int launch_chunk(const AttnParams &p0, int rows, hipStream_t st)
{
    const bool pairs = p0.pair_seq != nullptr;
    const int n_sel = pairs ? 1 : p0.n_sel;
    // the arrival counters are indexed by (row of the slice, head): a slice has no more
    // (row, head) combinations than there are counters
    const int slice = p0.arrivals ? std::min<int64_t>(kMaxPersistBatch, (int64_t)kArrivalSlots / n_sel)
                                  : kMaxPersistBatch;
    for (int row0 = 0; row0 < rows; row0 += slice) {
        const int n = std::min(slice, rows - row0);
        AttnParams p = p0;
        p.block_table += (int64_t)row0 * p.max_blocks_per_seq;
        const int64_t part0 = (int64_t)row0 * n_sel * p.max_segs * R;
        if (p.o_partial) p.o_partial += part0 * D;
        if (p.lse_partial) p.lse_partial += part0;
        if (pairs) {
            p.pair_seq += row0;
            p.pair_head += row0;
        } else {
            p.seq_lens += row0;
            p.q += (int64_t)row0 * p.n_q_heads * D;
            if (p.out) p.out += (int64_t)row0 * p.n_q_heads * D;
        }
        // the leanest instantiation that holds what this launch can need: the in-launch merge
        // when rows can leave partial results; the fixed second and third segments when the
        // launch may have few segments a workgroup (every row has at least one segment)
        const int64_t few_rows =
            (int64_t)HETIS_STATIC_SECOND_UPTO * std::max(device_cu_count(), 1) * wgs_per_cu_cap();
        const int variant = p.arrivals ? kVariantMerge
                                       : ((int64_t)n * n_sel <= few_rows ? kVariantFew : kVariantPlain);
        using Policy = std::conditional_t<(R >= 4), MfmaPolicy<D, R>, VecPolicy<D, R>>;
        int rc;
        if (pairs)
            rc = variant == kVariantMerge ? launch_persistent<Policy, true, kVariantMerge>(p, n, st)
                 : variant == kVariantFew ? launch_persistent<Policy, true, kVariantFew>(p, n, st)
                                          : launch_persistent<Policy, true, kVariantPlain>(p, n, st);
        else
            rc = variant == kVariantMerge ? launch_persistent<Policy, false, kVariantMerge>(p, n, st)
                 : variant == kVariantFew ? launch_persistent<Policy, false, kVariantFew>(p, n, st)
                                          : launch_persistent<Policy, false, kVariantPlain>(p, n, st);
        if (rc != HETIS_OK) return rc;
    }
    return HETIS_OK;
}

static int launch_chunks(const AttnParams &p, int D, int r, int rows, hipStream_t st)
{
#define HETIS_CASE(DD, RR) \
    if (D == DD && r == RR) return launch_chunk<DD, RR>(p, rows, st);
    HETIS_CASE(128, 1) HETIS_CASE(128, 2) HETIS_CASE(128, 4) HETIS_CASE(128, 8)
    HETIS_CASE(64, 1) HETIS_CASE(64, 2) HETIS_CASE(64, 4) HETIS_CASE(64, 8)
#undef HETIS_CASE
    return HETIS_ERR_UNSUPPORTED;
}

// `batch`: sequences, or pairs in pairs mode (p.n_sel is 1 there)
static void launch_merge(const AttnParams &p, int D, int r, int batch, hipStream_t st)
{
    dim3 grid(p.n_sel * r, batch);
    if (D == 128)
        launch_timed(attn_merge_kernel<128>, grid, dim3(128), 0, st, p, r);
    else
        launch_timed(attn_merge_kernel<64>, grid, dim3(64), 0, st, p, r);
}

// ---- workspaces.  Layout of a decode workspace (all offsets multiples of 256 bytes):
//   [0, kControlBytes)   control words (tickets drawn, workgroups finished, error word)
//   arrivals             uint32 [kArrivalSlots]: entry row * n_sel + head counts the partial
//                        results of that row that are stored.  The area has a fixed size so
//                        that it sits at the same place whatever the shape: calls of different
//                        shapes can then share one workspace, since no call's partial results
//                        ever land on another call's counters, and every launch leaves the
//                        counters it used at zero.
//   o_partial            fp32 [rows, n_sel, slots, r, D]
//   lse_partial          fp32 [rows, n_sel, slots, r]
// rows = sequences, or pairs in pairs mode (n_sel = 1 there).  Segment scheduling: slots =
// segments of the longest row the block table allows, and a shape whose rows fit one segment
// needs the control words only.  Spread scheduling (few rows): slots = chunks of the longest
// row, segment by segment.
// Launches with fewer rows (enumeration rows x selected heads) than this cut the work into
// single chunks instead of whole segments: with so few rows whole segments would leave most
// compute units without work.  Twice the number of compute units of the target.
#ifndef HETIS_SPREAD_BELOW_ROWS
#define HETIS_SPREAD_BELOW_ROWS 512
#endif
struct WsLayout {
    size_t arrivals = 0, o_partial = 0, lse_partial = 0, total = kControlBytes;
    size_t zeroed = kControlBytes;     // leading bytes this shape needs to be zero between launches
    int slots = 1;                     // partial-result slots per row
    int part_stride = 1;
    bool spread = false;
};
constexpr size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static int decode_max_segs(const hetis_attn_shape *s, int group)
{
    const int seg = decode_seg_tokens(group);
    const int64_t max_tokens = (int64_t)s->max_blocks_per_seq * kBlockTokens;
    return (int)((max_tokens + seg - 1) / seg);
}

// `spread`: lay the workspace out for spread scheduling.
static WsLayout decode_ws_layout(const hetis_attn_shape *s, int64_t rows, int n_sel, int group,
                                 bool spread)
{
    WsLayout w;
    const int max_segs = decode_max_segs(s, group);
    w.spread = spread;
    w.part_stride = spread ? decode_seg_tokens(group) / decode_chunk_tokens(group) : 1;
    w.slots = max_segs * w.part_stride;
    if (w.slots <= 1 || rows <= 0) return w;         // every row is written directly
    const size_t partial_rows = (size_t)rows * n_sel * group * w.slots;
    w.arrivals = kControlBytes;
    w.o_partial = kControlBytes + kArrivalBytes;
    // counters in use: one per (row, head) of a launch; spread scheduling: one more per segment
    w.zeroed = align256(w.arrivals + (size_t)std::min<int64_t>(rows, kMaxPersistBatch) * n_sel *
                                         (spread ? 1 + max_segs : 1) * sizeof(unsigned int));
    w.lse_partial = align256(w.o_partial + partial_rows * s->head_dim * sizeof(float));
    w.total = align256(w.lse_partial + partial_rows * sizeof(float));
    return w;
}

// Scheduling of a decode call over `rows` enumeration rows: spread when there are few rows and
// the workspace at hand (`have` bytes; SIZE_MAX: it will be made large enough) holds the chunk
// results, whole segments otherwise.  The choice never changes a result.
static WsLayout choose_layout(const hetis_attn_shape *s, int64_t rows, int n_sel, int group,
                              size_t have)
{
    if (rows * n_sel < HETIS_SPREAD_BELOW_ROWS) {
        const WsLayout w = decode_ws_layout(s, rows, n_sel, group, true);
        if (w.total <= have && w.zeroed <= kControlBytes + kArrivalBytes) return w;
    }
    return decode_ws_layout(s, rows, n_sel, group, false);
}

static int check_workspace(const void *ws, size_t have, size_t need)
{
    if (!ws) return HETIS_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0 || have < need) return HETIS_ERR_WORKSPACE;
    return HETIS_OK;
}

__global__ void zero_fill_kernel(uint4 *dst, size_t n16)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16;
         i += (size_t)gridDim.x * blockDim.x)
        dst[i] = make_uint4(0u, 0u, 0u, 0u);
}

static int zero_fill(void *ptr, size_t bytes, hipStream_t st)
{
    const size_t n16 = bytes / 16;
    const unsigned blocks = (unsigned)std::min<size_t>((n16 + 255) / 256, 2048);
    zero_fill_kernel<<<blocks, 256, 0, st>>>(static_cast<uint4 *>(ptr), n16);
    return hipGetLastError() == hipSuccess ? HETIS_OK : HETIS_ERR_LAUNCH;
}

// Library-owned workspace of the convenience entry points, one per device.  It only ever
// grows; a buffer that has been outgrown stays allocated until hetis_attn_release_workspace,
// because a HIP graph captured earlier holds its address.  Nothing is allocated on a
// capturing stream.
struct OwnedWs {
    void *ptr = nullptr;
    size_t bytes = 0;
    std::vector<void *> outgrown;
};
static std::mutex g_ws_mutex;
static std::vector<OwnedWs> g_ws;

static bool stream_is_capturing(hipStream_t st)
{
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &status) != hipSuccess) {
        (void)hipGetLastError();
        return true;      // e.g. the legacy stream while another stream captures: do not allocate
    }
    return status != hipStreamCaptureStatusNone;
}

// `st` == nullptr with `may_be_capturing` false: called outside any launch (reserve).
static int owned_workspace(size_t need, hipStream_t st, bool may_be_capturing, void **out)
{
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return HETIS_ERR_ALLOC;
    if ((size_t)dev >= g_ws.size()) g_ws.resize(dev + 1);
    OwnedWs &w = g_ws[dev];
    if (w.bytes < need) {
        if (may_be_capturing && stream_is_capturing(st)) return HETIS_ERR_WORKSPACE;
        const size_t want = align256(need + need / 4);
        void *ptr = nullptr;
        if (hipMalloc(&ptr, want) != hipSuccess) {
            (void)hipGetLastError();
            return HETIS_ERR_ALLOC;
        }
        // zero the whole buffer before its first use, in stream order with that use
        if (zero_fill(ptr, want, st) != HETIS_OK) {
            (void)hipFree(ptr);
            return HETIS_ERR_ALLOC;
        }
        if (!may_be_capturing && hipStreamSynchronize(st) != hipSuccess) {
            (void)hipGetLastError();
            (void)hipFree(ptr);
            return HETIS_ERR_ALLOC;
        }
        if (w.ptr) w.outgrown.push_back(w.ptr);
        w.ptr = ptr;
        w.bytes = want;
    }
    *out = w.ptr;
    return HETIS_OK;
}

// ---- static scratch of hetis_attn_decode_static: a workspace that exists from the moment the
// code object is loaded, so the entry point never allocates.  Every device the library runs on
// holds its own copy at its own address; `scratch` itself is only a host-side handle of the
// symbol and must never be passed to a kernel: host code uses the per-device address that
// hipGetSymbolAddress returned.
constexpr size_t kStaticScratchBytes = (size_t)HETIS_ATTN_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices];      // per device: address of its copy of `scratch`

// Device address of the current device's copy of `scratch` (looked up once per device, with
// that device current).
static int static_scratch(void **out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return HETIS_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return HETIS_ERR_LAUNCH;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return HETIS_OK;
}

static AttnParams make_params(const hetis_attn_shape *s, const Checked &c, const void *q,
                              const void *k, const void *v, const int32_t *bt,
                              const int32_t *sl, const int32_t *hid, int32_t n_sel, float scale,
                              void *out)
{
    AttnParams p{};
    p.q = (const __half *)q;
    p.k_cache = (const __half *)k;
    p.v_cache = (const __half *)v;
    p.block_table = bt;
    p.seq_lens = sl;
    p.head_ids = hid;
    p.out = (__half *)out;
    p.stride_block = c.stride_block;
    p.stride_head = c.stride_head;
    p.n_q_heads = s->n_q_heads;
    p.n_sel = n_sel;
    p.max_blocks_per_seq = s->max_blocks_per_seq;
    p.scale_log2 = scale * kLog2e;
    return p;
}

// Token cut, scheduling mode and workspace pointers of a decode call.
static void apply_layout(AttnParams &p, const WsLayout &lay, int group, void *workspace)
{
    p.chunk_tokens = decode_chunk_tokens(group);
    p.seg_tokens = decode_seg_tokens(group);
    p.max_segs = lay.slots;
    p.part_stride = lay.part_stride;
    p.mode = lay.spread ? kModeSpread : kModeSegments;
    p.direct_single = 1;
    unsigned char *base = static_cast<unsigned char *>(workspace);
    p.control = reinterpret_cast<unsigned int *>(base);
    if (lay.slots > 1) {
        // Rows cut into several pieces leave one partial result per piece; the wave that
        // stores a row's last one combines them, so there is no merge launch.
        p.o_partial = reinterpret_cast<float *>(base + lay.o_partial);
        p.lse_partial = reinterpret_cast<float *>(base + lay.lse_partial);
        p.arrivals = reinterpret_cast<unsigned int *>(base + lay.arrivals);
    }
}

}  // namespace hetis

using namespace hetis;

extern "C" {

int hetis_attn_version(void) { return 201; }

const char *hetis_attn_status_string(int status)
{
    switch (status) {
    case HETIS_OK: return "ok";
    case HETIS_ERR_NULL: return "null pointer argument";
    case HETIS_ERR_BAD_SHAPE: return "bad shape";
    case HETIS_ERR_UNSUPPORTED: return "unsupported head_dim, block_size, group size or chunk_tokens";
    case HETIS_ERR_BAD_HEADS: return "n_sel_heads outside [1, n_kv_heads]";
    case HETIS_ERR_WORKSPACE:
        return "max_seq_len inconsistent with shape or chunking, or workspace too small, "
               "misaligned or in need of growth during stream capture";
    case HETIS_ERR_LAUNCH: return "kernel launch failed";
    case HETIS_ERR_ALLOC: return "internal workspace allocation failed";
    case HETIS_ERR_BAD_CONTENT: return "device-side argument content out of range";
    case HETIS_ERR_INFEASIBLE: return "capacities cannot hold the requests";
    case HETIS_ERR_DEVICE_WAIT: return "a bounded wait inside a kernel expired";
    default: return "unknown status";
    }
}

// Shared body of hetis_attn_decode / hetis_attn_decode_ws.  `workspace` == nullptr: take the
// library-owned one.
static int decode_common(const hetis_attn_shape *shape, const void *q, const void *k_new,
                         const void *v_new, bool step, const void *k_cache, const void *v_cache,
                         const int32_t *block_table, const int32_t *seq_lens,
                         const int32_t *head_ids, int32_t n_sel_heads, float scale, void *out,
                         void *workspace, size_t workspace_bytes, bool owned, void *stream)
{
    Checked c;
    if (!shape || !q || !k_cache || !v_cache || !block_table || !seq_lens || !head_ids || !out)
        return HETIS_ERR_NULL;
    if (step && (!k_new || !v_new)) return HETIS_ERR_NULL;
    int rc = check_shape(shape, n_sel_heads, &c);
    if (rc != HETIS_OK) return rc;
    const WsLayout lay = choose_layout(shape, shape->batch, n_sel_heads, c.group,
                                       owned ? SIZE_MAX : workspace_bytes);
    hipStream_t st = (hipStream_t)stream;
    if (owned)
        rc = owned_workspace(lay.total, st, true, &workspace);
    else
        rc = check_workspace(workspace, workspace_bytes, lay.total);
    if (rc != HETIS_OK) return rc;

    AttnParams p = make_params(shape, c, q, k_cache, v_cache, block_table, seq_lens, head_ids,
                               n_sel_heads, scale, out);
    apply_layout(p, lay, c.group, workspace);
    if (step) {
        if (lay.spread) {
            // single chunks are handed out without regard to which of them reads the new rows:
            // the store runs as a launch of its own ahead of the Attention launch
            rc = hetis_kv_append(shape, k_new, v_new, block_table, seq_lens, head_ids, n_sel_heads,
                                 INT64_MAX, const_cast<void *>(k_cache), const_cast<void *>(v_cache),
                                 stream);
            if (rc != HETIS_OK) return rc;
        } else {
            p.k_new = static_cast<const __half *>(k_new);
            p.v_new = static_cast<const __half *>(v_new);
        }
    }
    rc = launch_chunks(p, shape->head_dim, c.group, shape->batch, st);
    if (rc != HETIS_OK) return rc;
    return hipGetLastError() == hipSuccess ? HETIS_OK : HETIS_ERR_LAUNCH;
}

int hetis_attn_decode(const hetis_attn_shape *shape, const void *q, const void *k_cache,
                      const void *v_cache, const int32_t *block_table, const int32_t *seq_lens,
                      const int32_t *head_ids, int32_t n_sel_heads, float scale, void *out,
                      void *stream)
{
    return decode_common(shape, q, nullptr, nullptr, false, k_cache, v_cache, block_table, seq_lens,
                         head_ids, n_sel_heads, scale, out, nullptr, 0, true, stream);
}

int hetis_attn_decode_ws(const hetis_attn_shape *shape, const void *q, const void *k_cache,
                         const void *v_cache, const int32_t *block_table,
                         const int32_t *seq_lens, const int32_t *head_ids, int32_t n_sel_heads,
                         float scale, void *out, void *workspace, size_t workspace_bytes,
                         void *stream)
{
    if (!workspace) return HETIS_ERR_NULL;
    return decode_common(shape, q, nullptr, nullptr, false, k_cache, v_cache, block_table, seq_lens,
                         head_ids, n_sel_heads, scale, out, workspace, workspace_bytes, false, stream);
}

int hetis_attn_decode_step(const hetis_attn_shape *shape, const void *q, const void *k_new,
                           const void *v_new, void *k_cache, void *v_cache,
                           const int32_t *block_table, const int32_t *seq_lens,
                           const int32_t *head_ids, int32_t n_sel_heads, float scale, void *out,
                           void *stream)
{
    return decode_common(shape, q, k_new, v_new, true, k_cache, v_cache, block_table, seq_lens,
                         head_ids, n_sel_heads, scale, out, nullptr, 0, true, stream);
}

int hetis_attn_decode_step_ws(const hetis_attn_shape *shape, const void *q, const void *k_new,
                              const void *v_new, void *k_cache, void *v_cache,
                              const int32_t *block_table, const int32_t *seq_lens,
                              const int32_t *head_ids, int32_t n_sel_heads, float scale,
                              void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!workspace) return HETIS_ERR_NULL;
    return decode_common(shape, q, k_new, v_new, true, k_cache, v_cache, block_table, seq_lens,
                         head_ids, n_sel_heads, scale, out, workspace, workspace_bytes, false,
                         stream);
}

int hetis_attn_decode_static(const hetis_attn_shape *shape, const void *q, const void *k_cache,
                             const void *v_cache, const int32_t *block_table,
                             const int32_t *seq_lens, const int32_t *head_ids,
                             int32_t n_sel_heads, float scale, void *out, void *stream)
{
    Checked c;
    if (!shape || !q || !k_cache || !v_cache || !block_table || !seq_lens || !head_ids || !out)
        return HETIS_ERR_NULL;
    int rc = check_shape(shape, n_sel_heads, &c);
    if (rc != HETIS_OK) return rc;
    const WsLayout lay = choose_layout(shape, shape->batch, n_sel_heads, c.group, kStaticScratchBytes);
    if (lay.total > kStaticScratchBytes) return HETIS_ERR_WORKSPACE;   // before any HIP call
    void *ws = nullptr;
    rc = static_scratch(&ws);
    if (rc != HETIS_OK) return rc;
    // The array keeps what the last call left.  Partial results are always written before they
    // are read; the control words and arrival counters must start at zero, and although every
    // launch re-arms them, they are cleared here (with a kernel, so that the call can be captured) to make each
    // call independent of how an earlier one ended.
    rc = zero_fill(ws, lay.zeroed, (hipStream_t)stream);
    if (rc != HETIS_OK) return rc;
    return decode_common(shape, q, nullptr, nullptr, false, k_cache, v_cache, block_table, seq_lens,
                         head_ids, n_sel_heads, scale, out, ws, kStaticScratchBytes, false, stream);
}

int hetis_attn_decode_workspace_bytes(const hetis_attn_shape *shape, int32_t n_sel_heads,
                                      size_t *bytes)
{
    Checked c;
    if (!shape || !bytes) return HETIS_ERR_NULL;
    const int rc = check_shape(shape, n_sel_heads, &c);
    if (rc != HETIS_OK) return rc;
    *bytes = choose_layout(shape, shape->batch, n_sel_heads, c.group, SIZE_MAX).total;
    return HETIS_OK;
}

static int check_pairs(const hetis_attn_shape *shape, int32_t n_pairs, Checked *c)
{
    int rc = check_shape(shape, 1, c);
    if (rc != HETIS_OK) return rc;
    if (n_pairs < 0) return HETIS_ERR_BAD_SHAPE;
    if (n_pairs > 65535) return HETIS_ERR_UNSUPPORTED;
    // the pool holds single-head tiles: one stride, no head term
    const int64_t tile = (int64_t)shape->block_size * shape->head_dim;
    c->stride_block = shape->kv_stride_block ? shape->kv_stride_block : tile;
    if (c->stride_block % 8 != 0 || c->stride_block < tile) return HETIS_ERR_BAD_SHAPE;
    c->stride_head = 0;
    return HETIS_OK;
}

int hetis_attn_decode_pairs_workspace_bytes(const hetis_attn_shape *shape, int32_t n_pairs,
                                            size_t *bytes)
{
    Checked c;
    if (!shape || !bytes) return HETIS_ERR_NULL;
    const int rc = check_pairs(shape, n_pairs, &c);
    if (rc != HETIS_OK) return rc;
    *bytes = choose_layout(shape, n_pairs, 1, c.group, SIZE_MAX).total;
    return HETIS_OK;
}

static int decode_pairs_common(const hetis_attn_shape *shape, const void *q, const void *k_new,
                               const void *v_new, bool step, const void *k_tiles,
                               const void *v_tiles, const int32_t *block_table,
                               const int32_t *seq_lens, const int32_t *pair_seq,
                               const int32_t *pair_head, int32_t n_pairs, float scale, void *out,
                               void *workspace, size_t workspace_bytes, bool owned, void *stream)
{
    Checked c;
    if (!shape || !q || !k_tiles || !v_tiles || !block_table || !seq_lens || !pair_seq ||
        !pair_head || !out)
        return HETIS_ERR_NULL;
    if (step && (!k_new || !v_new)) return HETIS_ERR_NULL;
    int rc = check_pairs(shape, n_pairs, &c);
    if (rc != HETIS_OK) return rc;
    const WsLayout lay = choose_layout(shape, n_pairs, 1, c.group, owned ? SIZE_MAX : workspace_bytes);
    if (!owned) {
        rc = check_workspace(workspace, workspace_bytes, lay.total);
        if (rc != HETIS_OK) return rc;
    }
    if (n_pairs == 0) return HETIS_OK;
    hipStream_t st = (hipStream_t)stream;
    if (owned) {
        rc = owned_workspace(lay.total, st, true, &workspace);
        if (rc != HETIS_OK) return rc;
    }

    AttnParams p = make_params(shape, c, q, k_tiles, v_tiles, block_table, seq_lens, nullptr, 1,
                               scale, out);
    p.pair_seq = pair_seq;
    p.pair_head = pair_head;
    apply_layout(p, lay, c.group, workspace);
    if (step) {
        if (lay.spread) {
            // as in decode_common: the store runs as a launch of its own ahead of the Attention launch
            rc = hetis_kv_append_pairs(shape, k_new, v_new, block_table, seq_lens, pair_seq, pair_head,
                                       n_pairs, INT64_MAX, const_cast<void *>(k_tiles),
                                       const_cast<void *>(v_tiles), stream);
            if (rc != HETIS_OK) return rc;
        } else {
            p.k_new = static_cast<const __half *>(k_new);
            p.v_new = static_cast<const __half *>(v_new);
        }
    }
    rc = launch_chunks(p, shape->head_dim, c.group, n_pairs, st);
    if (rc != HETIS_OK) return rc;
    return hipGetLastError() == hipSuccess ? HETIS_OK : HETIS_ERR_LAUNCH;
}

int hetis_attn_decode_pairs(const hetis_attn_shape *shape, const void *q, const void *k_tiles,
                            const void *v_tiles, const int32_t *block_table,
                            const int32_t *seq_lens, const int32_t *pair_seq,
                            const int32_t *pair_head, int32_t n_pairs, float scale, void *out,
                            void *stream)
{
    return decode_pairs_common(shape, q, nullptr, nullptr, false, k_tiles, v_tiles, block_table,
                               seq_lens, pair_seq, pair_head, n_pairs, scale, out, nullptr, 0, true,
                               stream);
}

int hetis_attn_decode_pairs_ws(const hetis_attn_shape *shape, const void *q, const void *k_tiles,
                               const void *v_tiles, const int32_t *block_table,
                               const int32_t *seq_lens, const int32_t *pair_seq,
                               const int32_t *pair_head, int32_t n_pairs, float scale, void *out,
                               void *workspace, size_t workspace_bytes, void *stream)
{
    if (!workspace) return HETIS_ERR_NULL;
    return decode_pairs_common(shape, q, nullptr, nullptr, false, k_tiles, v_tiles, block_table,
                               seq_lens, pair_seq, pair_head, n_pairs, scale, out, workspace,
                               workspace_bytes, false, stream);
}

int hetis_attn_decode_pairs_step(const hetis_attn_shape *shape, const void *q, const void *k_new,
                                 const void *v_new, void *k_tiles, void *v_tiles,
                                 const int32_t *block_table, const int32_t *seq_lens,
                                 const int32_t *pair_seq, const int32_t *pair_head,
                                 int32_t n_pairs, float scale, void *out, void *stream)
{
    return decode_pairs_common(shape, q, k_new, v_new, true, k_tiles, v_tiles, block_table,
                               seq_lens, pair_seq, pair_head, n_pairs, scale, out, nullptr, 0, true,
                               stream);
}

int hetis_attn_decode_pairs_step_ws(const hetis_attn_shape *shape, const void *q, const void *k_new,
                                    const void *v_new, void *k_tiles, void *v_tiles,
                                    const int32_t *block_table, const int32_t *seq_lens,
                                    const int32_t *pair_seq, const int32_t *pair_head,
                                    int32_t n_pairs, float scale, void *out, void *workspace,
                                    size_t workspace_bytes, void *stream)
{
    if (!workspace) return HETIS_ERR_NULL;
    return decode_pairs_common(shape, q, k_new, v_new, true, k_tiles, v_tiles, block_table,
                               seq_lens, pair_seq, pair_head, n_pairs, scale, out, workspace,
                               workspace_bytes, false, stream);
}

int hetis_attn_workspace_init(void *workspace, size_t bytes, void *stream)
{
    if (!workspace) return HETIS_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0 || bytes < (size_t)kControlBytes ||
        bytes % 16 != 0)
        return HETIS_ERR_WORKSPACE;
    return zero_fill(workspace, bytes, (hipStream_t)stream);
}

int hetis_attn_workspace_status(void *workspace, void *stream, uint32_t *flags)
{
    if (flags) *flags = 0;
    if (!workspace) {
        std::lock_guard<std::mutex> lock(g_ws_mutex);
        int dev = 0;
        if (g_ws.empty()) return HETIS_OK;             // nothing was ever allocated: no HIP call
        if (hipGetDevice(&dev) != hipSuccess) return HETIS_ERR_LAUNCH;
        if ((size_t)dev >= g_ws.size() || !g_ws[dev].ptr) return HETIS_OK;
        workspace = g_ws[dev].ptr;
    }
    hipStream_t st = (hipStream_t)stream;
    uint32_t word = 0;
    unsigned int *dev_word = static_cast<unsigned int *>(workspace) + kCtlError;
    if (hipStreamSynchronize(st) != hipSuccess ||
        hipMemcpy(&word, dev_word, sizeof(word), hipMemcpyDeviceToHost) != hipSuccess)
        return HETIS_ERR_LAUNCH;
    if (word != 0 && hipMemset(dev_word, 0, sizeof(word)) != hipSuccess) return HETIS_ERR_LAUNCH;
    if (flags) *flags = word;
    return word == 0 ? HETIS_OK : HETIS_ERR_DEVICE_WAIT;
}

int hetis_attn_reserve_workspace(size_t bytes)
{
    void *ws = nullptr;
    return owned_workspace(std::max<size_t>(bytes, kControlBytes), nullptr, false, &ws);
}

int hetis_attn_release_workspace(void)
{
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    bool any = false;
    for (const OwnedWs &w : g_ws)
        if (w.ptr || !w.outgrown.empty()) any = true;
    if (!any) return HETIS_OK;
    int cur = 0;
    if (hipGetDevice(&cur) != hipSuccess) return HETIS_ERR_ALLOC;
    for (size_t d = 0; d < g_ws.size(); ++d) {
        OwnedWs &w = g_ws[d];
        if (!w.ptr && w.outgrown.empty()) continue;
        (void)hipSetDevice((int)d);
        (void)hipDeviceSynchronize();
        if (w.ptr) (void)hipFree(w.ptr);
        for (void *old : w.outgrown) (void)hipFree(old);
        w = OwnedWs();
    }
    (void)hipSetDevice(cur);
    return HETIS_OK;
}

int hetis_attn_split_num_chunks(int32_t max_seq_len, int32_t chunk_tokens)
{
    if (chunk_tokens <= 0 || chunk_tokens % kBlockTokens != 0 || chunk_tokens > kMaxChunkTokens)
        return HETIS_ERR_UNSUPPORTED;
    if (max_seq_len < 1) return HETIS_ERR_WORKSPACE;
    return (int)(((int64_t)max_seq_len + chunk_tokens - 1) / chunk_tokens);
}

int hetis_attn_split_workspace_bytes(const hetis_attn_shape *shape, int32_t n_sel_heads,
                                     int32_t max_seq_len, int32_t chunk_tokens,
                                     size_t *o_partial_bytes, size_t *lse_partial_bytes)
{
    Checked c;
    if (!shape || !o_partial_bytes || !lse_partial_bytes) return HETIS_ERR_NULL;
    int rc = check_shape(shape, n_sel_heads, &c);
    if (rc != HETIS_OK) return rc;
    rc = check_chunking(shape, chunk_tokens, max_seq_len);
    if (rc != HETIS_OK) return rc;
    const size_t n_chunks = (size_t)hetis_attn_split_num_chunks(max_seq_len, chunk_tokens);
    const size_t rows = (size_t)shape->batch * n_sel_heads * c.group * n_chunks;
    *o_partial_bytes = rows * shape->head_dim * sizeof(float);
    *lse_partial_bytes = rows * sizeof(float);
    return HETIS_OK;
}

static int decode_split_common(const hetis_attn_shape *shape, const void *q, const void *k_cache,
                               const void *v_cache, const int32_t *block_table,
                               const int32_t *seq_lens, const int32_t *head_ids,
                               int32_t n_sel_heads, float scale, int32_t chunk_tokens,
                               int32_t max_seq_len, float *o_partial, float *lse_partial,
                               void *control, bool owned, void *stream)
{
    Checked c;
    if (!shape || !q || !k_cache || !v_cache || !block_table || !seq_lens || !head_ids ||
        !o_partial || !lse_partial)
        return HETIS_ERR_NULL;
    int rc = check_shape(shape, n_sel_heads, &c);
    if (rc != HETIS_OK) return rc;
    rc = check_chunking(shape, chunk_tokens, max_seq_len);
    if (rc != HETIS_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (owned)
        rc = owned_workspace(kControlBytes, st, true, &control);
    else
        rc = check_workspace(control, kControlBytes, kControlBytes);
    if (rc != HETIS_OK) return rc;
    AttnParams p = make_params(shape, c, q, k_cache, v_cache, block_table, seq_lens, head_ids,
                               n_sel_heads, scale, nullptr);
    p.chunk_tokens = chunk_tokens;      // every chunk is a segment of its own
    p.seg_tokens = chunk_tokens;
    p.mode = kModeSplit;
    p.part_stride = 1;
    p.max_segs = hetis_attn_split_num_chunks(max_seq_len, chunk_tokens);
    p.direct_single = 0;
    p.o_partial = o_partial;
    p.lse_partial = lse_partial;
    p.control = static_cast<unsigned int *>(control);
    rc = launch_chunks(p, shape->head_dim, c.group, shape->batch, st);
    if (rc != HETIS_OK) return rc;
    return hipGetLastError() == hipSuccess ? HETIS_OK : HETIS_ERR_LAUNCH;
}

int hetis_attn_decode_split(const hetis_attn_shape *shape, const void *q, const void *k_cache,
                            const void *v_cache, const int32_t *block_table,
                            const int32_t *seq_lens, const int32_t *head_ids, int32_t n_sel_heads,
                            float scale, int32_t chunk_tokens, int32_t max_seq_len,
                            float *o_partial, float *lse_partial, void *stream)
{
    return decode_split_common(shape, q, k_cache, v_cache, block_table, seq_lens, head_ids,
                               n_sel_heads, scale, chunk_tokens, max_seq_len, o_partial,
                               lse_partial, nullptr, true, stream);
}

int hetis_attn_decode_split_ws(const hetis_attn_shape *shape, const void *q, const void *k_cache,
                               const void *v_cache, const int32_t *block_table,
                               const int32_t *seq_lens, const int32_t *head_ids,
                               int32_t n_sel_heads, float scale, int32_t chunk_tokens,
                               int32_t max_seq_len, float *o_partial, float *lse_partial,
                               void *control, void *stream)
{
    if (!control) return HETIS_ERR_NULL;
    return decode_split_common(shape, q, k_cache, v_cache, block_table, seq_lens, head_ids,
                               n_sel_heads, scale, chunk_tokens, max_seq_len, o_partial,
                               lse_partial, control, false, stream);
}

int hetis_attn_merge(const hetis_attn_shape *shape, const float *o_partial,
                     const float *lse_partial, const int32_t *seq_lens, const int32_t *head_ids,
                     int32_t n_sel_heads, int32_t chunk_tokens, int32_t max_seq_len, void *out,
                     void *stream)
{
    Checked c;
    if (!shape || !o_partial || !lse_partial || !seq_lens || !head_ids || !out)
        return HETIS_ERR_NULL;
    int rc = check_shape(shape, n_sel_heads, &c);
    if (rc != HETIS_OK) return rc;
    rc = check_chunking(shape, chunk_tokens, max_seq_len);
    if (rc != HETIS_OK) return rc;
    AttnParams p = make_params(shape, c, nullptr, nullptr, nullptr, nullptr, seq_lens, head_ids,
                               n_sel_heads, 0.f, out);
    p.chunk_tokens = chunk_tokens;
    p.seg_tokens = chunk_tokens;
    p.max_segs = hetis_attn_split_num_chunks(max_seq_len, chunk_tokens);
    p.direct_single = 0;
    p.o_partial = const_cast<float *>(o_partial);
    p.lse_partial = const_cast<float *>(lse_partial);
    launch_merge(p, shape->head_dim, c.group, shape->batch, (hipStream_t)stream);
    return hipGetLastError() == hipSuccess ? HETIS_OK : HETIS_ERR_LAUNCH;
}

int hetis_attn_profile_events(void *begin, void *end)
{
    if ((begin == nullptr) != (end == nullptr)) return HETIS_ERR_NULL;
    t_prof_begin = (hipEvent_t)begin;
    t_prof_end = (hipEvent_t)end;
    return HETIS_OK;
}

int hetis_attn_validate(const hetis_attn_shape *shape, const int32_t *block_table,
                        const int32_t *seq_lens, const int32_t *head_ids, int32_t n_sel_heads,
                        int64_t num_blocks, void *stream)
{
    Checked c;
    if (!shape || !block_table || !seq_lens || !head_ids) return HETIS_ERR_NULL;
    int rc = check_shape(shape, n_sel_heads, &c);
    if (rc != HETIS_OK) return rc;
    if (num_blocks <= 0) return HETIS_ERR_BAD_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    const size_t B = (size_t)shape->batch, MB = (size_t)shape->max_blocks_per_seq;
    std::vector<int32_t> sl(B), hid((size_t)n_sel_heads), bt(B * MB);
    if (hipStreamSynchronize(st) != hipSuccess) return HETIS_ERR_LAUNCH;
    if (hipMemcpy(sl.data(), seq_lens, B * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(hid.data(), head_ids, hid.size() * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(bt.data(), block_table, bt.size() * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess)
        return HETIS_ERR_LAUNCH;
    for (int32_t h : hid)
        if (h < 0 || h >= shape->n_kv_heads) return HETIS_ERR_BAD_CONTENT;
    for (size_t b = 0; b < B; ++b) {
        const int64_t L = sl[b];
        if (L < 0 || L > (int64_t)MB * kBlockTokens) return HETIS_ERR_BAD_CONTENT;
        const size_t nb = (size_t)((L + kBlockTokens - 1) / kBlockTokens);
        for (size_t j = 0; j < nb; ++j) {
            const int64_t blk = bt[b * MB + j];
            if (blk < 0 || blk >= num_blocks) return HETIS_ERR_BAD_CONTENT;
        }
    }
    return HETIS_OK;
}

int hetis_attn_validate_pairs(const hetis_attn_shape *shape, const int32_t *block_table,
                              const int32_t *seq_lens, const int32_t *pair_seq,
                              const int32_t *pair_head, int32_t n_pairs, int64_t num_tiles,
                              void *stream)
{
    Checked c;
    if (!shape || !block_table || !seq_lens || !pair_seq || !pair_head) return HETIS_ERR_NULL;
    int rc = check_shape(shape, 1, &c);
    if (rc != HETIS_OK) return rc;
    if (num_tiles <= 0 || n_pairs < 0) return HETIS_ERR_BAD_SHAPE;
    if (n_pairs == 0) return HETIS_OK;
    hipStream_t st = (hipStream_t)stream;
    const size_t B = (size_t)shape->batch, MB = (size_t)shape->max_blocks_per_seq, P = (size_t)n_pairs;
    std::vector<int32_t> sl(B), ps(P), ph(P), bt(P * MB);
    if (hipStreamSynchronize(st) != hipSuccess) return HETIS_ERR_LAUNCH;
    if (hipMemcpy(sl.data(), seq_lens, B * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(ps.data(), pair_seq, P * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(ph.data(), pair_head, P * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(bt.data(), block_table, bt.size() * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess)
        return HETIS_ERR_LAUNCH;
    for (size_t b = 0; b < B; ++b)
        if (sl[b] < 0 || sl[b] > (int64_t)MB * kBlockTokens) return HETIS_ERR_BAD_CONTENT;
    for (size_t i = 0; i < P; ++i) {
        if (ps[i] < 0 || ps[i] >= shape->batch) return HETIS_ERR_BAD_CONTENT;
        if (ph[i] < 0 || ph[i] >= shape->n_kv_heads) return HETIS_ERR_BAD_CONTENT;
        const int64_t L = sl[(size_t)ps[i]];
        const size_t nb = (size_t)((L + kBlockTokens - 1) / kBlockTokens);
        for (size_t j = 0; j < nb; ++j) {
            const int64_t t = bt[i * MB + j];
            if (t < 0 || t >= num_tiles) return HETIS_ERR_BAD_CONTENT;
        }
    }
    return HETIS_OK;
}

}  // extern "C"
