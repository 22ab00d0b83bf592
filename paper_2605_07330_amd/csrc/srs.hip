// Host side of libsrs.so: argument checks, bucket / segment / tile tables, launches.
// The operations and their conventions are documented in include/srs.h.
#include "srs.h"
#include "device_guard.hpp"
#include "srs_kernels.hpp"

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

using namespace srs;

namespace {

constexpr uint64_t kMaxIndexable = 0x7fffffffull;   // int32 indices (Sec. 3.2: tensors below 2^31 elements)

#define SRS_HIP(expr)                                   \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) { (void)hipGetLastError(); return SRS_ERR_HIP; } \
    } while (0)

// Makes `device` current for the rest of the enclosing scope and puts the caller's device back afterwards.
struct HipDeviceApi {
    static bool get_device(int *out) { return hipGetDevice(out) == hipSuccess; }
    static bool set_device(int device) { return hipSetDevice(device) == hipSuccess; }
    static void clear_error() { (void)hipGetLastError(); }
};
typedef srs::BasicDeviceGuard<HipDeviceApi> DeviceGuard;

#define SRS_ON_DEVICE(device)            \
    DeviceGuard device_guard_(device);   \
    if (!device_guard_.ok) return SRS_ERR_HIP

}  // namespace

// Scratch of the entry point that may not allocate (srs_extract_noalloc): tile status words, then ticket counters.
// One copy per GPU, held until the process ends.  In host code `scratch` is only a handle for
// hipGetSymbolAddress: srs_create resolves it once per context, with the context's device current, and everything
// else (kernel arguments included) goes through the pointer kept in the context.
namespace {
constexpr uint64_t kStaticTiles = 1ull << 20;          // status words: 8 MiB
constexpr uint64_t kStaticTicketWords = 1ull << 18;    // ticket counters: 1 MiB
constexpr uint64_t kStaticScratchBytes = kStaticTiles * sizeof(unsigned long long) + kStaticTicketWords * sizeof(uint32_t);
}  // namespace
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

struct srs_ctx {
    int device = 0;
    unsigned char *static_scratch = nullptr;   // this device's address of `scratch`
    unsigned long long *status = nullptr;   // tile status words
    uint64_t status_cap = 0;
    uint32_t *tickets = nullptr;            // per-bucket ticket counters
    uint64_t tickets_cap = 0;               // in words
    uint32_t *flags = nullptr;              // device flag word (own 256-byte allocation)
    uint32_t *vc_scratch = nullptr;         // value codec: per-bucket histograms and codes
    uint64_t vc_cap = 0;                    // in words
    uint32_t spin_limit = 1u << 24;
    uint32_t tile_elems = 32768;
    uint32_t group = 64;                    // buckets whose tiles are interleaved over consecutive workgroups
    uint32_t refresh_group = 8;             // 8: snapshot refreshed by whole 128-byte lines (full, aligned tiles); 0: element by element
    uint32_t snapshot_mode = 0;             // 0: refreshed inside the scan; 1: left alone, the caller swaps buffers;
                                            // 2: left alone by the scan, then refreshed from the payload (second pass)
};

struct srs_plan {
    int device = 0;
    uint64_t total = 0, be = 0;
    uint32_t ntensors = 0, nbuckets = 0, nsegments = 0, ntiles = 0, tile_elems = 0;
    uint32_t max_bucket_tiles = 0;          // most tiles in any one bucket
    TileDesc *d_tiles = nullptr;
    uint64_t *d_tensor_base = nullptr;      // [ntensors] packed position of each tensor's element 0
    WgInfo *d_wg_info = nullptr;            // [ntiles] bucket served by each workgroup of extract, and that bucket's tiles
    uint32_t *d_bucket_first = nullptr;     // [nbuckets+1] first tile of each bucket
    SegDesc *d_segs = nullptr;
    uint32_t *d_seg_begin = nullptr;
    PtrPair *d_pairs = nullptr;             // extract-side pointer table
    uint16_t **d_wptrs = nullptr;           // apply-side pointer table
    std::vector<PtrPair> h_pairs;           // what d_pairs currently holds
    std::vector<uint16_t *> h_wptrs;
    bool pairs_valid = false, wptrs_valid = false;
    std::vector<uint8_t> has_elems;         // [ntensors] 1 where the tensor has elements, i.e. its pointers are used
};

namespace {

// ticket counters sit 256 bytes apart (atomics on one cache line serialise) unless there are very
// many buckets, which only happens with bucket sizes far below a tile
uint32_t ticket_stride_for(uint64_t nb) { return nb <= 65536 ? 64u : 1u; }

// make room for ntiles status words and nb ticket counters, then clear both on the stream
int prepare_extract(srs_ctx *ctx, uint64_t ntiles, uint64_t nb, hipStream_t st, uint32_t *stride) {
    *stride = ticket_stride_for(nb);
    const uint64_t words = nb * (*stride);
    if (words > ctx->tickets_cap) {
        SRS_HIP(hipDeviceSynchronize());
        if (ctx->tickets) SRS_HIP(hipFree(ctx->tickets));
        ctx->tickets = nullptr; ctx->tickets_cap = 0;
        const uint64_t cap = words + words / 4 + 4096;
        SRS_HIP(hipMalloc((void **)&ctx->tickets, cap * sizeof(uint32_t)));
        ctx->tickets_cap = cap;
    }
    if (ntiles > ctx->status_cap) {
        SRS_HIP(hipDeviceSynchronize());
        if (ctx->status) SRS_HIP(hipFree(ctx->status));
        ctx->status = nullptr; ctx->status_cap = 0;
        const uint64_t cap = ntiles + ntiles / 4 + 1024;
        SRS_HIP(hipMalloc((void **)&ctx->status, cap * sizeof(unsigned long long)));
        ctx->status_cap = cap;
    }
    const uint64_t n = ntiles > nb ? ntiles : nb;
    const uint32_t threads = 256;
    hipLaunchKernelGGL(prepare_extract_kernel, dim3((uint32_t)((n + threads - 1) / threads)), dim3(threads), 0, st,
                       ctx->tickets, nb, *stride, ctx->status, ntiles);
    SRS_HIP(hipGetLastError());
    return SRS_OK;
}

// The same on the static scratch: nothing is allocated, sizes beyond the array are refused.  Ticket counters sit
// 256 bytes apart while they fit, 4 bytes apart above that.
int prepare_extract_static(srs_ctx *ctx, uint64_t ntiles, uint64_t nb, hipStream_t st, uint32_t *stride,
                           unsigned long long **status, uint32_t **tickets) {
    if (!ctx->static_scratch) return SRS_ERR_HIP;
    if (ntiles > kStaticTiles || nb > kStaticTicketWords) return SRS_ERR_TOO_LARGE;
    *stride = (nb * 64u <= kStaticTicketWords) ? 64u : 1u;
    *status = reinterpret_cast<unsigned long long *>(ctx->static_scratch);
    *tickets = reinterpret_cast<uint32_t *>(ctx->static_scratch + kStaticTiles * sizeof(unsigned long long));
    const uint64_t n = ntiles > nb ? ntiles : nb;
    const uint32_t threads = 256;
    hipLaunchKernelGGL(prepare_extract_kernel, dim3((uint32_t)((n + threads - 1) / threads)), dim3(threads), 0, st,
                       *tickets, nb, *stride, *status, ntiles);
    SRS_HIP(hipGetLastError());
    return SRS_OK;
}

// One-byte elements: a tile of tile_elems elements is V = tile_elems / 4096 vectors per lane (16 elements each), so
// the smallest tile (4096) has no kernel (V is even by construction of the packed scan).  The snapshot is refreshed
// as for 16-bit elements: by whole lines, element by element, or not at all under the rotating-snapshot option.
template <bool MULTI>
int launch_extract_u8(const srs_ctx *ctx, uint32_t tile_elems, const ExtractArgs &a, hipStream_t st) {
    const dim3 grid(a.ntiles), block(kThreads);
#define SRS_LAUNCH8(VV)                                                                                               \
    do {                                                                                                              \
        if (ctx->snapshot_mode != 0) hipLaunchKernelGGL((extract_kernel<VV, MULTI, -1, kSrcBf16, 1>), grid, block, 0, st, a); \
        else if (ctx->refresh_group == 8) hipLaunchKernelGGL((extract_kernel<VV, MULTI, 8, kSrcBf16, 1>), grid, block, 0, st, a); \
        else hipLaunchKernelGGL((extract_kernel<VV, MULTI, 0, kSrcBf16, 1>), grid, block, 0, st, a);                   \
    } while (0)
    switch (tile_elems) {
        case 8192: SRS_LAUNCH8(2); break;
        case 16384: SRS_LAUNCH8(4); break;
        case 32768: SRS_LAUNCH8(8); break;
        default: return SRS_ERR_INVALID;
    }
#undef SRS_LAUNCH8
    SRS_HIP(hipGetLastError());
    return SRS_OK;
}

template <bool MULTI>
int launch_extract(const srs_ctx *ctx, uint32_t tile_elems, const ExtractArgs &a, hipStream_t st, int src, int eb = 2) {
    if (eb == 1) return launch_extract_u8<MULTI>(ctx, tile_elems, a, st);
    const dim3 grid(a.ntiles), block(kThreads);
    if (src == kSrcBitmap) {                   // the bitmap says where the changes are: gather, do not stream
        if (!MULTI) return SRS_ERR_INVALID;
        switch (tile_elems) {
            case 4096: hipLaunchKernelGGL((extract_marked_kernel<16>), grid, block, 0, st, a); break;
            case 8192: hipLaunchKernelGGL((extract_marked_kernel<32>), grid, block, 0, st, a); break;
            case 16384: hipLaunchKernelGGL((extract_marked_kernel<64>), grid, block, 0, st, a); break;
            case 32768: hipLaunchKernelGGL((extract_marked_kernel<128>), grid, block, 0, st, a); break;
            default: return SRS_ERR_INVALID;
        }
        SRS_HIP(hipGetLastError());
        return SRS_OK;
    }
#define SRS_LAUNCH(VV)                                                                                                \
    do {                                                                                                              \
        if (src == kSrcFp32) {                                                                                        \
            if (ctx->refresh_group == 8) hipLaunchKernelGGL((extract_kernel<VV, MULTI, 8, kSrcFp32>), grid, block, 0, st, a); \
            else hipLaunchKernelGGL((extract_kernel<VV, MULTI, 0, kSrcFp32>), grid, block, 0, st, a);                 \
        } else if (ctx->snapshot_mode != 0) hipLaunchKernelGGL((extract_kernel<VV, MULTI, -1>), grid, block, 0, st, a); \
        else if (ctx->refresh_group == 8) hipLaunchKernelGGL((extract_kernel<VV, MULTI, 8>), grid, block, 0, st, a);  \
        else hipLaunchKernelGGL((extract_kernel<VV, MULTI, 0>), grid, block, 0, st, a);                               \
    } while (0)
    switch (tile_elems) {
        case 4096: SRS_LAUNCH(2); break;
        case 8192: SRS_LAUNCH(4); break;
        case 16384: SRS_LAUNCH(8); break;
        case 32768: SRS_LAUNCH(16); break;
        default: return SRS_ERR_INVALID;
    }
#undef SRS_LAUNCH
    SRS_HIP(hipGetLastError());
    return SRS_OK;
}

bool valid_tile_elems(uint64_t v) { return v == 4096 || v == 8192 || v == 16384 || v == 32768; }

}  // namespace

namespace {
// Host tables of a tensor list: a segment is a maximal run of one tensor inside one bucket, a tile a run
// of at most tile_elems elements inside one segment; wg_bucket tells extract's workgroup i which bucket to
// serve: inside each group of `group` buckets consecutive workgroups rotate over the buckets that still
// have tiles left, so every bucket is served exactly once per tile.
struct Layout {
    std::vector<SegDesc> segs;
    std::vector<uint32_t> seg_begin, bucket_first, wg_bucket;
    std::vector<TileDesc> tiles;
    uint32_t nbuckets = 0, max_bucket_tiles = 0;
};

int build_layout(const uint64_t *numel, uint32_t ntensors, uint64_t bucket_elems, uint32_t tile_elems, uint32_t group,
                 Layout &L) {
    uint64_t total = 0;
    for (uint32_t k = 0; k < ntensors; ++k) {
        if (numel[k] > kMaxIndexable) return SRS_ERR_INVALID;
        total += numel[k];
    }
    const uint64_t nb64 = (total + bucket_elems - 1) / bucket_elems;
    if (nb64 > 0x7fffffffull || group == 0 || tile_elems == 0) return SRS_ERR_INVALID;
    L.nbuckets = (uint32_t)nb64;
    try {
        L.seg_begin.assign((size_t)L.nbuckets + 1, 0);
        L.bucket_first.assign((size_t)L.nbuckets + 1, 0);
        uint64_t g = 0;                       // packed position of the current tensor's element 0
        uint32_t cur_bucket = 0xffffffffu;
        for (uint32_t k = 0; k < ntensors; ++k) {
            uint64_t off = 0;
            while (off < numel[k]) {
                const uint64_t pos = g + off;
                const uint64_t b = pos / bucket_elems;
                const uint64_t boff = pos - b * bucket_elems;
                uint64_t len = numel[k] - off;
                if (len > bucket_elems - boff) len = bucket_elems - boff;
                if ((uint32_t)b != cur_bucket) {
                    cur_bucket = (uint32_t)b;
                    L.bucket_first[b] = (uint32_t)L.tiles.size();
                    L.seg_begin[b] = (uint32_t)L.segs.size();
                }
                L.segs.push_back(SegDesc{(uint32_t)boff, (uint32_t)len, k, (uint32_t)off});
                for (uint64_t t = 0; t < len; t += tile_elems) {
                    const uint64_t tl = (len - t < tile_elems) ? (len - t) : tile_elems;
                    L.tiles.push_back(TileDesc{k, (uint32_t)(off + t), (uint32_t)(boff + t), (uint32_t)tl});
                }
                if (L.tiles.size() > 0x7fffffffull) return SRS_ERR_INVALID;
                off += len;
            }
            g += numel[k];
        }
        L.seg_begin[L.nbuckets] = (uint32_t)L.segs.size();
        L.bucket_first[L.nbuckets] = (uint32_t)L.tiles.size();
        for (uint32_t b = 0; b < L.nbuckets; ++b) {
            const uint32_t nt = L.bucket_first[b + 1] - L.bucket_first[b];
            if (nt > L.max_bucket_tiles) L.max_bucket_tiles = nt;
        }
        L.wg_bucket.reserve(L.tiles.size());
        std::vector<uint32_t> left;
        for (uint32_t g0 = 0; g0 < L.nbuckets; g0 += group) {
            const uint32_t g1 = (L.nbuckets - g0 < group) ? L.nbuckets : g0 + group;
            left.assign(g1 - g0, 0);
            uint64_t remaining = 0;
            for (uint32_t b = g0; b < g1; ++b) {
                left[b - g0] = L.bucket_first[b + 1] - L.bucket_first[b];
                remaining += left[b - g0];
            }
            while (remaining) {
                for (uint32_t b = g0; b < g1; ++b)
                    if (left[b - g0]) { L.wg_bucket.push_back(b); --left[b - g0]; --remaining; }
            }
        }
    } catch (const std::bad_alloc &) {
        return SRS_ERR_NOMEM;
    }
    return SRS_OK;
}

// Pointer arrays of a call: every tensor that has elements needs its pointers, aligned to their element size
// (old_mask / new_mask / mask = alignment - 1).  Tensors without elements may carry anything.
bool pair_pointers_ok(const srs_plan *plan, const srs_tensor_pair *t, uintptr_t old_mask, uintptr_t new_mask, bool need_old) {
    for (uint32_t k = 0; k < plan->ntensors; ++k) {
        if (!plan->has_elems[k]) continue;
        if (!t[k].new_w || (need_old && !t[k].old_snapshot)) return false;
        if (((uintptr_t)t[k].old_snapshot & old_mask) || ((uintptr_t)t[k].new_w & new_mask)) return false;
    }
    return true;
}

bool weight_pointers_ok(const srs_plan *plan, const srs_tensor *t, uintptr_t mask) {
    for (uint32_t k = 0; k < plan->ntensors; ++k)
        if (plan->has_elems[k] && (!t[k].weights || ((uintptr_t)t[k].weights & mask))) return false;
    return true;
}

// keeps the device copy of the extract-side pointer table in step with the caller's array
int upload_pair_pointers(srs_plan *plan, const srs_tensor_pair *t, hipStream_t st) {
    bool same = plan->pairs_valid;
    for (uint32_t k = 0; same && k < plan->ntensors; ++k)
        same = plan->h_pairs[k].old_w == (uint16_t *)t[k].old_snapshot && plan->h_pairs[k].new_w == t[k].new_w;
    if (!same) {
        for (uint32_t k = 0; k < plan->ntensors; ++k)
            plan->h_pairs[k] = PtrPair{(uint16_t *)t[k].old_snapshot, t[k].new_w};
        plan->pairs_valid = false;
        SRS_HIP(hipMemcpyAsync(plan->d_pairs, plan->h_pairs.data(), plan->ntensors * sizeof(PtrPair), hipMemcpyHostToDevice, st));
        plan->pairs_valid = true;
    }
    return SRS_OK;
}

// keeps the device copy of the apply-side pointer table in step with the caller's array
int upload_weight_pointers(srs_plan *plan, const srs_tensor *t, hipStream_t st) {
    bool same = plan->wptrs_valid;
    for (uint32_t k = 0; same && k < plan->ntensors; ++k) same = plan->h_wptrs[k] == (uint16_t *)t[k].weights;
    if (!same) {
        for (uint32_t k = 0; k < plan->ntensors; ++k) plan->h_wptrs[k] = (uint16_t *)t[k].weights;
        plan->wptrs_valid = false;
        SRS_HIP(hipMemcpyAsync(plan->d_wptrs, plan->h_wptrs.data(), plan->ntensors * sizeof(uint16_t *), hipMemcpyHostToDevice, st));
        plan->wptrs_valid = true;
    }
    return SRS_OK;
}
}  // namespace

namespace {
template <bool PACK>
int launch_dense_copy(srs_ctx *ctx, srs_plan *plan, const int32_t *dense_bucket, const uint32_t *n_dense,
                      uint32_t max_dense, uint16_t *dense, hipStream_t st) {
    if (max_dense == 0 || plan->max_bucket_tiles == 0) return SRS_OK;
    if ((uint64_t)max_dense * plan->max_bucket_tiles > 0x7fffffffull) return SRS_ERR_INVALID;
    DenseCopyArgs a;
    std::memset(&a, 0, sizeof(a));
    a.tiles = plan->d_tiles; a.bucket_first = plan->d_bucket_first; a.pairs = plan->d_pairs; a.wptrs = plan->d_wptrs;
    a.dense_bucket = dense_bucket; a.n_dense = n_dense; a.max_dense = max_dense;
    a.tiles_per_bucket_max = plan->max_bucket_tiles; a.be = plan->be; a.dense = dense;
    hipLaunchKernelGGL((dense_copy_kernel<PACK>), dim3(max_dense * plan->max_bucket_tiles), dim3(kThreads), 0, st, a);
    SRS_HIP(hipGetLastError());
    (void)ctx;
    return SRS_OK;
}
}  // namespace

namespace {
bool encoded_args_ok(const uint16_t *D, const int32_t *I_wide, const uint16_t *V, const uint32_t *counts,
                     const uint32_t *max_gap, const int32_t *anchors) {
    if (!D || !I_wide || !V || !counts || !max_gap || !anchors) return false;
    if (((uintptr_t)D | (uintptr_t)V) & 1u) return false;
    if (((uintptr_t)I_wide | (uintptr_t)counts | (uintptr_t)max_gap | (uintptr_t)anchors) & 3u) return false;
    return true;
}
}  // namespace


namespace {
// workgroups apply_kernel needs per bucket: one per chunk of kApplyChunk payload slots
uint64_t apply_chunks_per_bucket(uint64_t cap, uint64_t be) {
    const uint64_t slots = cap < be ? cap : be;           // a bucket never holds more pairs than elements
    return (slots + kApplyChunk - 1) / kApplyChunk;
}

// do the grids of the second-pass snapshot refresh fit a launch?  (checked before anything is launched)
bool second_pass_fits(uint64_t nb, uint64_t cap, uint64_t be) {
    return nb * apply_chunks_per_bucket(cap, be) <= 0x7fffffffull && nb * kOverflowSplit <= 0x7fffffffull;
}

// Second-pass snapshot refresh (SRS_OPT_SNAPSHOT = 2), queued behind an extract that left the snapshot alone: the
// payload is scattered into the snapshot, and buckets whose payload was cut at cap are copied whole.  `a` is the
// extract's own argument block; for a list the scatter reads the snapshot pointers from the extract-side table.
template <bool MULTI>
int launch_second_pass(const srs_ctx *ctx, const srs_plan *plan, const ExtractArgs &a, uint64_t be, uint32_t tile_elems,
                       int eb, hipStream_t st) {
    const uint64_t cpb = apply_chunks_per_bucket(a.cap, be);
    ApplyArgs s;
    std::memset(&s, 0, sizeof(s));
    if (MULTI) {
        s.segs = plan->d_segs; s.seg_begin = plan->d_seg_begin; s.total = plan->total;
        s.wptrs = reinterpret_cast<uint16_t *const *>(plan->d_pairs); s.wptr_skip = 1;
        static_assert(sizeof(PtrPair) == 2 * sizeof(uint16_t *) && offsetof(PtrPair, old_w) == 0, "old_w of entry k is pointer 2k");
    } else {
        s.w = a.old_w; s.n = a.n;
    }
    s.be = (uint32_t)be; s.nb = a.nb; s.chunks_per_bucket = (uint32_t)cpb;
    s.I = a.I; s.V = a.V; s.counts = a.counts; s.cap = a.cap; s.flags = ctx->flags;
    const dim3 grid((uint32_t)((uint64_t)a.nb * cpb)), ogrid(a.nb * kOverflowSplit), block(kThreads);
    if (eb == 1) {
        hipLaunchKernelGGL((apply_kernel<MULTI, 1>), grid, block, 0, st, s);
        hipLaunchKernelGGL((refresh_overflow_kernel<MULTI, 1>), ogrid, block, 0, st, a, tile_elems);
    } else {
        hipLaunchKernelGGL((apply_kernel<MULTI, 2>), grid, block, 0, st, s);
        hipLaunchKernelGGL((refresh_overflow_kernel<MULTI, 2>), ogrid, block, 0, st, a, tile_elems);
    }
    SRS_HIP(hipGetLastError());
    return SRS_OK;
}

int extract_single(srs_ctx *ctx, void *old_snapshot, const void *new_w, uint64_t n, uint64_t bucket_elems,
                   int32_t *I, void *V, uint32_t *counts, uint64_t cap, void *stream, bool cast, int eb = 2,
                   bool static_scratch = false) {
    if (!ctx || bucket_elems == 0 || cap == 0 || n > kMaxIndexable || bucket_elems > kMaxIndexable) return SRS_ERR_INVALID;
    if (n == 0) return SRS_OK;
    if (!old_snapshot || !new_w || !I || !V || !counts) return SRS_ERR_INVALID;
    const uintptr_t amask = (uintptr_t)eb - 1u;                     // elements are naturally aligned
    if (((uintptr_t)old_snapshot | (uintptr_t)V) & amask) return SRS_ERR_INVALID;
    if ((uintptr_t)new_w & (cast ? 3u : amask)) return SRS_ERR_INVALID;
    if (((uintptr_t)I | (uintptr_t)counts) & 3u) return SRS_ERR_INVALID;
    if (eb == 1 && ctx->tile_elems < 8192) return SRS_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    SRS_ON_DEVICE(ctx->device);

    const uint64_t T = ctx->tile_elems;
    const uint64_t nb = (n + bucket_elems - 1) / bucket_elems;
    const uint64_t tpb = (bucket_elems + T - 1) / T;
    const uint64_t last_len = n - (nb - 1) * bucket_elems;
    const uint64_t ntiles = (nb - 1) * tpb + (last_len + T - 1) / T;
    if (ntiles > 0x7fffffffull) return SRS_ERR_INVALID;

    if (nb > 0x7fffffffull) return SRS_ERR_INVALID;
    const bool second_pass = !cast && ctx->snapshot_mode == 2;
    if (second_pass && !second_pass_fits(nb, cap, bucket_elems)) return SRS_ERR_INVALID;
    const uint64_t group = ctx->group < nb ? ctx->group : nb;     // group * tpb <= ntiles + tpb

    ExtractArgs a;
    std::memset(&a, 0, sizeof(a));
    int rc = static_scratch ? prepare_extract_static(ctx, ntiles, nb, st, &a.ticket_stride, &a.status, &a.tickets)
                            : prepare_extract(ctx, ntiles, nb, st, &a.ticket_stride);
    if (rc != SRS_OK) return rc;
    if (!static_scratch) { a.status = ctx->status; a.tickets = ctx->tickets; }
    a.old_w = (uint16_t *)old_snapshot; a.new_w = new_w; a.n = n;
    a.be = (uint32_t)bucket_elems; a.tiles_per_bucket = (uint32_t)tpb;
    a.nb = (uint32_t)nb; a.last_tiles = (uint32_t)((last_len + T - 1) / T); a.group = (uint32_t)group;
    a.ntiles = (uint32_t)ntiles;
    a.I = I; a.V = (uint16_t *)V; a.counts = counts; a.cap = cap;
    a.flags = ctx->flags;
    a.spin_limit = ctx->spin_limit;
    rc = launch_extract<false>(ctx, ctx->tile_elems, a, st, cast ? kSrcFp32 : kSrcBf16, eb);
    if (rc != SRS_OK || !second_pass) return rc;
    return launch_second_pass<false>(ctx, nullptr, a, bucket_elems, ctx->tile_elems, eb, st);
}
}  // namespace

namespace {
int extract_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor_pair *t,
                  int32_t *I, void *V, uint32_t *counts, uint64_t cap, void *stream, int src,
                  const uint32_t *bitmap = nullptr, int eb = 2) {
    const bool cast = (src == kSrcFp32);
    if (src == kSrcBitmap && (!bitmap || ((uintptr_t)bitmap & 3u))) return SRS_ERR_INVALID;
    if (!ctx || !plan || cap == 0 || plan->device != ctx->device) return SRS_ERR_INVALID;
    if (plan->total == 0) return SRS_OK;
    if (!t || !I || !V || !counts) return SRS_ERR_INVALID;
    const uintptr_t amask = (uintptr_t)eb - 1u;
    if (((uintptr_t)V & amask) || (((uintptr_t)I | (uintptr_t)counts) & 3u)) return SRS_ERR_INVALID;
    if (eb == 1 && plan->tile_elems < 8192) return SRS_ERR_INVALID;
    if (!pair_pointers_ok(plan, t, amask, cast ? 3u : amask, src != kSrcBitmap)) return SRS_ERR_INVALID;
    const bool second_pass = src == kSrcBf16 && ctx->snapshot_mode == 2;
    if (second_pass && !second_pass_fits(plan->nbuckets, cap, plan->be)) return SRS_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    SRS_ON_DEVICE(ctx->device);

    int rc_up = upload_pair_pointers(plan, t, st);
    if (rc_up != SRS_OK) return rc_up;

    ExtractArgs a;
    std::memset(&a, 0, sizeof(a));
    int rc = prepare_extract(ctx, plan->ntiles, plan->nbuckets, st, &a.ticket_stride);
    if (rc != SRS_OK) return rc;
    a.tiles = plan->d_tiles; a.ptrs = plan->d_pairs; a.ntiles = plan->ntiles;
    a.wg_info = plan->d_wg_info; a.bucket_first = plan->d_bucket_first; a.nb = plan->nbuckets;
    a.I = I; a.V = (uint16_t *)V; a.counts = counts; a.cap = cap;
    a.status = ctx->status; a.tickets = ctx->tickets; a.flags = ctx->flags;
    a.spin_limit = ctx->spin_limit;
    a.bitmap = const_cast<uint32_t *>(bitmap); a.bitmap_words = (plan->total + 31) / 32; a.tensor_base = plan->d_tensor_base;
    rc = launch_extract<true>(ctx, plan->tile_elems, a, st, src, eb);
    if (rc != SRS_OK || !second_pass) return rc;
    return launch_second_pass<true>(ctx, plan, a, plan->be, plan->tile_elems, eb, st);
}
}  // namespace

extern "C" {

int srs_version(void) { return 100; }

const char *srs_strerror(int err) {
    switch (err) {
        case SRS_OK: return "ok";
        case SRS_ERR_INVALID: return "invalid argument";
        case SRS_ERR_HIP: return "HIP runtime call failed";
        case SRS_ERR_NOMEM: return "out of host memory";
        case SRS_ERR_NO_DEVICE: return "no usable GPU";
        case SRS_ERR_TOO_LARGE: return "input needs more scratch than the no-allocation entry point holds";
        default: return "unknown error";
    }
}

int srs_create(srs_ctx **out, int device) {
    if (!out) return SRS_ERR_INVALID;
    *out = nullptr;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) { (void)hipGetLastError(); return SRS_ERR_NO_DEVICE; }
    if (device < 0 || device >= ndev) return SRS_ERR_INVALID;
    SRS_ON_DEVICE(device);
    srs_ctx *ctx = new (std::nothrow) srs_ctx();
    if (!ctx) return SRS_ERR_NOMEM;
    ctx->device = device;
    if (hipMalloc((void **)&ctx->flags, 256) != hipSuccess) {
        (void)hipGetLastError(); delete ctx; return SRS_ERR_HIP;
    }
    if (hipMemset(ctx->flags, 0, 256) != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
        (void)hipGetLastError(); (void)hipFree(ctx->flags); delete ctx; return SRS_ERR_HIP;
    }
    // this device's copy of the static scratch array (each GPU has its own, at its own address)
    void *sp = nullptr;
    if (hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)) != hipSuccess || !sp || ((uintptr_t)sp & 255u)) {
        (void)hipGetLastError(); (void)hipFree(ctx->flags); delete ctx; return SRS_ERR_HIP;
    }
    ctx->static_scratch = static_cast<unsigned char *>(sp);
    *out = ctx;
    return SRS_OK;
}

int srs_destroy(srs_ctx *ctx) {
    if (!ctx) return SRS_ERR_INVALID;
    DeviceGuard device_guard_(ctx->device);
    (void)hipDeviceSynchronize();
    if (ctx->status) (void)hipFree(ctx->status);
    if (ctx->tickets) (void)hipFree(ctx->tickets);
    if (ctx->vc_scratch) (void)hipFree(ctx->vc_scratch);
    if (ctx->flags) (void)hipFree(ctx->flags);
    delete ctx;
    return SRS_OK;
}

int srs_set_option(srs_ctx *ctx, int option, uint64_t value) {
    if (!ctx) return SRS_ERR_INVALID;
    switch (option) {
        case SRS_OPT_SPIN_LIMIT:
            if (value == 0 || value > 0xffffffffull) return SRS_ERR_INVALID;
            ctx->spin_limit = (uint32_t)value; return SRS_OK;
        case SRS_OPT_TILE_ELEMS:
            if (!valid_tile_elems(value)) return SRS_ERR_INVALID;
            ctx->tile_elems = (uint32_t)value; return SRS_OK;
        case SRS_OPT_REFRESH_GROUP:
            if (value != 0 && value != 8) return SRS_ERR_INVALID;
            ctx->refresh_group = (uint32_t)value; return SRS_OK;
        case SRS_OPT_INTERLEAVE:
            if (value == 0 || value > 4096) return SRS_ERR_INVALID;
            ctx->group = (uint32_t)value; return SRS_OK;
        case SRS_OPT_SNAPSHOT:
            if (value > 2) return SRS_ERR_INVALID;
            ctx->snapshot_mode = (uint32_t)value; return SRS_OK;
        default: return SRS_ERR_INVALID;
    }
}

int srs_status(srs_ctx *ctx, uint32_t *flags, void *stream) {
    if (!ctx || !flags) return SRS_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    SRS_ON_DEVICE(ctx->device);
    SRS_HIP(hipMemcpyAsync(flags, ctx->flags, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
    SRS_HIP(hipStreamSynchronize(st));
    hipLaunchKernelGGL(fill_u64_kernel, dim3(1), dim3(64), 0, st, (unsigned long long *)ctx->flags, (uint64_t)1, 0ull);
    SRS_HIP(hipGetLastError());
    return SRS_OK;
}

// ---------------------------------------------------------------------------------------------
// single tensor
// ---------------------------------------------------------------------------------------------


int srs_extract(srs_ctx *ctx, void *old_snapshot, const void *new_w, uint64_t n, uint64_t bucket_elems,
                int32_t *I, uint16_t *V, uint32_t *counts, uint64_t cap, void *stream) {
    return extract_single(ctx, old_snapshot, new_w, n, bucket_elems, I, V, counts, cap, stream, false);
}

int srs_extract_noalloc(srs_ctx *ctx, void *old_snapshot, const void *new_w, uint64_t n, uint64_t bucket_elems,
                        int32_t *I, uint16_t *V, uint32_t *counts, uint64_t cap, void *stream) {
    return extract_single(ctx, old_snapshot, new_w, n, bucket_elems, I, V, counts, cap, stream, false, 2, true);
}

int srs_extract_cast(srs_ctx *ctx, void *weights, const float *master, uint64_t n, uint64_t bucket_elems,
                     int32_t *I, uint16_t *V, uint32_t *counts, uint64_t cap, void *stream) {
    return extract_single(ctx, weights, master, n, bucket_elems, I, V, counts, cap, stream, true);
}

static int apply_single(srs_ctx *ctx, void *weights, uint64_t n, uint64_t bucket_elems,
                        const int32_t *I, const void *V, const uint32_t *counts, uint64_t cap, void *stream, int eb) {
    if (!ctx || bucket_elems == 0 || cap == 0 || n > kMaxIndexable || bucket_elems > kMaxIndexable) return SRS_ERR_INVALID;
    if (n == 0) return SRS_OK;
    if (!weights || !I || !V || !counts) return SRS_ERR_INVALID;
    if (((uintptr_t)weights | (uintptr_t)V) & ((uintptr_t)eb - 1u)) return SRS_ERR_INVALID;
    if (((uintptr_t)I | (uintptr_t)counts) & 3u) return SRS_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    SRS_ON_DEVICE(ctx->device);

    const uint64_t nb = (n + bucket_elems - 1) / bucket_elems;
    const uint64_t slots = cap < bucket_elems ? cap : bucket_elems;       // a bucket never holds more pairs than elements
    const uint64_t cpb = (slots + kApplyChunk - 1) / kApplyChunk;
    if (nb * cpb > 0x7fffffffull) return SRS_ERR_INVALID;
    ApplyArgs a;
    std::memset(&a, 0, sizeof(a));
    a.w = (uint16_t *)weights; a.n = n; a.be = (uint32_t)bucket_elems; a.nb = (uint32_t)nb;
    a.chunks_per_bucket = (uint32_t)cpb;
    a.I = I; a.V = (const uint16_t *)V; a.counts = counts; a.cap = cap; a.flags = ctx->flags;
    if (eb == 1) hipLaunchKernelGGL((apply_kernel<false, 1>), dim3((uint32_t)(nb * cpb)), dim3(kThreads), 0, st, a);
    else hipLaunchKernelGGL((apply_kernel<false>), dim3((uint32_t)(nb * cpb)), dim3(kThreads), 0, st, a);
    SRS_HIP(hipGetLastError());
    return SRS_OK;
}

int srs_apply(srs_ctx *ctx, void *weights, uint64_t n, uint64_t bucket_elems,
              const int32_t *I, const uint16_t *V, const uint32_t *counts, uint64_t cap, void *stream) {
    return apply_single(ctx, weights, n, bucket_elems, I, V, counts, cap, stream, 2);
}

// one-byte elements (FP8 synchronisation precision)
int srs_extract_u8(srs_ctx *ctx, void *old_snapshot, const void *new_w, uint64_t n, uint64_t bucket_elems,
                   int32_t *I, uint8_t *V, uint32_t *counts, uint64_t cap, void *stream) {
    return extract_single(ctx, old_snapshot, new_w, n, bucket_elems, I, V, counts, cap, stream, false, 1);
}

int srs_apply_u8(srs_ctx *ctx, void *weights, uint64_t n, uint64_t bucket_elems,
                 const int32_t *I, const uint8_t *V, const uint32_t *counts, uint64_t cap, void *stream) {
    return apply_single(ctx, weights, n, bucket_elems, I, V, counts, cap, stream, 1);
}

// ---------------------------------------------------------------------------------------------
// tensor lists
// ---------------------------------------------------------------------------------------------

int srs_plan_create(srs_ctx *ctx, const uint64_t *numel, uint32_t ntensors, uint64_t bucket_elems, srs_plan **out) {
    if (!ctx || !out || (!numel && ntensors) || bucket_elems == 0 || bucket_elems > kMaxIndexable) return SRS_ERR_INVALID;
    *out = nullptr;
    uint64_t total = 0;
    for (uint32_t k = 0; k < ntensors; ++k) {
        if (numel[k] > kMaxIndexable) return SRS_ERR_INVALID;
        total += numel[k];
    }
    const uint64_t nb64 = (total + bucket_elems - 1) / bucket_elems;
    if (nb64 > 0x7fffffffull) return SRS_ERR_INVALID;
    SRS_ON_DEVICE(ctx->device);

    srs_plan *p = new (std::nothrow) srs_plan();
    if (!p) return SRS_ERR_NOMEM;
    p->device = ctx->device; p->total = total; p->be = bucket_elems; p->ntensors = ntensors;
    p->nbuckets = (uint32_t)nb64; p->tile_elems = ctx->tile_elems;

    Layout L;
    {
        const int rc = build_layout(numel, ntensors, bucket_elems, p->tile_elems, ctx->group, L);
        if (rc != SRS_OK) { delete p; return rc; }
    }
    try {
        p->h_pairs.assign(ntensors, PtrPair{nullptr, nullptr});
        p->h_wptrs.assign(ntensors, nullptr);
        p->has_elems.resize(ntensors);
        for (uint32_t k = 0; k < ntensors; ++k) p->has_elems[k] = numel[k] != 0;
    } catch (const std::bad_alloc &) {
        delete p; return SRS_ERR_NOMEM;
    }
    p->max_bucket_tiles = L.max_bucket_tiles;
    std::vector<SegDesc> &segs = L.segs;
    std::vector<uint32_t> &seg_begin = L.seg_begin, &bucket_first = L.bucket_first, &wg_bucket = L.wg_bucket;
    std::vector<TileDesc> &tiles = L.tiles;
    if (tiles.size() > 0x7fffffffull) { delete p; return SRS_ERR_INVALID; }
    p->nsegments = (uint32_t)segs.size();
    p->ntiles = (uint32_t)tiles.size();

    auto upload = [](void **dst, const void *src, size_t bytes) -> bool {
        if (bytes == 0) bytes = 16;
        if (hipMalloc(dst, bytes) != hipSuccess) return false;
        if (src && hipMemcpy(*dst, src, bytes, hipMemcpyHostToDevice) != hipSuccess) return false;
        return true;
    };
    bool ok = true;
    ok = ok && upload((void **)&p->d_tiles, tiles.empty() ? nullptr : tiles.data(), tiles.size() * sizeof(TileDesc));
    ok = ok && upload((void **)&p->d_segs, segs.empty() ? nullptr : segs.data(), segs.size() * sizeof(SegDesc));
    ok = ok && upload((void **)&p->d_seg_begin, seg_begin.data(), seg_begin.size() * sizeof(uint32_t));
    ok = ok && upload((void **)&p->d_bucket_first, bucket_first.data(), bucket_first.size() * sizeof(uint32_t));
    // what extract's workgroup i needs before it can take its ticket, in one 16-byte load: the bucket it serves,
    // that bucket's first tile and its number of tiles
    std::vector<WgInfo> wg_info;
    try {
        wg_info.resize(wg_bucket.size());
    } catch (const std::bad_alloc &) {
        srs_plan_destroy(p); return SRS_ERR_NOMEM;
    }
    for (size_t i = 0; i < wg_bucket.size(); ++i) {
        const uint32_t b = wg_bucket[i];
        wg_info[i] = WgInfo{b, bucket_first[b], bucket_first[b + 1] - bucket_first[b], 0u};
    }
    ok = ok && upload((void **)&p->d_wg_info, wg_info.empty() ? nullptr : wg_info.data(), wg_info.size() * sizeof(WgInfo));
    std::vector<uint64_t> tensor_base((size_t)ntensors + 1, 0);
    for (uint32_t k = 0; k < ntensors; ++k) tensor_base[k + 1] = tensor_base[k] + numel[k];
    ok = ok && upload((void **)&p->d_tensor_base, tensor_base.data(), tensor_base.size() * sizeof(uint64_t));
    ok = ok && upload((void **)&p->d_pairs, nullptr, (size_t)ntensors * sizeof(PtrPair));
    ok = ok && upload((void **)&p->d_wptrs, nullptr, (size_t)ntensors * sizeof(uint16_t *));
    ok = ok && hipDeviceSynchronize() == hipSuccess;
    if (!ok) { (void)hipGetLastError(); srs_plan_destroy(p); return SRS_ERR_HIP; }
    *out = p;
    return SRS_OK;
}

int srs_plan_info(const srs_plan *plan, uint64_t *total_elems, uint32_t *nbuckets, uint32_t *nsegments, uint32_t *ntiles) {
    if (!plan) return SRS_ERR_INVALID;
    if (total_elems) *total_elems = plan->total;
    if (nbuckets) *nbuckets = plan->nbuckets;
    if (nsegments) *nsegments = plan->nsegments;
    if (ntiles) *ntiles = plan->ntiles;
    return SRS_OK;
}

int srs_plan_layout(const uint64_t *numel, uint32_t ntensors, uint64_t bucket_elems, uint32_t tile_elems,
                    uint32_t interleave, uint32_t *nbuckets, uint32_t *nsegments, uint32_t *ntiles, uint32_t *tiles,
                    uint32_t *segs, uint32_t *seg_begin, uint32_t *bucket_first, uint32_t *wg_bucket) {
    if ((!numel && ntensors) || bucket_elems == 0 || bucket_elems > kMaxIndexable || !valid_tile_elems(tile_elems) ||
        interleave == 0 || interleave > 4096)
        return SRS_ERR_INVALID;
    Layout L;
    const int rc = build_layout(numel, ntensors, bucket_elems, tile_elems, interleave, L);
    if (rc != SRS_OK) return rc;
    if (nbuckets) *nbuckets = L.nbuckets;
    if (nsegments) *nsegments = (uint32_t)L.segs.size();
    if (ntiles) *ntiles = (uint32_t)L.tiles.size();
    if (tiles) std::memcpy(tiles, L.tiles.data(), L.tiles.size() * sizeof(TileDesc));
    if (segs) std::memcpy(segs, L.segs.data(), L.segs.size() * sizeof(SegDesc));
    if (seg_begin) std::memcpy(seg_begin, L.seg_begin.data(), L.seg_begin.size() * sizeof(uint32_t));
    if (bucket_first) std::memcpy(bucket_first, L.bucket_first.data(), L.bucket_first.size() * sizeof(uint32_t));
    if (wg_bucket) std::memcpy(wg_bucket, L.wg_bucket.data(), L.wg_bucket.size() * sizeof(uint32_t));
    return SRS_OK;
}

int srs_plan_destroy(srs_plan *p) {
    if (!p) return SRS_ERR_INVALID;
    DeviceGuard device_guard_(p->device);
    (void)hipDeviceSynchronize();
    if (p->d_tiles) (void)hipFree(p->d_tiles);
    if (p->d_segs) (void)hipFree(p->d_segs);
    if (p->d_seg_begin) (void)hipFree(p->d_seg_begin);
    if (p->d_bucket_first) (void)hipFree(p->d_bucket_first);
    if (p->d_wg_info) (void)hipFree(p->d_wg_info);
    if (p->d_tensor_base) (void)hipFree(p->d_tensor_base);
    if (p->d_pairs) (void)hipFree(p->d_pairs);
    if (p->d_wptrs) (void)hipFree(p->d_wptrs);
    delete p;
    return SRS_OK;
}


int srs_extract_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor_pair *t,
                      int32_t *I, uint16_t *V, uint32_t *counts, uint64_t cap, void *stream) {
    return extract_multi(ctx, plan, t, I, V, counts, cap, stream, kSrcBf16);
}

int srs_extract_cast_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor_pair *t,
                           int32_t *I, uint16_t *V, uint32_t *counts, uint64_t cap, void *stream) {
    return extract_multi(ctx, plan, t, I, V, counts, cap, stream, kSrcFp32);
}

static int apply_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor *t,
                       const int32_t *I, const void *V, const uint32_t *counts, uint64_t cap, void *stream, int eb) {
    if (!ctx || !plan || cap == 0 || plan->device != ctx->device) return SRS_ERR_INVALID;
    if (plan->total == 0) return SRS_OK;
    if (!t || !I || !V || !counts) return SRS_ERR_INVALID;
    const uintptr_t amask = (uintptr_t)eb - 1u;
    if (((uintptr_t)V & amask) || (((uintptr_t)I | (uintptr_t)counts) & 3u)) return SRS_ERR_INVALID;
    if (!weight_pointers_ok(plan, t, amask)) return SRS_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    SRS_ON_DEVICE(ctx->device);

    int rc_up = upload_weight_pointers(plan, t, st);
    if (rc_up != SRS_OK) return rc_up;

    const uint64_t slots = cap < plan->be ? cap : plan->be;
    const uint64_t cpb = (slots + kApplyChunk - 1) / kApplyChunk;
    if ((uint64_t)plan->nbuckets * cpb > 0x7fffffffull) return SRS_ERR_INVALID;
    ApplyArgs a;
    std::memset(&a, 0, sizeof(a));
    a.segs = plan->d_segs; a.seg_begin = plan->d_seg_begin; a.wptrs = plan->d_wptrs; a.total = plan->total;
    a.be = (uint32_t)plan->be; a.nb = plan->nbuckets; a.chunks_per_bucket = (uint32_t)cpb;
    a.I = I; a.V = (const uint16_t *)V; a.counts = counts; a.cap = cap; a.flags = ctx->flags;
    const dim3 grid((uint32_t)((uint64_t)plan->nbuckets * cpb));
    if (eb == 1) hipLaunchKernelGGL((apply_kernel<true, 1>), grid, dim3(kThreads), 0, st, a);
    else hipLaunchKernelGGL((apply_kernel<true>), grid, dim3(kThreads), 0, st, a);
    SRS_HIP(hipGetLastError());
    return SRS_OK;
}

int srs_apply_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor *t,
                    const int32_t *I, const uint16_t *V, const uint32_t *counts, uint64_t cap, void *stream) {
    return apply_multi(ctx, plan, t, I, V, counts, cap, stream, 2);
}

int srs_tensor_indices(srs_ctx *ctx, srs_plan *plan, const int32_t *I, const uint32_t *counts, uint64_t cap,
                       uint32_t *tensor_id, int32_t *tensor_idx, void *stream) {
    if (!ctx || !plan || cap == 0 || plan->device != ctx->device) return SRS_ERR_INVALID;
    if (plan->total == 0) return SRS_OK;
    if (!I || !counts || !tensor_id || !tensor_idx) return SRS_ERR_INVALID;
    if (((uintptr_t)I | (uintptr_t)counts | (uintptr_t)tensor_id | (uintptr_t)tensor_idx) & 3u) return SRS_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    SRS_ON_DEVICE(ctx->device);
    const uint64_t slots = cap < plan->be ? cap : plan->be;
    const uint64_t cpb = (slots + kApplyChunk - 1) / kApplyChunk;
    if ((uint64_t)plan->nbuckets * cpb > 0x7fffffffull) return SRS_ERR_INVALID;
    ApplyArgs a;
    std::memset(&a, 0, sizeof(a));
    a.segs = plan->d_segs; a.seg_begin = plan->d_seg_begin; a.total = plan->total;
    a.be = (uint32_t)plan->be; a.nb = plan->nbuckets; a.chunks_per_bucket = (uint32_t)cpb;
    a.I = I; a.counts = counts; a.cap = cap; a.flags = ctx->flags;
    hipLaunchKernelGGL(tensor_view_kernel, dim3((uint32_t)((uint64_t)plan->nbuckets * cpb)), dim3(kThreads), 0, st, a,
                       tensor_id, tensor_idx);
    SRS_HIP(hipGetLastError());
    return SRS_OK;
}

int srs_extract_multi_u8(srs_ctx *ctx, srs_plan *plan, const srs_tensor_pair *t,
                         int32_t *I, uint8_t *V, uint32_t *counts, uint64_t cap, void *stream) {
    return extract_multi(ctx, plan, t, I, V, counts, cap, stream, kSrcBf16, nullptr, 1);
}

int srs_apply_multi_u8(srs_ctx *ctx, srs_plan *plan, const srs_tensor *t,
                       const int32_t *I, const uint8_t *V, const uint32_t *counts, uint64_t cap, void *stream) {
    return apply_multi(ctx, plan, t, I, V, counts, cap, stream, 1);
}

// ---------------------------------------------------------------------------------------------
// cumulative changed-index set (Alg. 1 as printed)
// ---------------------------------------------------------------------------------------------

uint64_t srs_bitmap_words(uint64_t total_elems) { return (total_elems + 31) / 32; }

static int mark_common(srs_ctx *ctx, srs_plan *plan, const srs_tensor_pair *t, uint32_t *bitmap, void *stream, bool cast) {
    if (!ctx || !plan || plan->device != ctx->device) return SRS_ERR_INVALID;
    if (plan->total == 0) return SRS_OK;
    if (!t || !bitmap || ((uintptr_t)bitmap & 3u)) return SRS_ERR_INVALID;
    if (!pair_pointers_ok(plan, t, 1u, cast ? 3u : 1u, true)) return SRS_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    SRS_ON_DEVICE(ctx->device);
    int rc = upload_pair_pointers(plan, t, st);
    if (rc != SRS_OK) return rc;
    ExtractArgs a;
    std::memset(&a, 0, sizeof(a));
    a.tiles = plan->d_tiles; a.ptrs = plan->d_pairs; a.ntiles = plan->ntiles;
    a.bitmap = bitmap; a.bitmap_words = (plan->total + 31) / 32; a.tensor_base = plan->d_tensor_base;
    const dim3 grid(plan->ntiles), block(kThreads);
#define SRS_MARK(VV)                                                                   \
    do {                                                                               \
        if (cast) hipLaunchKernelGGL((mark_kernel<VV, true>), grid, block, 0, st, a);  \
        else hipLaunchKernelGGL((mark_kernel<VV, false>), grid, block, 0, st, a);      \
    } while (0)
    switch (plan->tile_elems) {
        case 4096: SRS_MARK(2); break;
        case 8192: SRS_MARK(4); break;
        case 16384: SRS_MARK(8); break;
        case 32768: SRS_MARK(16); break;
        default: return SRS_ERR_INVALID;
    }
#undef SRS_MARK
    SRS_HIP(hipGetLastError());
    return SRS_OK;
}

int srs_mark_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor_pair *t, uint32_t *bitmap, void *stream) {
    return mark_common(ctx, plan, t, bitmap, stream, false);
}

int srs_cast_mark_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor_pair *t, uint32_t *bitmap, void *stream) {
    return mark_common(ctx, plan, t, bitmap, stream, true);
}

int srs_extract_marked_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor *t, const uint32_t *bitmap,
                             int32_t *I, uint16_t *V, uint32_t *counts, uint64_t cap, void *stream) {
    if (!ctx || !plan || cap == 0) return SRS_ERR_INVALID;
    if (plan->total == 0) return SRS_OK;
    if (!t) return SRS_ERR_INVALID;
    // the weights go in as the "new" side of a pair table; there is no snapshot in this mode
    std::vector<srs_tensor_pair> pairs;
    try {
        pairs.resize(plan->ntensors);
    } catch (const std::bad_alloc &) {
        return SRS_ERR_NOMEM;
    }
    for (uint32_t k = 0; k < plan->ntensors; ++k) { pairs[k].old_snapshot = nullptr; pairs[k].new_w = t[k].weights; }
    return extract_multi(ctx, plan, pairs.data(), I, V, counts, cap, stream, kSrcBitmap, bitmap);
}

// ---------------------------------------------------------------------------------------------
// 16-bit index coding
// ---------------------------------------------------------------------------------------------

uint64_t srs_anchor_count(uint32_t nbuckets, uint64_t cap) {
    return (uint64_t)nbuckets * ((cap + kApplyChunk - 1) / kApplyChunk);
}

int srs_encode_indices(srs_ctx *ctx, const int32_t *I, const uint32_t *counts, uint32_t nbuckets, uint64_t cap,
                       uint64_t base_stride, uint16_t *D, uint32_t *max_gap, int32_t *anchors, void *stream) {
    if (!ctx || cap == 0 || base_stride > kMaxIndexable) return SRS_ERR_INVALID;
    if (nbuckets == 0) return SRS_OK;
    if (!I || !counts || !D || !max_gap || !anchors) return SRS_ERR_INVALID;
    if (((uintptr_t)D & 1u) || (((uintptr_t)I | (uintptr_t)counts | (uintptr_t)max_gap | (uintptr_t)anchors) & 3u))
        return SRS_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    SRS_ON_DEVICE(ctx->device);
    const uint64_t cpb = (cap + kApplyChunk - 1) / kApplyChunk;
    if ((uint64_t)nbuckets * cpb > 0x7fffffffull) return SRS_ERR_INVALID;
    hipLaunchKernelGGL(zero_strided_kernel, dim3((nbuckets + 255) / 256), dim3(256), 0, st, max_gap, (uint64_t)nbuckets, 1u);
    SRS_HIP(hipGetLastError());
    ApplyArgs a;
    std::memset(&a, 0, sizeof(a));
    a.nb = nbuckets; a.chunks_per_bucket = (uint32_t)cpb;
    a.I = I; a.counts = counts; a.cap = cap; a.flags = ctx->flags; a.base_stride = base_stride;
    hipLaunchKernelGGL(encode_indices_kernel, dim3((uint32_t)((uint64_t)nbuckets * cpb)), dim3(kThreads), 0, st, a, D,
                       max_gap, anchors);
    SRS_HIP(hipGetLastError());
    return SRS_OK;
}

int srs_apply_encoded(srs_ctx *ctx, void *weights, uint64_t n, uint64_t bucket_elems, const uint16_t *D,
                      const int32_t *I_wide, const uint16_t *V, const uint32_t *counts, const uint32_t *max_gap,
                      const int32_t *anchors, uint64_t cap, void *stream) {
    if (!ctx || bucket_elems == 0 || cap == 0 || n > kMaxIndexable || bucket_elems > kMaxIndexable) return SRS_ERR_INVALID;
    if (n == 0) return SRS_OK;
    if (!weights || ((uintptr_t)weights & 1u) || !encoded_args_ok(D, I_wide, V, counts, max_gap, anchors)) return SRS_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    SRS_ON_DEVICE(ctx->device);
    const uint64_t nb = (n + bucket_elems - 1) / bucket_elems;
    const uint64_t cpb = (cap + kApplyChunk - 1) / kApplyChunk;       // the anchors' layout
    if (nb * cpb > 0x7fffffffull) return SRS_ERR_INVALID;
    ApplyArgs a;
    std::memset(&a, 0, sizeof(a));
    a.w = (uint16_t *)weights; a.n = n; a.be = (uint32_t)bucket_elems; a.nb = (uint32_t)nb;
    a.chunks_per_bucket = (uint32_t)cpb;
    a.I = I_wide; a.V = V; a.counts = counts; a.cap = cap; a.flags = ctx->flags;
    a.D = D; a.max_gap = max_gap; a.anchors = anchors; a.base_stride = bucket_elems;
    const dim3 grid((uint32_t)(nb * cpb));
    hipLaunchKernelGGL((apply_encoded_kernel<false>), grid, dim3(kThreads), 0, st, a);
    SRS_HIP(hipGetLastError());
    hipLaunchKernelGGL((apply_kernel<false>), grid, dim3(kThreads), 0, st, a);      // buckets that kept 32-bit indices
    SRS_HIP(hipGetLastError());
    return SRS_OK;
}

int srs_apply_multi_encoded(srs_ctx *ctx, srs_plan *plan, const srs_tensor *t, const uint16_t *D, const int32_t *I_wide,
                            const uint16_t *V, const uint32_t *counts, const uint32_t *max_gap, const int32_t *anchors,
                            uint64_t cap, void *stream) {
    if (!ctx || !plan || cap == 0 || plan->device != ctx->device) return SRS_ERR_INVALID;
    if (plan->total == 0) return SRS_OK;
    if (!t || !encoded_args_ok(D, I_wide, V, counts, max_gap, anchors)) return SRS_ERR_INVALID;
    if (!weight_pointers_ok(plan, t, 1u)) return SRS_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    SRS_ON_DEVICE(ctx->device);
    int rc = upload_weight_pointers(plan, t, st);
    if (rc != SRS_OK) return rc;
    const uint64_t cpb = (cap + kApplyChunk - 1) / kApplyChunk;
    if ((uint64_t)plan->nbuckets * cpb > 0x7fffffffull) return SRS_ERR_INVALID;
    ApplyArgs a;
    std::memset(&a, 0, sizeof(a));
    a.segs = plan->d_segs; a.seg_begin = plan->d_seg_begin; a.wptrs = plan->d_wptrs; a.total = plan->total;
    a.be = (uint32_t)plan->be; a.nb = plan->nbuckets; a.chunks_per_bucket = (uint32_t)cpb;
    a.I = I_wide; a.V = V; a.counts = counts; a.cap = cap; a.flags = ctx->flags;
    a.D = D; a.max_gap = max_gap; a.anchors = anchors; a.base_stride = 0;
    const dim3 grid((uint32_t)((uint64_t)plan->nbuckets * cpb));
    hipLaunchKernelGGL((apply_encoded_kernel<true>), grid, dim3(kThreads), 0, st, a);
    SRS_HIP(hipGetLastError());
    hipLaunchKernelGGL((apply_kernel<true>), grid, dim3(kThreads), 0, st, a);
    SRS_HIP(hipGetLastError());
    return SRS_OK;
}

// ---------------------------------------------------------------------------------------------
// density routing and the dense (full-copy) route
// ---------------------------------------------------------------------------------------------

int srs_route(srs_ctx *ctx, const uint32_t *counts, uint32_t nbuckets, uint64_t bucket_elems, uint64_t total_elems,
              uint64_t cap, uint32_t bytes_per_pair, uint32_t max_dense, int32_t *route_slot, uint32_t *sparse_counts,
              int32_t *dense_bucket, uint32_t *n_dense, void *stream) {
    if (!ctx || bucket_elems == 0 || cap == 0 || bytes_per_pair == 0) return SRS_ERR_INVALID;
    if (!n_dense || ((uintptr_t)n_dense & 3u)) return SRS_ERR_INVALID;
    if (nbuckets && (!counts || !route_slot || !sparse_counts || (!dense_bucket && max_dense))) return SRS_ERR_INVALID;
    if (((uintptr_t)counts | (uintptr_t)route_slot | (uintptr_t)sparse_counts | (uintptr_t)dense_bucket) & 3u) return SRS_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    SRS_ON_DEVICE(ctx->device);
    RouteArgs a;
    std::memset(&a, 0, sizeof(a));
    a.counts = counts; a.nb = nbuckets; a.be = bucket_elems; a.total = total_elems; a.cap = cap;
    a.bytes_per_pair = bytes_per_pair; a.max_dense = max_dense;
    a.route_slot = route_slot; a.sparse_counts = sparse_counts; a.dense_bucket = dense_bucket; a.n_dense = n_dense;
    a.flags = ctx->flags;
    hipLaunchKernelGGL(route_kernel, dim3(1), dim3(kThreads), 0, st, a);
    SRS_HIP(hipGetLastError());
    return SRS_OK;
}

int srs_pack_dense_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor_pair *t, const int32_t *dense_bucket,
                         const uint32_t *n_dense, uint32_t max_dense, uint16_t *dense, void *stream) {
    if (!ctx || !plan || plan->device != ctx->device) return SRS_ERR_INVALID;
    if (plan->total == 0 || max_dense == 0) return SRS_OK;
    if (!t || !dense_bucket || !n_dense || !dense || ((uintptr_t)dense & 1u)) return SRS_ERR_INVALID;
    if (!pair_pointers_ok(plan, t, 1u, 1u, false)) return SRS_ERR_INVALID;       // only the new weights are read
    hipStream_t st = (hipStream_t)stream;
    SRS_ON_DEVICE(ctx->device);
    int rc = upload_pair_pointers(plan, t, st);
    if (rc != SRS_OK) return rc;
    return launch_dense_copy<true>(ctx, plan, dense_bucket, n_dense, max_dense, dense, st);
}

int srs_unpack_dense_multi(srs_ctx *ctx, srs_plan *plan, const srs_tensor *t, const int32_t *dense_bucket,
                           const uint32_t *n_dense, uint32_t max_dense, const uint16_t *dense, void *stream) {
    if (!ctx || !plan || plan->device != ctx->device) return SRS_ERR_INVALID;
    if (plan->total == 0 || max_dense == 0) return SRS_OK;
    if (!t || !dense_bucket || !n_dense || !dense || ((uintptr_t)dense & 1u)) return SRS_ERR_INVALID;
    if (!weight_pointers_ok(plan, t, 1u)) return SRS_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    SRS_ON_DEVICE(ctx->device);
    int rc = upload_weight_pointers(plan, t, st);
    if (rc != SRS_OK) return rc;
    return launch_dense_copy<false>(ctx, plan, dense_bucket, n_dense, max_dense, const_cast<uint16_t *>(dense), st);
}

// ---------------------------------------------------------------------------------------------
// value entropy coding
// ---------------------------------------------------------------------------------------------

uint64_t srs_value_chunks(uint64_t cap) { return (cap + kVcChunk - 1) / kVcChunk; }

int srs_encode_values(srs_ctx *ctx, const uint16_t *V, const uint32_t *counts, uint32_t nbuckets, uint64_t cap,
                      uint8_t *lens, uint8_t *low, uint32_t *bits, uint32_t *chunk_words, uint16_t *sub, void *stream) {
    if (!ctx || cap == 0) return SRS_ERR_INVALID;
    if (nbuckets == 0) return SRS_OK;
    if (!V || !counts || !lens || !low || !bits || !chunk_words || !sub) return SRS_ERR_INVALID;
    if ((((uintptr_t)V | (uintptr_t)sub) & 1u) || (((uintptr_t)counts | (uintptr_t)bits | (uintptr_t)chunk_words) & 3u))
        return SRS_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    SRS_ON_DEVICE(ctx->device);
    const uint64_t nchunk = (cap + kVcChunk - 1) / kVcChunk;
    if ((uint64_t)nbuckets * nchunk > 0x7fffffffull) return SRS_ERR_INVALID;
    const uint64_t words = (uint64_t)nbuckets * 512;
    if (words > ctx->vc_cap) {
        SRS_HIP(hipDeviceSynchronize());
        if (ctx->vc_scratch) SRS_HIP(hipFree(ctx->vc_scratch));
        ctx->vc_scratch = nullptr; ctx->vc_cap = 0;
        SRS_HIP(hipMalloc((void **)&ctx->vc_scratch, words * sizeof(uint32_t)));
        ctx->vc_cap = words;
    }
    ValueCodecArgs a;
    std::memset(&a, 0, sizeof(a));
    a.V = V; a.counts = counts; a.nb = nbuckets; a.cap = cap; a.nchunk = (uint32_t)nchunk;
    a.lens = lens; a.low = low; a.bits = bits; a.chunk_words = chunk_words; a.sub = sub;
    a.hist = ctx->vc_scratch; a.rcode = ctx->vc_scratch + (uint64_t)nbuckets * 256; a.flags = ctx->flags;
    const uint64_t nh = (uint64_t)nbuckets * 256;
    hipLaunchKernelGGL(zero_strided_kernel, dim3((uint32_t)((nh + 255) / 256)), dim3(256), 0, st, a.hist, nh, 1u);
    SRS_HIP(hipGetLastError());
    const dim3 grid((uint32_t)((uint64_t)nbuckets * ((nchunk + kVcEncodeChunks - 1) / kVcEncodeChunks)));
    const dim3 hist_grid((uint32_t)((uint64_t)nbuckets * ((nchunk + kVcHistChunks - 1) / kVcHistChunks)));
    hipLaunchKernelGGL(vc_hist_kernel, hist_grid, dim3(kThreads), 0, st, a);
    SRS_HIP(hipGetLastError());
    hipLaunchKernelGGL(vc_build_kernel, dim3(nbuckets), dim3(kThreads), 0, st, a);
    SRS_HIP(hipGetLastError());
    hipLaunchKernelGGL(vc_encode_kernel, grid, dim3(kThreads), 0, st, a);
    SRS_HIP(hipGetLastError());
    return SRS_OK;
}

int srs_decode_values(srs_ctx *ctx, const uint8_t *lens, const uint8_t *low, const uint32_t *bits,
                      const uint32_t *chunk_words, const uint16_t *sub, const uint32_t *counts, uint32_t nbuckets,
                      uint64_t cap, uint16_t *V_out, void *stream) {
    if (!ctx || cap == 0) return SRS_ERR_INVALID;
    if (nbuckets == 0) return SRS_OK;
    if (!lens || !low || !bits || !chunk_words || !sub || !counts || !V_out) return SRS_ERR_INVALID;
    if ((((uintptr_t)V_out | (uintptr_t)sub) & 1u) || (((uintptr_t)counts | (uintptr_t)bits | (uintptr_t)chunk_words) & 3u))
        return SRS_ERR_INVALID;
    hipStream_t st = (hipStream_t)stream;
    SRS_ON_DEVICE(ctx->device);
    const uint64_t nchunk = (cap + kVcChunk - 1) / kVcChunk;
    if ((uint64_t)nbuckets * nchunk > 0x7fffffffull) return SRS_ERR_INVALID;
    ValueCodecArgs a;
    std::memset(&a, 0, sizeof(a));
    a.V_out = V_out; a.counts = counts; a.nb = nbuckets; a.cap = cap; a.nchunk = (uint32_t)nchunk;
    a.lens = const_cast<uint8_t *>(lens); a.low = const_cast<uint8_t *>(low); a.bits = const_cast<uint32_t *>(bits);
    a.chunk_words = const_cast<uint32_t *>(chunk_words); a.sub = const_cast<uint16_t *>(sub); a.flags = ctx->flags;
    const uint64_t groups = (nchunk + kVcDecodeChunks - 1) / kVcDecodeChunks;
    hipLaunchKernelGGL(vc_decode_kernel, dim3((uint32_t)((uint64_t)nbuckets * groups)), dim3(kThreads), 0, st, a);
    SRS_HIP(hipGetLastError());
    return SRS_OK;
}

// ---------------------------------------------------------------------------------------------
// measurement aid
// ---------------------------------------------------------------------------------------------

uint64_t srs_stream_probe_sink_words(uint64_t bytes) {
    const uint64_t tile_bytes = 16384ull * 2ull;
    return (bytes + tile_bytes - 1) / tile_bytes + 1;
}

int srs_stream_probe(srs_ctx *ctx, const void *a, const void *b, uint64_t bytes, uint32_t *sink, void *stream) {
    if (!ctx || !a || !b || !sink || (bytes & 15u) || (((uintptr_t)a | (uintptr_t)b) & 15u)) return SRS_ERR_INVALID;
    if (bytes == 0) return SRS_OK;
    hipStream_t st = (hipStream_t)stream;
    SRS_ON_DEVICE(ctx->device);
    const uint64_t nvec = bytes / 16;
    const uint64_t tile_bytes = 16384ull * 2ull;
    const uint64_t blocks = (bytes + tile_bytes - 1) / tile_bytes;
    if (blocks > 0x7fffffffull) return SRS_ERR_INVALID;
    // hinted loads, like extract's: 6.8 TB/s over two 61 GB buffers against 6.3 TB/s with ordinary loads
    hipLaunchKernelGGL((stream_probe_kernel<8, true>), dim3((uint32_t)blocks), dim3(kThreads), 0, st,
                       (const uint16_t *)a, (const uint16_t *)b, nvec, sink);
    SRS_HIP(hipGetLastError());
    return SRS_OK;
}

}  // extern "C"
