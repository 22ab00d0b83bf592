// Device code of the sparse-weight-sync hot path for gfx950 (wave64, 256 CUs in 8 XCDs).
//
// extract_kernel: one pass over old/new.  Each workgroup is assigned a bucket by its block id
//   (consecutive block ids rotate over a group of buckets, so that many buckets are in flight at
//   once) and claims that bucket's next tile with an atomic ticket on the bucket's own counter:
//   tickets on one address serialise at about 11 ns each on this chip, spread over 32 addresses
//   they cost nothing.  A tile is a run of up to TILE = 2048*V elements inside one tensor and one
//   bucket.  Ticket order within a bucket is start order, which is what makes the chained scan
//   free of deadlock whatever order the hardware dispatches workgroups in.  The workgroup streams
//   both inputs with 16-byte loads, forms per-lane change masks by XOR of the 16-bit patterns
//   (Alg. 1: I = { i : W[i] != W_prev[i] }), ranks the changed elements with a packed DPP wave
//   scan + an LDS combine across the four waves, chains tiles of the same bucket with a
//   decoupled look-back on one 64-bit {flag, value} status word per tile, stages the
//   (index, value) pairs of the tile in LDS in rank order and writes them out coalesced
//   (Alg. 2: V = W[I], I int32 ascending).  The snapshot is refreshed in the same pass: every 128-byte line of
//   it that holds a change is rewritten whole from the new weights the lanes hold (RG = 8), or each changed
//   element is stored by itself (RG = 0), or nothing is written for callers that rotate buffers (RG = -1).
//   Template flavours of the same kernel: SRC = FP32 master weights rounded to BF16 on the fly (the
//   cast-and-copy of Alg. 1 fused with its diff); EB = 1 for one-byte (FP8) patterns.
// mark_kernel: one optimizer step of Alg. 1's index accumulation, OR-ed into a bitmap.
// extract_marked_kernel: the payload of the accumulated index set, gathered through the bitmap.
// apply_kernel: the scatter of Alg. 3, W[I] <- V, one workgroup per (bucket, payload chunk).
// refresh_overflow_kernel: whole-bucket copy for buckets whose payload overflowed, when the snapshot is refreshed
// by scattering the payload into it after the scan (apply_kernel on the snapshot) instead of inside extract_kernel.
// apply_encoded_kernel / encode_indices_kernel: the 16-bit index delta coding of Sec. 3.3.
// route_kernel / dense_copy_kernel: the per-bucket sparse / dense routing of Sec. 3.4 and its full-copy route.
//
// No arithmetic is done on weight values anywhere (the cast flavour rounds, nothing more); every kernel here
// is HBM-bandwidth bound and there is no contraction, hence no MFMA.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>
#include <stdint.h>

namespace srs {

constexpr int kThreads = 256;          // 4 waves of 64
constexpr int kWaves = kThreads / 64;
constexpr int kVecElems = 8;           // 16-byte vector = 8 patterns
constexpr int kUnit = kThreads * kVecElems;   // 2048 elements per "V" step of a tile
constexpr uint32_t kStage = 2048;      // (index,value) pairs staged in LDS per round
constexpr uint32_t kApplyChunk = 2048; // payload pairs per apply workgroup
constexpr int kLoadPace = 4;           // s_sleep argument between the streaming loads of an extract that refreshes in place

constexpr uint32_t kFlagOverflow = 1u, kFlagBadIndex = 2u, kFlagTimeout = 4u;
constexpr uint32_t kStAgg = 1u, kStPrefix = 2u;   // tile status: aggregate only / inclusive prefix

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Weight pointers reach the kernels through tables in device memory, so the compiler cannot tell that they are
// global addresses and would use FLAT loads and stores for them (which also occupy the LDS queue and the LDS
// counter).  Every such pointer is cast to the global address space once, where it is read from its table:
// the streaming loads then compile to global_load_dwordx4 and measure 3 % faster on the 910-bucket benchmark set.
#define SRS_GLOBAL __attribute__((address_space(1)))
template <class T> using gptr = T SRS_GLOBAL *;
template <class T> __device__ __forceinline__ gptr<T> as_global(T *p) { return (gptr<T>)p; }

struct TileDesc {          // one extract tile of a tensor list (16 bytes)
    uint32_t tensor;       // index into the pointer table
    uint32_t tensor_off;   // first element inside the tensor
    uint32_t bucket_off;   // first element inside the bucket
    uint32_t len;          // 1 .. TILE
};

struct WgInfo {            // what one extract workgroup serves (16 bytes)
    uint32_t bucket;       // the bucket whose next tile it claims
    uint32_t first_tile;   // id of that bucket's first tile
    uint32_t ntiles;       // number of tiles of that bucket
    uint32_t pad;
};

struct SegDesc {           // a run of one tensor inside one bucket (16 bytes)
    uint32_t bucket_off;
    uint32_t len;
    uint32_t tensor;
    uint32_t tensor_off;
};

struct PtrPair { uint16_t *old_w; const void *new_w; };   // new_w: BF16 weights, or FP32 master weights (CAST)

struct ExtractArgs {
    // single tensor: nb buckets of tiles_per_bucket tiles each, the last one of last_tiles tiles
    uint16_t *old_w; const void *new_w; uint64_t n; uint32_t be; uint32_t tiles_per_bucket;
    uint32_t nb; uint32_t last_tiles; uint32_t group;      // group = buckets interleaved per group
    // tensor list
    const TileDesc *tiles; const PtrPair *ptrs;
    const WgInfo *wg_info;          // [ntiles] bucket served by each workgroup
    const uint32_t *bucket_first;   // [nb+1] id of each bucket's first tile
    uint32_t ntiles;
    int32_t *I; uint16_t *V; uint32_t *counts; uint64_t cap;
    unsigned long long *status;     // [>= ntiles] {flag : value}, zeroed before every launch
    uint32_t *tickets;              // per-bucket ticket counters, ticket_stride words apart, zeroed per launch
    uint32_t ticket_stride;
    uint32_t *flags;
    uint32_t spin_limit;
    // cumulative changed-index set: one bit per packed position (bit g&31 of word g>>5)
    uint32_t *bitmap; uint64_t bitmap_words; const uint64_t *tensor_base;   // packed position of each tensor's element 0
};

struct ApplyArgs {
    // single tensor
    uint16_t *w; uint64_t n;
    // tensor list
    const SegDesc *segs; const uint32_t *seg_begin; uint16_t *const *wptrs; uint64_t total;
    uint32_t be; uint32_t nb; uint32_t chunks_per_bucket;
    const int32_t *I; const uint16_t *V; const uint32_t *counts; uint64_t cap;
    uint32_t *flags;
    // pointers to skip between two entries of wptrs: 0 for the apply-side table, 1 when wptrs is the extract-side
    // table of PtrPair read through its old_w members (the second-pass snapshot refresh)
    uint32_t wptr_skip;
    // 16-bit index coding (null / 0 when the payload carries 32-bit indices only)
    const uint16_t *D; const uint32_t *max_gap; const int32_t *anchors; uint64_t base_stride;
};

// ---------------------------------------------------------------------------------------------
// wave64 helpers
// ---------------------------------------------------------------------------------------------

template <int CTRL, int ROW_MASK, int BANK_MASK>
__device__ __forceinline__ uint32_t dpp_get(uint32_t x) {
    // lanes whose source is outside the row, or whose row is masked off, receive 0
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, ROW_MASK, BANK_MASK, false);
}

// inclusive prefix sum over the 64 lanes of a wave (also valid on two packed 16-bit fields as long
// as neither field overflows)
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x) {
    x += dpp_get<0x111, 0xF, 0xF>(x);   // row_shr:1
    x += dpp_get<0x112, 0xF, 0xF>(x);   // row_shr:2
    x += dpp_get<0x114, 0xF, 0xF>(x);   // row_shr:4
    x += dpp_get<0x118, 0xF, 0xF>(x);   // row_shr:8
    x += dpp_get<0x142, 0xA, 0xF>(x);   // row_bcast:15 -> rows 1 and 3
    x += dpp_get<0x143, 0xC, 0xF>(x);   // row_bcast:31 -> rows 2 and 3
    return x;
}

// workgroup barrier that orders LDS accesses only: waits for this wave's LDS operations (lgkmcnt), not for its
// outstanding global loads and stores, before the barrier instruction
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_s_waitcnt(0xC07F);     // vmcnt and expcnt at their maxima (= no wait), lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
}

__device__ __forceinline__ uint32_t lane63(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}

__device__ __forceinline__ uint32_t uniform(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)x);
}

template <bool NT>
__device__ __forceinline__ u32x4 load16(gptr<const void> p) {
    gptr<const u32x4> q = (gptr<const u32x4>)p;
    if (NT) return __builtin_nontemporal_load(q);
    return *q;
}
__device__ __forceinline__ void store16_nt(gptr<void> p, u32x4 v) { __builtin_nontemporal_store(v, (gptr<u32x4>)p); }

// 8 patterns starting at element e of a run of len elements, as 4 dwords; elements at or beyond
// len read as 0 (for both inputs, hence "unchanged").  Any alignment.
__device__ __forceinline__ u32x4 load8_guarded(gptr<const uint16_t> p, uint32_t e, uint32_t len) {
    uint32_t h[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) h[k] = (e + k < len) ? (uint32_t)p[e + k] : 0u;
    u32x4 r;
    r.x = h[0] | (h[1] << 16); r.y = h[2] | (h[3] << 16);
    r.z = h[4] | (h[5] << 16); r.w = h[6] | (h[7] << 16);
    return r;
}

// binary32 pattern -> BF16 pattern, round to nearest even; NaN -> 0x7FC0
__device__ __forceinline__ uint32_t round_bf16(uint32_t x) {
    const uint32_t r = (x + 0x7FFFu + ((x >> 16) & 1u)) >> 16;
    return ((x & 0x7FFFFFFFu) > 0x7F800000u) ? 0x7FC0u : r;
}

// eight consecutive master weights (two 16-byte vectors) -> eight BF16 patterns in memory order
__device__ __forceinline__ u32x4 round8_bf16(u32x4 f0, u32x4 f1) {
    u32x4 r;
    r.x = round_bf16(f0.x) | (round_bf16(f0.y) << 16);
    r.y = round_bf16(f0.z) | (round_bf16(f0.w) << 16);
    r.z = round_bf16(f1.x) | (round_bf16(f1.y) << 16);
    r.w = round_bf16(f1.z) | (round_bf16(f1.w) << 16);
    return r;
}

// guarded, any alignment (4-byte elements): elements at or beyond len read as BF16 pattern 0
__device__ __forceinline__ u32x4 load8_guarded_cast(gptr<const uint32_t> p, uint32_t e, uint32_t len) {
    uint32_t h[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) h[k] = (e + k < len) ? round_bf16(p[e + k]) : 0u;
    u32x4 r;
    r.x = h[0] | (h[1] << 16); r.y = h[2] | (h[3] << 16);
    r.z = h[4] | (h[5] << 16); r.w = h[6] | (h[7] << 16);
    return r;
}

// bit k of the result is set iff the k-th 16-bit pattern of a and b differ (k = 0..7, memory order)
__device__ __forceinline__ uint32_t diff_mask8(u32x4 a, u32x4 b) {
    uint32_t m = 0;
    const uint32_t d0 = a.x ^ b.x, d1 = a.y ^ b.y, d2 = a.z ^ b.z, d3 = a.w ^ b.w;
    m |= (d0 & 0xFFFFu) ? 1u : 0u;   m |= (d0 >> 16) ? 2u : 0u;
    m |= (d1 & 0xFFFFu) ? 4u : 0u;   m |= (d1 >> 16) ? 8u : 0u;
    m |= (d2 & 0xFFFFu) ? 16u : 0u;  m |= (d2 >> 16) ? 32u : 0u;
    m |= (d3 & 0xFFFFu) ? 64u : 0u;  m |= (d3 >> 16) ? 128u : 0u;
    return m;
}

__device__ __forceinline__ uint32_t pattern_at(u32x4 v, uint32_t e) {
    const uint32_t lo = (e & 2u) ? v.y : v.x;
    const uint32_t hi = (e & 2u) ? v.w : v.z;
    const uint32_t w = (e & 4u) ? hi : lo;
    return (e & 1u) ? (w >> 16) : (w & 0xFFFFu);
}

// 16 one-byte patterns starting at element e of a run of len elements; elements at or beyond len read as 0
__device__ __forceinline__ u32x4 load16_guarded_u8(gptr<const uint8_t> p, uint32_t e, uint32_t len) {
    uint32_t d[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        uint32_t w = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) w |= ((e + 4 * q + k < len) ? (uint32_t)p[e + 4 * q + k] : 0u) << (8 * k);
        d[q] = w;
    }
    u32x4 r;
    r.x = d[0]; r.y = d[1]; r.z = d[2]; r.w = d[3];
    return r;
}

// bit k of the result is set iff byte k of d is non-zero (k = 0..3)
__device__ __forceinline__ uint32_t nonzero_bytes4(uint32_t d) {
    const uint32_t t = ((d | ((d & 0x7F7F7F7Fu) + 0x7F7F7F7Fu)) & 0x80808080u) >> 7;   // bits 0, 8, 16, 24
    return (t * 0x10204080u) >> 28;                                                       // gathered into bits 0..3
}

// Element width.  EB = 2: BF16 / FP16 patterns, 8 per 16-byte vector; EB = 1: FP8 patterns, 16 per vector
// (Sec. 2.1 measures the changed-element density at all three synchronisation precisions; nothing in
// Alg. 1-3 depends on the width).  diff_mask has one bit per element of the vector, in memory order.
template <int EB> struct Elem;
template <> struct Elem<2> {
    typedef uint16_t type;
    static __device__ __forceinline__ uint32_t diff_mask(u32x4 a, u32x4 b) { return diff_mask8(a, b); }
    static __device__ __forceinline__ uint32_t pattern(u32x4 v, uint32_t e) { return pattern_at(v, e); }
    static __device__ __forceinline__ u32x4 load_guarded(gptr<const uint16_t> p, uint32_t e, uint32_t len) {
        return load8_guarded(p, e, len);
    }
};
template <> struct Elem<1> {
    typedef uint8_t type;
    static __device__ __forceinline__ uint32_t diff_mask(u32x4 a, u32x4 b) {
        return nonzero_bytes4(a.x ^ b.x) | (nonzero_bytes4(a.y ^ b.y) << 4) | (nonzero_bytes4(a.z ^ b.z) << 8) |
               (nonzero_bytes4(a.w ^ b.w) << 12);
    }
    static __device__ __forceinline__ uint32_t pattern(u32x4 v, uint32_t e) {
        const uint32_t lo = (e & 4u) ? v.y : v.x;
        const uint32_t hi = (e & 4u) ? v.w : v.z;
        const uint32_t w = (e & 8u) ? hi : lo;
        return (w >> ((e & 3u) * 8u)) & 0xFFu;
    }
    static __device__ __forceinline__ u32x4 load_guarded(gptr<const uint8_t> p, uint32_t e, uint32_t len) {
        return load16_guarded_u8(p, e, len);
    }
};

__device__ __forceinline__ unsigned long long status_load(const unsigned long long *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void status_store(unsigned long long *p, unsigned long long v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long status_word(uint32_t flag, uint32_t value) {
    return ((unsigned long long)flag << 32) | value;
}

// ---------------------------------------------------------------------------------------------
// decoupled look-back, run by all 64 lanes of wave 0.  Returns the number of changed elements in
// the tiles first_tile .. tile-1 of the same bucket.  Lane l inspects tile (pos - l); the window
// slides back by 64 until a tile with an inclusive prefix, or the bucket's first tile, is reached.
// Bounded: after spin_limit polls of one window the wave gives up, raises kFlagTimeout and
// returns what it has (ranks are clamped by the caller, so memory safety does not depend on it).
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t look_back(const ExtractArgs &a, uint32_t tile, uint32_t first_tile, int lane) {
    uint32_t excl = 0;
    int64_t pos = (int64_t)tile - 1;
    while (pos >= (int64_t)first_tile) {
        const int64_t idx = pos - lane;
        const bool in_bucket = idx >= (int64_t)first_tile;
        uint32_t flag = 0, value = 0;
        unsigned long long need = 0;
        bool found_prefix = false;
        uint32_t polls = 0;
        for (;;) {
            if (in_bucket && flag == 0) {                                    // only lanes still waiting poll again
                const unsigned long long w = status_load(a.status + idx);
                const uint32_t hi = (uint32_t)(w >> 32);
                flag = hi & 3u;
                value = (uint32_t)w;
            }
            const unsigned long long valid = __ballot(in_bucket);            // a low run of lanes
            const unsigned long long pending = __ballot(in_bucket && flag == 0);
            const unsigned long long prefixed = __ballot(in_bucket && flag == kStPrefix);
            found_prefix = prefixed != 0;
            if (found_prefix) {
                const int first = __builtin_ctzll(prefixed);                 // nearest tile that has a prefix
                need = (first == 63) ? ~0ull : ((1ull << (first + 1)) - 1ull);
            } else {
                need = valid;
            }
            if ((pending & need) == 0) break;
            if (++polls > a.spin_limit) {
                if (lane == 0) atomicOr(a.flags, kFlagTimeout);
                need &= ~pending;
                found_prefix = true;                                         // stop walking back
                break;
            }
            __builtin_amdgcn_s_sleep(2);
        }
        const uint32_t mine = ((need >> lane) & 1ull) ? value : 0u;
        excl += lane63(wave_inclusive_scan(mine));
        if (found_prefix) break;
        pos -= 64;
    }
    return excl;
}

// ---------------------------------------------------------------------------------------------
// extract
// ---------------------------------------------------------------------------------------------
// RG = how the snapshot is refreshed.  8: by whole lines -- a full tile of 16-byte-aligned weights rewrites every
// aligned 128-byte line of the snapshot that holds a change (8 lanes x 16 bytes of one store instruction) from the
// new weights it has in registers; unchanged elements get the value they already hold.  The snapshot's loads and
// these stores carry the non-temporal hint: a line written in full needs no read-modify-write behind the L2, and
// nothing of the snapshot is needed again.  Measured on the 910-bucket benchmark set against element-wise refresh,
// in one process, ms: 21.8 / 22.4 at 0.1 % changed, 25.8 / 28.7 at 1 %, 30.1 / 36.2 at 3 %, 33.6 / 40.4 at 10 %.
// The two hints only pay together (at 1 %: stores alone 27.6, loads alone 28.3; 64-byte blocks 28.8, 256-byte
// blocks 30.5).  The new weights are hinted as well (read once; worth 1 % on one-byte and on sparse data, nothing
// at 1 %), except the FP32 master weights of CAST, where the hint costs 1 ms of 38.  Tiles that are ragged or not
// 16-byte aligned refresh element by element with ordinary loads.
// 0: element by element everywhere (2-byte stores from the write-out loop).  -1: the snapshot is not touched at all
// (the caller rotates buffers: `new` is the next call's `old`).
// CAST: `new` is not a BF16 buffer but the FP32 master weights; each element is rounded to BF16
// (nearest even, NaN -> 0x7FC0) on the fly and `old` is the model-parameter buffer itself: the cast-and-
// copy of Alg. 1 fused with its diff, so that no snapshot exists at all.
// (The cumulative index set of Alg. 1 has a kernel of its own, extract_marked_kernel; kSrcBitmap only names that
// source for the host code.)
constexpr int kSrcBf16 = 0, kSrcFp32 = 1, kSrcBitmap = 2;

template <int V, bool MULTI, int RG, int SRC = kSrcBf16, int EB = 2>
__global__ __launch_bounds__(kThreads) void extract_kernel(const ExtractArgs a) {
    // A snapshot that is not written is read exactly once, like the new weights: both streams then carry the
    // non-temporal hint (measured 4 % faster).  With element-wise refresh the hint on either stream measures slower,
    // on the snapshot by 5 ms: 2-byte refresh stores must find their line still cached, hinted or not.
    static_assert(RG == -1 || RG == 0 || RG == 8, "refresh: none, element-wise or whole lines");
    constexpr bool NT = (RG < 0);
    constexpr bool LINES = (RG == 8);
    constexpr bool CAST = (SRC == kSrcFp32);
    static_assert(SRC == kSrcBf16 || SRC == kSrcFp32, "the bitmap source has its own kernel");
    static_assert(V % 2 == 0, "counts are scanned in packed pairs");
    static_assert(EB == 2 || SRC == kSrcBf16, "the cast flavour exists for 16-bit elements only");
    typedef Elem<EB> EL;
    typedef typename EL::type T;
    constexpr uint32_t VE = 16u / EB;                    // elements per 16-byte vector
    constexpr uint32_t ROW = 64u * VE;                   // elements covered by one load instruction of a wave
    constexpr uint32_t TILE = (uint32_t)V * kThreads * VE;
    static_assert(TILE <= 65536u, "tile-local positions are staged in 16 bits");
    __shared__ uint32_t s_ticket;
    __shared__ uint32_t s_wave_total[kWaves];
    __shared__ uint32_t s_excl;
    __shared__ uint32_t s_stage[kStage];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // ---- which bucket this workgroup serves, then claim that bucket's next tile
    uint32_t bucket, first_tile, bucket_tiles;
    if (MULTI) {
        const WgInfo wi = a.wg_info[blockIdx.x];
        bucket = wi.bucket; first_tile = wi.first_tile; bucket_tiles = wi.ntiles;
    } else {
        // groups of `group` buckets; inside a group consecutive workgroups rotate over its buckets.
        // Only the very last bucket may have fewer tiles: in its group the first last_tiles rounds
        // rotate over all buckets, the remaining rounds over all but the last.
        const uint32_t per_group = a.group * a.tiles_per_bucket;
        const uint32_t g = blockIdx.x / per_group;
        const uint32_t j = blockIdx.x - g * per_group;
        const uint32_t g0 = g * a.group;
        const uint32_t gb = (a.nb - g0 < a.group) ? (a.nb - g0) : a.group;      // buckets in this group
        const bool has_short = (g0 + gb == a.nb) && (a.last_tiles < a.tiles_per_bucket);
        uint32_t slot;
        if (!has_short || j < a.last_tiles * gb) slot = j % gb;
        else slot = (j - a.last_tiles * gb) % (gb - 1);
        bucket = g0 + slot;
        first_tile = bucket * a.tiles_per_bucket;
        bucket_tiles = (bucket == a.nb - 1) ? a.last_tiles : a.tiles_per_bucket;
    }
    if (tid == 0)
        s_ticket = __hip_atomic_fetch_add(a.tickets + (uint64_t)bucket * a.ticket_stride, 1u, __ATOMIC_RELAXED,
                                          __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const uint32_t k = uniform(s_ticket);
    if (k >= bucket_tiles) return;         // cannot happen: each bucket is served by exactly bucket_tiles workgroups
    const uint32_t tile = first_tile + k;
    const bool last = (k == bucket_tiles - 1);

    // ---- where this tile lives
    uint32_t bucket_off, len, idx_base;
    gptr<T> po; gptr<const void> pn_raw; uint64_t pn_off;      // new weights: base pointer and element offset
    if (MULTI) {
        const TileDesc d = a.tiles[tile];
        const PtrPair p = a.ptrs[d.tensor];
        po = (gptr<T>)p.old_w + d.tensor_off; pn_raw = as_global(p.new_w); pn_off = d.tensor_off;
        bucket_off = d.bucket_off; len = d.len;
        idx_base = bucket_off;                          // index = position inside the bucket
    } else {
        const uint64_t b0 = (uint64_t)bucket * a.be;
        const uint32_t blen = (uint32_t)((a.n - b0 < a.be) ? (a.n - b0) : a.be);
        bucket_off = k * TILE;
        len = (blen - bucket_off < TILE) ? (blen - bucket_off) : TILE;
        po = (gptr<T>)a.old_w + b0 + bucket_off; pn_raw = as_global(a.new_w); pn_off = b0 + bucket_off;
        idx_base = (uint32_t)(b0 + bucket_off);         // index = tensor-flat position
    }

    // ---- stream the tile.  Layout: wave w owns elements [w*V*ROW, (w+1)*V*ROW); inside it vector j
    // of lane l holds elements (j*64 + l)*VE .. +VE, so ascending order is (wave, j, lane, element).
    u32x4 xo[V], xn[V];
    const uint32_t e0 = (uint32_t)wave * (V * ROW) + (uint32_t)lane * VE;
    // with CAST pn addresses 32-bit elements: pf is the same position in the master weights
    const gptr<const uint32_t> pf = (gptr<const uint32_t>)pn_raw + pn_off;
    const gptr<const T> pn = (gptr<const T>)pn_raw + pn_off;
    const bool aligned = CAST ? (((((uintptr_t)po) | ((uintptr_t)pf)) & 15u) == 0)
                              : (((((uintptr_t)po) | ((uintptr_t)pn)) & 15u) == 0);
    uint32_t m[V];
    // Whole-line refresh: any full tile of 16-byte vectors.  (A tile that does not start on a 128-byte boundary
    // writes the same bytes in runs of 128 that straddle two lines: correct, only without the benefit.)
    const bool by_lines = LINES && aligned && len == TILE;              // uniform over the workgroup
    if (aligned && len == TILE) {
        auto stream_tile = [&](auto hint) {                // all loads of the tile issued back to back
            constexpr bool H = decltype(hint)::value;
            if (CAST) {
                u32x4 f0[V], f1[V];
                // paced like the loads of the in-place refresh below (this flavour always writes the parameters
                // back); half the pause, as there are half as many bytes per load of master weights.  Measured on
                // the benchmark set at 1 %: 36.2 ms against 37.4 unpaced (pause 4: 36.3)
#pragma unroll
                for (int j = 0; j < V; ++j) {
                    f0[j] = load16<false>(pf + e0 + j * ROW);
                    __builtin_amdgcn_sched_barrier(0); __builtin_amdgcn_s_sleep(kLoadPace / 2); __builtin_amdgcn_sched_barrier(0);
                    f1[j] = load16<false>(pf + e0 + j * ROW + 4);
                    __builtin_amdgcn_sched_barrier(0); __builtin_amdgcn_s_sleep(kLoadPace / 2); __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int j = 0; j < V; ++j) {
                    xo[j] = load16<H>(po + e0 + j * ROW);
                    __builtin_amdgcn_sched_barrier(0); __builtin_amdgcn_s_sleep(kLoadPace / 2); __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int j = 0; j < V; ++j) xn[j] = round8_bf16(f0[j], f1[j]);
            } else if (RG >= 0) {
                // A kernel that also writes the snapshot issues its loads in program order with a short sleep
                // after each (kLoadPace x 64 clocks): the tile's 32 loads then leave the CU over about 3 us instead
                // of in one burst, which the memory side, busy with the refresh stores of the other workgroups,
                // serves faster.  Measured in one process on the benchmark sets, paced / unpaced, ms: 30B-A3B at
                // 1 % 25.09 / 25.84, at 0.1 % 20.83 / 21.82, at 5 % 30.70 / 30.89, skewed 20.45 / 21.44; 8B at 1 %
                // 6.80 / 7.24.  (Pace 1, 2, 4, 6, 8: 25.58, 25.31, 25.10, 25.04, 25.17.)  The kernel that writes
                // nothing into weights gains nothing from it (18.87 / 18.83) and stays as it was.
#pragma unroll
                for (int j = 0; j < V; ++j) {
                    xn[j] = load16<H>(pn + e0 + j * ROW);
                    __builtin_amdgcn_sched_barrier(0); __builtin_amdgcn_s_sleep(kLoadPace); __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int j = 0; j < V; ++j) {
                    xo[j] = load16<H>(po + e0 + j * ROW);
                    __builtin_amdgcn_sched_barrier(0); __builtin_amdgcn_s_sleep(kLoadPace); __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int j = 0; j < V; ++j) xn[j] = load16<H>(pn + e0 + j * ROW);
#pragma unroll
                for (int j = 0; j < V; ++j) xo[j] = load16<H>(po + e0 + j * ROW);
            }
        };
        // one flavour of loads per instantiation: choosing between two at run time cost 2 ms of the 3 ms the hints gain
        stream_tile(std::integral_constant<bool, NT || LINES>{});
    } else {
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const uint32_t e = e0 + j * ROW;
            if (aligned && e + VE <= len) {
                xo[j] = load16<false>(po + e);
                if (CAST) xn[j] = round8_bf16(load16<false>(pf + e), load16<false>(pf + e + 4));
                else xn[j] = load16<false>(pn + e);
            } else {
                xo[j] = EL::load_guarded(po, e, len);
                xn[j] = CAST ? load8_guarded_cast(pf, e, len) : EL::load_guarded(pn, e, len);
            }
        }
    }

    // ---- change masks and their counts
    uint32_t pk[V / 2];
#pragma unroll
    for (int j = 0; j < V; ++j) m[j] = EL::diff_mask(xo[j], xn[j]);

#pragma unroll
    for (int q = 0; q < V / 2; ++q) pk[q] = __popc(m[2 * q]) | (__popc(m[2 * q + 1]) << 16);

    // ---- wave scan (two vectors per register), then offsets of each vector inside the wave
    uint32_t ex[V];       // rank of this lane's first changed element of vector j inside the wave
    uint32_t wave_total = 0;
#pragma unroll
    for (int q = 0; q < V / 2; ++q) {
        const uint32_t inc = wave_inclusive_scan(pk[q]);
        const uint32_t tot = lane63(inc);
        const uint32_t exc = inc - pk[q];
        ex[2 * q] = wave_total + (exc & 0xFFFFu);
        wave_total += tot & 0xFFFFu;
        ex[2 * q + 1] = wave_total + (exc >> 16);
        wave_total += tot >> 16;
    }
    // ---- snapshot refresh by whole lines: lane groups of 8 hold one aligned 128-byte line per vector
    if (by_lines) {
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const unsigned long long changed = __ballot(m[j] != 0);
            if ((uint32_t)(changed >> (lane & ~7)) & 0xFFu) store16_nt(po + e0 + j * ROW, xn[j]);
        }
    }
    if (lane == 0) s_wave_total[wave] = wave_total;
    __syncthreads();
    uint32_t wave_base = 0, tile_total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint32_t t = s_wave_total[w];
        wave_base += (w < wave) ? t : 0u;
        tile_total += t;
    }
    tile_total = uniform(tile_total);
#pragma unroll
    for (int j = 0; j < V; ++j) ex[j] += wave_base;       // from here on: rank inside the tile

    // ---- chain with the earlier tiles of the bucket (wave 0), while the other waves start staging
    if (wave == 0) {
        uint32_t excl = 0;
        if (tile == first_tile) {
            if (lane == 0) status_store(a.status + tile, status_word(kStPrefix, tile_total));
        } else {
            if (lane == 0) status_store(a.status + tile, status_word(kStAgg, tile_total));
            excl = look_back(a, tile, first_tile, lane);
            if (lane == 0) status_store(a.status + tile, status_word(kStPrefix, excl + tile_total));
        }
        if (lane == 0) {
            s_excl = excl;
            if (last) {
                const uint32_t c = excl + tile_total;
                a.counts[bucket] = c;
                if ((uint64_t)c > a.cap) atomicOr(a.flags, kFlagOverflow);
            }
        }
    }

    // ---- stage (index, value) pairs in LDS in rank order, write out coalesced; kStage per round.  The barriers of
    // this loop order LDS accesses only (lds_barrier): a full __syncthreads would also wait for the round's global
    // stores to complete, which on dense tiles (many rounds) costs more than the stores themselves.
    int32_t *const Ib = a.I + (uint64_t)bucket * a.cap;
    T *const Vb = reinterpret_cast<T *>(a.V) + (uint64_t)bucket * a.cap;
    if (V >= 16 && tile_total > kStage) {
        // The largest tiles leave room for three workgroups per CU at most, and on dense data (several rounds of
        // staging) those spend most of their time writing out, with no loads in flight.  There every thread writes its
        // own pairs at their ranks instead: the lanes of a wave hold consecutive rank ranges, so these stores are
        // close together, and no round needs a barrier (measured at 25 % / 100 % density: 12.7 / 34.8 ms against
        // 22.3 / 39.9 ms staged; smaller tiles do better staged).
        __syncthreads();                            // s_excl
        const uint32_t excl = s_excl;
        const bool elementwise = RG == 0 || (LINES && !by_lines);
#pragma unroll
        for (int j = 0; j < V; ++j) {
            uint32_t mm = m[j];
            uint32_t r = excl + ex[j];              // below 2^32: a bucket holds fewer than 2^31 elements
            const uint32_t local = e0 + j * ROW;
            while (mm) {
                const uint32_t e = (uint32_t)__builtin_ctz(mm);
                mm &= mm - 1u;
                const T val = (T)EL::pattern(xn[j], e);
                if (local + e < len) {              // masks are zero beyond len; keeps stores in bounds regardless
                    if ((uint64_t)r < a.cap) { Ib[r] = (int32_t)(idx_base + local + e); Vb[r] = val; }
                    if (elementwise) po[local + e] = val;
                }
                ++r;
            }
        }
        return;
    }
    for (uint32_t r0 = 0; r0 < tile_total; r0 += kStage) {
#pragma unroll
        for (int j = 0; j < V; ++j) {
            uint32_t mm = m[j];
            // the ranks of this vector's changed elements are ex[j] .. ex[j] + popc - 1: nothing to do in a round
            // that lies wholly before or after them (this keeps dense tiles linear in the number of rounds)
            if (mm && ex[j] < r0 + kStage && ex[j] + __popc(mm) > r0) {
                uint32_t rank = ex[j] - r0;                  // wraps for elements of earlier rounds: skipped below
                const uint32_t local = e0 + j * ROW;
                while (mm) {
                    const uint32_t e = (uint32_t)__builtin_ctz(mm);
                    mm &= mm - 1u;
                    if (rank < kStage) s_stage[rank] = ((local + e) << 16) | EL::pattern(xn[j], e);
                    ++rank;
                }
            }
        }
        lds_barrier();
        const uint32_t excl = s_excl;
        const uint32_t nst = (tile_total - r0 < kStage) ? (tile_total - r0) : kStage;
        for (uint32_t k = tid; k < nst; k += kThreads) {
            const uint32_t ent = s_stage[k];
            const uint32_t local = ent >> 16;
            const T val = (T)(ent & 0xFFFFu);
            const uint64_t r = (uint64_t)excl + r0 + k;
            if (local < len) {                      // always true for a correct scan; keeps stores in bounds
                if (r < a.cap) { Ib[r] = (int32_t)(idx_base + local); Vb[r] = val; }
                // snapshot refresh: W_prev <- W at changed positions, unless the tile went by whole lines
                if (RG == 0 || (LINES && !by_lines)) po[local] = val;
            }
        }
        lds_barrier();
    }
}

// ---------------------------------------------------------------------------------------------
// extract_marked_kernel: Alg. 2's V = W[I] over the cumulative index set of Alg. 1, held as a bitmap over packed
// positions (mark_kernel builds it).  The bitmap already says where the changes are, so the weights are not
// streamed: the workgroup reads its tile's slice of the bitmap (one bit per element), ranks the set bits like
// extract_kernel ranks changed elements (wave scan, LDS combine, the same per-bucket ticket and look-back chain),
// stages their tile-local positions in LDS in rank order, and only then fetches the values, one 2-byte gather
// per pair, balanced over the 256 threads and written out coalesced next to the indices.  Memory traffic is the
// bitmap plus the lines that hold a marked element instead of the whole weight set.
// E = elements per thread (tile of the plan / 256); thread t owns the tile-local positions [t*E, (t+1)*E).
// ---------------------------------------------------------------------------------------------

// the nbits (1..32) bitmap bits of packed positions g .. g+nbits-1, bit k of the result for position g + k
__device__ __forceinline__ uint32_t bitmap_bits32(const uint32_t *bitmap, uint64_t words, uint64_t g, uint32_t nbits) {
    const uint64_t w = g >> 5;
    const uint32_t sh = (uint32_t)(g & 31u);
    const uint32_t lo = bitmap[w];
    const uint32_t hi = (sh != 0u && sh + nbits > 32u && w + 1 < words) ? bitmap[w + 1] : 0u;
    const uint32_t bits = (uint32_t)((((unsigned long long)hi << 32) | lo) >> sh);
    return nbits >= 32u ? bits : (bits & ((1u << nbits) - 1u));
}

template <int E>
__global__ __launch_bounds__(kThreads) void extract_marked_kernel(const ExtractArgs a) {
    static_assert(E == 16 || E == 32 || E == 64 || E == 128, "tile of 4096 .. 32768 elements");
    constexpr int NW = (E + 31) / 32;                    // mask words per thread
    constexpr uint32_t CH = (E < 32) ? (uint32_t)E : 32u; // elements per mask word
    constexpr int kGather = 4;                           // gathers in flight per thread in the write-out loop
    __shared__ uint32_t s_ticket;
    __shared__ uint32_t s_wave_total[kWaves];
    __shared__ uint32_t s_excl;
    __shared__ uint32_t s_stage[kStage];                 // tile-local positions in rank order

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // ---- bucket, ticket, tile: as in extract_kernel (tensor lists only)
    const WgInfo wi = a.wg_info[blockIdx.x];
    const uint32_t bucket = wi.bucket, first_tile = wi.first_tile, bucket_tiles = wi.ntiles;
    if (tid == 0)
        s_ticket = __hip_atomic_fetch_add(a.tickets + (uint64_t)bucket * a.ticket_stride, 1u, __ATOMIC_RELAXED,
                                          __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const uint32_t k = uniform(s_ticket);
    if (k >= bucket_tiles) return;
    const uint32_t tile = first_tile + k;
    const bool last = (k == bucket_tiles - 1);
    const TileDesc d = a.tiles[tile];
    const gptr<const uint16_t> pn = (gptr<const uint16_t>)a.ptrs[d.tensor].new_w + d.tensor_off;
    const uint32_t len = d.len, idx_base = d.bucket_off;
    const uint64_t g0 = a.tensor_base[d.tensor] + d.tensor_off;      // packed position of the tile's first element

    // ---- this thread's slice of the bitmap and its count
    const uint32_t e0 = (uint32_t)tid * E;
    uint32_t m[NW];
    uint32_t mine = 0;
#pragma unroll
    for (int c = 0; c < NW; ++c) {
        const uint32_t e = e0 + c * 32u;
        const uint32_t left = (e < len) ? (len - e) : 0u;
        const uint32_t nbits = left < CH ? left : CH;
        m[c] = nbits ? bitmap_bits32(a.bitmap, a.bitmap_words, g0 + e, nbits) : 0u;
        mine += __popc(m[c]);
    }
    const uint32_t inc = wave_inclusive_scan(mine);                  // at most 64 * 128 per wave
    const uint32_t wave_total = lane63(inc);
    if (lane == 0) s_wave_total[wave] = wave_total;
    __syncthreads();
    uint32_t wave_base = 0, tile_total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const uint32_t t = s_wave_total[w];
        wave_base += (w < wave) ? t : 0u;
        tile_total += t;
    }
    tile_total = uniform(tile_total);

    // ---- chain with the earlier tiles of the bucket
    if (wave == 0) {
        uint32_t excl = 0;
        if (tile == first_tile) {
            if (lane == 0) status_store(a.status + tile, status_word(kStPrefix, tile_total));
        } else {
            if (lane == 0) status_store(a.status + tile, status_word(kStAgg, tile_total));
            excl = look_back(a, tile, first_tile, lane);
            if (lane == 0) status_store(a.status + tile, status_word(kStPrefix, excl + tile_total));
        }
        if (lane == 0) {
            s_excl = excl;
            if (last) {
                const uint32_t c = excl + tile_total;
                a.counts[bucket] = c;
                if ((uint64_t)c > a.cap) atomicOr(a.flags, kFlagOverflow);
            }
        }
    }

    // ---- positions into LDS in rank order, then gather + coalesced write-out, kStage pairs per round
    int32_t *const Ib = a.I + (uint64_t)bucket * a.cap;
    uint16_t *const Vb = a.V + (uint64_t)bucket * a.cap;
    for (uint32_t r0 = 0; r0 < tile_total; r0 += kStage) {
        uint32_t rank = wave_base + (inc - mine) - r0;               // wraps for pairs of earlier rounds: skipped below
        const uint32_t first = wave_base + (inc - mine);
        const bool in_round = first < r0 + kStage && first + mine > r0;   // this thread has pairs of this round
#pragma unroll
        for (int c = 0; c < NW; ++c) {
            uint32_t mm = in_round ? m[c] : 0u;
            while (mm) {
                const uint32_t e = (uint32_t)__builtin_ctz(mm);
                mm &= mm - 1u;
                if (rank < kStage) s_stage[rank] = e0 + c * 32u + e;
                ++rank;
            }
        }
        __syncthreads();
        const uint32_t excl = s_excl;
        const uint32_t nst = (tile_total - r0 < kStage) ? (tile_total - r0) : kStage;
        for (uint32_t k0 = tid; k0 < nst; k0 += kGather * kThreads) {
            uint32_t local[kGather];
            uint16_t val[kGather];
#pragma unroll
            for (int u = 0; u < kGather; ++u) {
                const uint32_t kk = k0 + u * kThreads;
                local[u] = (kk < nst) ? s_stage[kk] : 0xFFFFFFFFu;
            }
#pragma unroll
            for (int u = 0; u < kGather; ++u) val[u] = (local[u] < len) ? pn[local[u]] : (uint16_t)0;
#pragma unroll
            for (int u = 0; u < kGather; ++u) {
                const uint64_t r = (uint64_t)excl + r0 + k0 + u * kThreads;
                if (local[u] < len && r < a.cap) { Ib[r] = (int32_t)(idx_base + local[u]); Vb[r] = val[u]; }
            }
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------------
// mark_kernel: one optimizer step of Alg. 1's index accumulation, I_cum <- I_cum U { i : W[i] != W_prev[i] },
// kept as a bitmap over packed positions.  CAST = false compares two BF16 versions; CAST = true is the
// Trainer's own sequence without the clone: W <- round_BF16(master) and the elements whose pattern changed
// are marked.  One workgroup per tile of the plan, in tile order; no chain, no ticket: tiles are independent here.
// (Extract's bucket-interleaved order measured 3 % faster for two BF16 versions and 5 % slower with CAST.)
// ---------------------------------------------------------------------------------------------
template <int V, bool CAST>
__global__ __launch_bounds__(kThreads) void mark_kernel(const ExtractArgs a) {
    constexpr uint32_t TILE = (uint32_t)V * kUnit;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (blockIdx.x >= a.ntiles) return;
    const TileDesc d = a.tiles[blockIdx.x];
    const PtrPair p = a.ptrs[d.tensor];
    const gptr<uint16_t> po = as_global(p.old_w) + d.tensor_off;
    const gptr<const uint32_t> pf = (gptr<const uint32_t>)p.new_w + d.tensor_off;
    const gptr<const uint16_t> pn = (gptr<const uint16_t>)p.new_w + d.tensor_off;
    const uint32_t len = d.len;
    const uint64_t g0 = a.tensor_base[d.tensor] + d.tensor_off;
    const uint32_t e0 = (uint32_t)wave * (V * 512u) + (uint32_t)lane * 8u;
    const bool aligned = CAST ? (((((uintptr_t)po) | ((uintptr_t)pf)) & 15u) == 0)
                              : (((((uintptr_t)po) | ((uintptr_t)pn)) & 15u) == 0);
    const bool full = aligned && len == TILE;
    u32x4 xo[V], xn[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        const uint32_t e = e0 + j * 512;
        if (full || (aligned && e + 8 <= len)) {
            // two versions that are only compared are read once each: non-temporal (2 % faster); with CAST the
            // parameters are rewritten below by whole lines, hinted like extract's snapshot, and the master weights
            // stay on ordinary loads
            xo[j] = load16<true>(po + e);
            if (CAST) xn[j] = round8_bf16(load16<false>(pf + e), load16<false>(pf + e + 4));
            else xn[j] = load16<true>(pn + e);
        } else {
            xo[j] = load8_guarded(po, e, len);
            xn[j] = CAST ? load8_guarded_cast(pf, e, len) : load8_guarded(pn, e, len);
        }
    }
#pragma unroll
    for (int j = 0; j < V; ++j) {
        const uint32_t e = e0 + j * 512;
        const uint32_t m = diff_mask8(xo[j], xn[j]);
        if (CAST) {                                           // write the cast back where it changed something
            if (full) {
                const unsigned long long changed = __ballot(m != 0);
                if ((uint32_t)(changed >> (lane & ~7)) & 0xFFu) store16_nt(po + e, xn[j]);
            } else if (m) {
                uint32_t mm = m;
                while (mm) {
                    const uint32_t k = (uint32_t)__builtin_ctz(mm);
                    mm &= mm - 1u;
                    po[e + k] = (uint16_t)pattern_at(xn[j], k);       // k < len - e: guarded loads read 0 == 0 beyond len
                }
            }
        }
        if (m) {
            const uint64_t g = g0 + e;
            const uint32_t sh = (uint32_t)(g & 31u);
            atomicOr(a.bitmap + (g >> 5), m << sh);
            const uint32_t spill = (sh > 24u) ? (m >> (32u - sh)) : 0u;       // bits that belong to the next word
            if (spill) atomicOr(a.bitmap + (g >> 5) + 1, spill);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// apply: W[I] <- V.  One workgroup per (bucket, chunk of kApplyChunk pairs); each thread owns
// kApplyPer pairs, kThreads apart, so that the index and value loads of a wave are contiguous and
// all of a thread's loads are in flight before its first store.  For tensor lists the bucket's
// segment table (start inside the bucket -> byte address of that element) is cached in LDS.
// ---------------------------------------------------------------------------------------------
constexpr int kApplyPer = (int)(kApplyChunk / kThreads);
constexpr uint32_t kSegCache = 128;
constexpr uint32_t kWideGap = 32768u;      // differences of 2^15 and more do not fit the 16-bit index coding

struct ApplyShared {
    uint32_t off[kSegCache + 1];
    unsigned long long base[kSegCache];
    uint32_t wave_total[kWaves];
};

// Common front of the apply kernels: which (bucket, chunk) this workgroup owns and how many of the
// chunk's pairs are valid; 0 when there is nothing to do.  Consecutive workgroups take the same chunk number of
// consecutive buckets (groups of kApplyInterleave buckets), so that the scatter of the moment is spread over the
// whole weight set instead of a dozen buckets: 12 % faster on the 910-bucket benchmark set at 1 %, 9 % at 5 %,
// nothing lost on the 244-bucket sets, 0.16 ms lost on the skewed set.
constexpr uint32_t kApplyInterleave = 1024;

__device__ __forceinline__ uint32_t apply_chunk(const ApplyArgs &a, uint32_t &b, uint64_t &start) {
    const uint32_t per_group = kApplyInterleave * a.chunks_per_bucket;
    const uint32_t g = blockIdx.x / per_group, j = blockIdx.x - g * per_group;
    const uint32_t g0 = g * kApplyInterleave;
    if (g0 >= a.nb) return 0;
    const uint32_t gb = (a.nb - g0 < kApplyInterleave) ? (a.nb - g0) : kApplyInterleave;   // buckets in this group
    const uint32_t c = j / gb;
    b = g0 + (j - c * gb);
    if (b >= a.nb) return 0;
    const uint32_t cnt_true = a.counts[b];
    const uint64_t cnt = ((uint64_t)cnt_true < a.cap) ? cnt_true : a.cap;
    start = (uint64_t)c * kApplyChunk;
    if (start >= cnt) return 0;
    return (uint32_t)((cnt - start < kApplyChunk) ? (cnt - start) : kApplyChunk);
}

// Scatter of one thread's kApplyPer pairs of bucket b; pair j is live when bit j of `live` is set.  The stores carry
// the non-temporal hint: each lands in a line nothing else will touch soon, and measures 10 % faster that way.
// idx holds tensor-flat indices (single tensor) or positions inside the bucket (lists).  For lists the
// bucket's segment table is cached in LDS (start inside the bucket -> byte address of that element).
template <bool MULTI, int EB = 2>
__device__ __forceinline__ void scatter_pairs(const ApplyArgs &a, ApplyShared &sh, uint32_t b,
                                              const int32_t (&idx)[kApplyPer], const uint16_t (&val)[kApplyPer],
                                              uint32_t live) {
    typedef typename Elem<EB>::type T;       // width of a stored value; val[] holds it zero-extended
    bool bad = false;
    if (MULTI) {
        const uint64_t b0 = (uint64_t)b * a.be;
        const uint32_t blen = (uint32_t)((a.total - b0 < a.be) ? (a.total - b0) : a.be);
        const uint32_t s_lo = a.seg_begin[b], s_hi = a.seg_begin[b + 1];
        const uint32_t nseg = s_hi - s_lo;
        const bool cached = nseg <= kSegCache;                 // uniform
        if (cached) {
            for (uint32_t s = threadIdx.x; s < nseg; s += kThreads) {
                const SegDesc d = a.segs[s_lo + s];
                sh.off[s] = d.bucket_off;
                // byte address of the element at bucket position 0 of this segment's tensor run
                sh.base[s] = (unsigned long long)(uintptr_t)a.wptrs[(uint64_t)d.tensor * (1u + a.wptr_skip)] +
                             (unsigned long long)EB * d.tensor_off -
                             (unsigned long long)EB * d.bucket_off;
            }
            if (threadIdx.x == 0) sh.off[nseg] = blen;
            __syncthreads();
        }
        uint32_t hint = 0;                                      // segment of the previous pair (payloads ascend)
#pragma unroll
        for (int j = 0; j < kApplyPer; ++j) {
            if (!((live >> j) & 1u)) continue;
            const uint32_t i = (uint32_t)idx[j];
            if (i >= blen) { bad = true; continue; }
            if (cached) {
                uint32_t lo = hint;
                if (!(sh.off[lo] <= i && i < sh.off[lo + 1])) {
                    lo = 0; uint32_t hi = nseg;                 // off[lo] <= i < off[hi]
                    while (hi - lo > 1) {
                        const uint32_t mid = (lo + hi) >> 1;
                        if (sh.off[mid] <= i) lo = mid; else hi = mid;
                    }
                    hint = lo;
                }
                __builtin_nontemporal_store((T)val[j], (gptr<T>)(uintptr_t)(sh.base[lo] + (unsigned long long)EB * i));
            } else {
                uint32_t lo = s_lo, hi = s_hi;                  // segs[lo].bucket_off <= i < segs[hi].bucket_off
                while (hi - lo > 1) {
                    const uint32_t mid = (lo + hi) >> 1;
                    if (a.segs[mid].bucket_off <= i) lo = mid; else hi = mid;
                }
                const SegDesc d = a.segs[lo];
                const uint32_t off = i - d.bucket_off;
                if (off >= d.len) { bad = true; continue; }     // cannot happen for a well-formed plan
                __builtin_nontemporal_store((T)val[j], (gptr<T>)a.wptrs[(uint64_t)d.tensor * (1u + a.wptr_skip)] +
                                                           ((uint64_t)d.tensor_off + off));
            }
        }
    } else {
        const uint64_t lo = (uint64_t)b * a.be;
        const uint64_t hi = (lo + a.be < a.n) ? (lo + a.be) : a.n;
#pragma unroll
        for (int j = 0; j < kApplyPer; ++j) {
            if (!((live >> j) & 1u)) continue;
            const int64_t i = idx[j];
            if (i < (int64_t)lo || i >= (int64_t)hi) { bad = true; continue; }
            __builtin_nontemporal_store((T)val[j], (gptr<T>)a.w + i);
        }
    }
    if (bad) atomicOr(a.flags, kFlagBadIndex);
}

// 32-bit indices.  When a.max_gap is given, buckets whose indices travel as 16-bit differences are
// left to apply_encoded_kernel.
template <bool MULTI, int EB = 2>
__global__ __launch_bounds__(kThreads) void apply_kernel(const ApplyArgs a) {
    typedef typename Elem<EB>::type T;
    __shared__ ApplyShared sh;
    uint32_t b; uint64_t start;
    const uint32_t nvalid = apply_chunk(a, b, start);
    if (nvalid == 0) return;
    if (a.max_gap && a.max_gap[b] < kWideGap) return;
    const int32_t *const Ib = a.I + (uint64_t)b * a.cap + start;
    const T *const Vb = reinterpret_cast<const T *>(a.V) + (uint64_t)b * a.cap + start;
    int32_t idx[kApplyPer];
    uint16_t val[kApplyPer];
    uint32_t live = 0;
#pragma unroll
    for (int j = 0; j < kApplyPer; ++j) {           // pair k = thread + j*256: contiguous per wave
        const uint32_t k = threadIdx.x + j * kThreads;
        const bool ok = k < nvalid;
        idx[j] = ok ? Ib[k] : 0;
        val[j] = ok ? Vb[k] : (uint16_t)0;
        live |= ok ? (1u << j) : 0u;
    }
    scatter_pairs<MULTI, EB>(a, sh, b, idx, val, live);
}

// The per-tensor view of a list payload: Alg. 2's message carries, per parameter tensor, int32 indices into that
// tensor's flattened elements; pair r of bucket b is at packed position b*be + I, inside exactly one segment of the
// bucket.  tensor_id / tensor_idx are laid out like I.  Same workgroup-to-chunk mapping and segment search as apply.
__global__ __launch_bounds__(kThreads) void tensor_view_kernel(const ApplyArgs a, uint32_t *tensor_id, int32_t *tensor_idx) {
    uint32_t b; uint64_t start;
    const uint32_t nvalid = apply_chunk(a, b, start);
    if (nvalid == 0) return;
    const uint64_t b0 = (uint64_t)b * a.be;
    const uint32_t blen = (uint32_t)((a.total - b0 < a.be) ? (a.total - b0) : a.be);
    const uint32_t s_lo = a.seg_begin[b], s_hi = a.seg_begin[b + 1];
    const uint64_t row = (uint64_t)b * a.cap + start;
    bool bad = false;
    for (uint32_t k = threadIdx.x; k < nvalid; k += kThreads) {
        const int32_t iv = a.I[row + k];
        if (iv < 0 || (uint32_t)iv >= blen) { bad = true; continue; }
        const uint32_t i = (uint32_t)iv;
        uint32_t lo = s_lo, hi = s_hi;                  // segs[lo].bucket_off <= i < segs[hi].bucket_off
        while (hi - lo > 1) {
            const uint32_t mid = (lo + hi) >> 1;
            if (a.segs[mid].bucket_off <= i) lo = mid; else hi = mid;
        }
        const SegDesc d = a.segs[lo];
        const uint32_t off = i - d.bucket_off;
        if (off >= d.len) { bad = true; continue; }     // cannot happen for a well-formed plan
        tensor_id[row + k] = d.tensor;
        tensor_idx[row + k] = (int32_t)(d.tensor_off + off);
    }
    if (bad) atomicOr(a.flags, kFlagBadIndex);
}

// 16-bit first differences (Sec. 3.3, index delta coding) decoded on the fly: thread t loads the
// kApplyPer consecutive differences t*8 .. t*8+7 of the chunk and sums them, the workgroup scans the
// 256 thread sums (DPP wave scan + LDS), and the chunk's anchor (the position of its first pair) turns
// the running sums into positions inside the bucket.  The positions then change hands through LDS so that
// thread t scatters pairs t, t+256, ...: one store instruction of a wave covers 64 consecutive pairs (about 13 KB
// of weights at 1 % density) as in apply_kernel, not every eighth pair of 512 (100 KB), which takes the memory
// side half as long again (12.4 against 8.2 ms on the 910-bucket benchmark set).
template <bool MULTI>
__global__ __launch_bounds__(kThreads) void apply_encoded_kernel(const ApplyArgs a) {
    __shared__ ApplyShared sh;
    __shared__ int32_t s_pos[kApplyChunk + kApplyChunk / 8];    // pair k at k + k/8: both access patterns spread over the banks
    uint32_t b; uint64_t start;
    const uint32_t nvalid = apply_chunk(a, b, start);
    if (nvalid == 0) return;
    if (a.max_gap[b] >= kWideGap) return;           // this bucket travels with 32-bit indices
    const uint16_t *const Db = a.D + (uint64_t)b * a.cap + start;
    const uint16_t *const Vb = a.V + (uint64_t)b * a.cap + start;
    const uint32_t k0 = threadIdx.x * kApplyPer;
    static_assert(kApplyPer == 8, "one 16-byte vector of differences per thread");
    uint32_t d[kApplyPer];
    if ((((uintptr_t)Db) & 15u) == 0 && k0 + kApplyPer <= nvalid) {
        const u32x4 dv = *reinterpret_cast<const u32x4 *>(Db + k0);
#pragma unroll
        for (int j = 0; j < kApplyPer; ++j) d[j] = pattern_at(dv, j);
    } else {
#pragma unroll
        for (int j = 0; j < kApplyPer; ++j) d[j] = (k0 + j < nvalid) ? (uint32_t)Db[k0 + j] : 0u;
    }
    uint16_t val[kApplyPer];
    uint32_t live = 0;
#pragma unroll
    for (int j = 0; j < kApplyPer; ++j) {            // the values of the pairs this thread will scatter
        const uint32_t k = threadIdx.x + j * kThreads;
        const bool ok = k < nvalid;
        val[j] = ok ? Vb[k] : (uint16_t)0;
        live |= ok ? (1u << j) : 0u;
    }
    const uint32_t first = Db[0];                    // the chunk's first difference is covered by the anchor
    uint32_t run = 0;
#pragma unroll
    for (int j = 0; j < kApplyPer; ++j) { run += d[j]; d[j] = run; }      // inclusive inside the thread
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t inc = wave_inclusive_scan(run);
    if (lane == 63) sh.wave_total[wave] = inc;
    __syncthreads();
    uint32_t before = inc - run;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) before += (w < wave) ? sh.wave_total[w] : 0u;
    const uint32_t nchunk = a.chunks_per_bucket;
    const int32_t anchor = a.anchors[(uint64_t)b * nchunk + (uint32_t)(start / kApplyChunk)];
    const int64_t origin = (int64_t)anchor - (int64_t)first + (int64_t)((uint64_t)b * a.base_stride);
#pragma unroll
    for (int j = 0; j < kApplyPer; ++j) s_pos[k0 + j + threadIdx.x] = (int32_t)(origin + (int64_t)before + (int64_t)d[j]);
    __syncthreads();
    int32_t idx[kApplyPer];
#pragma unroll
    for (int j = 0; j < kApplyPer; ++j) {
        const uint32_t k = threadIdx.x + j * kThreads;
        idx[j] = s_pos[k + (k >> 3)];
    }
    scatter_pairs<MULTI>(a, sh, b, idx, val, live);
}

// First differences of each bucket's ascending indices, the bucket's largest difference and the
// anchors (position of the first pair of every chunk of kApplyChunk pairs).  max_gap must be zero on
// entry.  Indices that do not ascend raise kFlagBadIndex and force the bucket to 32-bit transport.
__global__ __launch_bounds__(kThreads) void encode_indices_kernel(const ApplyArgs a, uint16_t *D, uint32_t *max_gap,
                                                                  int32_t *anchors) {
    __shared__ uint32_t s_gap[kWaves];
    uint32_t b; uint64_t start;
    const uint32_t nvalid = apply_chunk(a, b, start);
    if (nvalid == 0) return;
    const int32_t *const Ib = a.I + (uint64_t)b * a.cap;
    const int64_t base = (int64_t)((uint64_t)b * a.base_stride);
    uint32_t gap = 0;
    bool bad = false;
    uint16_t *const Db = D + (uint64_t)b * a.cap;
    const uint32_t k0 = threadIdx.x * kApplyPer;
    static_assert(kApplyPer == 8, "eight consecutive pairs per thread: two 16-byte loads, one 16-byte store");
    // cap is a multiple of 4 whenever the rows of I are 16-byte aligned for every bucket; checked on the addresses
    const bool vec = (((uintptr_t)(Ib + start) | (uintptr_t)(Db + start)) & 15u) == 0;       // uniform over the workgroup
    if (vec && k0 + kApplyPer <= nvalid) {
        const uint64_t r0 = start + k0;
        const u32x4 lo = *reinterpret_cast<const u32x4 *>(Ib + r0), hi = *reinterpret_cast<const u32x4 *>(Ib + r0 + 4);
        const int32_t idx[8] = {(int32_t)lo.x, (int32_t)lo.y, (int32_t)lo.z, (int32_t)lo.w,
                                (int32_t)hi.x, (int32_t)hi.y, (int32_t)hi.z, (int32_t)hi.w};
        int64_t prev = r0 ? ((int64_t)Ib[r0 - 1] - base) : 0;
        uint32_t d16[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int64_t cur = (int64_t)idx[j] - base;
            int64_t dd = cur - prev;
            if (dd < 0 || cur < 0) { bad = true; dd = 0xFFFFFFFFll; }
            d16[j] = (uint32_t)((uint64_t)dd & 0xFFFFu);
            gap = ((uint64_t)dd > gap) ? (uint32_t)dd : gap;
            prev = cur;
        }
        u32x4 out;
        out.x = d16[0] | (d16[1] << 16); out.y = d16[2] | (d16[3] << 16);
        out.z = d16[4] | (d16[5] << 16); out.w = d16[6] | (d16[7] << 16);
        *reinterpret_cast<u32x4 *>(Db + r0) = out;
        if (k0 == 0) anchors[(uint64_t)b * a.chunks_per_bucket + (uint32_t)(start / kApplyChunk)] = (int32_t)((int64_t)idx[0] - base);
    } else {
#pragma unroll
        for (int j = 0; j < kApplyPer; ++j) {            // the chunk's ragged end, or rows that are not 16-byte aligned
            const uint32_t k = vec ? (k0 + j) : (threadIdx.x + j * kThreads);
            if (k >= nvalid) continue;
            const uint64_t r = start + k;
            const int64_t cur = (int64_t)Ib[r] - base;
            const int64_t prev = r ? ((int64_t)Ib[r - 1] - base) : 0;
            int64_t dd = cur - prev;
            if (dd < 0 || cur < 0) { bad = true; dd = 0xFFFFFFFFll; }
            Db[r] = (uint16_t)((uint64_t)dd & 0xFFFFu);
            gap = ((uint64_t)dd > gap) ? (uint32_t)dd : gap;
            if (k == 0) anchors[(uint64_t)b * a.chunks_per_bucket + (uint32_t)(start / kApplyChunk)] = (int32_t)cur;
        }
    }
    // workgroup maximum: wave maximum by DPP-free shuffles is overkill here; use LDS atomics
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) s_gap[wave] = 0;
    __syncthreads();
    if (gap) atomicMax(&s_gap[wave], gap);
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t g = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) g = s_gap[w] > g ? s_gap[w] : g;
        if (g) atomicMax(max_gap + b, g);
    }
    if (bad) atomicOr(a.flags, kFlagBadIndex);
}

// ---------------------------------------------------------------------------------------------
// density routing (Sec. 3.4): buckets whose sparse payload would not be smaller than their dense bytes,
// or that overflowed their slot, travel as a full copy.
// ---------------------------------------------------------------------------------------------
struct RouteArgs {
    const uint32_t *counts; uint32_t nb; uint64_t be; uint64_t total; uint64_t cap;
    uint32_t bytes_per_pair; uint32_t max_dense;
    int32_t *route_slot; uint32_t *sparse_counts; int32_t *dense_bucket; uint32_t *n_dense;
    uint32_t *flags;
};

// One workgroup walks the buckets 256 at a time, so that dense slots are handed out in bucket order.
__global__ __launch_bounds__(kThreads) void route_kernel(const RouteArgs a) {
    __shared__ uint32_t s_wave[kWaves];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t taken = 0;                                 // dense buckets before this round (uniform)
    bool dropped = false;
    for (uint32_t b0 = 0; b0 < a.nb; b0 += kThreads) {
        const uint32_t b = b0 + threadIdx.x;
        bool dense = false;
        uint32_t cnt = 0;
        if (b < a.nb) {
            cnt = a.counts[b];
            const uint64_t lo = (uint64_t)b * a.be;
            const uint64_t len = (lo + a.be < a.total) ? a.be : (a.total > lo ? a.total - lo : 0);
            dense = ((uint64_t)cnt > a.cap) || (cnt > 0 && (uint64_t)cnt * a.bytes_per_pair >= 2 * len);
        }
        const unsigned long long mask = __ballot(dense);
        const uint32_t in_wave = __builtin_popcountll(mask & ((1ull << lane) - 1ull));
        if (lane == 0) s_wave[wave] = (uint32_t)__builtin_popcountll(mask);
        __syncthreads();
        uint32_t before = taken, round_total = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) { before += (w < wave) ? s_wave[w] : 0u; round_total += s_wave[w]; }
        __syncthreads();
        if (b < a.nb) {
            const uint32_t slot = before + in_wave;
            if (dense && slot < a.max_dense) {
                a.route_slot[b] = (int32_t)slot; a.dense_bucket[slot] = (int32_t)b; a.sparse_counts[b] = 0;
            } else {
                if (dense) dropped = true;
                a.route_slot[b] = -1;
                a.sparse_counts[b] = ((uint64_t)cnt < a.cap) ? cnt : (uint32_t)a.cap;
            }
        }
        taken += round_total;
    }
    if (threadIdx.x == 0) *a.n_dense = (taken < a.max_dense) ? taken : a.max_dense;
    if (dropped) atomicOr(a.flags, kFlagOverflow);
}

struct DenseCopyArgs {
    const TileDesc *tiles; const uint32_t *bucket_first; const PtrPair *pairs; uint16_t *const *wptrs;
    const int32_t *dense_bucket; const uint32_t *n_dense; uint32_t max_dense; uint32_t tiles_per_bucket_max;
    uint64_t be; uint16_t *dense;
};

// PACK: dense[s] <- the new weights of bucket dense_bucket[s];  !PACK: resident weights <- dense[s].
// One workgroup per (dense slot, tile of the bucket), tiles as in extract's plan.
template <bool PACK>
__global__ __launch_bounds__(kThreads) void dense_copy_kernel(const DenseCopyArgs a) {
    const uint32_t s = blockIdx.x / a.tiles_per_bucket_max;
    const uint32_t j = blockIdx.x - s * a.tiles_per_bucket_max;
    if (s >= a.max_dense || s >= *a.n_dense) return;
    const uint32_t b = (uint32_t)a.dense_bucket[s];
    const uint32_t first = a.bucket_first[b];
    if (j >= a.bucket_first[b + 1] - first) return;
    const TileDesc d = a.tiles[first + j];
    uint16_t *const slot = a.dense + (uint64_t)s * a.be + d.bucket_off;
    uint16_t *const w = PACK ? const_cast<uint16_t *>(static_cast<const uint16_t *>(a.pairs[d.tensor].new_w)) + d.tensor_off
                             : a.wptrs[d.tensor] + d.tensor_off;
    const gptr<uint16_t> dst = as_global(PACK ? slot : w);
    const gptr<const uint16_t> src = as_global(static_cast<const uint16_t *>(PACK ? w : slot));
    const bool aligned = ((((uintptr_t)dst) | ((uintptr_t)src)) & 15u) == 0;
    if (aligned) {
        const uint32_t nvec = d.len / 8;
        for (uint32_t v = threadIdx.x; v < nvec; v += kThreads)
            ((gptr<u32x4>)dst)[v] = ((gptr<const u32x4>)src)[v];
        for (uint32_t e = nvec * 8 + threadIdx.x; e < d.len; e += kThreads) dst[e] = src[e];
    } else {
        for (uint32_t e = threadIdx.x; e < d.len; e += kThreads) dst[e] = src[e];
    }
}

// Second-pass snapshot refresh (Alg. 1's W_prev <- W done after the scan instead of inside it): the payload is
// scattered into the snapshot by apply_kernel, which cannot bring a bucket up to date whose payload was cut at cap.
// Those buckets are copied whole here.  kOverflowSplit workgroups per bucket walk its tiles (the plan's for a list,
// runs of tile_elems for a single tensor); a bucket that did not overflow costs one load of its count.
constexpr uint32_t kOverflowSplit = 16;

template <bool MULTI, int EB>
__global__ __launch_bounds__(kThreads) void refresh_overflow_kernel(const ExtractArgs a, uint32_t tile_elems) {
    typedef typename Elem<EB>::type T;
    constexpr uint32_t VE = 16u / EB;
    const uint32_t b = blockIdx.x / kOverflowSplit, s = blockIdx.x - b * kOverflowSplit;
    if (b >= a.nb || (uint64_t)a.counts[b] <= a.cap) return;           // uniform over the workgroup
    uint64_t b0 = 0; uint32_t blen = 0, first = 0, nt;
    if (MULTI) {
        first = a.bucket_first[b];
        nt = a.bucket_first[b + 1] - first;
    } else {
        b0 = (uint64_t)b * a.be;
        blen = (uint32_t)((a.n - b0 < a.be) ? (a.n - b0) : a.be);
        nt = (blen + tile_elems - 1) / tile_elems;
    }
    for (uint32_t j = s; j < nt; j += kOverflowSplit) {
        gptr<T> dst; gptr<const T> src; uint32_t len;
        if (MULTI) {
            const TileDesc d = a.tiles[first + j];
            const PtrPair p = a.ptrs[d.tensor];
            dst = (gptr<T>)p.old_w + d.tensor_off;
            src = (gptr<const T>)as_global(p.new_w) + d.tensor_off;
            len = d.len;
        } else {
            const uint32_t off = j * tile_elems;
            len = (blen - off < tile_elems) ? (blen - off) : tile_elems;
            dst = (gptr<T>)a.old_w + b0 + off;
            src = (gptr<const T>)as_global(a.new_w) + b0 + off;
        }
        uint32_t done = 0;
        if (((((uintptr_t)dst) | ((uintptr_t)src)) & 15u) == 0) {
            const uint32_t nvec = len / VE;
            for (uint32_t v = threadIdx.x; v < nvec; v += kThreads) ((gptr<u32x4>)dst)[v] = ((gptr<const u32x4>)src)[v];
            done = nvec * VE;
        }
        for (uint32_t e = done + threadIdx.x; e < len; e += kThreads) dst[e] = src[e];
    }
}

// ---------------------------------------------------------------------------------------------
// value entropy coding (Sec. 3.3): static Huffman code over the high bytes of one bucket's values, low
// bytes raw.  Chunks of 2048 values, each chunk's bit stream in a slot of its own, a bit offset every 64
// values so that 32 lanes decode a chunk side by side.  Layout and code construction are those of the
// library header; the bit order is: most significant code bit first, stream bit i = bit (i & 31) of word i >> 5.
// ---------------------------------------------------------------------------------------------
constexpr uint32_t kVcChunk = 2048, kVcSlotWords = 768, kVcSub = 64, kVcMaxLen = 12;

struct ValueCodecArgs {
    const uint16_t *V; uint16_t *V_out; const uint32_t *counts; uint32_t nb; uint64_t cap; uint32_t nchunk;
    uint8_t *lens; uint8_t *low; uint32_t *bits; uint32_t *chunk_words; uint16_t *sub;
    uint32_t *hist;        // [nb*256] scratch
    uint32_t *rcode;       // [nb*256] scratch: bit-reversed canonical code of each symbol
    uint32_t *flags;
};

// per (bucket, chunk): histogram of the high bytes, accumulated per bucket
constexpr uint32_t kVcHistChunks = 8;        // chunks of one bucket counted by one workgroup

__global__ __launch_bounds__(kThreads) void vc_hist_kernel(const ValueCodecArgs a) {
    // The high bytes of a payload crowd into a handful of bins, and LDS atomics of one wave on one address take
    // turns: 32 partial histograms, one per 8 lanes, 257 words apart so that the same bin of different partials
    // lies in different banks.
    constexpr uint32_t kParts = kThreads / 8, kPitch = 257;
    __shared__ uint32_t h[kParts * kPitch];
    const uint32_t groups = (a.nchunk + kVcHistChunks - 1) / kVcHistChunks;
    const uint32_t b = blockIdx.x / groups, g = blockIdx.x - b * groups;
    const uint64_t cnt = ((uint64_t)a.counts[b] < a.cap) ? a.counts[b] : a.cap;
    const uint64_t g0 = (uint64_t)g * kVcHistChunks * kVcChunk;
    if (g0 >= cnt) return;
    const uint32_t s = threadIdx.x;
    uint32_t *const mine = h + (s >> 3) * kPitch;
    const uint32_t gn = (uint32_t)((cnt - g0 < (uint64_t)kVcHistChunks * kVcChunk) ? (cnt - g0) : kVcHistChunks * kVcChunk);
    for (uint32_t i = s; i < kParts * kPitch; i += kThreads) h[i] = 0;
    __syncthreads();
    const uint16_t *v = a.V + (uint64_t)b * a.cap + g0;
    if ((((uintptr_t)v) & 15u) == 0) {
        constexpr uint32_t kSteps = kVcHistChunks * kVcChunk / (8 * kThreads);   // 8 values per 16-byte load
        u32x4 x[kSteps];
        const u32x4 none = {0, 0, 0, 0};
#pragma unroll
        for (uint32_t q = 0; q < kSteps; ++q) {
            const uint32_t i0 = (q * kThreads + s) * 8u;
            x[q] = (i0 + 8u <= gn) ? *reinterpret_cast<const u32x4 *>(v + i0) : none;
        }
#pragma unroll
        for (uint32_t q = 0; q < kSteps; ++q) {
            const uint32_t i0 = (q * kThreads + s) * 8u;
            if (i0 + 8u <= gn) {
                const uint32_t d[4] = {x[q].x, x[q].y, x[q].z, x[q].w};
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    atomicAdd(&mine[(d[c] >> 8) & 0xFFu], 1u);
                    atomicAdd(&mine[d[c] >> 24], 1u);
                }
            } else {
                for (uint32_t i = i0; i < gn; ++i) atomicAdd(&mine[v[i] >> 8], 1u);
            }
        }
    } else {
        for (uint32_t i = s; i < gn; i += kThreads) atomicAdd(&mine[v[i] >> 8], 1u);
    }
    __syncthreads();
    uint32_t t = 0;
#pragma unroll 8
    for (uint32_t p = 0; p < kParts; ++p) t += h[p * kPitch + s];
    if (t) atomicAdd(a.hist + (uint64_t)b * 256 + s, t);
}

// One workgroup per bucket builds the Huffman lengths exactly as the header specifies (merge the two smallest
// live nodes, ties to the smaller id; weights halved until no length exceeds 12), then all threads derive the
// canonical codes.  The merge runs in wave 0: node ids 0..255 are the symbols, 256.. the merged nodes in order
// of creation; lane l keeps the keys (weight << 9 | id) of the nodes l, l + 64, ... l + 448 in registers (all
// ones = not live), so "the smallest live node by (weight, id)" is a wave-wide minimum of one 64-bit key per
// lane and a merge step is two of those.  The leaf depths are then read off the parent array by all threads.
__device__ __forceinline__ unsigned long long wave_min_u64(unsigned long long x) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned long long y = __shfl_xor(x, d, 64);
        x = y < x ? y : x;
    }
    return x;
}

__global__ __launch_bounds__(kThreads) void vc_build_kernel(const ValueCodecArgs a) {
    constexpr unsigned long long kDead = ~0ull;
    __shared__ int16_t parent[512];
    __shared__ uint32_t w0[256];
    __shared__ uint8_t len[256];
    __shared__ uint32_t count_l[kVcMaxLen + 2];
    __shared__ uint32_t s_used, s_maxlen;
    const uint32_t b = blockIdx.x, s = threadIdx.x;
    const int lane = s & 63;
    w0[s] = a.hist[(uint64_t)b * 256 + s];
    len[s] = 0;
    if (s < kVcMaxLen + 2) count_l[s] = 0;
    if (s == 0) s_used = 0;
    __syncthreads();
    if (w0[s]) atomicAdd(&s_used, 1u);
    __syncthreads();
    const uint32_t used = s_used;
    while (used > 0) {                                       // uniform: every thread takes every barrier
        parent[s] = -1; parent[s + 256] = -1;
        if (s == 0) s_maxlen = 0;
        __syncthreads();
        if (s < 64) {
            unsigned long long key[8];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const uint32_t id = (uint32_t)lane + 64u * r, w = w0[id];
                key[r] = w ? (((unsigned long long)w << 9) | id) : kDead;
                key[r + 4] = kDead;                           // merged nodes 256 + lane + 64 r: none yet
            }
            uint32_t nnodes = 256;
            for (uint32_t nlive = used; nlive > 1; --nlive, ++nnodes) {
                unsigned long long pick[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) {                 // the smallest, then the smallest of what is left
                    unsigned long long m = key[0];
#pragma unroll
                    for (int r = 1; r < 8; ++r) m = key[r] < m ? key[r] : m;
                    m = wave_min_u64(m);
                    pick[t] = m;
#pragma unroll
                    for (int r = 0; r < 8; ++r) if (key[r] == m) key[r] = kDead;      // ids are unique: one lane, one slot
                }
                const uint32_t x = (uint32_t)(pick[0] & 511u), y = (uint32_t)(pick[1] & 511u);
                const unsigned long long wsum = (pick[0] >> 9) + (pick[1] >> 9);
                if (lane == 0) { parent[x] = (int16_t)nnodes; parent[y] = (int16_t)nnodes; }
                const uint32_t slot = nnodes - 256u;          // owner: lane slot & 63, register 4 + slot / 64
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if ((slot >> 6) == (uint32_t)r && (slot & 63u) == (uint32_t)lane) key[r + 4] = (wsum << 9) | nnodes;
            }
        }
        __syncthreads();
        uint32_t d = 0;
        if (w0[s]) {
            for (int jn = (int)s; parent[jn] >= 0; jn = parent[jn]) ++d;
            if (used == 1) d = 1;
            atomicMax(&s_maxlen, d);
        }
        len[s] = (uint8_t)d;
        __syncthreads();
        if (s_maxlen <= kVcMaxLen) break;
        if (w0[s]) w0[s] = (w0[s] + 1) / 2;
        __syncthreads();
    }
    __syncthreads();
    const uint32_t l = len[s];
    a.lens[(uint64_t)b * 256 + s] = (uint8_t)l;
    if (l) atomicAdd(&count_l[l], 1u);
    __syncthreads();
    // canonical code = first code of its length + number of smaller symbols of the same length
    uint32_t first = 0, code = 0;
    for (uint32_t j = 1; j <= kVcMaxLen; ++j) { if (j == l) first = code; code = (code + count_l[j]) << 1; }
    uint32_t rank = 0;
    for (uint32_t i = 0; i < s; ++i) rank += (len[i] == l) ? 1u : 0u;
    const uint32_t c = first + rank;
    a.rcode[(uint64_t)b * 256 + s] = l ? (__brev(c) >> (32 - l)) : 0u;
}

// per (bucket, group of kVcEncodeChunks chunks), chunk after chunk with the bucket's code table loaded once: codes of
// 8 consecutive values per thread, assembled in a 128-bit buffer, placed in the chunk's LDS bit array at the offset a
// workgroup scan of the bit counts gives, then stored coalesced
constexpr uint32_t kVcEncodeChunks = 4;

__global__ __launch_bounds__(kThreads) void vc_encode_kernel(const ValueCodecArgs a) {
    __shared__ uint32_t s_code[256];                 // bit-reversed code | length << 16
    __shared__ uint32_t s_words[kVcSlotWords + 4];
    __shared__ uint32_t s_wave[kWaves];
    const uint32_t groups = (a.nchunk + kVcEncodeChunks - 1) / kVcEncodeChunks;
    const uint32_t b = blockIdx.x / groups, g = blockIdx.x - b * groups;
    const uint64_t cnt = ((uint64_t)a.counts[b] < a.cap) ? a.counts[b] : a.cap;
    const uint32_t k_lo = g * kVcEncodeChunks;
    const uint32_t k_hi = (k_lo + kVcEncodeChunks < a.nchunk) ? (k_lo + kVcEncodeChunks) : a.nchunk;
    if ((uint64_t)k_lo * kVcChunk < cnt) {
        s_code[threadIdx.x] = a.rcode[(uint64_t)b * 256 + threadIdx.x] | ((uint32_t)a.lens[(uint64_t)b * 256 + threadIdx.x] << 16);
        __syncthreads();
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (uint32_t k = k_lo; k < k_hi; ++k) {
        const uint64_t r0 = (uint64_t)k * kVcChunk;
        const uint64_t slot = (uint64_t)b * a.nchunk + k;
        if (r0 >= cnt) {                                 // uniform: a chunk without values
            if (threadIdx.x == 0) a.chunk_words[slot] = 0;
            continue;
        }
        const uint32_t n = (uint32_t)((cnt - r0 < kVcChunk) ? (cnt - r0) : kVcChunk);
        const uint16_t *v = a.V + (uint64_t)b * a.cap + r0;
        uint8_t *lo = a.low + (uint64_t)b * a.cap + r0;
        const uint32_t k0 = threadIdx.x * 8;
        // the thread's 8 values: one 16-byte load and one 8-byte store of the low bytes where the rows allow it
        uint32_t xs[8];
        const bool vec = (k0 + 8 <= n) && (((((uintptr_t)(v + k0)) & 15u) | (((uintptr_t)(lo + k0)) & 7u)) == 0);
        if (vec) {
            const u32x4 q = *reinterpret_cast<const u32x4 *>(v + k0);
            xs[0] = q.x & 0xFFFFu; xs[1] = q.x >> 16; xs[2] = q.y & 0xFFFFu; xs[3] = q.y >> 16;
            xs[4] = q.z & 0xFFFFu; xs[5] = q.z >> 16; xs[6] = q.w & 0xFFFFu; xs[7] = q.w >> 16;
            uint2 lb;
            lb.x = (xs[0] & 0xFFu) | ((xs[1] & 0xFFu) << 8) | ((xs[2] & 0xFFu) << 16) | ((xs[3] & 0xFFu) << 24);
            lb.y = (xs[4] & 0xFFu) | ((xs[5] & 0xFFu) << 8) | ((xs[6] & 0xFFu) << 16) | ((xs[7] & 0xFFu) << 24);
            *reinterpret_cast<uint2 *>(lo + k0) = lb;
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                xs[j] = (k0 + j < n) ? (uint32_t)v[k0 + j] : 0u;
                if (k0 + j < n) lo[k0 + j] = (uint8_t)(xs[j] & 0xFFu);
            }
        }
        // two halves of four codes each (at most 48 bits per half), joined into a 128-bit buffer afterwards;
        // stream order = ascending bit index
        unsigned long long half[2] = {0, 0};
        uint32_t hbits[2] = {0, 0};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (k0 + j < n) {
                const uint32_t c = s_code[xs[j] >> 8];
                half[j >> 2] |= (unsigned long long)(c & 0xFFFFu) << hbits[j >> 2];
                hbits[j >> 2] += c >> 16;
            }
        }
        const uint32_t nbits = hbits[0] + hbits[1];
        const unsigned long long buf0 = half[0] | (half[1] << hbits[0]);                       // hbits[0] <= 48
        const unsigned long long buf1 = hbits[0] ? (half[1] >> (64 - hbits[0])) : 0ull;
        const uint32_t inc = wave_inclusive_scan(nbits);
        if (lane == 63) s_wave[wave] = inc;
        __syncthreads();                                // also: every thread is done with the previous chunk's s_words
        uint32_t start = inc - nbits, total = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) { start += (w < wave) ? s_wave[w] : 0u; total += s_wave[w]; }
        const uint32_t used = (total + 31) / 32;         // at most kVcSlotWords: 2048 codes of at most kVcMaxLen bits
        for (uint32_t i = threadIdx.x; i < used + 4; i += kThreads) s_words[i] = 0;     // what this chunk can touch
        __syncthreads();
        if ((threadIdx.x & 7) == 0 && k0 < n) a.sub[slot * 32 + (threadIdx.x >> 3)] = (uint16_t)start;
        if (nbits) {
            const uint32_t w = start >> 5, sh = start & 31;
            // the thread's bits shifted to their place: up to 96 + 31 bits -> four words
            const uint32_t p0 = (uint32_t)buf0, p1 = (uint32_t)(buf0 >> 32), p2 = (uint32_t)buf1, p3 = (uint32_t)(buf1 >> 32);
            atomicOr(&s_words[w], p0 << sh);
            atomicOr(&s_words[w + 1], sh ? ((p0 >> (32 - sh)) | (p1 << sh)) : p1);
            atomicOr(&s_words[w + 2], sh ? ((p1 >> (32 - sh)) | (p2 << sh)) : p2);
            atomicOr(&s_words[w + 3], sh ? ((p2 >> (32 - sh)) | (p3 << sh)) : p3);
            if (sh && (p3 >> (32 - sh))) atomicOr(&s_words[w + 4], p3 >> (32 - sh));
        }
        __syncthreads();
        uint32_t *out = a.bits + slot * kVcSlotWords;
        for (uint32_t i = threadIdx.x; i < used; i += kThreads) out[i] = s_words[i];
        if (threadIdx.x == 0) a.chunk_words[slot] = used;
    }
}

// per (bucket, group of kVcDecodeChunks chunks): rebuild the code from its lengths, fill a 4096-entry table
// indexed by the next 12 stream bits, bring the group's bit streams into LDS, then all 256 threads decode at
// once -- 32 threads per chunk, 64 values each, every thread starting at its own recorded bit offset -- and the
// values (decoded high byte | stored low byte) are written coalesced
constexpr uint32_t kVcDecodeChunks = 8;
static_assert(kVcDecodeChunks * 32 == kThreads, "one thread per sub-block of the group");

__global__ __launch_bounds__(kThreads) void vc_decode_kernel(const ValueCodecArgs a) {
    __shared__ uint16_t s_lut[1u << kVcMaxLen];      // symbol << 4 | length
    __shared__ uint32_t s_cnt[kVcMaxLen + 1][kWaves];
    __shared__ uint8_t s_sorted[256];                // symbols in (length, symbol) order
    __shared__ uint32_t s_first[kVcMaxLen + 2], s_off[kVcMaxLen + 2];   // per length: first code, start in s_sorted
    __shared__ uint32_t s_words[kVcDecodeChunks][kVcSlotWords + 1];
    // decoded high bytes: value q*4 + c of thread t is byte c of word q * kSymPitch + t (the odd pitch keeps both
    // the decoders' stores and the write-out's loads off each other's LDS banks)
    constexpr uint32_t kSymPitch = kThreads + 1;
    __shared__ uint32_t s_sym[(kVcSub / 4) * kSymPitch];
    const uint32_t groups = (a.nchunk + kVcDecodeChunks - 1) / kVcDecodeChunks;
    const uint32_t b = blockIdx.x / groups, g = blockIdx.x - b * groups;
    const uint64_t cnt = ((uint64_t)a.counts[b] < a.cap) ? a.counts[b] : a.cap;
    const uint64_t g0 = (uint64_t)g * kVcDecodeChunks * kVcChunk;        // first value of the group
    if (g0 >= cnt) return;
    const uint32_t s = threadIdx.x;
    const int lane = s & 63, wave = s >> 6;
    uint32_t l = a.lens[(uint64_t)b * 256 + s];
    if (l > kVcMaxLen) l = 0;                        // not a length this format can hold: treated as absent
    // canonical code of symbol s = first code of its length + number of smaller symbols of that length
    uint32_t rank = 0;
    for (uint32_t j = 1; j <= kVcMaxLen; ++j) {
        const unsigned long long m = __ballot(l == j);
        if (l == j) rank = __builtin_popcountll(m & ((1ull << lane) - 1ull));
        if (lane == 0) s_cnt[j][wave] = (uint32_t)__builtin_popcountll(m);
    }
    // the group's streams: chunk kk of the group is chunk g*8 + kk of the bucket; chunks past the end read as empty
    const uint32_t gn = (uint32_t)((cnt - g0 < (uint64_t)kVcDecodeChunks * kVcChunk) ? (cnt - g0) : kVcDecodeChunks * kVcChunk);
    const uint32_t nch = (gn + kVcChunk - 1) / kVcChunk;                  // chunks of this group that hold values
    const uint64_t slot0 = (uint64_t)b * a.nchunk + (uint64_t)g * kVcDecodeChunks;
    {   // every load of the group's streams is issued before the first is stored (3 words per thread and chunk)
        static_assert(kVcSlotWords == 3 * kThreads, "three stream words per thread");
        uint32_t used[kVcDecodeChunks], tmp[kVcDecodeChunks][3];
#pragma unroll
        for (uint32_t kk = 0; kk < kVcDecodeChunks; ++kk) {
            used[kk] = (kk < nch) ? a.chunk_words[slot0 + kk] : 0u;
            used[kk] = used[kk] > kVcSlotWords ? kVcSlotWords : used[kk];
        }
#pragma unroll
        for (uint32_t kk = 0; kk < kVcDecodeChunks; ++kk) {
            const uint32_t *in = a.bits + (slot0 + kk) * kVcSlotWords;
#pragma unroll
            for (uint32_t r = 0; r < 3; ++r) tmp[kk][r] = (s + r * kThreads < used[kk]) ? in[s + r * kThreads] : 0u;
        }
#pragma unroll
        for (uint32_t kk = 0; kk < kVcDecodeChunks; ++kk) {
#pragma unroll
            for (uint32_t r = 0; r < 3; ++r) s_words[kk][s + r * kThreads] = tmp[kk][r];
        }
        if (s < kVcDecodeChunks) s_words[s][kVcSlotWords] = 0u;
    }
    __syncthreads();
    // Per length j: how many symbols have it, the first code of that length and where its symbols start in the
    // list of symbols sorted by (length, symbol) -- every thread keeps the three small tables in registers.
    // end_j[j]: one past the last code of length j, left-aligned to kVcMaxLen bits.  The runs of canonical codes of
    // the lengths 1, 2, ... follow one another in that space, so end_j never decreases.
    uint32_t off_j[kVcMaxLen + 1], end_j[kVcMaxLen + 1];
    {
        uint32_t code = 0, off = 0;
#pragma unroll
        for (uint32_t j = 1; j <= kVcMaxLen; ++j) {
            uint32_t cj = 0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) { cj += s_cnt[j][w]; if (j == l && w < wave) rank += s_cnt[j][w]; }
            off_j[j] = off; end_j[j] = (code + cj) << (kVcMaxLen - j);
            if (s == j) { s_first[j] = code; s_off[j] = off; }
            code = (code + cj) << 1; off += cj;
        }
        if (s == 0) { s_first[kVcMaxLen + 1] = 0; s_off[kVcMaxLen + 1] = 0; }
    }
#pragma unroll
    for (uint32_t j = 1; j <= kVcMaxLen; ++j)
        if (l == j) s_sorted[off_j[j] + rank] = (uint8_t)s;            // off + rank < 256: each symbol has one length
    __syncthreads();
    // Table entry i: the 12 stream bits i, first bit in bit 0, are a code word's bits most significant first;
    // the entry's length is the first length whose run ends above them (none: not a code of this table, entry 0).
    for (uint32_t i = s; i < (1u << kVcMaxLen); i += kThreads) {
        const uint32_t c12 = __brev(i) >> (32 - kVcMaxLen);
        uint32_t len = 1;
#pragma unroll
        for (uint32_t j = 1; j <= kVcMaxLen; ++j) len += (c12 >= end_j[j]) ? 1u : 0u;
        uint32_t e = 0;
        if (len <= kVcMaxLen) {
            const uint32_t d = (c12 >> (kVcMaxLen - len)) - s_first[len];      // below the count of that length
            e = ((uint32_t)s_sorted[(s_off[len] + d) & 255u] << 4) | len;
        }
        s_lut[i] = (uint16_t)e;
    }
    __syncthreads();
    bool bad = false;
    {
        const uint32_t kk = s >> 5, sb = s & 31u;                         // chunk of the group, sub-block of the chunk
        const uint32_t v0 = kk * kVcChunk + sb * kVcSub;                  // first value of this thread, inside the group
        if (v0 < gn) {
            const uint32_t v1 = (v0 + kVcSub < gn) ? (v0 + kVcSub) : gn;  // a chunk holds a multiple of kVcSub unless it is the last
            uint32_t pos = a.sub[(slot0 + kk) * 32 + sb];
            // one value: the next kVcMaxLen stream bits index the table.  A pattern that is no code of the table has
            // length 0: the position then stands still and the remaining values of the sub-block come out as that
            // entry's symbol -- the flag tells the caller that the output means nothing.  (The loop is bound by
            // instruction issue, so it carries no early exit and, for full sub-blocks, no per-value bookkeeping.)
            auto next = [&]() -> uint32_t {
                const uint32_t w = pos >> 5, sh = pos & 31;
                uint32_t x = 0;
                if (w < kVcSlotWords) x = (uint32_t)((((unsigned long long)s_words[kk][w + 1] << 32) | s_words[kk][w]) >> sh);
                const uint32_t e = s_lut[x & ((1u << kVcMaxLen) - 1u)];
                bad = bad || (e & 15u) == 0;
                pos += e & 15u;
                return e >> 4;
            };
            if (v1 - v0 == kVcSub) {
#pragma unroll 4
                for (uint32_t q = 0; q < kVcSub / 4; ++q) {
                    uint32_t pack = next();
                    pack |= next() << 8;
                    pack |= next() << 16;
                    pack |= next() << 24;
                    s_sym[q * kSymPitch + s] = pack;
                }
            } else {
                uint32_t pack = 0;
                for (uint32_t i = v0; i < v1; ++i) {
                    const uint32_t it = i - v0;
                    pack |= next() << (8u * (it & 3u));
                    if ((it & 3u) == 3u || i + 1 == v1) { s_sym[(it >> 2) * kSymPitch + s] = pack; pack = 0; }
                }
            }
        }
    }
    __syncthreads();
    const uint8_t *lo = a.low + (uint64_t)b * a.cap + g0;
    uint16_t *out = a.V_out + (uint64_t)b * a.cap + g0;
    if (((((uintptr_t)lo) & 7u) | (((uintptr_t)out) & 15u)) == 0) {
        // 8 consecutive values per thread and step: one 8-byte load of low bytes, two words of symbols, one
        // 16-byte store; all of a thread's loads are issued first
        constexpr uint32_t kSteps = kVcDecodeChunks * kVcChunk / (8 * kThreads);
        uint2 lw[kSteps];
#pragma unroll
        for (uint32_t q = 0; q < kSteps; ++q) {
            const uint32_t i0 = (q * kThreads + s) * 8u;
            lw[q] = (i0 + 8u <= gn) ? *reinterpret_cast<const uint2 *>(lo + i0) : make_uint2(0u, 0u);
        }
#pragma unroll
        for (uint32_t q = 0; q < kSteps; ++q) {
            const uint32_t i0 = (q * kThreads + s) * 8u;
            if (i0 + 8u <= gn) {
                const uint32_t t = i0 / kVcSub, w0 = (i0 % kVcSub) >> 2;
                const uint32_t lwq[2] = {lw[q].x, lw[q].y};
                uint32_t o[4];
#pragma unroll
                for (uint32_t c = 0; c < 2; ++c) {                        // 4 values per word of symbols / of low bytes
                    const uint32_t sy = s_sym[(w0 + c) * kSymPitch + t], lb = lwq[c];
                    o[2 * c] = ((sy & 0xFFu) << 8) | (lb & 0xFFu) | ((sy & 0xFF00u) << 16) | ((lb & 0xFF00u) << 8);
                    o[2 * c + 1] = ((sy >> 8) & 0xFF00u) | ((lb >> 16) & 0xFFu) | (sy & 0xFF000000u) | ((lb >> 8) & 0xFF0000u);
                }
                u32x4 a0;
                a0.x = o[0]; a0.y = o[1]; a0.z = o[2]; a0.w = o[3];
                *reinterpret_cast<u32x4 *>(out + i0) = a0;
            } else {
                for (uint32_t i = i0; i < gn; ++i) {                      // the ragged end of the bucket's payload
                    const uint32_t t = i / kVcSub, it = i % kVcSub;
                    out[i] = (uint16_t)((((s_sym[(it >> 2) * kSymPitch + t] >> (8u * (it & 3u))) & 0xFFu) << 8) | lo[i]);
                }
            }
        }
    } else {
        // any alignment: 8 loads in flight per thread
        for (uint32_t base = 0; base < gn; base += 8 * kThreads) {
            uint32_t lb[8];
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u) {
                const uint32_t i = base + u * kThreads + s;
                lb[u] = (i < gn) ? (uint32_t)lo[i] : 0u;
            }
#pragma unroll
            for (uint32_t u = 0; u < 8; ++u) {
                const uint32_t i = base + u * kThreads + s;
                if (i < gn) {
                    const uint32_t t = i / kVcSub, it = i % kVcSub;       // decoding thread, its it-th value
                    const uint32_t sym = (s_sym[(it >> 2) * kSymPitch + t] >> (8u * (it & 3u))) & 0xFFu;
                    out[i] = (uint16_t)((sym << 8) | lb[u]);
                }
            }
        }
    }
    if (bad) atomicOr(a.flags, kFlagBadIndex);
}

// ---------------------------------------------------------------------------------------------
// small utilities
// ---------------------------------------------------------------------------------------------
__global__ void fill_u64_kernel(unsigned long long *p, uint64_t n, unsigned long long v) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// p[i*stride] = 0 for i < n
__global__ void zero_strided_kernel(uint32_t *p, uint64_t n, uint32_t stride) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i * stride] = 0u;
}

// Before every extract launch: rewinds the per-bucket ticket counters and clears the tile status words.
// Part of the stream's work (not of host state), so a captured graph replays correctly.
__global__ void prepare_extract_kernel(uint32_t *tickets, uint64_t nb, uint32_t stride, unsigned long long *status,
                                       uint64_t ntiles) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nb) tickets[i * stride] = 0u;
    if (i < ntiles) status[i] = 0ull;
}

// two-stream read probe with extract's load shape; the XOR-reduction keeps the loads alive
template <int V, bool NT>
__global__ __launch_bounds__(kThreads) void stream_probe_kernel(const uint16_t *pa, const uint16_t *pb, uint64_t nvec,
                                                                 uint32_t *sink) {
    constexpr uint32_t TILE = (uint32_t)V * kUnit;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t base = (uint64_t)blockIdx.x * TILE + (uint32_t)wave * (V * 512u) + (uint32_t)lane * 8u;
    u32x4 acc = {0, 0, 0, 0};
    u32x4 xa[V], xb[V];
#pragma unroll
    for (int j = 0; j < V; ++j) {
        const uint64_t e = base + j * 512;
        const bool ok = e / 8 < nvec;
        xa[j] = ok ? load16<NT>(as_global(pa) + e) : acc;
        xb[j] = ok ? load16<NT>(as_global(pb) + e) : acc;
    }
#pragma unroll
    for (int j = 0; j < V; ++j) acc ^= xa[j] ^ xb[j];
    uint32_t r = acc.x ^ acc.y ^ acc.z ^ acc.w;
    r = lane63(wave_inclusive_scan(r & 0xFFu));
    if (lane == 0 && wave == 0) sink[blockIdx.x] = r;
}

}  // namespace srs
