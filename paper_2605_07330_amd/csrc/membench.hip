// membench -- measurement aid, not part of the method.  Prints the memory-system figures of the box
// that the extract / apply kernels are designed around:
//   1. workgroup dispatch rate and the cost of an atomic ticket on 1..64 distinct addresses
//      (why each bucket has its own ticket counter and buckets are interleaved over workgroups);
//   2. streaming read and write bandwidth;
//   3. the cost of writing a sparse subset of 64-byte blocks, as 2-byte stores or as full 64-byte
//      stores, alone and mixed with a streaming read (what the snapshot refresh and the scatter
//      apply cost, and why they cost the same whatever the store width: the memory side pays per
//      128-byte line touched);
//   4. the same sparse blocks updated by an explicit read-modify-write of the whole 64-byte block or 128-byte
//      line in the kernel, with ordinary or hinted accesses (no cheaper than the masked 2-byte store, so the scatter
//      keeps its 2-byte stores);
//   5. what extract's snapshot refresh does now -- both buffers streamed with the non-temporal hint, chosen 128-byte
//      lines of one of them rewritten whole with the hint -- with the same number of lines chosen one by one or in
//      runs of 4 .. 256 consecutive lines (how much of the cost goes with the line and how much with the stretch of
//      memory it lies in).
// Everything is in bounds by construction; no input, no arguments.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

#define CK(x)                                                                      \
    do {                                                                           \
        hipError_t e_ = (x);                                                       \
        if (e_ != hipSuccess) {                                                    \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 1;                                                              \
        }                                                                          \
    } while (0)

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void k_empty(uint32_t *out) {
    if (threadIdx.x == 1000) out[0] = 1;
}

__global__ __launch_bounds__(256) void k_ticket(uint32_t *ctr, uint32_t addresses, uint32_t *out) {
    __shared__ uint32_t s;
    if (threadIdx.x == 0)
        s = __hip_atomic_fetch_add(ctr + (blockIdx.x % addresses) * 64, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s == 0xffffffffu) out[0] = 1;
}

// One workgroup per tile of 16384 16-bit elements.  STORE: 0 none, 1 one 2-byte store per chosen
// 64-byte block, 2 the whole chosen block (4 lanes x 16 bytes), 3 every block (dense).
// A block is chosen when hash(block) % keep == 0.
template <int STORE, bool READ>
__global__ __launch_bounds__(256) void k_mix(uint16_t *dst, const uint16_t *src, uint32_t keep, uint32_t *sink) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t tile = (uint64_t)blockIdx.x * 16384;
    const uint32_t e0 = wave * 4096 + lane * 8;
    u32x4 acc = {0, 0, 0, 0};
    if (READ) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc ^= *reinterpret_cast<const u32x4 *>(src + tile + e0 + j * 512);
    }
    if (STORE) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t e = e0 + j * 512;
            const uint32_t blk = (uint32_t)((tile + e) >> 5);
            const bool hit = (STORE == 3) || (((blk * 2654435761u) >> 8) % keep == 0);
            if (STORE == 1) {
                if (hit && (lane & 3) == ((blk >> 3) & 3)) dst[tile + e + (blk & 7)] = (uint16_t)(blk + acc.x);
            } else if (hit) {
                const u32x4 v = {blk, acc.x, acc.y, acc.z};
                *reinterpret_cast<u32x4 *>(dst + tile + e) = v;
            }
        }
    }
    if (READ && (acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345u) sink[0] = 1;
}

// dst <- src, 16 bytes per lane and step, loads and stores with or without the non-temporal hint
template <bool HINT>
__global__ __launch_bounds__(256) void k_copy(uint16_t *dst, const uint16_t *src) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t tile = (uint64_t)blockIdx.x * 16384;
    const uint32_t e0 = wave * 4096 + lane * 8;
    u32x4 x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const u32x4 *p = reinterpret_cast<const u32x4 *>(src + tile + e0 + j * 512);
        x[j] = HINT ? __builtin_nontemporal_load(p) : *p;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        u32x4 *q = reinterpret_cast<u32x4 *>(dst + tile + e0 + j * 512);
        if (HINT) __builtin_nontemporal_store(x[j], q); else *q = x[j];
    }
}

// UNIT = 4: read, change and rewrite each chosen 64-byte block (4 lanes x 16 bytes); UNIT = 8: each 128-byte
// line that holds a chosen block; UNIT = 0: only read the chosen blocks.
template <int UNIT, bool HINT = false>
__global__ __launch_bounds__(256) void k_rmw(uint16_t *dst, uint32_t keep, uint32_t *sink) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t tile = (uint64_t)blockIdx.x * 16384;
    const uint32_t e0 = wave * 4096 + lane * 8;
    uint32_t acc = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t e = e0 + j * 512;
        const uint32_t blk = (uint32_t)((tile + e) >> 5);
        bool hit = ((blk * 2654435761u) >> 8) % keep == 0;
        if (UNIT == 8) hit = hit || ((((blk ^ 1u) * 2654435761u) >> 8) % keep == 0);
        if (hit) {
            u32x4 *p = reinterpret_cast<u32x4 *>(dst + tile + e);
            u32x4 v = HINT ? __builtin_nontemporal_load(p) : *p;
            if (UNIT == 0) acc ^= v.x ^ v.w;
            else { v.x ^= blk; if (HINT) __builtin_nontemporal_store(v, p); else *p = v; }
        }
    }
    if (UNIT == 0 && acc == 0x12345u) sink[0] = 1;
}

// Two hinted read streams over dst and src; the chosen 128-byte lines of dst are rewritten whole (8 lanes x 16 bytes,
// hinted).  Lines are chosen in runs of G: run r (lines r*G .. r*G+G-1) is chosen when hash(r) % keep == 0.
// WRITE = false: the two reads only.
template <int G, bool WRITE>
__global__ __launch_bounds__(256) void k_lines(uint16_t *dst, const uint16_t *src, uint32_t keep, uint32_t *sink) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t tile = (uint64_t)blockIdx.x * 16384;
    const uint32_t e0 = wave * 4096 + lane * 8;
    u32x4 xo[8], xn[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) xn[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + tile + e0 + j * 512));
#pragma unroll
    for (int j = 0; j < 8; ++j) xo[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(dst + tile + e0 + j * 512));
    u32x4 acc = {0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 8; ++j) acc ^= xo[j] ^ xn[j];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        if (WRITE) {
            const uint32_t line = (uint32_t)((tile + e0 + j * 512) >> 6);
            const uint32_t run = line / G;
            if (((run * 2654435761u) >> 8) % keep == 0)
                __builtin_nontemporal_store(xn[j], reinterpret_cast<u32x4 *>(dst + tile + e0 + j * 512));
        }
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345u) sink[0] = 1;
}

int main() {
    const uint64_t N = 8ull << 30;   // elements per buffer (16 GB)
    const uint32_t nwg = (uint32_t)(N / 16384);
    uint16_t *dst, *src;
    uint32_t *sink, *ctr;
    CK(hipMalloc(&dst, N * 2)); CK(hipMalloc(&src, N * 2)); CK(hipMalloc(&sink, 64)); CK(hipMalloc(&ctr, 64 * 64 * 4));
    CK(hipMemset(dst, 0, N * 2)); CK(hipMemset(src, 1, N * 2)); CK(hipMemset(ctr, 0, 64 * 64 * 4));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    float ms = 0;
#define TIME(...)                                                          \
    for (int rep_ = 0; rep_ < 2; ++rep_) {                                 \
        CK(hipEventRecord(e0)); __VA_ARGS__; CK(hipEventRecord(e1));       \
        CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1)); \
    }

    std::printf("## dispatch and tickets (2,000,000 workgroups of 256 threads)\n");
    const uint32_t M = 2000000;
    TIME(hipLaunchKernelGGL(k_empty, dim3(M), dim3(256), 0, 0, sink));
    std::printf("empty workgroups: %.3f ms = %.2f ns per workgroup\n", ms, ms * 1e6 / M);
    for (uint32_t a : {1u, 2u, 4u, 8u, 16u, 32u, 64u}) {
        TIME(hipLaunchKernelGGL(k_ticket, dim3(M), dim3(256), 0, 0, ctr, a, sink));
        std::printf("one agent-scope fetch_add per workgroup on %2u address(es): %.3f ms = %.2f ns per ticket\n", a, ms,
                    ms * 1e6 / M);
    }

    std::printf("## streaming (16 GB buffers)\n");
    TIME(hipLaunchKernelGGL((k_mix<0, true>), dim3(nwg), dim3(256), 0, 0, dst, src, 1u, sink));
    const float t_read = ms;
    std::printf("read only: %.3f ms = %.0f GB/s\n", ms, N * 2 / (ms * 1e-3) / 1e9);
    TIME(hipLaunchKernelGGL((k_mix<3, false>), dim3(nwg), dim3(256), 0, 0, dst, src, 1u, sink));
    std::printf("write only (dense 16-byte stores): %.3f ms = %.0f GB/s\n", ms, N * 2 / (ms * 1e-3) / 1e9);
    TIME(hipLaunchKernelGGL((k_mix<3, true>), dim3(nwg), dim3(256), 0, 0, dst, src, 1u, sink));
    std::printf("read + dense write: %.3f ms = %.0f GB/s (both directions)\n", ms, N * 4 / (ms * 1e-3) / 1e9);
    TIME(hipLaunchKernelGGL((k_copy<false>), dim3(nwg), dim3(256), 0, 0, dst, src));
    std::printf("copy, ordinary loads and stores: %.3f ms = %.0f GB/s (both directions)\n", ms, N * 4 / (ms * 1e-3) / 1e9);
    TIME(hipLaunchKernelGGL((k_copy<true>), dim3(nwg), dim3(256), 0, 0, dst, src));
    std::printf("copy, hinted loads and stores: %.3f ms = %.0f GB/s (both directions)\n", ms, N * 4 / (ms * 1e-3) / 1e9);

    std::printf("## sparse block writes: 1/keep of the 64-byte blocks of a 16 GB buffer\n");
    std::printf("%-5s %-9s %-10s | %-22s | %-22s | %-26s | %-26s\n", "keep", "blocks", "128B lines", "2B stores alone",
                "64B stores alone", "2B stores + 16 GB read", "64B stores + 16 GB read");
    for (uint32_t keep : {2u, 4u, 8u, 16u}) {
        const double blocks = (double)N / 32 / keep;
        const double lines = (double)N / 64 * (1.0 - (1.0 - 1.0 / keep) * (1.0 - 1.0 / keep));
        float t1, t2, t3, t4;
        TIME(hipLaunchKernelGGL((k_mix<1, false>), dim3(nwg), dim3(256), 0, 0, dst, src, keep, sink)); t1 = ms;
        TIME(hipLaunchKernelGGL((k_mix<2, false>), dim3(nwg), dim3(256), 0, 0, dst, src, keep, sink)); t2 = ms;
        TIME(hipLaunchKernelGGL((k_mix<1, true>), dim3(nwg), dim3(256), 0, 0, dst, src, keep, sink)); t3 = ms;
        TIME(hipLaunchKernelGGL((k_mix<2, true>), dim3(nwg), dim3(256), 0, 0, dst, src, keep, sink)); t4 = ms;
        std::printf("1/%-3u %6.1f M  %6.1f M   | %6.3f ms %5.1f ps/line | %6.3f ms %5.1f ps/line | +%6.3f ms %5.1f ps/line    | +%6.3f ms %5.1f ps/line\n",
                    keep, blocks / 1e6, lines / 1e6, t1, t1 * 1e9 / lines, t2, t2 * 1e9 / lines, t3 - t_read,
                    (t3 - t_read) * 1e9 / lines, t4 - t_read, (t4 - t_read) * 1e9 / lines);
    }
    std::printf("## the same sparse blocks by explicit read-modify-write in the kernel (no other traffic)\n");
    std::printf("%-5s %-10s | %-22s | %-22s | %-22s | %-22s | %-22s\n", "keep", "128B lines", "2B stores", "RMW of 64B blocks",
                "RMW of 128B lines", "reads of 64B blocks only", "RMW of 128B lines, hinted");
    for (uint32_t keep : {2u, 4u, 8u, 16u}) {
        const double lines = (double)N / 64 * (1.0 - (1.0 - 1.0 / keep) * (1.0 - 1.0 / keep));
        float t1, t2, t3, t4, t5;
        TIME(hipLaunchKernelGGL((k_mix<1, false>), dim3(nwg), dim3(256), 0, 0, dst, src, keep, sink)); t1 = ms;
        TIME(hipLaunchKernelGGL((k_rmw<4>), dim3(nwg), dim3(256), 0, 0, dst, keep, sink)); t2 = ms;
        TIME(hipLaunchKernelGGL((k_rmw<8>), dim3(nwg), dim3(256), 0, 0, dst, keep, sink)); t3 = ms;
        TIME(hipLaunchKernelGGL((k_rmw<0>), dim3(nwg), dim3(256), 0, 0, dst, keep, sink)); t4 = ms;
        TIME(hipLaunchKernelGGL((k_rmw<8, true>), dim3(nwg), dim3(256), 0, 0, dst, keep, sink)); t5 = ms;
        std::printf("1/%-3u %6.1f M   | %6.3f ms %5.1f ps/line | %6.3f ms %5.1f ps/line | %6.3f ms %5.1f ps/line | %6.3f ms %5.1f ps/line | %6.3f ms %5.1f ps/line\n",
                    keep, lines / 1e6, t1, t1 * 1e9 / lines, t2, t2 * 1e9 / lines, t3, t3 * 1e9 / lines, t4,
                    t4 * 1e9 / lines, t5, t5 * 1e9 / lines);
    }
    std::printf("## two hinted read streams (2 x 16 GB) + 1/keep of the 128-byte lines of one of them rewritten whole, hinted,\n");
    std::printf("## the lines chosen in runs of G consecutive lines; time added to the two reads, per line and per run\n");
    TIME(hipLaunchKernelGGL((k_lines<1, false>), dim3(nwg), dim3(256), 0, 0, dst, src, 1u, sink));
    const float t_two = ms;
    std::printf("the two reads alone: %.3f ms = %.0f GB/s\n", t_two, N * 4 / (t_two * 1e-3) / 1e9);
    for (uint32_t keep : {2u, 4u, 16u, 64u}) {
        const double lines = (double)N / 64 / keep;
        float t[5];
        TIME(hipLaunchKernelGGL((k_lines<1, true>), dim3(nwg), dim3(256), 0, 0, dst, src, keep, sink)); t[0] = ms - t_two;
        TIME(hipLaunchKernelGGL((k_lines<4, true>), dim3(nwg), dim3(256), 0, 0, dst, src, keep, sink)); t[1] = ms - t_two;
        TIME(hipLaunchKernelGGL((k_lines<16, true>), dim3(nwg), dim3(256), 0, 0, dst, src, keep, sink)); t[2] = ms - t_two;
        TIME(hipLaunchKernelGGL((k_lines<64, true>), dim3(nwg), dim3(256), 0, 0, dst, src, keep, sink)); t[3] = ms - t_two;
        TIME(hipLaunchKernelGGL((k_lines<256, true>), dim3(nwg), dim3(256), 0, 0, dst, src, keep, sink)); t[4] = ms - t_two;
        std::printf("1/%-3u %6.1f M lines |", keep, lines / 1e6);
        const int g[5] = {1, 4, 16, 64, 256};
        for (int i = 0; i < 5; ++i)
            std::printf(" G=%-3d +%6.3f ms %5.1f ps/line %6.0f ps/run |", g[i], t[i], t[i] * 1e9 / lines, t[i] * 1e9 / (lines / g[i]));
        std::printf("\n");
    }
    CK(hipDeviceSynchronize());
    std::printf("done\n");
    return 0;
}
