/*
 * A plain C consumer of libsrs.so: no Python, no C++, only include/srs.h and the HIP runtime's C API.
 * It shows that the boundary is what the header says (device pointers and sizes) and gives the GPU tests
 * one caller that is not the ctypes binding.
 *
 *   roundtrip <old.u16> <new.u16> <n> <bucket_elems> <cap> <out.bin> [noalloc|secondpass]
 *
 * old / new: n 16-bit patterns each (host byte order).  The program extracts the difference on the GPU
 * (Alg. 1-2: indices and values of the changed elements, per bucket; the snapshot is refreshed), applies the
 * payload to a second copy of the old weights (Alg. 3) and writes, one after the other,
 *   counts[nb] (u32), I[nb*cap] (i32), V[nb*cap] (u16), snapshot[n] (u16), patched[n] (u16), flags (u32)
 * to out.bin.  Payload slots are pre-filled with -1 / 0xFFFF so that untouched slots can be checked.
 * With the trailing word `noalloc` the extraction goes through srs_extract_noalloc (static scratch) instead of
 * srs_extract; with `secondpass` the context is first given SRS_OPT_SNAPSHOT = 2 (snapshot refreshed by a scatter
 * of the payload after the scan).  The output is the same in all three.  Exit status 0 when every call returned SRS_OK.
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>

#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "srs.h"

#define CHECK_HIP(x)                                                                   \
    do {                                                                               \
        hipError_t e_ = (x);                                                           \
        if (e_ != hipSuccess) {                                                        \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                    \
            return 2;                                                                  \
        }                                                                              \
    } while (0)

#define CHECK_SRS(x)                                                                   \
    do {                                                                               \
        int r_ = (x);                                                                  \
        if (r_ != SRS_OK) {                                                            \
            fprintf(stderr, "%s: %s\n", #x, srs_strerror(r_));                         \
            return 3;                                                                  \
        }                                                                              \
    } while (0)

static int read_file(const char *path, void *dst, size_t bytes) {
    FILE *f = fopen(path, "rb");
    if (!f) return -1;
    const size_t got = fread(dst, 1, bytes, f);
    fclose(f);
    return got == bytes ? 0 : -1;
}

int main(int argc, char **argv) {
    if (argc != 7 && !(argc == 8 && (strcmp(argv[7], "noalloc") == 0 || strcmp(argv[7], "secondpass") == 0))) {
        fprintf(stderr, "usage: %s old.u16 new.u16 n bucket_elems cap out.bin [noalloc|secondpass]\n", argv[0]);
        return 1;
    }
    const int noalloc = argc == 8 && strcmp(argv[7], "noalloc") == 0;
    const int secondpass = argc == 8 && strcmp(argv[7], "secondpass") == 0;
    const uint64_t n = strtoull(argv[3], NULL, 10), be = strtoull(argv[4], NULL, 10), cap = strtoull(argv[5], NULL, 10);
    if (n == 0 || be == 0 || cap == 0) return 1;
    const uint64_t nb = (n + be - 1) / be;
    const size_t wbytes = (size_t)n * 2, slots = (size_t)(nb * cap);

    uint16_t *h_old = malloc(wbytes), *h_new = malloc(wbytes);
    if (!h_old || !h_new || read_file(argv[1], h_old, wbytes) || read_file(argv[2], h_new, wbytes)) {
        fprintf(stderr, "cannot read the inputs\n");
        return 1;
    }

    void *d_snap, *d_new, *d_roll, *d_I, *d_V, *d_counts;
    CHECK_HIP(hipSetDevice(0));
    CHECK_HIP(hipMalloc(&d_snap, wbytes));
    CHECK_HIP(hipMalloc(&d_new, wbytes));
    CHECK_HIP(hipMalloc(&d_roll, wbytes));
    CHECK_HIP(hipMalloc(&d_I, slots * 4));
    CHECK_HIP(hipMalloc(&d_V, slots * 2));
    CHECK_HIP(hipMalloc(&d_counts, (size_t)nb * 4));
    CHECK_HIP(hipMemcpy(d_snap, h_old, wbytes, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_roll, h_old, wbytes, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_new, h_new, wbytes, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemset(d_I, 0xFF, slots * 4));
    CHECK_HIP(hipMemset(d_V, 0xFF, slots * 2));
    CHECK_HIP(hipMemset(d_counts, 0, (size_t)nb * 4));

    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));
    srs_ctx *ctx = NULL;
    CHECK_SRS(srs_create(&ctx, 0));
    if (secondpass) CHECK_SRS(srs_set_option(ctx, SRS_OPT_SNAPSHOT, 2));
    if (noalloc)
        CHECK_SRS(srs_extract_noalloc(ctx, d_snap, d_new, n, be, (int32_t *)d_I, (uint16_t *)d_V, (uint32_t *)d_counts, cap,
                                      stream));
    else
        CHECK_SRS(srs_extract(ctx, d_snap, d_new, n, be, (int32_t *)d_I, (uint16_t *)d_V, (uint32_t *)d_counts, cap, stream));
    CHECK_SRS(srs_apply(ctx, d_roll, n, be, (const int32_t *)d_I, (const uint16_t *)d_V, (const uint32_t *)d_counts, cap,
                        stream));
    uint32_t flags = 0;
    CHECK_SRS(srs_status(ctx, &flags, stream));            /* synchronises the stream */

    uint32_t *h_counts = malloc((size_t)nb * 4);
    int32_t *h_I = malloc(slots * 4);
    uint16_t *h_V = malloc(slots * 2), *h_snap = malloc(wbytes), *h_roll = malloc(wbytes);
    if (!h_counts || !h_I || !h_V || !h_snap || !h_roll) return 1;
    CHECK_HIP(hipMemcpy(h_counts, d_counts, (size_t)nb * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(h_I, d_I, slots * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(h_V, d_V, slots * 2, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(h_snap, d_snap, wbytes, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(h_roll, d_roll, wbytes, hipMemcpyDeviceToHost));

    FILE *out = fopen(argv[6], "wb");
    if (!out) return 1;
    int ok = fwrite(h_counts, 4, (size_t)nb, out) == (size_t)nb && fwrite(h_I, 4, slots, out) == slots &&
             fwrite(h_V, 2, slots, out) == slots && fwrite(h_snap, 2, (size_t)n, out) == (size_t)n &&
             fwrite(h_roll, 2, (size_t)n, out) == (size_t)n && fwrite(&flags, 4, 1, out) == 1;
    ok = (fclose(out) == 0) && ok;

    CHECK_SRS(srs_destroy(ctx));
    CHECK_HIP(hipStreamDestroy(stream));
    CHECK_HIP(hipFree(d_snap)); CHECK_HIP(hipFree(d_new)); CHECK_HIP(hipFree(d_roll));
    CHECK_HIP(hipFree(d_I)); CHECK_HIP(hipFree(d_V)); CHECK_HIP(hipFree(d_counts));
    free(h_old); free(h_new); free(h_counts); free(h_I); free(h_V); free(h_snap); free(h_roll);
    printf("roundtrip: n=%llu buckets=%llu flags=%u\n", (unsigned long long)n, (unsigned long long)nb, flags);
    return ok ? 0 : 1;
}
