/*
 * A plain-C client of the C ABI in include/lioncub.h: no C++, no Python, no torch in the
 * process.  It reads one optimizer state from a file, runs one 1-bit step on the GPU
 * (lc_local_update_pack, then lc_vote_apply_1bit) and writes the results to another file,
 * for the test that drives it to compare with the CPU oracle.
 *
 * Input file:  uint64 n, uint64 W, uint64 step, then theta[n], m[W][n], g[W][n] as float32.
 * Output file: theta[n], m[W][n] as float32, then q[W][nw] as uint64 (nw = ceil(n / 64)).
 * Exit status 0 on success; any failure prints what failed and exits with 1.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "lioncub.h"

#define CHECK_HIP(call)                                                                   \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess) {                                                           \
            fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));             \
            return 1;                                                                     \
        }                                                                                 \
    } while (0)

#define CHECK_LC(call)                                                                    \
    do {                                                                                  \
        int s_ = (call);                                                                  \
        if (s_ != LC_OK) {                                                                \
            fprintf(stderr, "%s failed: %s\n", #call, lc_status_string(s_));              \
            return 1;                                                                     \
        }                                                                                 \
    } while (0)

static int read_all(FILE *f, void *dst, size_t bytes) { return fread(dst, 1, bytes, f) == bytes ? 0 : 1; }

int main(int argc, char **argv)
{
    if (argc != 3) {
        fprintf(stderr, "usage: %s state.bin result.bin\n", argv[0]);
        return 1;
    }
    FILE *in = fopen(argv[1], "rb");
    if (!in) { perror(argv[1]); return 1; }
    uint64_t head[3];
    if (read_all(in, head, sizeof head)) { fprintf(stderr, "short header\n"); return 1; }
    const size_t n = (size_t)head[0];
    const int W = (int)head[1];
    const uint64_t step = head[2];
    if (n == 0 || n > ((size_t)1 << 28) || W < 1 || W > LC_MAX_W) { fprintf(stderr, "bad header\n"); return 1; }
    const size_t nw = (n + 63) / 64;
    const size_t stride = (n + 63) / 64 * 64;          /* elements per row: keeps every row 256-byte aligned */

    float *h_theta = malloc(n * sizeof(float));
    float *h_rows = malloc((size_t)W * n * sizeof(float));
    uint64_t *h_q = malloc((size_t)W * nw * sizeof(uint64_t));
    if (!h_theta || !h_rows || !h_q) { fprintf(stderr, "out of host memory\n"); return 1; }

    float *theta, *m, *g;
    uint64_t *q;
    CHECK_HIP(hipMalloc((void **)&theta, stride * sizeof(float)));
    CHECK_HIP(hipMalloc((void **)&m, (size_t)W * stride * sizeof(float)));
    CHECK_HIP(hipMalloc((void **)&g, (size_t)W * stride * sizeof(float)));
    CHECK_HIP(hipMalloc((void **)&q, (size_t)W * nw * sizeof(uint64_t)));

    if (read_all(in, h_theta, n * sizeof(float))) { fprintf(stderr, "short theta\n"); return 1; }
    CHECK_HIP(hipMemcpy(theta, h_theta, n * sizeof(float), hipMemcpyHostToDevice));
    for (int pass = 0; pass < 2; ++pass) {             /* m rows, then g rows */
        if (read_all(in, h_rows, (size_t)W * n * sizeof(float))) { fprintf(stderr, "short rows\n"); return 1; }
        for (int w = 0; w < W; ++w)
            CHECK_HIP(hipMemcpy((pass ? g : m) + (size_t)w * stride, h_rows + (size_t)w * n, n * sizeof(float),
                                hipMemcpyHostToDevice));
    }
    fclose(in);

    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));
    /* An error that an unrelated call of the host program leaves pending (here: a copy with
     * a direction that does not exist, refused on the host before anything reaches the GPU)
     * must not show up as the status of the library's calls, which report their own
     * launches only. */
    const hipError_t planted = hipMemcpy(theta, h_theta, sizeof(float), (hipMemcpyKind)77);
    if (planted == hipSuccess) { fprintf(stderr, "the copy with an invalid direction was accepted\n"); return 1; }
    CHECK_LC(lc_local_update_pack(g, stride, LC_F32, m, stride, W, n, 0.9f, 1, 0.99f, 1, q, nw * 8, step, LC_ZERO_ALT, stream));
    CHECK_LC(lc_vote_apply_1bit(q, nw, W, n, step, LC_TIE_ZERO, theta, 1e-4f, 0.1f, NULL, 0, NULL, 0, LC_F32, 0, 0.99f, stream));
    const hipError_t pending = hipGetLastError();      /* read (and cleared) by the host program, not by the library */
    printf("planted error %d, pending after the library calls: %d\n", (int)planted, (int)pending);
    if (pending != hipSuccess && pending != planted) { fprintf(stderr, "unexpected pending error %d\n", (int)pending); return 1; }
    CHECK_HIP(hipStreamSynchronize(stream));

    FILE *out = fopen(argv[2], "wb");
    if (!out) { perror(argv[2]); return 1; }
    CHECK_HIP(hipMemcpy(h_theta, theta, n * sizeof(float), hipMemcpyDeviceToHost));
    fwrite(h_theta, sizeof(float), n, out);
    for (int w = 0; w < W; ++w) {
        CHECK_HIP(hipMemcpy(h_rows, m + (size_t)w * stride, n * sizeof(float), hipMemcpyDeviceToHost));
        fwrite(h_rows, sizeof(float), n, out);
    }
    CHECK_HIP(hipMemcpy(h_q, q, (size_t)W * nw * sizeof(uint64_t), hipMemcpyDeviceToHost));
    fwrite(h_q, sizeof(uint64_t), (size_t)W * nw, out);
    if (fclose(out) != 0) { perror("close"); return 1; }
    printf("lioncub %d: n = %zu, W = %d, step %llu done\n", lc_version(), n, W, (unsigned long long)step);
    CHECK_HIP(hipStreamDestroy(stream));
    CHECK_HIP(hipFree(theta)); CHECK_HIP(hipFree(m)); CHECK_HIP(hipFree(g)); CHECK_HIP(hipFree(q));
    free(h_theta); free(h_rows); free(h_q);
    return 0;
}
