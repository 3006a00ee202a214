// Bare streaming kernels in the shape of the library's streaming kernels (one wave per
// 256-element tile, 16-byte non-temporal accesses): what this device reaches when a kernel
// does nothing but move the data.  A calibration aid for measurements, beside the
// datasheet peak; no step of the method runs here.
#include "lc_launch.hpp"

namespace lc {

// kind: 0 read a, 1 write a, 2 copy b to a, 3 scale a in place, 4 a <- s a + (1 - s) b
// (two streams read, one written: update+pack without the packing).
// THREADS: one-wave workgroups where a wave moves 2 KiB or more; four-wave workgroups for the
// kinds that move 1 KiB per wave, which would otherwise be bound by the rate at which
// workgroups are dispatched (about 2.4 per ns on this part) and not by memory.
template <int KIND, int THREADS>
__global__ __launch_bounds__(THREADS) void stream_probe_kernel(float *__restrict__ a, const float *__restrict__ b, size_t n, float s,
                                                            float never)
{
    const size_t e = (static_cast<size_t>(blockIdx.x) * THREADS + threadIdx.x) * 4;
    if (e >= n) return;
    if (e + 4 <= n) {
        f32x4 v = {s, s, s, s};
        if (KIND == 0 || KIND == 3 || KIND == 4) v = load4(a + e);
        if (KIND == 2) v = load4(b + e);
        if (KIND == 0) {  // `never` is a NaN: the comparison is false, but the loads must be made to find that out
            if (v[0] + v[1] + v[2] + v[3] == never) a[e] = 0.0f;
            return;
        }
        if (KIND == 3) v *= s;
        if (KIND == 4) {
            const f32x4 w = load4(b + e);
            const float t = 1.0f - s;
#pragma unroll
            for (int k = 0; k < 4; ++k) v[k] = __builtin_fmaf(s, v[k], t * w[k]);
        }
        store4(a + e, v);
        return;
    }
    for (size_t i = e; i < n; ++i) {  // ragged end, one element at a time
        float v = s;
        if (KIND == 0 || KIND == 3 || KIND == 4) v = a[i];
        if (KIND == 2) v = b[i];
        if (KIND == 0) {
            if (v == never) a[i] = 0.0f;
            continue;
        }
        if (KIND == 3) v *= s;
        if (KIND == 4) v = __builtin_fmaf(s, v, (1.0f - s) * b[i]);
        a[i] = v;
    }
}

hipError_t launch_stream_probe(int kind, float *a, const float *b, size_t n, float s, hipStream_t st)
{
    const unsigned grid1 = static_cast<unsigned>((n + 255) / 256), grid4 = static_cast<unsigned>((n + 1023) / 1024);
    const float never = __builtin_nanf("");
    switch (kind) {
    case 0: return launch(stream_probe_kernel<0, 4 * kWave>, grid4, 4 * kWave, 0, st, a, b, n, s, never);
    case 1: return launch(stream_probe_kernel<1, 4 * kWave>, grid4, 4 * kWave, 0, st, a, b, n, s, never);
    case 2: return launch(stream_probe_kernel<2, kWave>, grid1, kWave, 0, st, a, b, n, s, never);
    case 3: return launch(stream_probe_kernel<3, kWave>, grid1, kWave, 0, st, a, b, n, s, never);
    default: return launch(stream_probe_kernel<4, kWave>, grid1, kWave, 0, st, a, b, n, s, never);
    }
}

}  // namespace lc
