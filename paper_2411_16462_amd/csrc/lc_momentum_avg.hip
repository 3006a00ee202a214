// Momentum synchronisation (Section 5): every worker's momentum row becomes the mean of
// the W rows -- what an averaging allreduce leaves on every worker.
//
// Streaming kernel: reads W rows and writes W rows, 8 W bytes per element.  A lane owns
// 4 consecutive elements (16-byte accesses); rows are summed in row order in fp32 with
// 8 loads in flight, and the sum is multiplied once by 1/W.
#include "lc_launch.hpp"

namespace lc {

#ifndef LC_AVG_THREADS
#define LC_AVG_THREADS 256
#endif
constexpr int kAvgThreads = LC_AVG_THREADS;  // workgroup size
constexpr int kAvgBlock = kAvgThreads * 4;   // elements per workgroup

__global__ __launch_bounds__(kAvgThreads) void momentum_avg_kernel(float *__restrict__ m, size_t stride, int W, size_t n, float inv_w)
{
    const size_t e = static_cast<size_t>(blockIdx.x) * kAvgBlock + threadIdx.x * 4;
    if (e >= n) return;
    if (e + 4 <= n) {
        f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
        int w = 0;
        for (; w + 8 <= W; w += 8) {
            f32x4 x[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) x[k] = load4(m + static_cast<size_t>(w + k) * stride + e);
#pragma unroll
            for (int k = 0; k < 8; ++k) acc += x[k];
        }
        for (; w < W; ++w) acc += load4(m + static_cast<size_t>(w) * stride + e);
        acc *= inv_w;
        for (w = 0; w < W; ++w) store4(m + static_cast<size_t>(w) * stride + e, acc);
    } else {
        for (size_t i = e; i < n; ++i) {
            float acc = 0.0f;
            for (int w = 0; w < W; ++w) acc += m[static_cast<size_t>(w) * stride + i];
            acc *= inv_w;
            for (int w = 0; w < W; ++w) m[static_cast<size_t>(w) * stride + i] = acc;
        }
    }
}

hipError_t launch_momentum_avg(float *m, size_t stride, int W, size_t n, hipStream_t s)
{
    const unsigned grid = static_cast<unsigned>((n + kAvgBlock - 1) / kAvgBlock);
    momentum_avg_kernel<<<grid, kAvgThreads, 0, s>>>(m, stride, W, n, 1.0f / static_cast<float>(W));
    return hipGetLastError();
}

}  // namespace lc
