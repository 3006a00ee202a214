// Momentum synchronisation (Section 5): every worker's momentum row becomes the mean of
// the W rows -- what an averaging allreduce leaves on every worker.
//
// Streaming kernel: reads W rows and writes W rows, 8 W bytes per element.  A workgroup
// owns 256 consecutive elements (lane l of every wave holds elements 4l..4l+3, 16-byte
// accesses) and splits the ROWS over its waves: wave r sums rows r, r + R, r + 2R, ...,
// the R partial sums meet in LDS, and each wave writes the mean back to the rows it
// read.  Keeping every wave's share of the traffic small (a few KiB) is what lets the
// kernel stream at DRAM speed; one wave that walks all W rows is 14 % slower.
#include "lc_launch.hpp"

namespace lc {

constexpr int kAvgTile = 256;  // elements per workgroup
// Unused dynamic LDS per 8-wave workgroup: with the 8 KiB of partial sums it lets three
// workgroups (24 waves) share a compute unit's 160 KiB instead of four -- measured +3 %
// (6.2 against 6.0 TB/s at 16 rows); two workgroups lose 12 %.
#ifndef LC_AVG_LDS
#define LC_AVG_LDS 40960
#endif

__device__ __forceinline__ f32x4 load4_guarded(const float *p, size_t e, size_t n)
{
    if (e + 4 <= n) return load4(p + e);
    f32x4 v = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int k = 0; k < 4; ++k)
        if (e + k < n) v[k] = ld_stream(p + e + k);
    return v;
}

__device__ __forceinline__ void store4_guarded(float *p, size_t e, size_t n, f32x4 v)
{
    if (e + 4 <= n) {
        store4(p + e, v);
        return;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
        if (e + k < n) st_stream(p + e + k, v[k]);
}

template <int R>
__global__ __launch_bounds__(R *kWave) void momentum_avg_kernel(float *__restrict__ m, size_t stride, int W, size_t n, float inv_w)
{
    __shared__ f32x4 part[R][kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_index();
    const size_t e = static_cast<size_t>(blockIdx.x) * kAvgTile + lane * 4;
    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    if (e < n) {
        int w = wave;
        for (; w + 3 * R < W; w += 4 * R) {
            f32x4 x[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) x[k] = load4_guarded(m + static_cast<size_t>(w + k * R) * stride, e, n);
#pragma unroll
            for (int k = 0; k < 4; ++k) acc += x[k];
        }
        for (; w < W; w += R) acc += load4_guarded(m + static_cast<size_t>(w) * stride, e, n);
    }
    part[wave][lane] = acc;
    __syncthreads();
    if (e >= n) return;
    f32x4 mean = part[0][lane];
#pragma unroll
    for (int r = 1; r < R; ++r) mean += part[r][lane];
    mean *= inv_w;
    for (int w = wave; w < W; w += R) store4_guarded(m + static_cast<size_t>(w) * stride, e, n, mean);
}

hipError_t launch_momentum_avg(float *m, size_t stride, int W, size_t n, hipStream_t s)
{
    const unsigned grid = static_cast<unsigned>((n + kAvgTile - 1) / kAvgTile);
    const float inv_w = 1.0f / static_cast<float>(W);
    if (W >= 8) return launch(momentum_avg_kernel<8>, grid, 8 * kWave, LC_AVG_LDS, s, m, stride, W, n, inv_w);
    if (W >= 4) return launch(momentum_avg_kernel<4>, grid, 4 * kWave, 0, s, m, stride, W, n, inv_w);
    return launch(momentum_avg_kernel<2>, grid, 2 * kWave, 0, s, m, stride, W, n, inv_w);
}

// ---- divergence of the workers' momenta (Section 5.1, the quantity of Figure 6) --------
// max over elements of the standard deviation across the W workers (divisor W), in fp64
// with the workers taken in order, so that the result equals a sequential evaluation bit
// for bit; the maximum is order-free.  Reads W * 4 bytes per element, writes one double.
__global__ void divergence_zero_kernel(double *out, int count)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) out[i] = 0.0;
}

// non-negative doubles order like their bit patterns
__device__ __forceinline__ unsigned long long wave_max_bits(unsigned long long bits, int lane)
{
#pragma unroll
    for (int mask = 1; mask < kWave; mask <<= 1) {
        const int addr = (lane ^ mask) << 2;
        const unsigned lo = static_cast<unsigned>(__builtin_amdgcn_ds_bpermute(addr, static_cast<int>(bits & 0xFFFFFFFFull)));
        const unsigned hi = static_cast<unsigned>(__builtin_amdgcn_ds_bpermute(addr, static_cast<int>(bits >> 32)));
        const unsigned long long o = (static_cast<unsigned long long>(hi) << 32) | lo;
        bits = o > bits ? o : bits;
    }
    return bits;
}

// Raise *dst to the standard deviation that belongs to the sum of squares `ss`.  The plain
// read first spares the atomic once the running maximum has passed this value (a stale
// read can only cause a superfluous atomic, never a lost one: the value only grows).
__device__ __forceinline__ void publish_std(double *dst, double ss, int W)
{
    if (!(ss > 0.0)) return;
    const double sd = sqrt(ss / static_cast<double>(W));
    const unsigned long long bits = static_cast<unsigned long long>(__double_as_longlong(sd));
    unsigned long long *p = reinterpret_cast<unsigned long long *>(dst);
    if (bits > *reinterpret_cast<volatile unsigned long long *>(p)) atomicMax(p, bits);
}

// GROUPED: out[s] receives the maximum over segment s of a group table (segment ends in
// units of 64 elements).  A wave whose 256 elements lie in one segment reduces first; a wave
// that straddles a boundary lets every lane publish its own value.
template <bool GROUPED>
__global__ __launch_bounds__(256) void momentum_divergence_kernel(const float *__restrict__ m, size_t stride, int W, size_t n,
                                                                  double *__restrict__ out,
                                                                  const uint32_t *__restrict__ end64, int G)
{
    __shared__ double s_max[4];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_index();
    const size_t e = (static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x) * 4;
    double worst = 0.0;  // largest sum of squared deviations of this lane's elements
    if (e < n) {
        double sum[4] = {0.0, 0.0, 0.0, 0.0};
        for (int w = 0; w < W; ++w) {
            const f32x4 v = load4_guarded(m + static_cast<size_t>(w) * stride, e, n);
#pragma unroll
            for (int k = 0; k < 4; ++k) sum[k] += static_cast<double>(v[k]);
        }
        double mean[4], ss[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int k = 0; k < 4; ++k) mean[k] = sum[k] / static_cast<double>(W);
        for (int w = 0; w < W; ++w) {  // second pass: the rows are still in cache
            const f32x4 v = load4_guarded(m + static_cast<size_t>(w) * stride, e, n);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const double d = static_cast<double>(v[k]) - mean[k];
                ss[k] += d * d;
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (e + k < n && ss[k] > worst) worst = ss[k];
    }
    unsigned long long bits = static_cast<unsigned long long>(__double_as_longlong(worst));
    if (GROUPED) {
        // segment of the wave's first 64-element block by bisection (uniform), then each
        // lane walks on to the segment of its own block; lanes past n stay with the last
        const size_t first = (static_cast<size_t>(blockIdx.x) * 256 + static_cast<size_t>(wave) * kWave) * 4;
        int seg = group_find(end64, G, static_cast<uint32_t>(first / 64));
        if (e < n) {
            seg = group_walk(end64, G, seg, static_cast<uint32_t>(e / 64));
        } else {
            seg = G - 1;
        }
        const int seg0 = __builtin_amdgcn_readfirstlane(seg);
        if (__ballot(seg != seg0) == 0) {
            bits = wave_max_bits(bits, lane);
            if (lane == 0) publish_std(out + seg0, __longlong_as_double(static_cast<long long>(bits)), W);
        } else {
            publish_std(out + seg, worst, W);
        }
        return;
    }
    bits = wave_max_bits(bits, lane);
    if (lane == 0) s_max[wave] = __longlong_as_double(static_cast<long long>(bits));
    __syncthreads();
    if (threadIdx.x == 0) {
        double b = s_max[0];
        for (int r = 1; r < 4; ++r) b = s_max[r] > b ? s_max[r] : b;
        publish_std(out, b, W);
    }
}

hipError_t launch_momentum_divergence(const float *m, size_t stride, int W, size_t n, double *out, const uint32_t *end64,
                                      int n_groups, hipStream_t s)
{
    const int count = n_groups > 0 ? n_groups : 1;
    hipError_t e = launch(divergence_zero_kernel, (count + 255) / 256, 256, 0, s, out, count);
    if (e != hipSuccess || n == 0) return e;
    const unsigned grid = static_cast<unsigned>((n + 1023) / 1024);
    if (n_groups > 0) return launch(momentum_divergence_kernel<true>, grid, 256, 0, s, m, stride, W, n, out, end64, n_groups);
    return launch(momentum_divergence_kernel<false>, grid, 256, 0, s, m, stride, W, n, out, static_cast<const uint32_t *>(nullptr), 0);
}

}  // namespace lc
