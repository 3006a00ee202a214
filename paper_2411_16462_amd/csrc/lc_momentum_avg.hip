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

// the workgroup's tile: elements [block * 256, block * 256 + 256) of rows that hold n elements
template <int R>
__device__ __forceinline__ void momentum_avg_tile(float *__restrict__ m, size_t stride, int W, size_t n, float inv_w, size_t block)
{
    __shared__ f32x4 part[R][kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_index();
    const size_t e = block * kAvgTile + lane * 4;
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

template <int R>
__global__ __launch_bounds__(R *kWave) void momentum_avg_kernel(float *__restrict__ m, size_t stride, int W, size_t n, float inv_w)
{
    momentum_avg_tile<R>(m, stride, W, n, inv_w, blockIdx.x);
}

// Several ranges of the rows in one launch (selective synchronisation, Section 6.2): the
// ranges travel in the kernel arguments, workgroup b belongs to the range r with
// first[r] <= b < first[r + 1] and handles that range's tile b - first[r] exactly as a
// launch of its own on the range would.
constexpr int kAvgRanges = 32;
struct AvgRanges {
    size_t off[kAvgRanges];         // first element of the range (a multiple of 4)
    size_t size[kAvgRanges];        // its length in elements
    uint32_t first[kAvgRanges + 1]; // running count of tiles
    int count;
};

template <int R>
__global__ __launch_bounds__(R *kWave) void momentum_avg_ranges_kernel(float *__restrict__ m, size_t stride, int W, float inv_w,
                                                                       const AvgRanges ranges)
{
    int lo = 0, hi = ranges.count - 1;  // uniform bisection over at most 32 entries
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (ranges.first[mid] <= blockIdx.x) lo = mid;
        else hi = mid - 1;
    }
    momentum_avg_tile<R>(m + ranges.off[lo], stride, W, ranges.size[lo], inv_w, blockIdx.x - ranges.first[lo]);
}

hipError_t launch_momentum_avg(float *m, size_t stride, int W, size_t n, hipStream_t s)
{
    const unsigned grid = static_cast<unsigned>((n + kAvgTile - 1) / kAvgTile);
    const float inv_w = 1.0f / static_cast<float>(W);
    if (W >= 8) return launch(momentum_avg_kernel<8>, grid, 8 * kWave, LC_AVG_LDS, s, m, stride, W, n, inv_w);
    if (W >= 4) return launch(momentum_avg_kernel<4>, grid, 4 * kWave, 0, s, m, stride, W, n, inv_w);
    return launch(momentum_avg_kernel<2>, grid, 2 * kWave, 0, s, m, stride, W, n, inv_w);
}

// Ranges in batches of kAvgRanges per launch; empty ranges are skipped.  A batch also ends
// before its tile count would pass what one grid holds.
hipError_t launch_momentum_avg_ranges(float *m, size_t stride, int W, const size_t *offsets, const size_t *sizes, int n_ranges,
                                      hipStream_t s)
{
    const float inv_w = 1.0f / static_cast<float>(W);
    int r = 0;
    while (r < n_ranges) {
        AvgRanges batch;
        batch.count = 0;
        uint64_t tiles = 0;
        for (; r < n_ranges && batch.count < kAvgRanges; ++r) {
            if (sizes[r] == 0) continue;
            const uint64_t t = (sizes[r] + kAvgTile - 1) / kAvgTile;
            if (tiles + t > 0x7FFFFFFFull) break;  // a grid holds 2^31 - 1 workgroups
            batch.off[batch.count] = offsets[r];
            batch.size[batch.count] = sizes[r];
            batch.first[batch.count] = static_cast<uint32_t>(tiles);
            tiles += t;
            ++batch.count;
        }
        if (batch.count == 0) continue;  // only empty ranges were left
        for (int k = batch.count; k < kAvgRanges; ++k) batch.off[k] = batch.size[k] = 0;
        for (int k = batch.count; k <= kAvgRanges; ++k) batch.first[k] = static_cast<uint32_t>(tiles);
        const unsigned grid = static_cast<unsigned>(tiles);
        hipError_t e;
        if (W >= 8) e = launch(momentum_avg_ranges_kernel<8>, grid, 8 * kWave, LC_AVG_LDS, s, m, stride, W, inv_w, batch);
        else if (W >= 4) e = launch(momentum_avg_ranges_kernel<4>, grid, 4 * kWave, 0, s, m, stride, W, inv_w, batch);
        else e = launch(momentum_avg_ranges_kernel<2>, grid, 2 * kWave, 0, s, m, stride, W, inv_w, batch);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---- divergence of the workers' momenta (Section 5.1, the quantity of Figure 6) --------
// max over elements of the standard deviation across the W workers (divisor W), in fp64
// with the workers taken in order, so that the result equals a sequential evaluation bit
// for bit; the maximum is order-free.  Reads W * 4 bytes per element, writes one double
// (or one per segment of a group table).
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

#ifndef LC_DIV_STREAMS
#define LC_DIV_STREAMS 1024  // measured alike from 256 to 2048; 8 and 64 are slower
#endif
constexpr unsigned kDivStreams = LC_DIV_STREAMS;
#ifndef LC_DIV_LDS
#define LC_DIV_LDS 0  // unused dynamic LDS per workgroup: a tuning knob that caps occupancy
#endif

// Largest sum of squared deviations among the lane's four elements e .. e + 3.  CAP > 0:
// the wave's 256 elements all lie below n and W <= CAP; every row is requested once, up
// front, and both passes (sum, then squared deviations, workers in order) run from
// registers -- 6.8 TB/s at 16 rows against 3.3 TB/s for the form that reads the rows a
// second time.  A row index at or beyond W re-reads the last row (a cache hit) and is left
// out of the arithmetic.  CAP = 0: any W, ragged end; the second pass reads the rows again.
template <int CAP, class Between>
__device__ __forceinline__ double divergence_worst(const float *__restrict__ m, size_t stride, int W, size_t n, size_t tile,
                                                   unsigned lane_off, Between &&between)
{
    const size_t e = tile + lane_off;
    double worst = 0.0;
    const double dw = static_cast<double>(W);
    if constexpr (CAP > 0) {
        f32x4 x[CAP];
#pragma unroll
        for (int w = 0; w < CAP; ++w) {
            // uniform row address plus a 32-bit lane offset: no address registers per row
            const float *row = m + static_cast<size_t>(w < W ? w : W - 1) * stride + tile;
            x[w] = load4(row + lane_off);
        }
        __builtin_amdgcn_sched_barrier(0);  // every row is requested before the first is used
        between();                          // work that does not depend on the rows runs while they are in flight
        double sum[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int w = 0; w < CAP; ++w) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (w < W) sum[k] += static_cast<double>(x[w][k]);
        }
        double mean[4], ss[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int k = 0; k < 4; ++k) mean[k] = sum[k] / dw;
        // the second pass converts the rows again: keeping the first pass's doubles would
        // triple the registers per lane
#pragma unroll
        for (int w = 0; w < CAP; ++w) asm volatile("" : "+v"(x[w]));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int w = 0; w < CAP; ++w) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if (w < W) {
                    const double d = static_cast<double>(x[w][k]) - mean[k];
                    ss[k] += d * d;
                }
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (ss[k] > worst) worst = ss[k];
    } else {
        between();
        double sum[4] = {0.0, 0.0, 0.0, 0.0};
        for (int w = 0; w < W; ++w) {
            const f32x4 v = load4_guarded(m + static_cast<size_t>(w) * stride, e, n);
#pragma unroll
            for (int k = 0; k < 4; ++k) sum[k] += static_cast<double>(v[k]);
        }
        double mean[4], ss[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int k = 0; k < 4; ++k) mean[k] = sum[k] / dw;
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
    return worst;
}

// GROUPED: out[s] receives the maximum over segment s of a group table (segment ends in
// units of 64 elements).  A wave whose 256 elements lie in one segment reduces first; a wave
// that straddles a boundary lets every lane publish its own value.
template <int CAP, bool GROUPED>
__global__ __launch_bounds__(256) void momentum_divergence_kernel(const float *__restrict__ m, size_t stride, int W, size_t n,
                                                                  double *__restrict__ out,
                                                                  const uint32_t *__restrict__ end64, int G)
{
    __shared__ double s_max[4];
    __shared__ int s_seg[4];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_index();
    // GROUPED: workgroup b works in stream b % S at position b / S, so that the workgroups in
    // flight at one time lie in S distant places.  In launch order the workgroups of a segment
    // would all run at once, every one of them would read the segment's slot before any has
    // written it, and every one would then send its atomic to that one address (measured on
    // 148 equal segments of 124 M elements: 1.27 ms against 0.58 ms).
    size_t wg = blockIdx.x;
    if (GROUPED) wg = static_cast<size_t>(blockIdx.x % kDivStreams) * (gridDim.x / kDivStreams) + blockIdx.x / kDivStreams;
    const size_t tile = (wg * 4 + wave) * 256;  // the wave's first element (uniform)
    const size_t e = tile + static_cast<size_t>(lane) * 4;
    // GROUPED: the segment of the wave's first 64-element block (uniform), then each lane
    // walks on to the segment of its own block; lanes past n stay with the last.  Small
    // tables are requested here, ahead of the rows, and resolved with lane masks once the
    // rows are requested; large ones are bisected, a chain of dependent loads that runs
    // between the request for the rows and their use.
    int seg = G - 1;
    GroupEnds ends;
    const bool counted = GROUPED && G <= kGroupCountMax;
    if (counted) ends.load(end64, G, lane);
    auto find_group = [&] {
        if (GROUPED) {
            const uint32_t b = static_cast<uint32_t>(tile / 64);
            int first;
            bool one = false;  // the wave's four blocks lie in one segment
            if (counted) {
                first = ends.count(G, b);
                one = ends.count(G, b + 3) == first;
            } else {
                first = group_find(end64, G, b);
            }
            if (e < n) seg = one ? first : group_walk(end64, G, first, static_cast<uint32_t>(e / 64));
        }
    };
    double worst = 0.0;  // largest sum of squared deviations of this lane's elements
    if (CAP > 0 && tile + 256 <= n) worst = divergence_worst<CAP>(m, stride, W, n, tile, lane * 4u, find_group);
    else {
        find_group();  // with every lane active
        if (e < n) worst = divergence_worst<0>(m, stride, W, n, tile, lane * 4u, [] {});
    }
    unsigned long long bits = static_cast<unsigned long long>(__double_as_longlong(worst));
    if (GROUPED) {
        // A wave inside one segment reduces and hands its value to the workgroup; a wave
        // across a boundary publishes lane by lane.  Waves of one segment are neighbours:
        // one publication per run of equal segments, so that the segment's slot -- one
        // address for every reader on the chip -- is touched once per workgroup at most.
        const int seg0 = __builtin_amdgcn_readfirstlane(seg);
        int mine = -1;
        if (__ballot(seg != seg0) == 0) {
            bits = wave_max_bits(bits, lane);
            mine = seg0;
        } else {
            publish_std(out + seg, worst, W);
        }
        if (lane == 0) {
            s_max[wave] = __longlong_as_double(static_cast<long long>(bits));
            s_seg[wave] = mine;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int r = 0; r < 4;) {
                const int sg = s_seg[r];
                double b = s_max[r];
                int q = r + 1;
                for (; q < 4 && s_seg[q] == sg; ++q) b = s_max[q] > b ? s_max[q] : b;
                if (sg >= 0) publish_std(out + sg, b, W);
                r = q;
            }
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
    unsigned grid = static_cast<unsigned>((n + 1023) / 1024);
    if (n_groups > 0) grid = (grid + kDivStreams - 1) / kDivStreams * kDivStreams;  // whole streams; the surplus workgroups lie beyond n
    const uint32_t *none = nullptr;
#define LC_LAUNCH(CAP)                                                                                                       \
    return n_groups > 0 ? launch(momentum_divergence_kernel<CAP, true>, grid, 256, LC_DIV_LDS, s, m, stride, W, n, out, end64, n_groups) \
                        : launch(momentum_divergence_kernel<CAP, false>, grid, 256, LC_DIV_LDS, s, m, stride, W, n, out, none, 0)
    if (W <= 4) LC_LAUNCH(4);
    if (W <= 8) LC_LAUNCH(8);
    if (W <= 16) LC_LAUNCH(16);
    if (W <= 32) LC_LAUNCH(32);
    if (W <= 64) LC_LAUNCH(64);
    LC_LAUNCH(0);
#undef LC_LAUNCH
}

}  // namespace lc
