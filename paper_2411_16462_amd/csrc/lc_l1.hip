// L1 quantisation of the update (Section 4.2, Equation 1 with p = 1; Appendix F.1):
//   pass 1  M_1 = mean_i |c_i| per worker, with the sum formed WITHOUT rounding, so that the
//           result does not depend on the order in which a GPU adds and equals what a
//           sequential exact summation gives;
//   pass 2  level_i = clamp(round(L / (2 M_1) * c_i), L), stored as the byte level_i + L,
//           fused with the momentum update of Algorithm 1 line 6.
// c = beta1 * m + (1 - beta1) * g as in the 1-bit path (same fixed fp32 evaluation).
//
// Exact sum.  A finite binary32 is an integer M < 2^24 times 2^(P-149), P = max(E, 1) - 1 the
// bit position of M's lowest bit.  Integers add exactly, so the sum is kept as one long
// integer in units of 2^-149: 64-bit accumulators 32 bits apart ("limbs"), each of which
// only ever receives pieces below 2^32 and therefore cannot overflow for any n < 2^32
// additions.  Each lane of a wave sums its elements as 64-bit integers relative to a base
// position chosen from the wave's first tile (elements whose magnitude lies outside a
// window of 28 binary orders above that base -- rare -- go to the limbs one by one); the
// wave adds its 64 lane sums, shifts the total to the base and adds it to the workgroup's
// limbs in LDS; the workgroup adds its limbs, carries propagated, to the worker's limbs
// in global memory with 64-bit atomics.  A one-thread kernel rounds the long integer once to fp64
// (nearest, ties to even) and divides by n.
//
// Groups.  With a table of parameter groups (consecutive segments of the arena that end on
// multiples of 64 elements) every (worker, group) pair gets its own M_1 in the same three
// launches: a one-workgroup kernel turns the segment ends into a running count of
// workgroups per group (the "plan"), each workgroup of the summing kernel bisects the plan
// for its group and works inside that segment only, and the finalising kernel runs one
// thread per pair.  The second pass looks the group of each 64-element block up by
// bisection on the segment ends while its loads of m and g are in flight.
#include "lc_launch.hpp"

#include <mutex>

namespace lc {

#ifndef LC_L1_TILES
#define LC_L1_TILES 8
#endif
constexpr int kL1Threads = 256;
constexpr int kL1Waves = kL1Threads / kWave;
constexpr int kL1Tiles = LC_L1_TILES;                       // 256-element tiles per wave
constexpr int kL1Block = kL1Waves * kL1Tiles * 256;         // elements per workgroup

__device__ __forceinline__ float interpolate_c(float m, float g, float beta1, float omb1)
{
    return __builtin_fmaf(beta1, m, omb1 * g);
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t v)
{
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(static_cast<int>(v), static_cast<int>(v), CTRL, 0xF, 0xF, false));
}

// min and max over the wave, uniform result
__device__ __forceinline__ void wave_min_max(uint32_t lo, uint32_t hi, uint32_t &wmin, uint32_t &wmax)
{
#define LC_STEP(CTRL)                          \
    {                                          \
        const uint32_t a = dpp_mov<CTRL>(lo);  \
        const uint32_t b = dpp_mov<CTRL>(hi);  \
        lo = a < lo ? a : lo;                  \
        hi = b > hi ? b : hi;                  \
    }
    LC_STEP(0xB1)   // quad_perm [1,0,3,2]
    LC_STEP(0x4E)   // quad_perm [2,3,0,1]
    LC_STEP(0x141)  // row_half_mirror
    LC_STEP(0x140)  // row_mirror: every lane of a row of 16 now holds the row's result
#undef LC_STEP
    uint32_t a0 = __builtin_amdgcn_readlane(lo, 0), a1 = __builtin_amdgcn_readlane(lo, 16);
    uint32_t a2 = __builtin_amdgcn_readlane(lo, 32), a3 = __builtin_amdgcn_readlane(lo, 48);
    uint32_t b0 = __builtin_amdgcn_readlane(hi, 0), b1 = __builtin_amdgcn_readlane(hi, 16);
    uint32_t b2 = __builtin_amdgcn_readlane(hi, 32), b3 = __builtin_amdgcn_readlane(hi, 48);
    a0 = a0 < a1 ? a0 : a1;
    a2 = a2 < a3 ? a2 : a3;
    b0 = b0 > b1 ? b0 : b1;
    b2 = b2 > b3 ? b2 : b3;
    wmin = a0 < a2 ? a0 : a2;
    wmax = b0 > b2 ? b0 : b2;
}

__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t v, int lane)
{
#pragma unroll
    for (int mask = 1; mask < kWave; mask <<= 1) {
        const int addr = (lane ^ mask) << 2;
        const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(addr, static_cast<int>(static_cast<uint32_t>(v))));
        const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(addr, static_cast<int>(static_cast<uint32_t>(v >> 32))));
        v += (static_cast<uint64_t>(hi) << 32) | lo;
    }
    return v;
}

// value << pos added to the limbs (pieces of 32 bits)
__device__ __forceinline__ void limbs_add(uint64_t *limbs, uint64_t value, uint32_t pos)
{
    const uint32_t l = pos >> 5, sh = pos & 31u;
    const unsigned __int128 v = static_cast<unsigned __int128>(value) << sh;
    const uint64_t p0 = static_cast<uint64_t>(v) & 0xFFFFFFFFull;
    const uint64_t p1 = static_cast<uint64_t>(v >> 32) & 0xFFFFFFFFull;
    const uint64_t p2 = static_cast<uint64_t>(v >> 64);
    if (p0) atomicAdd(reinterpret_cast<unsigned long long *>(limbs + l), static_cast<unsigned long long>(p0));
    if (p1) atomicAdd(reinterpret_cast<unsigned long long *>(limbs + l + 1), static_cast<unsigned long long>(p1));
    if (p2) atomicAdd(reinterpret_cast<unsigned long long *>(limbs + l + 2), static_cast<unsigned long long>(p2));
}

__global__ void l1_zero_kernel(uint64_t *workspace, size_t words)
{
    const size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < words) workspace[i] = 0;
}

// plan[s] = number of summing workgroups of the groups before s, plan[G] = their total.
// One workgroup: each thread adds a contiguous share of the groups, thread 0 scans the
// shares.
constexpr uint32_t kL1Block64 = kL1Block / 64;
__global__ __launch_bounds__(256) void l1_plan_kernel(const uint32_t *__restrict__ end64, int G, uint32_t n64,
                                                      uint32_t *__restrict__ plan)
{
    __shared__ uint32_t part[256];
    const int per = (G + 255) / 256;
    const int lo = static_cast<int>(threadIdx.x) * per;
    const int hi = lo + per < G ? lo + per : G;
    uint32_t sum = 0;
    for (int s = lo; s < hi; ++s) sum += (group_hi64(end64, G, s, n64) - group_lo64(end64, s, n64) + kL1Block64 - 1) / kL1Block64;
    part[threadIdx.x] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int i = 0; i < 256; ++i) {
            const uint32_t t = part[i];
            part[i] = run;
            run += t;
        }
        plan[G] = run;
    }
    __syncthreads();
    uint32_t run = part[threadIdx.x];
    for (int s = lo; s < hi; ++s) {
        plan[s] = run;
        run += (group_hi64(end64, G, s, n64) - group_lo64(end64, s, n64) + kL1Block64 - 1) / kL1Block64;
    }
}

// How far above the wave's base position a magnitude may sit to take the fast path: a
// lane then adds at most kL1Tiles * 4 integers below 2^(24 + kL1Window) to its private
// 64-bit sum, and 64 such sums still fit 64 bits.
constexpr uint32_t kL1Window = 28;
static_assert(kL1Tiles * 4 <= 32, "lane sums must stay below 2^57");

template <int GDT, bool GROUPED>
__global__ __launch_bounds__(kL1Threads) void l1_abs_sum_kernel(const void *__restrict__ g, size_t g_stride,
                                                                const float *__restrict__ m, size_t m_stride, size_t n_all,
                                                                float beta1, float omb1, uint64_t *__restrict__ workspace,
                                                                const uint32_t *__restrict__ end64,
                                                                const uint32_t *__restrict__ plan, int G)
{
    __shared__ uint64_t s_limbs[kL1Limbs];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_index();
    const size_t w = blockIdx.y;

    // the range [first, n) this workgroup's accumulator covers, and which accumulator
    size_t first = 0, n = n_all, acc = w;
    uint32_t local_block = blockIdx.x;
    if (GROUPED) {
        if (blockIdx.x >= plan[G]) return;  // the grid is an upper bound; uniform in the workgroup
        int lo = 0, hi = G;                 // last group whose first workgroup is <= blockIdx.x
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (plan[mid] <= blockIdx.x) lo = mid;
            else hi = mid;
        }
        const uint32_t n64 = static_cast<uint32_t>((n_all + 63) / 64);
        first = static_cast<size_t>(group_lo64(end64, lo, n64)) * 64;
        const size_t last = static_cast<size_t>(group_hi64(end64, G, lo, n64)) * 64;
        n = last < n_all ? last : n_all;
        local_block = blockIdx.x - plan[lo];
        acc = w * static_cast<size_t>(G) + static_cast<size_t>(lo);
    }
    if (threadIdx.x < kL1Limbs) s_limbs[threadIdx.x] = 0;
    __syncthreads();

    const float *mrow = m + w * m_stride;
    const void *grow = static_cast<const char *>(g) + w * g_stride * Grad<GDT>::kBytes;
    const size_t wave_base = first + static_cast<size_t>(local_block) * kL1Block + static_cast<size_t>(wave) * (kL1Tiles * 256);

    // The wave's base position comes from its first tile: 22 binary orders below that
    // tile's largest magnitude, so the window reaches 64 times above it.  Elements outside
    // the window (tiny or huge against the rest) go to the limbs one by one: still exact.
    uint32_t base = 0;
    uint64_t lane_sum = 0;
    bool have_base = false;
#pragma unroll 2
    for (int t = 0; t < kL1Tiles; ++t) {
        const size_t tile = wave_base + static_cast<size_t>(t) * 256;
        if (tile >= n) break;  // uniform in the wave
        const size_t e = tile + lane * 4;
        f32x4 mv = {0.0f, 0.0f, 0.0f, 0.0f}, gv = {0.0f, 0.0f, 0.0f, 0.0f};
        if (e + 4 <= n) {
            mv = ld_grad(reinterpret_cast<const f32x4 *>(mrow + e));
            gv = Grad<GDT>::load4(grow, e);
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (e + k < n) {
                    mv[k] = mrow[e + k];
                    gv[k] = Grad<GDT>::load1(grow, e + k);
                }
        }
        uint32_t mant[4], pos[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t b = __float_as_uint(interpolate_c(mv[k], gv[k], beta1, omb1)) & 0x7FFFFFFFu;
            const uint32_t ex = b >> 23;
            mant[k] = ex ? ((b & 0x7FFFFFu) | 0x800000u) : b;
            pos[k] = ex ? ex - 1u : 0u;
        }
        if (!have_base) {  // uniform
            uint32_t pmin = 0xFFFFu, pmax = 0u;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (mant[k]) {
                    pmin = pos[k] < pmin ? pos[k] : pmin;
                    pmax = pos[k] > pmax ? pos[k] : pmax;
                }
            uint32_t wmin, wmax;
            wave_min_max(pmin, pmax, wmin, wmax);
            if (wmin == 0xFFFFu) continue;  // the whole tile is zero: nothing to add, no base yet
            base = wmax > 22u ? wmax - 22u : 0u;
            have_base = true;
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t rel = pos[k] - base;  // wraps for positions below the base
            if (rel <= kL1Window || mant[k] == 0u) {
                lane_sum += static_cast<uint64_t>(mant[k]) << (rel & 31u);
            } else {
                limbs_add(s_limbs, mant[k], pos[k]);
            }
        }
    }
    if (have_base) {
        const uint64_t total = wave_sum_u64(lane_sum, lane);
        if (lane == 0 && total) limbs_add(s_limbs, total, base);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        // one of kL1Slots accumulators per worker, so that the atomics of neighbouring
        // workgroups do not queue on the same addresses
        uint64_t carry = 0;
        uint64_t *dst = workspace + (acc * kL1Slots + blockIdx.x % kL1Slots) * kL1Limbs;
#pragma unroll
        for (int l = 0; l < kL1Limbs; ++l) {
            const uint64_t v = s_limbs[l] + carry;
            const uint64_t piece = v & 0xFFFFFFFFull;
            carry = v >> 32;
            if (piece) atomicAdd(reinterpret_cast<unsigned long long *>(dst + l), static_cast<unsigned long long>(piece));
        }
    }
}

// One thread per accumulator (worker, or worker x group when G > 0): the limbs as one
// integer (units of 2^-149), rounded once to fp64 (nearest, ties to even), divided by the
// element count (of the call; of the group's segment; or the caller's count for the group).
__global__ void l1_finalize_kernel(uint64_t *workspace, int n_acc, size_t n_all, double *mean_abs, const uint32_t *end64,
                                   const uint64_t *count, int G)
{
    const int w = blockIdx.x * blockDim.x + threadIdx.x;
    if (w >= n_acc) return;
    size_t n = n_all;
    if (G > 0) {
        const int s = w % G;
        if (count) {
            n = count[s];
        } else {
            const uint32_t n64 = static_cast<uint32_t>((n_all + 63) / 64);
            const size_t lo = static_cast<size_t>(group_lo64(end64, s, n64)) * 64;
            size_t hi = static_cast<size_t>(group_hi64(end64, G, s, n64)) * 64;
            hi = hi < n_all ? hi : n_all;
            n = hi - lo;
        }
    }
    uint64_t *limb = workspace + static_cast<size_t>(w) * kL1Slots * kL1Limbs;  // slot 0 receives the total
    for (int s = 1; s < kL1Slots; ++s)
        for (int l = 0; l < kL1Limbs; ++l) limb[l] += limb[s * kL1Limbs + l];
    uint64_t carry = 0;
    int top = -1;
    for (int l = 0; l < kL1Limbs; ++l) {  // after this every limb is below 2^32
        const uint64_t v = limb[l] + carry;
        limb[l] = v & 0xFFFFFFFFull;
        carry = v >> 32;
        if (limb[l]) top = l;
    }
    double sum = 0.0;
    if (top >= 0) {
        const int tb = 32 * top + (31 - __builtin_clz(static_cast<uint32_t>(limb[top])));  // index of the highest set bit
        if (tb <= 52) {
            sum = static_cast<double>(limb[0] | (limb[1] << 32));
        } else {
            const int shift = tb - 52;  // bits below `shift` are rounded away
            const int li = shift >> 5, off = shift & 31;
            unsigned __int128 window = static_cast<unsigned __int128>(limb[li]);
            if (li + 1 < kL1Limbs) window |= static_cast<unsigned __int128>(limb[li + 1]) << 32;
            if (li + 2 < kL1Limbs) window |= static_cast<unsigned __int128>(limb[li + 2]) << 64;
            uint64_t mant = static_cast<uint64_t>(window >> off) & ((1ull << 53) - 1ull);
            const int rb = shift - 1;
            const bool round_bit = (limb[rb >> 5] >> (rb & 31)) & 1ull;
            bool sticky = false;
            for (int l = 0; l <= (rb >> 5); ++l) {
                uint64_t v = limb[l];
                if (l == (rb >> 5)) v &= (1ull << (rb & 31)) - 1ull;
                sticky = sticky || v != 0;
            }
            if (round_bit && (sticky || (mant & 1ull))) mant += 1;
            sum = ldexp(static_cast<double>(mant), shift);
        }
        sum = ldexp(sum, -149);
    }
    mean_abs[w] = n ? sum / static_cast<double>(n) : 0.0;
}

hipError_t launch_l1_mean_abs(const void *g, size_t g_stride, int g_dtype, const float *m, size_t m_stride, int W, size_t n,
                              float beta1, double *mean_abs, uint64_t *workspace, const L1Groups &grp, hipStream_t s)
{
    const int G = grp.n;
    const size_t n_acc = static_cast<size_t>(W) * static_cast<size_t>(G > 0 ? G : 1);
    const size_t words = n_acc * kL1Slots * kL1Limbs;
    uint32_t *plan = reinterpret_cast<uint32_t *>(workspace + words);
    hipError_t e = launch(l1_zero_kernel, static_cast<unsigned>((words + 255) / 256), 256, 0, s, workspace, words);
    if (e != hipSuccess) return e;
    if (n > 0) {
        const float omb1 = 1.0f - beta1;
        size_t blocks = (n + kL1Block - 1) / kL1Block;
        if (G > 0) {
            blocks += static_cast<size_t>(G);  // every group may end in a partly filled workgroup
            e = launch(l1_plan_kernel, 1, 256, 0, s, grp.end64, G, static_cast<uint32_t>((n + 63) / 64), plan);
            if (e != hipSuccess) return e;
        }
        const dim3 grid(static_cast<unsigned>(blocks), static_cast<unsigned>(W));
#define LC_LAUNCH(GDT, GROUPED)                                                                                      \
    launch(l1_abs_sum_kernel<GDT, GROUPED>, grid, kL1Threads, 0, s, g, g_stride, m, m_stride, n, beta1, omb1, workspace, \
           grp.end64, static_cast<const uint32_t *>(plan), G)
        if (g_dtype == LC_BF16) e = G > 0 ? LC_LAUNCH(LC_BF16, true) : LC_LAUNCH(LC_BF16, false);
        else e = G > 0 ? LC_LAUNCH(LC_F32, true) : LC_LAUNCH(LC_F32, false);
#undef LC_LAUNCH
        if (e != hipSuccess) return e;
    }
    return launch(l1_finalize_kernel, static_cast<unsigned>((n_acc + 63) / 64), 64, 0, s, workspace, static_cast<int>(n_acc), n,
                  mean_abs, grp.end64, grp.count, G);
}

// ---- pass 1 for callers that cannot allocate -------------------------------------------
// The workspace of lc_l1_mean_abs as a file-scope device array: every GPU the library runs
// on holds its own copy at its own address until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; kernels and launches always take
// the resolved device pointer, which is looked up once per device (with that device
// current) and kept.
static __device__ __align__(256) uint64_t scratch[LC_L1_STATIC_MAX_W * kL1Slots * kL1Limbs];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
uint64_t *g_scratch_ptr[kMaxDevices];  // device address of `scratch` per device ordinal; null = not yet resolved
}  // namespace

static hipError_t static_workspace(uint64_t **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        uint64_t *p = nullptr;
        e = hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

hipError_t launch_l1_mean_abs_static(const void *g, size_t g_stride, int g_dtype, const float *m, size_t m_stride, int W,
                                     size_t n, float beta1, double *mean_abs, hipStream_t s)
{
    uint64_t *ws = nullptr;
    const hipError_t e = static_workspace(&ws);
    if (e != hipSuccess) return e;
    // the summing kernels clear the W accumulator sets they use first (a fill kernel, so the
    // call can be captured into a graph), whatever the previous call left there
    return launch_l1_mean_abs(g, g_stride, g_dtype, m, m_stride, W, n, beta1, mean_abs, ws, L1Groups(), s);
}

// ---- pass 2: levels --------------------------------------------------------------------
#ifndef LC_L1Q_XCD
#define LC_L1Q_XCD 4  // consecutive tiles per XCD (measured: +2.5 %)
#endif
constexpr int kQuantThreads = 64;  // one wave, one 256-element tile: same shape as the 1-bit pack kernel

// Level of one element: scale * c rounded to the nearest integer (ties to even), clamped.
__device__ __forceinline__ int l1_level(float c, float scale, float fl, bool live)
{
    float r = __builtin_rintf(scale * c);
    r = r > fl ? fl : r;
    r = r < -fl ? -fl : r;
    return live ? static_cast<int>(r) : 0;
}

template <int GDT, bool UPDATE_M, bool GROUPED>
__global__ __launch_bounds__(kQuantThreads) void l1_quantize_pack_kernel(const void *__restrict__ g, size_t g_stride,
                                                                         float *__restrict__ m, size_t m_stride, size_t n,
                                                                         float beta1, float omb1, float beta2, float omb2,
                                                                         int L, const double *__restrict__ mean_abs,
                                                                         uint8_t *__restrict__ q, size_t q_stride_bytes,
                                                                         const uint32_t *__restrict__ end64, int G)
{
    const int lane = threadIdx.x;
    const size_t w = blockIdx.y;
    const size_t tile = xcd_chunk_index<LC_L1Q_XCD>(blockIdx.x, gridDim.x) * 256;
    const size_t e = tile + lane * 4;
    if (e >= n) return;
    float *mrow = m + w * m_stride;
    const void *grow = static_cast<const char *>(g) + w * g_stride * Grad<GDT>::kBytes;
    uint8_t *qrow = q + w * q_stride_bytes;
    const bool full = e + 4 <= n;
    f32x4 mv = {0.0f, 0.0f, 0.0f, 0.0f}, gv = {0.0f, 0.0f, 0.0f, 0.0f};
    if (full) {  // issued first: the group look-up below runs while these are in flight
        mv = load4(mrow + e);
        gv = Grad<GDT>::load4(grow, e);
    }
    size_t mean_index = w;
    if (GROUPED) {
        // first group that ends beyond the tile's first 64-element block (uniform), then
        // each lane walks on to the group of its own block
        const int first = group_find(end64, G, static_cast<uint32_t>(tile / 64));
        const int sgm = group_walk(end64, G, first, static_cast<uint32_t>(e / 64));
        mean_index = w * static_cast<size_t>(G) + static_cast<size_t>(sgm);
    }
    const double mean = mean_abs[mean_index];
    const bool live = mean > 0.0;                       // all-zero input: every level is 0
    const float scale = live ? static_cast<float>(static_cast<double>(L) / (2.0 * mean)) : 0.0f;
    const float fl = static_cast<float>(L);
    if (full) {
        uint32_t bytes = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float c = interpolate_c(mv[k], gv[k], beta1, omb1);
            bytes |= static_cast<uint32_t>(l1_level(c, scale, fl, live) + L) << (8 * k);
            if (UPDATE_M) mv[k] = momentum_step(mv[k], gv[k], beta2, omb2);
        }
        if (UPDATE_M) store4(mrow + e, mv);
        st_stream(reinterpret_cast<uint32_t *>(qrow + e), bytes);
    } else {
        for (int k = 0; k < 4 && e + k < n; ++k) {
            const float mm = mrow[e + k];
            const float gg = Grad<GDT>::load1(grow, e + k);
            const float c = interpolate_c(mm, gg, beta1, omb1);
            qrow[e + k] = static_cast<uint8_t>(l1_level(c, scale, fl, live) + L);
            if (UPDATE_M) mrow[e + k] = momentum_step(mm, gg, beta2, omb2);
        }
    }
}

hipError_t launch_l1_quantize_pack(const void *g, size_t g_stride, int g_dtype, float *m, size_t m_stride, int W, size_t n,
                                   float beta1, bool update_m, float beta2, int levels, const double *mean_abs, uint8_t *q,
                                   size_t q_stride_bytes, const L1Groups &grp, hipStream_t s)
{
    const dim3 grid(static_cast<unsigned>((n + 255) / 256), static_cast<unsigned>(W));
    const float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
#define LC_LAUNCH(GDT, UPD, GRP)                                                                                     \
    return launch(l1_quantize_pack_kernel<GDT, UPD, GRP>, grid, kQuantThreads, 0, s, g, g_stride, m, m_stride, n, beta1, omb1, \
                  beta2, omb2, levels, mean_abs, q, q_stride_bytes, grp.end64, grp.n)
#define LC_LAUNCH2(GDT, UPD)                  \
    if (grp.n > 0) LC_LAUNCH(GDT, UPD, true); \
    LC_LAUNCH(GDT, UPD, false)
    if (g_dtype == LC_BF16) {
        if (update_m) { LC_LAUNCH2(LC_BF16, true); }
        LC_LAUNCH2(LC_BF16, false);
    }
    if (update_m) { LC_LAUNCH2(LC_F32, true); }
    LC_LAUNCH2(LC_F32, false);
#undef LC_LAUNCH2
#undef LC_LAUNCH
}

}  // namespace lc
