// Local interpolation, sign, zero rule and packing for all W workers in one launch
// (Algorithm 1 lines 3 and 6; Section 3 for the 1-bit form; Appendix F.1 for p-bit fields).
//
// Memory-bound streaming kernel: per worker and element it reads m (4 B) and g (4 or
// 2 B), optionally writes m (4 B), and writes 1/8 .. 1 byte of packed output.
//
// Work split.  grid.y = worker, grid.x = chunk of kPackBlock elements.  A wave owns
// kPackTiles tiles of 256 consecutive elements: in a tile lane l holds elements
// 4l..4l+3 (one 16-byte load per operand, 1 KiB per wave instruction), so a tile's
// 1-bit output is 32 bytes.  The default is one tile per wave and one wave per
// workgroup: many short, independent waves measured fastest for this read-modify-write
// stream (longer waves, 2..8 tiles, lose 3..10 %).
//
// 1-bit packing.  Each lane forms the 4 bits of its elements, shifts them to
// 4*(l mod 8) and an OR butterfly over each aligned group of 8 lanes (three DPP steps)
// leaves the dword that covers the group's 32 elements in every lane of the group.
// Lane 8h+t (t < kPackTiles) then stores tile t's dword h.
#include "lc_launch.hpp"

namespace lc {

#ifndef LC_PACK_TILES
#define LC_PACK_TILES 1
#endif
#ifndef LC_PACK_THREADS
#define LC_PACK_THREADS 64
#endif
#ifndef LC_PACK_LDS
#define LC_PACK_LDS 0  // unused dynamic LDS per workgroup: a tuning knob that caps occupancy
#endif
constexpr int kPackTiles = LC_PACK_TILES;             // 256-element tiles per wave
constexpr int kPackThreads = LC_PACK_THREADS;         // workgroup size
constexpr int kPackWave = kPackTiles * 256;           // elements per wave
constexpr int kPackBlock = kPackWave * (kPackThreads / kWave);
static_assert(kPackTiles >= 1 && kPackTiles <= 8, "a lane of each 8-lane group stores one tile's dword");

// The workgroup index is remapped so that 4 consecutive tiles -- whose 1-bit output shares
// one 128-byte line -- run on the same XCD (measured: +1..3 %; 2 gains nothing, 8 and more lose).
#ifndef LC_PACK_XCD
#define LC_PACK_XCD 4
#endif
__device__ __forceinline__ size_t pack_chunk_index(unsigned b, unsigned nblocks)
{
    return xcd_chunk_index<LC_PACK_XCD>(b, nblocks);
}

// bit that a value of the interpolation c maps to: 1 if c > 0, 0 if c < 0, and the
// zero rule's bit when c is zero (either sign) or NaN.
__device__ __forceinline__ uint32_t sign_to_bit(float c, bool zero_is_one)
{
    return zero_is_one ? !(c < 0.0f) : (c > 0.0f);
}

// c = beta1*m + (1-beta1)*g with the fixed order of two roundings: fl(omb1*g), then fma.
__device__ __forceinline__ float interpolate(float m, float g, float beta1, float omb1)
{
    return __builtin_fmaf(beta1, m, omb1 * g);
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_or(uint32_t v)
{
    return v | static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xF, 0xF, false));
}

// OR over each aligned group of 8 lanes, result in all 8.
__device__ __forceinline__ uint32_t or_reduce8(uint32_t v)
{
    v = dpp_or<0xB1>(v);   // quad_perm [1,0,3,2]
    v = dpp_or<0x4E>(v);   // quad_perm [2,3,0,1]
    v = dpp_or<0x141>(v);  // row_half_mirror: lane i <-> 7-i inside each half row
    return v;
}

template <int GDT, int OUT_BITS, bool UPDATE_M>
__global__ __launch_bounds__(kPackThreads) void local_update_pack_kernel(
    const void *__restrict__ g, size_t g_stride, float *__restrict__ m, size_t m_stride, size_t n,
    float beta1, float omb1, float beta2, float omb2, void *__restrict__ q, size_t q_stride_bytes,
    int zero_bit)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_index();
    const size_t w = blockIdx.y;
    const size_t wave_base = pack_chunk_index(blockIdx.x, gridDim.x) * kPackBlock + static_cast<size_t>(wave) * kPackWave;
    if (wave_base >= n) return;

    float *mrow = m + w * m_stride;
    const void *grow = static_cast<const char *>(g) + w * g_stride * Grad<GDT>::kBytes;
    char *qrow = q ? static_cast<char *>(q) + w * q_stride_bytes : nullptr;
    const bool z1 = zero_bit != 0;

    if (wave_base + kPackWave <= n) {
        f32x4 mv[kPackTiles], gv[kPackTiles];
#pragma unroll
        for (int t = 0; t < kPackTiles; ++t) {
            const size_t e = wave_base + t * 256 + lane * 4;
            mv[t] = load4(mrow + e);
            gv[t] = Grad<GDT>::load4(grow, e);
        }
        uint32_t fld[kPackTiles];
#pragma unroll
        for (int t = 0; t < kPackTiles; ++t) {
            fld[t] = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float c = interpolate(mv[t][k], gv[t][k], beta1, omb1);
                fld[t] |= sign_to_bit(c, z1) << (OUT_BITS * k);
                if (UPDATE_M) mv[t][k] = momentum_step(mv[t][k], gv[t][k], beta2, omb2);
            }
        }
        if (UPDATE_M) {
#pragma unroll
            for (int t = 0; t < kPackTiles; ++t) store4(mrow + wave_base + t * 256 + lane * 4, mv[t]);
        }
        if (qrow) {
            if (OUT_BITS == 1) {
                uint32_t mine = 0;
#pragma unroll
                for (int t = 0; t < kPackTiles; ++t) {
                    const uint32_t d = or_reduce8(fld[t] << (4 * (lane & 7)));
                    if ((lane & 7) == t) mine = d;
                }
                if ((lane & 7) < kPackTiles) {
                    uint32_t *q32 = reinterpret_cast<uint32_t *>(qrow) + wave_base / 32;
                    q32[(lane & 7) * 8 + (lane >> 3)] = mine;
                }
            } else {
#pragma unroll
                for (int t = 0; t < kPackTiles; ++t) {
                    const size_t quad = (wave_base + t * 256) / 4 + lane;  // index of this lane's 4 elements
                    if (OUT_BITS == 2) reinterpret_cast<uint8_t *>(qrow)[quad] = static_cast<uint8_t>(fld[t]);
                    if (OUT_BITS == 4) reinterpret_cast<uint16_t *>(qrow)[quad] = static_cast<uint16_t>(fld[t]);
                    if (OUT_BITS == 8) reinterpret_cast<uint32_t *>(qrow)[quad] = fld[t];
                }
            }
        }
        return;
    }

    // Ragged end of the range: 64 elements at a time, one per lane; the lane mask of
    // the comparison is the packed word.
    const size_t wave_end = (wave_base + kPackWave < n) ? wave_base + kPackWave : n;
    for (size_t b = wave_base; b < wave_end; b += kWave) {
        const size_t i = b + lane;
        const bool valid = i < n;
        uint32_t bit = 0;
        if (valid) {
            const float mm = ld_stream(mrow + i);
            const float gg = Grad<GDT>::load1(grow, i);
            bit = sign_to_bit(interpolate(mm, gg, beta1, omb1), z1);
            if (UPDATE_M) st_stream(mrow + i, momentum_step(mm, gg, beta2, omb2));
        }
        const uint64_t mask = __ballot(bit != 0);
        if (!qrow) continue;
        if (OUT_BITS == 1) {
            if (lane == 0) reinterpret_cast<uint64_t *>(qrow)[b / 64] = mask;
        } else {
            constexpr int per = 8 / OUT_BITS;  // fields per byte
            if (valid && lane % per == 0) {
                uint32_t byte = 0;
#pragma unroll
                for (int k = 0; k < per; ++k) byte |= static_cast<uint32_t>((mask >> (lane + k)) & 1u) << (OUT_BITS * k);
                reinterpret_cast<uint8_t *>(qrow)[i / per] = static_cast<uint8_t>(byte);
            }
        }
    }
}

// Ternary wire format (Appendix B.1's allreduce that transmits exact zeros): the sign
// s = sign(c) in {-1, 0, +1} leaves the worker as two 1-bit planes, pos (s > 0) and nz
// (s != 0); nothing is forced.  Same tiling and packing as the 1-bit kernel.
template <int GDT, bool UPDATE_M>
__global__ __launch_bounds__(kPackThreads) void local_update_pack_ternary_kernel(
    const void *__restrict__ g, size_t g_stride, float *__restrict__ m, size_t m_stride, size_t n, float beta1, float omb1,
    float beta2, float omb2, uint64_t *__restrict__ pos, uint64_t *__restrict__ nz, size_t stride_words)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_index();
    const size_t w = blockIdx.y;
    const size_t wave_base = pack_chunk_index(blockIdx.x, gridDim.x) * kPackBlock + static_cast<size_t>(wave) * kPackWave;
    if (wave_base >= n) return;
    float *mrow = m + w * m_stride;
    const void *grow = static_cast<const char *>(g) + w * g_stride * Grad<GDT>::kBytes;
    uint64_t *prow = pos + w * stride_words;
    uint64_t *zrow = nz + w * stride_words;

    if (wave_base + kPackWave <= n) {
        f32x4 mv[kPackTiles], gv[kPackTiles];
#pragma unroll
        for (int t = 0; t < kPackTiles; ++t) {
            const size_t e = wave_base + t * 256 + lane * 4;
            mv[t] = load4(mrow + e);
            gv[t] = Grad<GDT>::load4(grow, e);
        }
        uint32_t pb[kPackTiles], zb[kPackTiles];
#pragma unroll
        for (int t = 0; t < kPackTiles; ++t) {
            pb[t] = 0;
            zb[t] = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float c = interpolate(mv[t][k], gv[t][k], beta1, omb1);
                pb[t] |= static_cast<uint32_t>(c > 0.0f) << k;
                zb[t] |= static_cast<uint32_t>(c > 0.0f || c < 0.0f) << k;
                if (UPDATE_M) mv[t][k] = momentum_step(mv[t][k], gv[t][k], beta2, omb2);
            }
        }
        if (UPDATE_M) {
#pragma unroll
            for (int t = 0; t < kPackTiles; ++t) store4(mrow + wave_base + t * 256 + lane * 4, mv[t]);
        }
#pragma unroll
        for (int t = 0; t < kPackTiles; ++t) {
            const uint32_t pd = or_reduce8(pb[t] << (4 * (lane & 7)));
            const uint32_t zd = or_reduce8(zb[t] << (4 * (lane & 7)));
            const size_t d = (wave_base + t * 256) / 32 + (lane >> 3);  // dword of this group of 8 lanes
            if ((lane & 7) == 0) reinterpret_cast<uint32_t *>(prow)[d] = pd;
            if ((lane & 7) == 1) reinterpret_cast<uint32_t *>(zrow)[d] = zd;
        }
        return;
    }
    const size_t wave_end = (wave_base + kPackWave < n) ? wave_base + kPackWave : n;
    for (size_t b = wave_base; b < wave_end; b += kWave) {
        const size_t i = b + lane;
        bool p = false, z = false;
        if (i < n) {
            const float mm = ld_stream(mrow + i);
            const float gg = Grad<GDT>::load1(grow, i);
            const float c = interpolate(mm, gg, beta1, omb1);
            p = c > 0.0f;
            z = c > 0.0f || c < 0.0f;
            if (UPDATE_M) st_stream(mrow + i, momentum_step(mm, gg, beta2, omb2));
        }
        const uint64_t pm = __ballot(p), zm = __ballot(z);
        if (lane == 0) {
            prow[b / 64] = pm;
            zrow[b / 64] = zm;
        }
    }
}

hipError_t launch_local_update_pack_ternary(const void *g, size_t g_stride, int g_dtype, float *m, size_t m_stride, int W,
                                            size_t n, float beta1, bool update_m, float beta2, uint64_t *pos, uint64_t *nz,
                                            size_t stride_words, hipStream_t s)
{
    const dim3 grid(static_cast<unsigned>((n + kPackBlock - 1) / kPackBlock), static_cast<unsigned>(W));
    const float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
#define LC_LAUNCH(GDT, UPD)                                                                                         \
    return launch(local_update_pack_ternary_kernel<GDT, UPD>, grid, kPackThreads, LC_PACK_LDS, s, g, g_stride, m, m_stride, \
                  n, beta1, omb1, beta2, omb2, pos, nz, stride_words)
    if (g_dtype == LC_BF16) {
        if (update_m) LC_LAUNCH(LC_BF16, true);
        LC_LAUNCH(LC_BF16, false);
    }
    if (update_m) LC_LAUNCH(LC_F32, true);
    LC_LAUNCH(LC_F32, false);
#undef LC_LAUNCH
}

template <int GDT, int OUT_BITS>
static hipError_t launch_pack(bool update_m, dim3 grid, hipStream_t s, const void *g, size_t g_stride, float *m,
                              size_t m_stride, size_t n, float beta1, float omb1, float beta2, float omb2, void *q,
                              size_t q_stride_bytes, int zero_bit)
{
    if (update_m)
        return launch(local_update_pack_kernel<GDT, OUT_BITS, true>, grid, kPackThreads, LC_PACK_LDS, s, g, g_stride, m, m_stride, n,
                      beta1, omb1, beta2, omb2, q, q_stride_bytes, zero_bit);
    return launch(local_update_pack_kernel<GDT, OUT_BITS, false>, grid, kPackThreads, LC_PACK_LDS, s, g, g_stride, m, m_stride, n,
                  beta1, omb1, beta2, omb2, q, q_stride_bytes, zero_bit);
}

template <int GDT>
static hipError_t launch_pack_bits(int out_bits, bool update_m, dim3 grid, hipStream_t s, const void *g, size_t g_stride,
                                   float *m, size_t m_stride, size_t n, float beta1, float omb1, float beta2, float omb2,
                                   void *q, size_t q_stride_bytes, int zero_bit)
{
    switch (out_bits) {
    case 1: return launch_pack<GDT, 1>(update_m, grid, s, g, g_stride, m, m_stride, n, beta1, omb1, beta2, omb2, q, q_stride_bytes, zero_bit);
    case 2: return launch_pack<GDT, 2>(update_m, grid, s, g, g_stride, m, m_stride, n, beta1, omb1, beta2, omb2, q, q_stride_bytes, zero_bit);
    case 4: return launch_pack<GDT, 4>(update_m, grid, s, g, g_stride, m, m_stride, n, beta1, omb1, beta2, omb2, q, q_stride_bytes, zero_bit);
    default: return launch_pack<GDT, 8>(update_m, grid, s, g, g_stride, m, m_stride, n, beta1, omb1, beta2, omb2, q, q_stride_bytes, zero_bit);
    }
}

// Host launcher; arguments were validated by the caller.
hipError_t launch_local_update_pack(const void *g, size_t g_stride, int g_dtype, float *m, size_t m_stride, int W, size_t n,
                                    float beta1, bool update_m, float beta2, int out_bits, void *q, size_t q_stride_bytes,
                                    int zero_bit, hipStream_t s)
{
    const dim3 grid(static_cast<unsigned>((n + kPackBlock - 1) / kPackBlock), static_cast<unsigned>(W));
    const float omb1 = 1.0f - beta1;
    const float omb2 = 1.0f - beta2;
    if (g_dtype == LC_BF16)
        return launch_pack_bits<LC_BF16>(out_bits, update_m, grid, s, g, g_stride, m, m_stride, n, beta1, omb1, beta2, omb2, q,
                                         q_stride_bytes, zero_bit);
    return launch_pack_bits<LC_F32>(out_bits, update_m, grid, s, g, g_stride, m, m_stride, n, beta1, omb1, beta2, omb2, q,
                                    q_stride_bytes, zero_bit);
}

}  // namespace lc
