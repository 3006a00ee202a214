// Shared device helpers for the Lion Cub kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lioncub.h"

namespace lc {

// Every buffer of this path is streamed: read once and (for m and theta) written once
// per call, with no reuse.  Marking BOTH the loads and the stores non-temporal is what
// lets the kernels run at DRAM speed on MI355X (measured: +30 % over plain accesses;
// either one alone gains nothing).
#ifndef LC_NT
#define LC_NT 1
#endif
#ifndef LC_NT_G
#define LC_NT_G 1  // gradient rows (read only)
#endif
#ifndef LC_NT_Q
#define LC_NT_Q 0  // packed rows and vote planes (read only)
#endif

constexpr int kWave = 64;

using f32x4 = __attribute__((ext_vector_type(4))) float;
using u32x4 = __attribute__((ext_vector_type(4))) uint32_t;
using u32x2 = __attribute__((ext_vector_type(2))) uint32_t;

__device__ __forceinline__ float bits_f32(uint32_t b) { return __uint_as_float(b); }

// streaming load / store of any scalar or vector type
template <typename T>
__device__ __forceinline__ T ld_stream(const T *p)
{
#if LC_NT
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}
// loads from streams that a call only reads: gradients, packed rows
template <typename T>
__device__ __forceinline__ T ld_grad(const T *p)
{
#if LC_NT_G
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}
template <typename T>
__device__ __forceinline__ T ld_packed(const T *p)
{
#if LC_NT_Q
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}
template <typename T>
__device__ __forceinline__ void st_stream(T *p, T v)
{
#if LC_NT
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}

// Gradient rows are fp32 or bfloat16; a bfloat16 is the upper half of a binary32, so
// widening is a shift (exact).
template <int GDT>
struct Grad;

template <>
struct Grad<LC_F32> {
    static constexpr int kBytes = 4;
    static __device__ __forceinline__ f32x4 load4(const void *row, size_t i)
    {
        return ld_grad(reinterpret_cast<const f32x4 *>(static_cast<const float *>(row) + i));
    }
    static __device__ __forceinline__ float load1(const void *row, size_t i)
    {
        return ld_grad(static_cast<const float *>(row) + i);
    }
};

template <>
struct Grad<LC_BF16> {
    static constexpr int kBytes = 2;
    static __device__ __forceinline__ f32x4 load4(const void *row, size_t i)
    {
        const u32x2 v = ld_grad(reinterpret_cast<const u32x2 *>(static_cast<const uint16_t *>(row) + i));
        f32x4 r;
        r.x = bits_f32(v.x << 16);
        r.y = bits_f32(v.x & 0xffff0000u);
        r.z = bits_f32(v.y << 16);
        r.w = bits_f32(v.y & 0xffff0000u);
        return r;
    }
    static __device__ __forceinline__ float load1(const void *row, size_t i)
    {
        return bits_f32(static_cast<uint32_t>(ld_grad(static_cast<const uint16_t *>(row) + i)) << 16);
    }
};

__device__ __forceinline__ f32x4 load4(const float *p) { return ld_stream(reinterpret_cast<const f32x4 *>(p)); }
__device__ __forceinline__ void store4(float *p, f32x4 v) { st_stream(reinterpret_cast<f32x4 *>(p), v); }

// Index of the wave in its workgroup as a value the compiler knows to be uniform (it lives
// in a scalar register), so that what depends on it -- tile bases, row pointers, the search
// through a group table -- stays on the scalar unit and its loads in the scalar cache.
// threadIdx.x / 64 alone is uniform too, but the compiler cannot tell and would make every
// such load a vector load that waits behind the wave's streaming loads.
__device__ __forceinline__ int wave_index()
{
    return __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) / kWave);
}

// Workgroups are handed to the 8 XCDs (each with its own L2) round-robin by index.  This
// remaps the workgroup index so that G consecutive chunks (G a power of two) run on the
// same XCD; G = 0 or 1 leaves the order alone.  Only whole groups of 8 G workgroups are
// remapped, so the map is a bijection for any grid size.
template <unsigned G>
__device__ __forceinline__ size_t xcd_chunk_index(unsigned b, unsigned nblocks)
{
    if constexpr (G > 1) {
        constexpr unsigned group = 8u * G;
        const unsigned full = nblocks & ~(group - 1u);
        if (b < full) return (b & ~(group - 1u)) + (b & 7u) * G + ((b >> 3) & (G - 1u));
    }
    (void)nblocks;
    return b;
}

// Group tables (per-tensor rates, scales, divergences): G consecutive segments of the range,
// segment s ending at element 64 * end64[s], ends ascending.  One rule in every kernel: a
// 64-element block b belongs to the first segment whose end lies beyond it, and to the last
// segment if there is none (a last end short of n stretches to n; ends beyond n mean n).
// group_find bisects (uniform when b is); group_walk moves on from a segment at or before
// the right one, for lanes whose block lies a little further on.
__device__ __forceinline__ int group_find(const uint32_t *end64, int G, uint32_t b)
{
    int lo = 0, hi = G - 1;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (end64[mid] > b) hi = mid;
        else lo = mid + 1;
    }
    return lo;
}
__device__ __forceinline__ int group_walk(const uint32_t *end64, int G, int s, uint32_t b)
{
    while (s < G - 1 && b >= end64[s]) ++s;
    return s;
}
// group_find for a whole wave without a chain of dependent loads: for ascending ends the
// segment of block b is the number of ends (the last one aside, which counts as infinite) at
// or before b.  The 64 lanes hold up to kGroupEndsPerLane ends each -- lane l the ends
// l, l + 64, ... -- requested in one go (GroupEnds::load, which a kernel places ahead of its
// bulk loads so that the table arrives first); GroupEnds::count then needs only lane masks.
// Every lane must be active in both.  A table that does not ascend still gives an index in
// [0, G - 1].
constexpr int kGroupEndsPerLane = 16;
constexpr int kGroupCountMax = 64 * kGroupEndsPerLane;
struct GroupEnds {
    uint32_t v[kGroupEndsPerLane];
    __device__ __forceinline__ void load(const uint32_t *end64, int G, int lane)
    {
#pragma unroll
        for (int k = 0; k < kGroupEndsPerLane; ++k) {
            const int idx = lane + 64 * k;
            v[k] = 0xFFFFFFFFu;  // beyond every block
            if (64 * k < G - 1 && idx < G - 1) v[k] = end64[idx];
        }
    }
    __device__ __forceinline__ int count(int G, uint32_t b) const
    {
        int s = 0;
#pragma unroll
        for (int k = 0; k < kGroupEndsPerLane; ++k)
            if (64 * k < G - 1) s += __builtin_popcountll(__ballot(v[k] <= b));
        return s;
    }
};
// the blocks [lo, hi) of segment s under the same rule (n64 = blocks in the range)
__device__ __forceinline__ uint32_t group_lo64(const uint32_t *end64, int s, uint32_t n64)
{
    if (s == 0) return 0u;
    const uint32_t v = end64[s - 1];
    return v < n64 ? v : n64;
}
__device__ __forceinline__ uint32_t group_hi64(const uint32_t *end64, int G, int s, uint32_t n64)
{
    const uint32_t v = s == G - 1 ? n64 : end64[s];
    const uint32_t hi = v < n64 ? v : n64, lo = group_lo64(end64, s, n64);
    return hi > lo ? hi : lo;
}

// Algorithm 1 line 6 in fp32: one rounded product, one fused multiply-add.
__device__ __forceinline__ float momentum_step(float m, float g, float beta2, float omb2)
{
    return __builtin_fmaf(beta2, m, omb2 * g);
}

}  // namespace lc
