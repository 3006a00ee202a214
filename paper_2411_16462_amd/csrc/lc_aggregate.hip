// W-way aggregation (majority vote over packed bits, or p-bit sum then sign) and the
// apply step (Algorithm 1 lines 4-6; Section 3; Appendix A.1, B.1 and F.1).
//
// Four kernels, chosen by launch_aggregate() at the end of this file:
//   aggregate_kernel    the general one, described next: any input kind, any W, optional
//                       planes / counts out, optional momentum streams;
//   vote_only_kernel    1-bit rows in, planes out, nothing applied;
//   apply_only_kernel   planes in, theta (and momentum rows) updated;
//   tile_apply_kernel   aggregate + apply for few workers without momentum streams.
// The last three are the general kernel's special cases with a wave shape that suits them
// better; their results are the same bits.
//
// General kernel.
// Every wave works alone on 1024 consecutive elements (16 packed words, four 256-element
// tiles; 512 elements for 32 and more 1-bit rows) and is short-lived: on MI355X many small independent waves stream
// faster than few long ones.  Three phases:
//
//  A  count   1-bit rows: lane = 16 * phase + j.  Lane (phase, j) loads word j of rows
//             phase, phase + 4, phase + 8, ... (one load instruction fetches 128
//             contiguous bytes from each of 4 rows) and counts them bit-sliced:
//             carry-save adders fold 8 words at a time into planes c[0..7]
//             (c[k] bit i = bit k of the count for element i).  Two butterfly steps
//             over the lane pairs 16 and 32 apart add the four partial counts, also
//             bit-sliced.  K is compared with W/2 plane by plane, giving the `pos`
//             (S > 0) and `nz` (S != 0) words directly.
//             Field rows: a lane owns 16 consecutive fields of every row (4, 8 or 16
//             bytes) and adds the rows as 32-bit integers -- no carry crosses a field
//             because K <= W <= 2^p - 1 -- then compares field by field.
//  B  stage   pos / nz (and, if the counts K are wanted from 1-bit rows, the count
//             planes) go to the wave's slice of LDS in the canonical 1-bit layout;
//             the planes are also stored to global memory if the caller asked.
//  C  apply   Lanes own elements: in tile t lane l holds elements 256 t + 4 l .. + 3
//             (16-byte accesses of theta, m, g) and fetches its 4 pos / nz bits from
//             LDS.  This is the only place where the word-per-lane and the
//             element-per-lane layouts meet, and the only use of LDS.  The loads of
//             theta are issued before phase A so that they overlap the counting.
#include "lc_launch.hpp"

namespace lc {

#ifndef LC_AGG_THREADS
#define LC_AGG_THREADS 128
#endif
// Unused dynamic LDS per workgroup: a tuning knob that caps how many workgroups share a
// compute unit (160 KiB of LDS each); 0 leaves occupancy to the register count.  Kernels
// whose waves are short (one tile: a load or two, a store) want every wave slot filled;
// kernels whose waves walk many rows stream faster with FEWER waves per compute unit, each
// of which keeps many loads in flight (measured on the W = 64 vote: 32 waves per unit
// 5.35 TB/s, 12 waves 5.47, 8 waves 5.6, 4 waves 5.0).
#ifndef LC_AGG_LDS
#define LC_AGG_LDS 32768  // general kernel on 32 and more 1-bit rows with 16 words per wave: 10 waves per compute unit (+1.5 %)
#endif
#ifndef LC_AGG_BATCH16
#define LC_AGG_BATCH16 1  // 1-bit rows of the general kernel: sixteen loads in flight per lane instead of eight (+1.5 % at W = 64)
#endif
#ifndef LC_VOTE_LDS
#define LC_VOTE_LDS 65536  // two 256-thread workgroups = 8 waves per compute unit
#endif
#ifndef LC_APPLY_LDS
#define LC_APPLY_LDS 0
#endif
#ifndef LC_TILE_LDS
#define LC_TILE_LDS 0
#endif
#ifndef LC_AGG_XCD
#define LC_AGG_XCD 2  // consecutive workgroups per XCD (measured: +3..5 % on the W = 64 and p = 4 workloads)
#endif
constexpr int kAggThreads = LC_AGG_THREADS;   // workgroup size; waves are independent
constexpr int kWaves = kAggThreads / kWave;
#ifndef LC_AGG_WORDS
#define LC_AGG_WORDS 16
#endif
constexpr int kAggWordsDefault = LC_AGG_WORDS;  // packed words per wave
#ifndef LC_AGG_WORDS_MANY
#define LC_AGG_WORDS_MANY 8
#endif
constexpr int kAggWordsMany = LC_AGG_WORDS_MANY;  // ... for 32 and more 1-bit rows
constexpr int kAggManyRows = 32;

enum { IN_PLANES = 0, IN_BITS = 1 /* 2, 4, 8: field width */, IN_TERNARY = 16 /* pos + nz rows */ };

// a + b + c = 2 h + l, bitwise in every position
__device__ __forceinline__ void csa(uint64_t &h, uint64_t &l, uint64_t a, uint64_t b, uint64_t c)
{
    const uint64_t u = a ^ b;
    h = (a & b) | (u & c);
    l = u ^ c;
}

// add one word of weight 2^from into the planes
__device__ __forceinline__ void ripple(uint64_t (&c)[8], uint64_t x, int from)
{
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        if (k < from) continue;
        const uint64_t t = c[k] & x;
        c[k] ^= x;
        x = t;
    }
}

// eight more words into the planes: seven carry-save adders and one ripple from plane 3
__device__ __forceinline__ void csa8(uint64_t (&c)[8], const uint64_t (&x)[8])
{
    uint64_t ta, tb, fa, fb, e;
    csa(ta, c[0], c[0], x[0], x[1]);
    csa(tb, c[0], c[0], x[2], x[3]);
    csa(fa, c[1], c[1], ta, tb);
    csa(ta, c[0], c[0], x[4], x[5]);
    csa(tb, c[0], c[0], x[6], x[7]);
    csa(fb, c[1], c[1], ta, tb);
    csa(e, c[2], c[2], fa, fb);
    ripple(c, e, 3);
}

// A > B and A == B for two bit-sliced counts, scanning from the top plane down.
__device__ __forceinline__ void compare_two(const uint64_t (&a)[8], const uint64_t (&b)[8], uint64_t &gt, uint64_t &eq)
{
    gt = 0;
    eq = ~0ull;
#pragma unroll
    for (int k = 7; k >= 0; --k) {
        const uint64_t d = a[k] ^ b[k];
        gt |= eq & d & a[k];
        eq &= ~d;
    }
}

// K > T and K == T for the bit-sliced count, scanning from the top plane down.
__device__ __forceinline__ void compare_planes(const uint64_t (&c)[8], int T, uint64_t &gt, uint64_t &eq)
{
    gt = 0;
    eq = ~0ull;
#pragma unroll
    for (int k = 7; k >= 0; --k) {
        if ((T >> k) & 1) {
            eq &= c[k];
        } else {
            gt |= eq & c[k];
            eq &= ~c[k];
        }
    }
}

// From "K > T" and "K == T" to the two vote planes.  K == T is a tie only if the
// caller says so (for an odd number of 0/1 votes K == floor(W/2) means S = -1).
__device__ __forceinline__ void vote_planes(uint64_t gt, uint64_t eq, bool tie_possible, int tie, uint64_t &pos, uint64_t &nz)
{
    pos = gt;
    nz = ~0ull;
    if (tie_possible) {
        if (tie < 0) nz = ~eq;
        else if (tie > 0) pos |= eq;
    }
}

__device__ __forceinline__ uint64_t valid_mask(size_t first, size_t n)
{
    if (first >= n) return 0;
    const size_t left = n - first;
    return left >= 64 ? ~0ull : ((1ull << left) - 1ull);
}

// 4 bits -> 4 bytes holding 0/1
__device__ __forceinline__ uint32_t spread4(uint32_t nib)
{
    return (nib & 1u) | ((nib & 2u) << 7) | ((nib & 4u) << 14) | ((nib & 8u) << 21);
}


// LDS traffic of one wave is ordered by the hardware; this keeps the compiler from
// moving the reads above the writes and waits for the writes to land.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

__device__ __forceinline__ uint64_t lane_xor64(uint64_t v, int lane, int mask)
{
    const int addr = (lane ^ mask) << 2;
    const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(addr, static_cast<int>(static_cast<uint32_t>(v))));
    const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(addr, static_cast<int>(static_cast<uint32_t>(v >> 32))));
    return (static_cast<uint64_t>(hi) << 32) | lo;
}

// c += the planes of the lane `mask` away (bit-sliced ripple-carry add); np planes hold the total
__device__ __forceinline__ void add_partner(uint64_t (&c)[8], int lane, int mask, int np)
{
    uint64_t carry = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        if (k >= np) break;
        const uint64_t o = lane_xor64(c[k], lane, mask);
        const uint64_t t = c[k] ^ o;
        const uint64_t cy = (c[k] & o) | (t & carry);
        c[k] = t ^ carry;
        carry = cy;
    }
}

template <int NWD>
__device__ __forceinline__ void load_words(const char *p, uint32_t (&x)[NWD])
{
    if constexpr (NWD == 1) {
        x[0] = ld_packed(reinterpret_cast<const uint32_t *>(p));
    } else if constexpr (NWD == 2) {
        const u32x2 v = ld_packed(reinterpret_cast<const u32x2 *>(p));
        x[0] = v.x;
        x[1] = v.y;
    } else {
#pragma unroll
        for (int h = 0; h < NWD / 4; ++h) {
            const u32x4 v = ld_packed(reinterpret_cast<const u32x4 *>(p) + h);
            x[4 * h + 0] = v.x;
            x[4 * h + 1] = v.y;
            x[4 * h + 2] = v.z;
            x[4 * h + 3] = v.w;
        }
    }
}

template <int NWD>
__device__ __forceinline__ void store_words(char *p, const uint32_t (&x)[NWD])
{
    if constexpr (NWD == 1) {
        st_stream(reinterpret_cast<uint32_t *>(p), x[0]);
    } else if constexpr (NWD == 2) {
        u32x2 v = {x[0], x[1]};
        st_stream(reinterpret_cast<u32x2 *>(p), v);
    } else {
#pragma unroll
        for (int h = 0; h < NWD / 4; ++h) {
            u32x4 v = {x[4 * h + 0], x[4 * h + 1], x[4 * h + 2], x[4 * h + 3]};
            st_stream(reinterpret_cast<u32x4 *>(p) + h, v);
        }
    }
}

template <int IN, int GDT, bool APPLY, bool MOM, bool KOUT, int WORDS>
__global__ __launch_bounds__(kAggThreads) void aggregate_kernel(const AggParams P)
{
    // WORDS packed words per wave: 16 (1024 elements, four tiles) in general, 8 for 32 and more
    // 1-bit rows, where shorter waves with the same loads in flight per lane stream faster
    constexpr int kAggWords = WORDS;
    constexpr int kAggWave = kAggWords * 64;    // elements per wave
    constexpr int kAggTiles = kAggWave / 256;
    constexpr int kPhases = kWave / kAggWords;  // lanes that share a word in phase A
    __shared__ uint64_t s_pos[kWaves][kAggWords];
    __shared__ uint64_t s_nz[kWaves][kAggWords];
    __shared__ uint64_t s_cnt[KOUT ? kWaves : 1][KOUT ? 8 : 1][KOUT ? kAggWords : 1];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_index();
    const size_t n = P.n;
    const size_t wave_base = (xcd_chunk_index<LC_AGG_XCD>(blockIdx.x, gridDim.x) * kWaves + wave) * kAggWave;
    if (wave_base >= n) return;
    const bool full_wave = wave_base + kAggWave <= n;
    const int W = P.W;
    const int T = P.thresh;  // the count at which the sum of signs (or of levels) is zero

    // theta first: these loads overlap all of phase A
    f32x4 th[kAggTiles];
    if (APPLY && full_wave) {
#pragma unroll
        for (int t = 0; t < kAggTiles; ++t) th[t] = load4(P.theta + wave_base + t * 256 + lane * 4);
    }

    // ... and so do the loads of the first momentum / gradient stream
    f32x4 mv0[MOM ? kAggTiles : 1], gv0[MOM ? kAggTiles : 1];
    if (MOM && full_wave) {
#pragma unroll
        for (int t = 0; t < kAggTiles; ++t) {
            const size_t e = wave_base + t * 256 + lane * 4;
            mv0[MOM ? t : 0] = load4(P.m + e);
            gv0[MOM ? t : 0] = Grad<GDT>::load4(P.g, e);
        }
    }

    // ---------------------------------------------------------------- phase A + B
    if constexpr (IN == IN_PLANES) {
        if (lane < 2 * kAggWords) {
            const int j = lane & (kAggWords - 1);
            const size_t jw = wave_base / 64 + j;
            const uint64_t vm = valid_mask(jw * 64, n);
            uint64_t v = 0;
            if (lane < kAggWords) {
                if (vm) v = ld_packed(P.in_pos + jw);
                s_pos[wave][j] = v & vm;
            } else {
                if (vm) v = P.in_nz ? ld_packed(P.in_nz + jw) : ~0ull;
                s_nz[wave][j] = v & vm;
            }
        }
    } else if constexpr (IN == IN_BITS) {
        const int j = lane & (kAggWords - 1);
        const int ph = lane / kAggWords;
        const size_t jw = wave_base / 64 + j;
        const uint64_t vm = valid_mask(jw * 64, n);
        const size_t stride = P.q_stride_bytes / 8;
        const uint64_t *qp = static_cast<const uint64_t *>(P.q) + jw + static_cast<size_t>(ph) * stride;
        const size_t step4 = stride * kPhases;
        const int np = 32 - __builtin_clz(static_cast<unsigned>(W));  // planes that hold a count up to W
        uint64_t c[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        const int most = (W + kPhases - 1) / kPhases;  // rows of phase 0; later phases may have one fewer
        // sixteen rows at a time (two sets of eight), their loads in flight together; a row
        // that does not exist counts as zero
        int k = 0;
#if LC_AGG_BATCH16
        for (; k + 8 < most; k += 16) {
            uint64_t x[8], y[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const bool have = vm && (ph + (k + i) * kPhases < W);
                x[i] = have ? ld_packed(qp + static_cast<size_t>(k + i) * step4) : 0ull;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const bool have = vm && (ph + (k + 8 + i) * kPhases < W);
                y[i] = have ? ld_packed(qp + static_cast<size_t>(k + 8 + i) * step4) : 0ull;
            }
            csa8(c, x);
            csa8(c, y);
        }
#endif
        for (; k < most; k += 8) {
            uint64_t x[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const bool have = vm && (ph + (k + i) * kPhases < W);
                x[i] = have ? ld_packed(qp + static_cast<size_t>(k + i) * step4) : 0ull;
            }
            csa8(c, x);
        }
#pragma unroll
        for (int mask = kAggWords; mask < kWave; mask <<= 1) add_partner(c, lane, mask, np);
        uint64_t gt, eq, pos, nz;
        compare_planes(c, T, gt, eq);
        vote_planes(gt, eq, P.tie_possible != 0, P.tie, pos, nz);
        pos &= vm;
        nz &= vm;
        if (ph == 0) {
            s_pos[wave][j] = pos;
            s_nz[wave][j] = nz;
            if (KOUT) {
#pragma unroll
                for (int i = 0; i < 8; ++i) s_cnt[KOUT ? wave : 0][KOUT ? i : 0][KOUT ? j : 0] = c[i] & vm;
                if (P.sum_bits == 1 && vm) static_cast<uint64_t *>(P.sum_out)[jw] = c[0] & vm;  // W = 1: K is the bit
            }
            if (vm) {
                if (P.vote_pos) P.vote_pos[jw] = pos;
                if (P.vote_nz) P.vote_nz[jw] = nz;
            }
        }
    } else if constexpr (IN == IN_TERNARY) {
        // Every worker sends two planes, pos (s > 0) and nz (s != 0): count the +1 votes and
        // the -1 votes separately, the update is the sign of their difference.
        const int j = lane & (kAggWords - 1);
        const int ph = lane / kAggWords;
        const size_t jw = wave_base / 64 + j;
        const uint64_t vm = valid_mask(jw * 64, n);
        const size_t stride = P.q_stride_bytes / 8;
        const uint64_t *pp = static_cast<const uint64_t *>(P.q) + jw + static_cast<size_t>(ph) * stride;
        const uint64_t *zp = static_cast<const uint64_t *>(P.q2) + jw + static_cast<size_t>(ph) * stride;
        const size_t step4 = stride * kPhases;
        const int np = 32 - __builtin_clz(static_cast<unsigned>(W));
        uint64_t cp[8] = {0, 0, 0, 0, 0, 0, 0, 0}, cn[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        const int every = W / kPhases;
        const int most = (W + kPhases - 1) / kPhases;
        int k = 0;
        for (; k + 8 <= every; k += 8) {
            uint64_t xp[8], xn[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint64_t a = vm ? ld_packed(pp + static_cast<size_t>(k + i) * step4) : 0ull;
                const uint64_t z = vm ? ld_packed(zp + static_cast<size_t>(k + i) * step4) : 0ull;
                xp[i] = a & z;
                xn[i] = z & ~a;
            }
            csa8(cp, xp);
            csa8(cn, xn);
        }
        for (; k < most; ++k) {
            const bool have = vm && (ph + k * kPhases < W);
            const uint64_t a = have ? ld_packed(pp + static_cast<size_t>(k) * step4) : 0ull;
            const uint64_t z = have ? ld_packed(zp + static_cast<size_t>(k) * step4) : 0ull;
            ripple(cp, a & z, 0);
            ripple(cn, z & ~a, 0);
        }
#pragma unroll
        for (int mask = kAggWords; mask < kWave; mask <<= 1) {
            add_partner(cp, lane, mask, np);
            add_partner(cn, lane, mask, np);
        }
        uint64_t gt, eq;
        compare_two(cp, cn, gt, eq);
        const uint64_t pos = gt & vm, nz = ~eq & vm;
        if (ph == 0) {
            s_pos[wave][j] = pos;
            s_nz[wave][j] = nz;
            if (vm) {
                if (P.vote_pos) P.vote_pos[jw] = pos;
                if (P.vote_nz) P.vote_nz[jw] = nz;
            }
        }
    } else {
        // field rows: a lane owns kFpl consecutive fields of every row
        constexpr int C = IN;
        constexpr int kFpl = kAggWave / kWave;   // fields per lane
        constexpr int kLaneBytes = kFpl * C / 8;
        constexpr int NWD = kLaneBytes / 4;      // 32-bit words per lane
        static_assert(kLaneBytes >= 4, "a lane needs at least one 32-bit word of fields");
        constexpr uint32_t fmask = (1u << C) - 1u;
        const size_t valid_bytes = (n * C + 7) / 8;
        const size_t e0 = wave_base + static_cast<size_t>(lane) * kFpl;
        const size_t off = e0 / 8 * C;  // e0 is a multiple of 16
        const char *qb = static_cast<const char *>(P.q) + off;
        uint32_t acc[NWD];
#pragma unroll
        for (int i = 0; i < NWD; ++i) acc[i] = 0;
        if (off + kLaneBytes <= valid_bytes) {
            int w = 0;
            for (; w + 4 <= W; w += 4) {
                uint32_t x[4][NWD];
#pragma unroll
                for (int k = 0; k < 4; ++k) load_words<NWD>(qb + static_cast<size_t>(w + k) * P.q_stride_bytes, x[k]);
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int i = 0; i < NWD; ++i) acc[i] += x[k][i];
            }
            for (; w < W; ++w) {
                uint32_t x[NWD];
                load_words<NWD>(qb + static_cast<size_t>(w) * P.q_stride_bytes, x);
#pragma unroll
                for (int i = 0; i < NWD; ++i) acc[i] += x[i];
            }
            if (P.sum_out) store_words<NWD>(static_cast<char *>(P.sum_out) + off, acc);
        } else if (off < valid_bytes) {
            // the lane that holds the end of the row: byte by byte, pad fields dropped
            const int nb = static_cast<int>(valid_bytes - off);
            for (int w = 0; w < W; ++w) {
                const uint8_t *src = reinterpret_cast<const uint8_t *>(qb + static_cast<size_t>(w) * P.q_stride_bytes);
#pragma unroll
                for (int b = 0; b < kLaneBytes; ++b)
                    if (b < nb) acc[b >> 2] += static_cast<uint32_t>(src[b]) << (8 * (b & 3));
            }
#pragma unroll
            for (int f = 0; f < kFpl; ++f)
                if (e0 + f >= n) acc[(f * C) >> 5] &= ~(fmask << ((f * C) & 31));
            if (P.sum_out) {
                uint8_t *dst = reinterpret_cast<uint8_t *>(static_cast<char *>(P.sum_out) + off);
#pragma unroll
                for (int b = 0; b < kLaneBytes; ++b)
                    if (b < nb) dst[b] = static_cast<uint8_t>(acc[b >> 2] >> (8 * (b & 3)));
            }
        }
        uint64_t gt = 0, eq = 0;
#pragma unroll
        for (int f = 0; f < kFpl; ++f) {
            const uint32_t K = (acc[(f * C) >> 5] >> ((f * C) & 31)) & fmask;
            gt |= static_cast<uint64_t>(K > static_cast<uint32_t>(T)) << f;
            eq |= static_cast<uint64_t>(K == static_cast<uint32_t>(T)) << f;
        }
        uint64_t pos, nz;
        vote_planes(gt, eq, P.tie_possible != 0, P.tie, pos, nz);
        const uint64_t vm = valid_mask(e0, n) & ((1ull << kFpl) - 1ull);
        if constexpr (kFpl == 16) {
            reinterpret_cast<uint16_t *>(s_pos[wave])[lane] = static_cast<uint16_t>(pos & vm);
            reinterpret_cast<uint16_t *>(s_nz[wave])[lane] = static_cast<uint16_t>(nz & vm);
        } else {
            static_assert(kFpl == 32, "16 or 32 fields per lane");
            reinterpret_cast<uint32_t *>(s_pos[wave])[lane] = static_cast<uint32_t>(pos & vm);
            reinterpret_cast<uint32_t *>(s_nz[wave])[lane] = static_cast<uint32_t>(nz & vm);
        }
    }
    wave_lds_sync();

    if (IN != IN_PLANES && IN != IN_BITS && IN != IN_TERNARY && lane < kAggWords) {
        // planes for the caller, from LDS in word order
        const size_t jw = wave_base / 64 + lane;
        if (jw * 64 < n) {
            if (P.vote_pos) P.vote_pos[jw] = s_pos[wave][lane];
            if (P.vote_nz) P.vote_nz[jw] = s_nz[wave][lane];
        }
    }

    // ---------------------------------------------------------------- phase C
    if (!(APPLY || KOUT)) return;
    const uint8_t *pos8 = reinterpret_cast<const uint8_t *>(s_pos[wave]);
    const uint8_t *nz8 = reinterpret_cast<const uint8_t *>(s_nz[wave]);
    const int sh = (lane & 1) * 4;

    // Learning rate and weight decay: one pair for the call, or one per parameter group.
    // Groups are consecutive segments of the range that end at multiples of 64 elements,
    // so the 4 elements of a lane always share a group.  The group of the wave's first
    // element is found by bisection (uniform); lanes whose elements lie further on walk
    // forward from there, which is rare.
    int seg0 = 0;
    if (APPLY && P.n_seg > 0) {
        seg0 = group_find(P.seg_end64, P.n_seg, static_cast<uint32_t>(wave_base / 64));
    }
    auto rates = [&](size_t e, float &lr, float &wd) {
        lr = P.lr;
        wd = P.wd;
        if (P.n_seg > 0) {
            const int sgm = group_walk(P.seg_end64, P.n_seg, seg0, static_cast<uint32_t>(e / 64));
            lr = P.seg_lr[sgm];
            wd = P.seg_wd[sgm];
        }
    };

    if (APPLY && full_wave) {
#pragma unroll
        for (int t = 0; t < kAggTiles; ++t) {
            const int byte = t * 32 + (lane >> 1);
            const uint32_t pn = pos8[byte] >> sh, zn = nz8[byte] >> sh;
            float lr, wd;
            rates(wave_base + t * 256 + lane * 4, lr, wd);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float uf = ((zn >> k) & 1u) ? (((pn >> k) & 1u) ? 1.0f : -1.0f) : 0.0f;
                th[t][k] = __builtin_fmaf(-lr, __builtin_fmaf(wd, th[t][k], uf), th[t][k]);
            }
        }
#pragma unroll
        for (int t = 0; t < kAggTiles; ++t) store4(P.theta + wave_base + t * 256 + lane * 4, th[t]);
        if (MOM) {
#pragma unroll
            for (int t = 0; t < kAggTiles; ++t) {
                f32x4 &mv = mv0[MOM ? t : 0];
                const f32x4 gv = gv0[MOM ? t : 0];
#pragma unroll
                for (int k = 0; k < 4; ++k) mv[k] = momentum_step(mv[k], gv[k], P.beta2, P.omb2);
                store4(P.m + wave_base + t * 256 + lane * 4, mv);
            }
        }
        for (int w = 1; MOM && w < P.n_m; ++w) {
            float *mrow = P.m + static_cast<size_t>(w) * P.m_stride;
            const void *grow = static_cast<const char *>(P.g) + static_cast<size_t>(w) * P.g_stride * Grad<GDT>::kBytes;
            f32x4 mv[kAggTiles], gv[kAggTiles];
#pragma unroll
            for (int t = 0; t < kAggTiles; ++t) {
                const size_t e = wave_base + t * 256 + lane * 4;
                mv[t] = load4(mrow + e);
                gv[t] = Grad<GDT>::load4(grow, e);
            }
#pragma unroll
            for (int t = 0; t < kAggTiles; ++t) {
#pragma unroll
                for (int k = 0; k < 4; ++k) mv[t][k] = momentum_step(mv[t][k], gv[t][k], P.beta2, P.omb2);
                store4(mrow + wave_base + t * 256 + lane * 4, mv[t]);
            }
        }
    } else if (APPLY) {
        // ragged end: element by element
        for (int t = 0; t < kAggTiles; ++t) {
            const size_t e = wave_base + t * 256 + lane * 4;
            if (e >= n) break;
            const int byte = t * 32 + (lane >> 1);
            const uint32_t pn = pos8[byte] >> sh, zn = nz8[byte] >> sh;
            float lr, wd;
            rates(e, lr, wd);
            for (int k = 0; k < 4 && e + k < n; ++k) {
                const float uf = ((zn >> k) & 1u) ? (((pn >> k) & 1u) ? 1.0f : -1.0f) : 0.0f;
                const float v = P.theta[e + k];
                P.theta[e + k] = __builtin_fmaf(-lr, __builtin_fmaf(wd, v, uf), v);
                for (int w = 0; MOM && w < P.n_m; ++w) {
                    float *mrow = P.m + static_cast<size_t>(w) * P.m_stride;
                    const void *grow = static_cast<const char *>(P.g) + static_cast<size_t>(w) * P.g_stride * Grad<GDT>::kBytes;
                    mrow[e + k] = momentum_step(mrow[e + k], Grad<GDT>::load1(grow, e + k), P.beta2, P.omb2);
                }
            }
        }
    }

    if (KOUT && P.sum_bits > 1) {
        // counts K from the bit-sliced planes, as fields of sum_bits bits
        const int C = P.sum_bits;
        uint8_t *out = static_cast<uint8_t *>(P.sum_out);
        for (int t = 0; t < kAggTiles; ++t) {
            const size_t e = wave_base + t * 256 + lane * 4;
            if (e >= n) break;
            const int byte = t * 32 + (lane >> 1);
            uint32_t kb = 0;  // 4 counts, one per byte
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const uint8_t *pl = reinterpret_cast<const uint8_t *>(s_cnt[KOUT ? wave : 0][KOUT ? k : 0]);
                kb |= spread4((pl[byte] >> sh) & 0xFu) << k;
            }
            const int left = (n - e >= 4) ? 4 : static_cast<int>(n - e);
            if (C == 8) {
                if (left == 4) *reinterpret_cast<uint32_t *>(out + e) = kb;
                else for (int k = 0; k < left; ++k) out[e + k] = static_cast<uint8_t>(kb >> (8 * k));
            } else if (C == 4) {
                const uint32_t v = (kb & 0xFu) | ((kb >> 4) & 0xF0u) | ((kb >> 8) & 0xF00u) | ((kb >> 12) & 0xF000u);
                if (left > 2) *reinterpret_cast<uint16_t *>(out + e / 2) = static_cast<uint16_t>(v);
                else out[e / 2] = static_cast<uint8_t>(v);
            } else {
                const uint32_t v = (kb & 0x3u) | ((kb >> 6) & 0xCu) | ((kb >> 12) & 0x30u) | ((kb >> 18) & 0xC0u);
                out[e / 4] = static_cast<uint8_t>(v);
            }
        }
    }
}

// Vote only (planes out, nothing applied): the local reduction of the 1-bit compressed
// allreduce between its all-to-all and its allgather (Section 3).  There is no element-wise
// phase, so the word-per-lane layout is kept throughout: a lane owns one 64-bit word of every
// row (512 contiguous bytes per row and wave instruction).  Rows are fetched eight at a time;
// for W a multiple of 16 two register sets take turns, the next eight rows requested before
// the current eight are counted, so that a wave always has loads in flight.  (Letting a wave
// walk on through 2 .. 8 further columns, with the first rows of the next column requested
// before a column's planes are stored, was slower: 5.1 .. 4.9 against 5.4 TB/s.)
#ifndef LC_VOTE_THREADS
#define LC_VOTE_THREADS 256
#endif
#ifndef LC_VOTE_PIPE
#define LC_VOTE_PIPE 1
#endif
constexpr int kVoteThreads = LC_VOTE_THREADS;

// eight consecutive rows of the lane's word, no guards: straight-line loads (a guard on each
// load makes the compiler wait after every one of them)
__device__ __forceinline__ void vote_load8(uint64_t (&x)[8], const uint64_t *src, size_t stride)
{
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = ld_packed(src + static_cast<size_t>(i) * stride);
}

// PIPE: W is a multiple of 16.  Otherwise eight rows at a time through one register set, rows
// at or beyond W (uniform) skipped.
template <bool PIPE>
__global__ __launch_bounds__(kVoteThreads) void vote_only_kernel(const AggParams P)
{
    const size_t jw = static_cast<size_t>(blockIdx.x) * kVoteThreads + threadIdx.x;
    const size_t n = P.n;
    if (jw * 64 >= n) return;
    const int W = P.W;
    const size_t stride = P.q_stride_bytes / 8;
    const uint64_t *cur = static_cast<const uint64_t *>(P.q) + jw;
    uint64_t c[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if constexpr (PIPE) {
        const size_t half = 8 * stride;
        uint64_t xa[8], xb[8];
        vote_load8(xa, cur, stride);
        for (int w = 16; w < W; w += 16) {  // every group of sixteen rows but the last
            vote_load8(xb, cur + half, stride);
            csa8(c, xa);
            cur += 2 * half;
            vote_load8(xa, cur, stride);
            csa8(c, xb);
        }
        vote_load8(xb, cur + half, stride);
        csa8(c, xa);
        csa8(c, xb);
    } else {
        for (int w = 0; w < W; w += 8) {
            uint64_t x[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = (w + i < W) ? ld_packed(cur + static_cast<size_t>(w + i) * stride) : 0ull;
            csa8(c, x);
        }
    }
    const uint64_t vm = valid_mask(jw * 64, n);
    uint64_t gt, eq, pos, nz;
    compare_planes(c, P.thresh, gt, eq);
    vote_planes(gt, eq, P.tie_possible != 0, P.tie, pos, nz);
    if (P.vote_pos) P.vote_pos[jw] = pos & vm;
    if (P.vote_nz) P.vote_nz[jw] = nz & vm;
}

// The same for the ternary wire format (Appendix B.1): row w is a pair of words, pos and nz;
// pos & nz are the votes for +1, nz & ~pos the votes for -1, counted in two sets of planes
// and compared plane by plane.  K+ == K- is a zero of the vote, whatever W is.
__device__ __forceinline__ void vote_load8_ternary(uint64_t (&plus)[8], uint64_t (&minus)[8], const uint64_t *pos, const uint64_t *nz,
                                                   size_t stride)
{
    uint64_t p[8], z[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        p[i] = ld_packed(pos + static_cast<size_t>(i) * stride);
        z[i] = ld_packed(nz + static_cast<size_t>(i) * stride);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        plus[i] = p[i] & z[i];
        minus[i] = z[i] & ~p[i];
    }
}

template <bool WHOLE8>
__global__ __launch_bounds__(kVoteThreads) void vote_only_ternary_kernel(const AggParams P)
{
    const size_t jw = static_cast<size_t>(blockIdx.x) * kVoteThreads + threadIdx.x;
    const size_t n = P.n;
    if (jw * 64 >= n) return;
    const int W = P.W;
    const size_t stride = P.q_stride_bytes / 8;
    const uint64_t *pcur = static_cast<const uint64_t *>(P.q) + jw;
    const uint64_t *zcur = static_cast<const uint64_t *>(P.q2) + jw;
    uint64_t cp[8] = {0, 0, 0, 0, 0, 0, 0, 0}, cn[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if constexpr (WHOLE8) {  // W is a multiple of 8: sixteen straight-line loads per step
        for (int w = 0; w < W; w += 8) {
            uint64_t plus[8], minus[8];
            vote_load8_ternary(plus, minus, pcur + static_cast<size_t>(w) * stride, zcur + static_cast<size_t>(w) * stride, stride);
            csa8(cp, plus);
            csa8(cn, minus);
        }
    } else {
        for (int w = 0; w < W; w += 8) {
            uint64_t plus[8], minus[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint64_t pw = (w + i < W) ? ld_packed(pcur + static_cast<size_t>(w + i) * stride) : 0ull;
                const uint64_t zw = (w + i < W) ? ld_packed(zcur + static_cast<size_t>(w + i) * stride) : 0ull;
                plus[i] = pw & zw;
                minus[i] = zw & ~pw;
            }
            csa8(cp, plus);
            csa8(cn, minus);
        }
    }
    const uint64_t vm = valid_mask(jw * 64, n);
    uint64_t gt, eq;
    compare_two(cp, cn, gt, eq);
    if (P.vote_pos) P.vote_pos[jw] = gt & vm;
    if (P.vote_nz) P.vote_nz[jw] = ~eq & vm;
}

#ifndef LC_VOTE_TERNARY
#define LC_VOTE_TERNARY 1
#endif
static hipError_t launch_vote_only(const AggParams &P, hipStream_t s)
{
    const size_t nw = (P.n + 63) / 64;
    const unsigned grid = static_cast<unsigned>((nw + kVoteThreads - 1) / kVoteThreads);
    if (LC_VOTE_PIPE && P.W % 16 == 0) return launch(vote_only_kernel<true>, grid, kVoteThreads, LC_VOTE_LDS, s, P);
    return launch(vote_only_kernel<false>, grid, kVoteThreads, LC_VOTE_LDS, s, P);
}

// Apply only (planes in): Algorithm 1 lines 5 and 6 after the allgather of the vote.  Nothing
// is counted, so the element-per-lane layout is kept throughout and a wave is as short as in
// the update+pack kernel: one 256-element tile of one row.  grid.y = row: row 0 also moves
// theta, every row below n_m updates its momentum.  Lane l takes its four sign bits from
// byte l / 2 of the tile's 32 plane bytes.  Four consecutive tiles (one 128-byte line of
// each plane) share an XCD.
#ifndef LC_APPLY_ONLY
#define LC_APPLY_ONLY 1  // 0: planes-in applies go through the general kernel
#endif
constexpr int kApplyThreads = 64;

// u of the lane's elements e .. e + left - 1.  IN = 0: from the two planes (byte e / 8 of each,
// the lane's nibble).  IN = 2, 4, 8: from one buffer of counts in IN-bit fields (what a summing
// allreduce leaves), u = sign of K against the threshold.
template <int IN>
__device__ __forceinline__ void apply_signs(const AggParams &P, size_t e, int left, int lane, float (&uf)[4])
{
    if constexpr (IN == 0) {
        const uint8_t *pos8 = reinterpret_cast<const uint8_t *>(P.in_pos);
        const uint8_t *nz8 = reinterpret_cast<const uint8_t *>(P.in_nz);
        const uint32_t sh = (lane & 1) * 4;
        const uint32_t pn = static_cast<uint32_t>(pos8[e / 8]) >> sh;
        const uint32_t zn = nz8 ? static_cast<uint32_t>(nz8[e / 8]) >> sh : 0xFu;
#pragma unroll
        for (int k = 0; k < 4; ++k) uf[k] = ((zn >> k) & 1u) ? (((pn >> k) & 1u) ? 1.0f : -1.0f) : 0.0f;
    } else {
        const uint8_t *src = static_cast<const uint8_t *>(P.q) + e * IN / 8;
        uint32_t x = 0;
        if (left == 4) {
            if (IN == 8) x = *reinterpret_cast<const uint32_t *>(src);
            else if (IN == 4) x = *reinterpret_cast<const uint16_t *>(src);
            else x = *src;
        } else {
            for (int b = 0; b < (left * IN + 7) / 8; ++b) x |= static_cast<uint32_t>(src[b]) << (8 * b);
        }
        const float tie_u = !P.tie_possible ? -1.0f : (P.tie < 0 ? 0.0f : (P.tie > 0 ? 1.0f : -1.0f));
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int K = static_cast<int>((x >> (IN * k)) & ((1u << IN) - 1u));
            uf[k] = K > P.thresh ? 1.0f : (K == P.thresh ? tie_u : -1.0f);
        }
    }
}

template <int GDT, bool MOM, int IN>
__global__ __launch_bounds__(kApplyThreads) void apply_only_kernel(const AggParams P)
{
    const int lane = threadIdx.x;
    const size_t n = P.n;
    const size_t tile = xcd_chunk_index<4>(blockIdx.x, gridDim.x) * 256;
    if (tile >= n) return;
    const size_t e = tile + static_cast<size_t>(lane) * 4;
    const size_t r = blockIdx.y;
    float *mrow = MOM ? P.m + r * P.m_stride : nullptr;
    const void *grow = MOM ? static_cast<const char *>(P.g) + r * P.g_stride * Grad<GDT>::kBytes : nullptr;

    if (tile + 256 <= n) {
        f32x4 th = {0.0f, 0.0f, 0.0f, 0.0f}, mv = th, gv = th;
        if (r == 0) th = load4(P.theta + e);
        if (MOM) {
            mv = load4(mrow + e);
            gv = Grad<GDT>::load4(grow, e);
        }
        if (r == 0) {
            float uf[4];
            apply_signs<IN>(P, e, 4, lane, uf);
#pragma unroll
            for (int k = 0; k < 4; ++k) th[k] = __builtin_fmaf(-P.lr, __builtin_fmaf(P.wd, th[k], uf[k]), th[k]);
            store4(P.theta + e, th);
        }
        if (MOM) {
#pragma unroll
            for (int k = 0; k < 4; ++k) mv[k] = momentum_step(mv[k], gv[k], P.beta2, P.omb2);
            store4(mrow + e, mv);
        }
        return;
    }
    if (e >= n) return;
    const int left = n - e >= 4 ? 4 : static_cast<int>(n - e);
    float uf[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (r == 0) apply_signs<IN>(P, e, left, lane, uf);
    for (int k = 0; k < left; ++k) {
        if (r == 0) {
            const float v = P.theta[e + k];
            P.theta[e + k] = __builtin_fmaf(-P.lr, __builtin_fmaf(P.wd, v, uf[k]), v);
        }
        if (MOM) mrow[e + k] = momentum_step(mrow[e + k], Grad<GDT>::load1(grow, e + k), P.beta2, P.omb2);
    }
}

template <int IN>
static hipError_t launch_apply_only(const AggParams &P, int g_dtype, hipStream_t s)
{
    const dim3 grid(static_cast<unsigned>((P.n + 255) / 256), static_cast<unsigned>(P.n_m > 0 ? P.n_m : 1));
    if (P.n_m == 0) return launch(apply_only_kernel<LC_F32, false, IN>, grid, kApplyThreads, LC_APPLY_LDS, s, P);
    if (g_dtype == LC_BF16) return launch(apply_only_kernel<LC_BF16, true, IN>, grid, kApplyThreads, LC_APPLY_LDS, s, P);
    return launch(apply_only_kernel<LC_F32, true, IN>, grid, kApplyThreads, LC_APPLY_LDS, s, P);
}

// Aggregate + apply for few workers, one 256-element tile per wave (no momentum streams).
// With W small the packed rows are a small part of the traffic (W/8 .. W bytes per element
// against 8 for theta), so the kernel takes the shape that streams theta fastest -- the
// update+pack kernel's: lane l owns elements 4l..4l+3, a wave lives for one tile -- and each
// lane counts its own four elements in four byte-wide counters of one register:
//   1-bit rows   one byte load per row and lane (lanes 2k, 2k+1 share it), the lane's nibble
//                spread to bit 0 of each counter byte (multiply by 2^0 + 2^7 + 2^14 + 2^21);
//   ternary      the same for pos & nz and for nz & ~pos;
//   field rows   the lane's 1 / 2 / 4 bytes of fields are added as integers (no carry
//                crosses a field), then spread to bytes.
// One byte load and about four vector instructions per row and lane: measured with cold
// caches on 124 M elements this beats the bit-sliced kernel above up to about 24 row loads
// per lane (W = 8: 0.195 against 0.212 ms, W = 16: 0.243 against 0.259, W = 24: 0.282 against
// 0.283, W = 32: 0.328 against 0.309), so that kernel takes over beyond 24.
#ifndef LC_TILE_THREADS
#define LC_TILE_THREADS 128
#endif
constexpr int kTileThreads = LC_TILE_THREADS;  // waves of a workgroup are independent: one tile each
#ifndef LC_TILE_BATCH
#define LC_TILE_BATCH 8
#endif
constexpr int kTileBatch = LC_TILE_BATCH;  // row loads in flight per lane
#ifndef LC_TILE_MAX_W_BITS
#define LC_TILE_MAX_W_BITS 24  // most row loads per lane (W for 1-bit rows, 2 W for ternary) served by the tile kernel; 0 disables it
#endif
#ifndef LC_TILE_FIELDS
#define LC_TILE_FIELDS 1       // field rows through the tile kernel
#endif
#ifndef LC_TILE_NT_FIELDS
#define LC_TILE_NT_FIELDS 1    // non-temporal loads of 4- and 8-bit field rows
#endif

__device__ __forceinline__ uint32_t nibble_to_bytes(uint32_t nib) { return (nib * 0x00204081u) & 0x01010101u; }

#ifndef LC_TILE_PER_WAVE
#define LC_TILE_PER_WAVE 2  // measured: 2 is 1..3 % faster than 1, 4 is slower
#endif
template <int IN, bool KOUT, bool GROUPED>
__device__ __forceinline__ void tile_apply_one(const AggParams &P, size_t tile, int lane);

// Tiles per wave: two without a group table; one with it, because the group search of a
// second tile would wait for the first tile to finish (measured on the 1-bit vote of the
// GPT-2-small shapes: 0.240 against 0.179 ms).
#ifndef LC_TILE_PER_WAVE_GROUPED
#define LC_TILE_PER_WAVE_GROUPED 1
#endif
template <bool GROUPED>
constexpr int kTilesPerWave = GROUPED ? LC_TILE_PER_WAVE_GROUPED : LC_TILE_PER_WAVE;

template <int IN, bool KOUT, bool GROUPED>
__global__ __launch_bounds__(kTileThreads) void tile_apply_kernel(const AggParams P)
{
    constexpr int kTileWaves = kTileThreads / kWave;
    constexpr int T = kTilesPerWave<GROUPED>;
    constexpr unsigned kShare = 4 / kTileWaves / T > 0 ? 4 / kTileWaves / T : 1;  // workgroups per XCD that share a line of 1-bit rows
    const int lane = threadIdx.x & (kWave - 1);
    const size_t first = (xcd_chunk_index<kShare>(blockIdx.x, gridDim.x) * kTileWaves + wave_index()) * T;
#pragma unroll
    for (int t = 0; t < T; ++t) tile_apply_one<IN, KOUT, GROUPED>(P, (first + t) * 256, lane);
}

template <int IN, bool KOUT, bool GROUPED>
__device__ __forceinline__ void tile_apply_one(const AggParams &P, size_t tile, int lane)
{
    const size_t n = P.n;
    if (tile >= n) return;
    const size_t e = tile + static_cast<size_t>(lane) * 4;
    if (e >= n) return;
    const int left = n - e >= 4 ? 4 : static_cast<int>(n - e);
    const bool full = left == 4;
    const int W = P.W;
    const size_t stride = P.q_stride_bytes;
    const uint8_t *q8 = static_cast<const uint8_t *>(P.q);
    const uint8_t *z8 = static_cast<const uint8_t *>(P.q2);
    const uint32_t sh = (lane & 1) * 4;

    f32x4 th = {0.0f, 0.0f, 0.0f, 0.0f};
    if (full) th = load4(P.theta + e);
    else for (int k = 0; k < left; ++k) th[k] = P.theta[e + k];

    // Rates of the lane's group.  Placed here, between the issue of the theta loads and the
    // row loads, so that the search (a chain of dependent scalar loads) runs while those
    // are in flight; after the counting it would wait for them first.
    float lr = P.lr, wd = P.wd;
    if (GROUPED) {
        // first group that ends beyond the tile's first 64-element block (uniform), then
        // each lane walks on to the group of its own block
        const int first = group_find(P.seg_end64, P.n_seg, static_cast<uint32_t>(tile / 64));
        const int sgm = group_walk(P.seg_end64, P.n_seg, first, static_cast<uint32_t>(e / 64));
        lr = P.seg_lr[sgm];
        wd = P.seg_wd[sgm];
    }
    // counts: byte k of kp = K (or K+) of element e + k, byte k of kn = K- (ternary only)
    uint32_t kp = 0, kn = 0;
    if constexpr (IN == IN_BITS || IN == IN_TERNARY) {
        // every byte that holds a bit of an element below n lies inside the row
        const size_t off = e / 8;
        // kTileBatch rows at a time, all loads of a batch in flight together; a row index
        // at or beyond W (uniform) loads nothing and counts as zero
        for (int w = 0; w < W; w += kTileBatch) {
            uint32_t x[kTileBatch], z[kTileBatch];
#pragma unroll
            for (int i = 0; i < kTileBatch; ++i) {
                x[i] = 0;
                z[i] = 0;
                if (w + i < W) {
                    x[i] = q8[static_cast<size_t>(w + i) * stride + off];
                    if (IN == IN_TERNARY) z[i] = z8[static_cast<size_t>(w + i) * stride + off];
                }
            }
#pragma unroll
            for (int i = 0; i < kTileBatch; ++i) {
                if (IN == IN_TERNARY) {
                    kp += nibble_to_bytes(((x[i] & z[i]) >> sh) & 0xFu);
                    kn += nibble_to_bytes(((z[i] & ~x[i]) >> sh) & 0xFu);
                } else {
                    kp += nibble_to_bytes((x[i] >> sh) & 0xFu);
                }
            }
        }
    } else {
        // IN-bit fields: the lane's four fields are IN / 2 bytes at byte e * IN / 8; in a
        // ragged lane only the bytes that hold elements below n are read
        const size_t off = e * IN / 8;
        const int bytes = full ? IN / 2 : (left * IN + 7) / 8;
        uint32_t acc = 0;
        if (full) {
            for (int w = 0; w < W; w += kTileBatch) {
                uint32_t x[kTileBatch];
#pragma unroll
                for (int i = 0; i < kTileBatch; ++i) {
                    x[i] = 0;
                    if (w + i < W) {
                        const uint8_t *src = q8 + static_cast<size_t>(w + i) * stride + off;
                        // 4- and 8-bit field rows: every line belongs to one wave, and the
                        // non-temporal hint is worth +14 % here (1-bit rows, whose lines are
                        // shared by four tiles, lose 11 % with it and keep plain loads)
                        if (IN == 8) x[i] = LC_TILE_NT_FIELDS ? __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(src)) : *reinterpret_cast<const uint32_t *>(src);
                        else if (IN == 4) x[i] = LC_TILE_NT_FIELDS ? __builtin_nontemporal_load(reinterpret_cast<const uint16_t *>(src)) : *reinterpret_cast<const uint16_t *>(src);
                        else x[i] = *src;
                    }
                }
#pragma unroll
                for (int i = 0; i < kTileBatch; ++i) acc += x[i];
            }
        } else {
            for (int w = 0; w < W; ++w) {
                const uint8_t *src = q8 + static_cast<size_t>(w) * stride + off;
                uint32_t x = 0;
                for (int b = 0; b < bytes; ++b) x |= static_cast<uint32_t>(src[b]) << (8 * b);
                acc += x;
            }
        }
        if (!full) acc &= (1u << (left * IN)) - 1u;  // fields of elements at and beyond n do not count
        if (IN == 8) kp = acc;
        else if (IN == 4) kp = (acc & 0xFu) | ((acc & 0xF0u) << 4) | ((acc & 0xF00u) << 8) | ((acc & 0xF000u) << 12);
        else kp = (acc & 0x3u) | ((acc & 0xCu) << 6) | ((acc & 0x30u) << 12) | ((acc & 0xC0u) << 18);
        if (P.sum_out) {  // the summed fields, in the rows' own format
            uint8_t *dst = static_cast<uint8_t *>(P.sum_out) + off;
            if (full && IN == 8) *reinterpret_cast<uint32_t *>(dst) = acc;
            else if (full && IN == 4) *reinterpret_cast<uint16_t *>(dst) = static_cast<uint16_t>(acc);
            else for (int b = 0; b < bytes; ++b) dst[b] = static_cast<uint8_t>(acc >> (8 * b));
        }
    }
    if constexpr (KOUT) {  // counts from 1-bit rows as C-bit fields, C = 2, 4 or 8
        const int C = P.sum_bits;
        uint8_t *out = static_cast<uint8_t *>(P.sum_out);
        const uint32_t valid = left == 4 ? 0xFFFFFFFFu : ((1u << (8 * left)) - 1u);
        const uint32_t kb = kp & valid;
        if (C == 8) {
            if (full) *reinterpret_cast<uint32_t *>(out + e) = kb;
            else for (int k = 0; k < left; ++k) out[e + k] = static_cast<uint8_t>(kb >> (8 * k));
        } else if (C == 4) {
            const uint32_t v = (kb & 0xFu) | ((kb >> 4) & 0xF0u) | ((kb >> 8) & 0xF00u) | ((kb >> 12) & 0xF000u);
            if (left > 2) *reinterpret_cast<uint16_t *>(out + e / 2) = static_cast<uint16_t>(v);
            else out[e / 2] = static_cast<uint8_t>(v);
        } else {
            const uint32_t v = (kb & 0x3u) | ((kb >> 6) & 0xCu) | ((kb >> 12) & 0x30u) | ((kb >> 18) & 0xC0u);
            out[e / 4] = static_cast<uint8_t>(v);
        }
    }

    // u per element: K against the threshold (or K+ against K-); what a tie gives is uniform
    const float tie_u = (IN == IN_TERNARY) ? 0.0f : (!P.tie_possible ? -1.0f : (P.tie < 0 ? 0.0f : (P.tie > 0 ? 1.0f : -1.0f)));
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int a = static_cast<int>((kp >> (8 * k)) & 0xFFu);
        const int b = (IN == IN_TERNARY) ? static_cast<int>((kn >> (8 * k)) & 0xFFu) : P.thresh;
        const float uf = a > b ? 1.0f : (a == b ? tie_u : -1.0f);
        th[k] = __builtin_fmaf(-lr, __builtin_fmaf(wd, th[k], uf), th[k]);
    }
    if (full) store4(P.theta + e, th);
    else for (int k = 0; k < left; ++k) P.theta[e + k] = th[k];
}

template <int IN, bool KOUT>
static hipError_t launch_tile(const AggParams &P, hipStream_t s)
{
    constexpr size_t waves = kTileThreads / kWave;
    if (P.n_seg > 0) {
        constexpr size_t per = 256 * waves * kTilesPerWave<true>;
        return launch(tile_apply_kernel<IN, KOUT, true>, static_cast<unsigned>((P.n + per - 1) / per), kTileThreads, LC_TILE_LDS, s, P);
    }
    constexpr size_t per = 256 * waves * kTilesPerWave<false>;
    return launch(tile_apply_kernel<IN, KOUT, false>, static_cast<unsigned>((P.n + per - 1) / per), kTileThreads, LC_TILE_LDS, s, P);
}

template <int IN, int GDT, bool APPLY, bool MOM, bool KOUT>
static hipError_t launch_one(const AggParams &P, hipStream_t s)
{
    if constexpr (IN == IN_BITS) {
        if (P.W >= kAggManyRows) {
            // many rows: shorter waves; with 16 words per wave fewer waves per compute unit (dynamic LDS as a cap)
            constexpr size_t block = static_cast<size_t>(kAggWordsMany) * 64 * kWaves;
            const unsigned lds = kAggWordsMany >= 16 ? LC_AGG_LDS : 0;
            return launch(aggregate_kernel<IN, GDT, APPLY, MOM, KOUT, kAggWordsMany>, static_cast<unsigned>((P.n + block - 1) / block),
                          kAggThreads, lds, s, P);
        }
    }
    constexpr size_t block = static_cast<size_t>(kAggWordsDefault) * 64 * kWaves;  // elements per workgroup
    return launch(aggregate_kernel<IN, GDT, APPLY, MOM, KOUT, kAggWordsDefault>, static_cast<unsigned>((P.n + block - 1) / block),
                  kAggThreads, 0, s, P);
}

template <int IN, bool KOUT>
static hipError_t launch_in(const AggParams &P, bool apply, int g_dtype, hipStream_t s)
{
    if (!apply) return launch_one<IN, LC_F32, false, false, KOUT>(P, s);
    if (P.n_m == 0) return launch_one<IN, LC_F32, true, false, KOUT>(P, s);
    if (g_dtype == LC_BF16) return launch_one<IN, LC_BF16, true, true, KOUT>(P, s);
    return launch_one<IN, LC_F32, true, true, KOUT>(P, s);
}

// Host launcher; arguments were validated by the caller.  in_kind: 0 planes, 1 bits,
// 2/4/8 fields, 16 ternary (pos + nz rows).  kout: counts wanted from 1-bit rows.
hipError_t launch_aggregate(const AggParams &P, int in_kind, bool apply, bool kout, int g_dtype, hipStream_t s)
{
    // few workers, apply, no momentum streams, no planes wanted: one tile per wave
    const bool tile_ok = apply && P.n_m == 0 && !P.vote_pos && !P.vote_nz;
    if (tile_ok && (in_kind == IN_BITS || in_kind == IN_TERNARY) && P.W * (in_kind == IN_TERNARY ? 2 : 1) <= LC_TILE_MAX_W_BITS &&
        !(kout && P.sum_bits == 1)) {
        if (in_kind == IN_TERNARY) return launch_tile<IN_TERNARY, false>(P, s);
        return kout ? launch_tile<IN_BITS, true>(P, s) : launch_tile<IN_BITS, false>(P, s);
    }
    if (tile_ok && LC_TILE_FIELDS && (in_kind == 2 || in_kind == 4 || in_kind == 8)) {
        if (in_kind == 2) return launch_tile<2, false>(P, s);
        if (in_kind == 4) return launch_tile<4, false>(P, s);
        return launch_tile<8, false>(P, s);
    }
    // one buffer of counts and momentum rows to update: a row per grid line, as from planes
    if (LC_APPLY_ONLY && apply && P.W == 1 && P.n_m > 0 && P.n_seg == 0 && !P.vote_pos && !P.vote_nz && !P.sum_out &&
        (in_kind == 2 || in_kind == 4 || in_kind == 8)) {
        if (in_kind == 2) return launch_apply_only<2>(P, g_dtype, s);
        if (in_kind == 4) return launch_apply_only<4>(P, g_dtype, s);
        return launch_apply_only<8>(P, g_dtype, s);
    }
    switch (in_kind) {
    case IN_PLANES:
        if (LC_APPLY_ONLY && apply && P.n_seg == 0 && !P.vote_pos && !P.vote_nz) return launch_apply_only<0>(P, g_dtype, s);
        return launch_in<IN_PLANES, false>(P, apply, g_dtype, s);
    case IN_BITS:
        if (!apply && !kout) return launch_vote_only(P, s);
        return kout ? launch_in<IN_BITS, true>(P, apply, g_dtype, s) : launch_in<IN_BITS, false>(P, apply, g_dtype, s);
    case IN_TERNARY:
        if (LC_VOTE_TERNARY && !apply) {
            const size_t nw = (P.n + 63) / 64;
            const unsigned grid = static_cast<unsigned>((nw + kVoteThreads - 1) / kVoteThreads);
            if (P.W % 8 == 0) return launch(vote_only_ternary_kernel<true>, grid, kVoteThreads, LC_VOTE_LDS, s, P);
            return launch(vote_only_ternary_kernel<false>, grid, kVoteThreads, LC_VOTE_LDS, s, P);
        }
        return launch_in<IN_TERNARY, false>(P, apply, g_dtype, s);
    case 2: return launch_in<2, false>(P, apply, g_dtype, s);
    case 4: return launch_in<4, false>(P, apply, g_dtype, s);
    default: return launch_in<8, false>(P, apply, g_dtype, s);
    }
}

}  // namespace lc
