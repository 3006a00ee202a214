// W-way aggregation (majority vote over packed bits, or p-bit sum then sign) and the
// apply step, as one kernel family (Algorithm 1 lines 4-6; Section 3; Appendix A.1, B.1
// and F.1).
//
// A wave owns kAggWave = 4096 consecutive elements (64 packed words) and runs three phases:
//
//  A  count   Lanes own packed input.  1-bit rows: lane j holds word j of every worker
//             and counts bit-sliced: carry-save adders fold 8 words at a time into
//             planes c[0..7] (c[k] bit i = bit k of K_i), about 6 bitwise ops per word
//             for 64 elements.  K is compared with W/2 bit-sliced as well, giving the
//             `pos` (S > 0) and `nz` (S != 0) words directly.  Field rows: lane holds 16
//             bytes of fields per worker and adds them as four 32-bit integers -- no
//             carry crosses a field because K <= W <= 2^p - 1 -- then compares field
//             by field.
//  B  stage   pos / nz (and, if the counts K are wanted from 1-bit rows, the count
//             planes) go to LDS in the canonical 1-bit layout; the planes are also
//             stored to global memory if the caller asked for them.
//  C  apply   Lanes own elements: tile t, lane l holds elements 256 t + 4 l .. + 3
//             (16-byte accesses of theta, m, g) and fetches its 4 pos / nz bits from
//             LDS.  This is the only place where the word-per-lane and element-per-lane
//             layouts meet, and the only use of LDS.
#include "lc_launch.hpp"

namespace lc {

constexpr int kAggWords = 64;                 // packed words per wave
constexpr int kAggWave = kAggWords * 64;      // elements per wave
constexpr int kAggBlock = kAggWave * kWaves;  // elements per workgroup
constexpr int kAggTiles = kAggWave / 256;

enum { IN_PLANES = 0, IN_BITS = 1 /* 2, 4, 8: field width */ };


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

// From "K > W/2" and "K == W/2" to the two vote planes.  For odd W, K == floor(W/2)
// means S = -1: not a tie.
__device__ __forceinline__ void vote_planes(uint64_t gt, uint64_t eq, int W, int tie, uint64_t &pos, uint64_t &nz)
{
    pos = gt;
    nz = ~0ull;
    if ((W & 1) == 0) {
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

template <int IN, int GDT, bool APPLY, bool KOUT>
__global__ __launch_bounds__(kBlock) void aggregate_kernel(const AggParams P)
{
    __shared__ uint64_t s_pos[kWaves][kAggWords];
    __shared__ uint64_t s_nz[kWaves][kAggWords];
    __shared__ uint64_t s_cnt[KOUT ? kWaves : 1][KOUT ? 8 : 1][KOUT ? kAggWords : 1];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const size_t n = P.n;
    const size_t wave_base = (static_cast<size_t>(blockIdx.x) * kWaves + wave) * kAggWave;
    const bool active = wave_base < n;
    const int W = P.W;
    const int T = W >> 1;

    // ---------------------------------------------------------------- phase A + B
    if (active) {
        if constexpr (IN == IN_PLANES) {
            const size_t jw = wave_base / 64 + lane;
            const uint64_t vm = valid_mask(jw * 64, n);
            uint64_t pos = 0, nz = 0;
            if (vm) {
                pos = P.in_pos[jw];
                nz = P.in_nz ? P.in_nz[jw] : ~0ull;
            }
            s_pos[wave][lane] = pos & nz & vm;
            s_nz[wave][lane] = nz & vm;
        } else if constexpr (IN == IN_BITS) {
            const size_t jw = wave_base / 64 + lane;
            const uint64_t vm = valid_mask(jw * 64, n);
            const size_t stride = P.q_stride_bytes / 8;
            const uint64_t *qp = static_cast<const uint64_t *>(P.q) + jw;
            uint64_t c[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            int w = 0;
            for (; w + 8 <= W; w += 8) {
                uint64_t x[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) x[k] = vm ? qp[static_cast<size_t>(w + k) * stride] : 0ull;
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
            for (; w < W; ++w) ripple(c, vm ? qp[static_cast<size_t>(w) * stride] : 0ull, 0);
            uint64_t gt, eq, pos, nz;
            compare_planes(c, T, gt, eq);
            vote_planes(gt, eq, W, P.tie, pos, nz);
            pos &= vm;
            nz &= vm;
            s_pos[wave][lane] = pos;
            s_nz[wave][lane] = nz;
            if (KOUT) {
#pragma unroll
                for (int k = 0; k < 8; ++k) s_cnt[KOUT ? wave : 0][KOUT ? k : 0][KOUT ? lane : 0] = c[k] & vm;
                if (P.sum_bits == 1 && vm) static_cast<uint64_t *>(P.sum_out)[jw] = c[0] & vm;  // W = 1: K is the bit
            }
            if (vm) {
                if (P.vote_pos) P.vote_pos[jw] = pos;
                if (P.vote_nz) P.vote_nz[jw] = nz;
            }
        } else {
            // field rows: lane owns 16 bytes = kFpl fields per round
            constexpr int C = IN;
            constexpr int kFpl = 128 / C;            // fields per lane per round
            constexpr int kRound = kWave * kFpl;     // elements per round
            constexpr int kRounds = kAggWave / kRound;
            constexpr uint32_t fmask = (1u << C) - 1u;
            const size_t valid_bytes = (n * C + 7) / 8;
            const char *qb = static_cast<const char *>(P.q);
#pragma unroll 1
            for (int r = 0; r < kRounds; ++r) {
                const size_t e0 = wave_base + static_cast<size_t>(r) * kRound + static_cast<size_t>(lane) * kFpl;
                const size_t off = e0 / 8 * C;  // e0 is a multiple of 16
                u32x4 acc = {0, 0, 0, 0};
                const bool full = off + 16 <= valid_bytes;
                if (full) {
                    int w = 0;
                    for (; w + 4 <= W; w += 4) {
                        u32x4 x[4];
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            x[k] = *reinterpret_cast<const u32x4 *>(qb + static_cast<size_t>(w + k) * P.q_stride_bytes + off);
#pragma unroll
                        for (int k = 0; k < 4; ++k) acc += x[k];
                    }
                    for (; w < W; ++w) acc += *reinterpret_cast<const u32x4 *>(qb + static_cast<size_t>(w) * P.q_stride_bytes + off);
                    if (P.sum_out) *reinterpret_cast<u32x4 *>(static_cast<char *>(P.sum_out) + off) = acc;
                } else if (off < valid_bytes) {
                    // the lane that holds the end of the row: byte by byte, pad fields dropped
                    const int nb = static_cast<int>(valid_bytes - off);
                    for (int w = 0; w < W; ++w) {
                        const uint8_t *src = reinterpret_cast<const uint8_t *>(qb + static_cast<size_t>(w) * P.q_stride_bytes + off);
#pragma unroll
                        for (int b = 0; b < 16; ++b)
                            if (b < nb) acc[b >> 2] += static_cast<uint32_t>(src[b]) << (8 * (b & 3));
                    }
#pragma unroll
                    for (int f = 0; f < kFpl; ++f)
                        if (e0 + f >= n) acc[(f * C) >> 5] &= ~(fmask << ((f * C) & 31));
                    if (P.sum_out) {
                        uint8_t *dst = reinterpret_cast<uint8_t *>(static_cast<char *>(P.sum_out) + off);
#pragma unroll
                        for (int b = 0; b < 16; ++b)
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
                vote_planes(gt, eq, W, P.tie, pos, nz);
                const uint64_t vm = valid_mask(e0, n) & (kFpl == 64 ? ~0ull : ((1ull << (kFpl & 63)) - 1ull));
                pos &= vm;
                nz &= vm;
                if (kFpl == 64) {
                    s_pos[wave][lane] = pos;
                    s_nz[wave][lane] = nz;
                } else if (kFpl == 32) {
                    reinterpret_cast<uint32_t *>(s_pos[wave])[r * kWave + lane] = static_cast<uint32_t>(pos);
                    reinterpret_cast<uint32_t *>(s_nz[wave])[r * kWave + lane] = static_cast<uint32_t>(nz);
                } else {
                    reinterpret_cast<uint16_t *>(s_pos[wave])[r * kWave + lane] = static_cast<uint16_t>(pos);
                    reinterpret_cast<uint16_t *>(s_nz[wave])[r * kWave + lane] = static_cast<uint16_t>(nz);
                }
            }
        }
    }
    __syncthreads();

    if (IN != IN_PLANES && IN != IN_BITS && active) {
        // planes for the caller, from LDS in word order
        const size_t jw = wave_base / 64 + lane;
        if (jw * 64 < n) {
            if (P.vote_pos) P.vote_pos[jw] = s_pos[wave][lane];
            if (P.vote_nz) P.vote_nz[jw] = s_nz[wave][lane];
        }
    }

    // ---------------------------------------------------------------- phase C
    if (!(APPLY || KOUT) || !active) return;
    const uint8_t *pos8 = reinterpret_cast<const uint8_t *>(s_pos[wave]);
    const uint8_t *nz8 = reinterpret_cast<const uint8_t *>(s_nz[wave]);
    const float lr = P.lr, wd = P.wd;
    const int sh = (lane & 1) * 4;

    if (APPLY && wave_base + kAggWave <= n) {
        constexpr int U = 4;
#pragma unroll 1
        for (int t0 = 0; t0 < kAggTiles; t0 += U) {
            f32x4 th[U];
#pragma unroll
            for (int u = 0; u < U; ++u) th[u] = load4(P.theta + wave_base + (t0 + u) * 256 + lane * 4);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int byte = (t0 + u) * 32 + (lane >> 1);
                const uint32_t pn = pos8[byte] >> sh, zn = nz8[byte] >> sh;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float uf = ((zn >> k) & 1u) ? (((pn >> k) & 1u) ? 1.0f : -1.0f) : 0.0f;
                    th[u][k] = __builtin_fmaf(-lr, __builtin_fmaf(wd, th[u][k], uf), th[u][k]);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) store4(P.theta + wave_base + (t0 + u) * 256 + lane * 4, th[u]);
            for (int w = 0; w < P.n_m; ++w) {
                float *mrow = P.m + static_cast<size_t>(w) * P.m_stride;
                const void *grow = static_cast<const char *>(P.g) + static_cast<size_t>(w) * P.g_stride * Grad<GDT>::kBytes;
                f32x4 mv[U], gv[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const size_t e = wave_base + (t0 + u) * 256 + lane * 4;
                    mv[u] = load4(mrow + e);
                    gv[u] = Grad<GDT>::load4(grow, e);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) mv[u][k] = momentum_step(mv[u][k], gv[u][k], P.beta2, P.omb2);
                    store4(mrow + wave_base + (t0 + u) * 256 + lane * 4, mv[u]);
                }
            }
        }
    } else if (APPLY) {
        // ragged end: element by element
        for (int t = 0; t < kAggTiles; ++t) {
            const size_t e = wave_base + t * 256 + lane * 4;
            if (e >= n) break;
            const int byte = t * 32 + (lane >> 1);
            const uint32_t pn = pos8[byte] >> sh, zn = nz8[byte] >> sh;
            for (int k = 0; k < 4 && e + k < n; ++k) {
                const float uf = ((zn >> k) & 1u) ? (((pn >> k) & 1u) ? 1.0f : -1.0f) : 0.0f;
                const float th = P.theta[e + k];
                P.theta[e + k] = __builtin_fmaf(-lr, __builtin_fmaf(wd, th, uf), th);
                for (int w = 0; w < P.n_m; ++w) {
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

template <int IN, int GDT, bool APPLY, bool KOUT>
static hipError_t launch_one(const AggParams &P, hipStream_t s)
{
    const unsigned grid = static_cast<unsigned>((P.n + kAggBlock - 1) / kAggBlock);
    aggregate_kernel<IN, GDT, APPLY, KOUT><<<grid, kBlock, 0, s>>>(P);
    return hipGetLastError();
}

template <int IN, bool KOUT>
static hipError_t launch_in(const AggParams &P, bool apply, int g_dtype, hipStream_t s)
{
    if (!apply) return launch_one<IN, LC_F32, false, KOUT>(P, s);
    if (g_dtype == LC_BF16) return launch_one<IN, LC_BF16, true, KOUT>(P, s);
    return launch_one<IN, LC_F32, true, KOUT>(P, s);
}

// Host launcher; arguments were validated by the caller.  in_kind: 0 planes, 1 bits,
// 2/4/8 fields.  kout: counts wanted from 1-bit rows.
hipError_t launch_aggregate(const AggParams &P, int in_kind, bool apply, bool kout, int g_dtype, hipStream_t s)
{
    switch (in_kind) {
    case IN_PLANES: return launch_in<IN_PLANES, false>(P, apply, g_dtype, s);
    case IN_BITS: return kout ? launch_in<IN_BITS, true>(P, apply, g_dtype, s) : launch_in<IN_BITS, false>(P, apply, g_dtype, s);
    case 2: return launch_in<2, false>(P, apply, g_dtype, s);
    case 4: return launch_in<4, false>(P, apply, g_dtype, s);
    default: return launch_in<8, false>(P, apply, g_dtype, s);
    }
}

}  // namespace lc
