// Host-side launchers of the kernel files and the parameter block of the aggregation
// kernels.  Arguments are validated by the C-ABI layer before any of these is called.
#pragma once

#include "lc_common.hpp"

#include <tuple>
#include <utility>

namespace lc {

// Kernel launch that reports what THIS launch returned.  The <<< >>> form leaves its status
// in the runtime's per-thread "last error", which also holds -- and, once read, forgets --
// whatever an unrelated earlier call of the host program left there; hipLaunchKernel's own
// return value neither sees nor clears that.
template <typename... KArgs, size_t... I, typename Tuple>
inline hipError_t launch_impl(void (*kernel)(KArgs...), dim3 grid, dim3 block, unsigned lds, hipStream_t s, Tuple &vals,
                              std::index_sequence<I...>)
{
    void *ptrs[] = {const_cast<void *>(static_cast<const void *>(&std::get<I>(vals)))...};
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, lds, s);
}
template <typename... KArgs, typename... Args>
inline hipError_t launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, unsigned lds, hipStream_t s, Args &&...args)
{
    static_assert(sizeof...(KArgs) == sizeof...(Args), "one argument per kernel parameter");
    std::tuple<std::remove_cv_t<KArgs>...> vals(static_cast<std::remove_cv_t<KArgs>>(std::forward<Args>(args))...);
    return launch_impl(kernel, grid, block, lds, s, vals, std::index_sequence_for<KArgs...>());
}

struct AggParams {
    const void *q;          // packed rows (1-bit words or fields); unused for IN_PLANES
    const void *q2;         // ternary input: the nz rows (q holds the pos rows), same stride
    size_t q_stride_bytes;
    int W;
    size_t n;
    int sum_bits;           // container width of sum_out fields
    void *sum_out;          // may be null
    uint64_t *vote_pos;     // may be null
    uint64_t *vote_nz;      // may be null
    const uint64_t *in_pos; // IN_PLANES only
    const uint64_t *in_nz;  // IN_PLANES only; null = every element non-zero
    int tie;                // -1: tie -> 0 ; 0: tie -> -1 ; +1: tie -> +1
    int thresh;             // count K at which the summed signs / levels are zero
    int tie_possible;       // K == thresh is a tie (even W for 0/1 votes; always for levels)
    float *theta;
    float lr, wd;
    const uint32_t *seg_end64;  // parameter groups: end of each segment in units of 64 elements, ascending
    const float *seg_lr;        // per-segment learning rate and weight decay (device arrays)
    const float *seg_wd;
    int n_seg;                  // 0: lr / wd above hold for the whole range
    float *m;
    size_t m_stride;
    const void *g;
    size_t g_stride;
    int n_m;
    float beta2, omb2;
};

hipError_t launch_local_update_pack(const void *g, size_t g_stride, int g_dtype, float *m, size_t m_stride, int W, size_t n,
                                    float beta1, bool update_m, float beta2, int out_bits, void *q, size_t q_stride_bytes,
                                    int zero_bit, hipStream_t s);
// in_kind: 0 = vote planes, 1 = 1-bit rows, 2 / 4 / 8 = field rows of that width,
// 16 = ternary rows (pos in q, nz in q2).
// kout: the counts K are wanted as fields from 1-bit rows.
hipError_t launch_aggregate(const AggParams &P, int in_kind, bool apply, bool kout, int g_dtype, hipStream_t s);
hipError_t launch_momentum_avg(float *m, size_t stride, int W, size_t n, hipStream_t s);
hipError_t launch_stream_probe(int kind, float *a, const float *b, size_t n, float s, hipStream_t st);
hipError_t launch_momentum_avg_ranges(float *m, size_t stride, int W, const size_t *offsets, const size_t *sizes, int n_ranges,
                                      hipStream_t s);
// n_groups = 0: one maximum over the whole range; else one per segment of the group table
hipError_t launch_momentum_divergence(const float *m, size_t stride, int W, size_t n, double *out, const uint32_t *end64,
                                      int n_groups, hipStream_t s);
hipError_t launch_local_update_pack_ternary(const void *g, size_t g_stride, int g_dtype, float *m, size_t m_stride, int W,
                                            size_t n, float beta1, bool update_m, float beta2, uint64_t *pos, uint64_t *nz,
                                            size_t stride_words, hipStream_t s);

// L1 quantisation (Equation 1, p = 1)
constexpr int kL1Limbs = 12;  // 64-bit accumulators, 32 bits apart
constexpr int kL1Slots = 32;  // independent sets of limbs per worker (spreads the atomics)
static_assert(kL1Limbs * kL1Slots == LC_L1_WORKSPACE_WORDS, "workspace size in the header");
// Optional table of parameter groups for the L1 calls (n = 0: none).  Segment s ends at
// element 64 * end64[s]; count[s], if given, is the number of elements its mean divides by.
struct L1Groups {
    const uint32_t *end64 = nullptr;
    const uint64_t *count = nullptr;
    int n = 0;
};
hipError_t launch_l1_mean_abs(const void *g, size_t g_stride, int g_dtype, const float *m, size_t m_stride, int W, size_t n,
                              float beta1, double *mean_abs, uint64_t *workspace, const L1Groups &grp, hipStream_t s);
// lc_l1_mean_abs with the library's own per-device workspace (W <= LC_L1_STATIC_MAX_W)
hipError_t launch_l1_mean_abs_static(const void *g, size_t g_stride, int g_dtype, const float *m, size_t m_stride, int W,
                                     size_t n, float beta1, double *mean_abs, hipStream_t s);
hipError_t launch_l1_quantize_pack(const void *g, size_t g_stride, int g_dtype, float *m, size_t m_stride, int W, size_t n,
                                   float beta1, bool update_m, float beta2, int levels, const double *mean_abs, uint8_t *q,
                                   size_t q_stride_bytes, const L1Groups &grp, hipStream_t s);

}  // namespace lc
