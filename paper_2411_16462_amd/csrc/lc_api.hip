// C ABI of the library: argument validation on the host, then one kernel launch per
// call.  Nothing here allocates, synchronises or keeps state.
#include "lc_launch.hpp"

namespace lc {


namespace {

struct Groups {
    const uint32_t *end64 = nullptr;
    const float *lr = nullptr;
    const float *wd = nullptr;
    int n = 0;
};

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline int from_hip(hipError_t e) { return e == hipSuccess ? LC_OK : -static_cast<int>(e); }
inline size_t gbytes(int g_dtype) { return g_dtype == LC_BF16 ? 2 : 4; }

int container(int p)
{
    if (p < 1 || p > 8) return -1;
    return p == 1 ? 1 : p == 2 ? 2 : p <= 4 ? 4 : 8;
}

// rows of fp32 momentum and of gradients, `rows` of them
int check_mg(const float *m, size_t m_stride, const void *g, size_t g_stride, int g_dtype, int rows)
{
    if (g_dtype != LC_F32 && g_dtype != LC_BF16) return LC_ERR_DTYPE;
    if (!m || !g) return LC_ERR_NULL;
    if (!aligned(m, 16) || !aligned(g, 16)) return LC_ERR_ALIGN;
    if (rows > 1 && ((m_stride * 4) % 16 != 0 || (g_stride * gbytes(g_dtype)) % 16 != 0)) return LC_ERR_ALIGN;
    return LC_OK;
}

int tie_code(int tie_rule, uint64_t step)
{
    if (tie_rule == LC_TIE_ZERO) return -1;
    return (step & 1u) ? 1 : 0;
}

// Segment ends are uint32 in units of 64 elements: a group table cannot describe more.
constexpr size_t kMaxGroupedN = static_cast<size_t>(64) * 0xFFFFFFFFull;

// One aggregation call, filled in by name by its entry point (whatever an entry point does
// not have keeps the default: no second plane buffer, no sum, no planes out, nothing
// applied, no momentum rows, no group table).
struct AggCall {
    const void *q = nullptr;        // packed rows: 1-bit words, fields, or the pos rows of the ternary format
    const void *q2 = nullptr;       // ternary format: the nz rows
    size_t q_stride_bytes = 0;
    int in_bits = 1;                // 1, 2 / 4 / 8 (fields), 16 (ternary)
    int W = 0;
    size_t n = 0;
    int p = 0;                      // p-bit sum: range rule W <= 2^p - 1; 0 = not a p-bit sum
    int levels = 0;                 // summed level bytes: L; 0 = not a level sum
    void *sum_out = nullptr;
    uint64_t *vote_pos = nullptr;
    uint64_t *vote_nz = nullptr;
    uint64_t step = 1;
    int tie_rule = LC_TIE_ZERO;
    bool apply = false;
    float *theta = nullptr;
    float lr = 0.0f, wd = 0.0f;
    float *m = nullptr;
    size_t m_stride = 0;
    const void *g = nullptr;
    size_t g_stride = 0;
    int g_dtype = LC_F32;
    int n_m = 0;
    float beta2 = 0.0f;
    bool grouped = false;           // a *_groups entry point: the table below is required
    Groups groups;
    void *stream = nullptr;
};

// shared by the aggregation entry points
int aggregate(const AggCall &c)
{
    const int W = c.W, p = c.p, levels = c.levels, in_bits = c.in_bits;
    if (W < 1 || W > LC_MAX_W || c.n > LC_MAX_N) return LC_ERR_SIZE;
    if (c.grouped) {
        if (c.groups.n < 1 || c.groups.n > LC_MAX_GROUPS || c.n > kMaxGroupedN) return LC_ERR_SIZE;
        if (!c.groups.end64 || !c.groups.lr || !c.groups.wd) return LC_ERR_NULL;
        if (!aligned(c.groups.end64, 4) || !aligned(c.groups.lr, 4) || !aligned(c.groups.wd, 4)) return LC_ERR_ALIGN;
    }
    if (c.tie_rule != LC_TIE_ZERO && c.tie_rule != LC_TIE_ALT) return LC_ERR_MODE;
    int sum_bits = 0;
    if (levels != 0) {  // summed level bytes: every row holds level + L in [0, 2L]
        if (levels < 1 || levels > 127 || 2 * levels * W > 255) return LC_ERR_RANGE;
        sum_bits = 8;
    } else if (p != 0) {  // p-bit sum: range rule of the direct allreduce
        sum_bits = container(p);
        if (sum_bits < 0) return LC_ERR_RANGE;
        if (W > (1 << p) - 1) return LC_ERR_RANGE;
        if (in_bits != 1 && in_bits != sum_bits) return LC_ERR_MODE;
    } else if (in_bits != 1 && in_bits != 16) {
        return LC_ERR_MODE;
    }
    if (!c.q || (in_bits == 16 && !c.q2)) return LC_ERR_NULL;
    if (in_bits == 16 && !aligned(c.q2, 8)) return LC_ERR_ALIGN;
    if (in_bits == 1 || in_bits == 16) {
        if (!aligned(c.q, 8) || (W > 1 && c.q_stride_bytes % 8 != 0)) return LC_ERR_ALIGN;
    } else {
        if (!aligned(c.q, 16) || (W > 1 && c.q_stride_bytes % 16 != 0)) return LC_ERR_ALIGN;
    }
    if (c.sum_out && !aligned(c.sum_out, 16)) return LC_ERR_ALIGN;
    if (!aligned(c.vote_pos, 8) || !aligned(c.vote_nz, 8)) return LC_ERR_ALIGN;
    if (c.apply) {
        if (!c.theta) return LC_ERR_NULL;
        if (!aligned(c.theta, 16)) return LC_ERR_ALIGN;
        if (c.n_m < 0 || c.n_m > LC_MAX_W) return LC_ERR_SIZE;
        if (c.n_m > 0) {
            const int rc = check_mg(c.m, c.m_stride, c.g, c.g_stride, c.g_dtype, c.n_m);
            if (rc) return rc;
        }
    }
    if (c.n == 0) return LC_OK;
    AggParams P{};
    P.q = c.q;
    P.q2 = c.q2;
    P.q_stride_bytes = c.q_stride_bytes;
    P.W = W;
    P.n = c.n;
    P.sum_bits = sum_bits;
    P.sum_out = c.sum_out;
    P.vote_pos = c.vote_pos;
    P.vote_nz = c.vote_nz;
    P.tie = tie_code(c.tie_rule, c.step);
    P.thresh = levels > 0 ? W * levels : (W >> 1);
    P.tie_possible = levels > 0 ? 1 : ((W & 1) == 0);
    P.theta = c.theta;
    P.lr = c.lr;
    P.wd = c.wd;
    P.seg_end64 = c.groups.end64;
    P.seg_lr = c.groups.lr;
    P.seg_wd = c.groups.wd;
    P.n_seg = c.grouped ? c.groups.n : 0;
    P.m = c.m;
    P.m_stride = c.m_stride;
    P.g = c.g;
    P.g_stride = c.g_stride;
    P.n_m = c.apply ? c.n_m : 0;
    P.beta2 = c.beta2;
    P.omb2 = 1.0f - c.beta2;
    const bool kout = in_bits == 1 && c.sum_out != nullptr;
    return from_hip(launch_aggregate(P, in_bits, c.apply, kout, (c.apply && c.n_m > 0) ? c.g_dtype : LC_F32,
                                     static_cast<hipStream_t>(c.stream)));
}

// the momentum / gradient rows of an apply call
void set_streams(AggCall &c, float *m, size_t m_stride, const void *g, size_t g_stride, int g_dtype, int n_m, float beta2)
{
    c.m = m;
    c.m_stride = m_stride;
    c.g = g;
    c.g_stride = g_stride;
    c.g_dtype = g_dtype;
    c.n_m = n_m;
    c.beta2 = beta2;
}

void set_groups(AggCall &c, const uint32_t *end64, const float *lr, const float *wd, int n_groups)
{
    c.grouped = true;
    c.groups.end64 = end64;
    c.groups.lr = lr;
    c.groups.wd = wd;
    c.groups.n = n_groups;
}

}  // namespace
}  // namespace lc

using namespace lc;

extern "C" {

int lc_local_update_pack(const void *g, size_t g_stride_elems, int g_dtype, float *m, size_t m_stride_elems, int W,
                         size_t n, float beta1, int update_m, float beta2, int out_bits, void *q, size_t q_stride_bytes,
                         uint64_t step, int zero_rule, void *stream)
{
    if (W < 1 || W > LC_MAX_W || n > LC_MAX_N) return LC_ERR_SIZE;
    if (out_bits != 1 && out_bits != 2 && out_bits != 4 && out_bits != 8) return LC_ERR_MODE;
    if (zero_rule != LC_ZERO_ALT && zero_rule != LC_ZERO_POS && zero_rule != LC_ZERO_NEG) return LC_ERR_MODE;
    if (!q && !update_m) return LC_ERR_NULL;
    const int rc = check_mg(m, m_stride_elems, g, g_stride_elems, g_dtype, W);
    if (rc) return rc;
    if (q) {
        const size_t a = out_bits == 1 ? 8 : 16;
        if (!aligned(q, a) || (W > 1 && q_stride_bytes % a != 0)) return LC_ERR_ALIGN;
    }
    if (n == 0) return LC_OK;
    const int zero_bit = zero_rule == LC_ZERO_POS ? 1 : zero_rule == LC_ZERO_NEG ? 0 : static_cast<int>(step & 1u);
    return from_hip(launch_local_update_pack(g, g_stride_elems, g_dtype, m, m_stride_elems, W, n, beta1, update_m != 0, beta2,
                                             out_bits, q, q_stride_bytes, zero_bit, static_cast<hipStream_t>(stream)));
}

int lc_vote_1bit(const uint64_t *q, size_t q_stride_words, int W, size_t n, uint64_t *vote_pos, uint64_t *vote_nz,
                 uint64_t step, int tie_rule, void *stream)
{
    AggCall c;
    c.q = q;
    c.q_stride_bytes = q_stride_words * 8;
    c.in_bits = 1;
    c.W = W;
    c.n = n;
    c.vote_pos = vote_pos;
    c.vote_nz = vote_nz;
    c.step = step;
    c.tie_rule = tie_rule;
    c.stream = stream;
    return aggregate(c);
}

int lc_pbit_sum_sign(const void *q, size_t q_stride_bytes, int in_bits, int W, size_t n, int p, void *sum_out,
                     uint64_t *vote_pos, uint64_t *vote_nz, uint64_t step, int tie_rule, void *stream)
{
    if (p == 0) return LC_ERR_RANGE;
    AggCall c;
    c.q = q;
    c.q_stride_bytes = q_stride_bytes;
    c.in_bits = in_bits;
    c.W = W;
    c.n = n;
    c.p = p;
    c.sum_out = sum_out;
    c.vote_pos = vote_pos;
    c.vote_nz = vote_nz;
    c.step = step;
    c.tie_rule = tie_rule;
    c.stream = stream;
    return aggregate(c);
}

int lc_vote_apply_1bit(const uint64_t *q, size_t q_stride_words, int W, size_t n, uint64_t step, int tie_rule, float *theta,
                       float lr, float wd, float *m, size_t m_stride_elems, const void *g, size_t g_stride_elems, int g_dtype,
                       int n_m, float beta2, void *stream)
{
    AggCall c;
    c.q = q;
    c.q_stride_bytes = q_stride_words * 8;
    c.in_bits = 1;
    c.W = W;
    c.n = n;
    c.step = step;
    c.tie_rule = tie_rule;
    c.apply = true;
    c.theta = theta;
    c.lr = lr;
    c.wd = wd;
    set_streams(c, m, m_stride_elems, g, g_stride_elems, g_dtype, n_m, beta2);
    c.stream = stream;
    return aggregate(c);
}

int lc_pbit_sum_apply(const void *q, size_t q_stride_bytes, int in_bits, int W, size_t n, int p, void *sum_out, uint64_t step,
                      int tie_rule, float *theta, float lr, float wd, float *m, size_t m_stride_elems, const void *g,
                      size_t g_stride_elems, int g_dtype, int n_m, float beta2, void *stream)
{
    if (p == 0) return LC_ERR_RANGE;
    AggCall c;
    c.q = q;
    c.q_stride_bytes = q_stride_bytes;
    c.in_bits = in_bits;
    c.W = W;
    c.n = n;
    c.p = p;
    c.sum_out = sum_out;
    c.step = step;
    c.tie_rule = tie_rule;
    c.apply = true;
    c.theta = theta;
    c.lr = lr;
    c.wd = wd;
    set_streams(c, m, m_stride_elems, g, g_stride_elems, g_dtype, n_m, beta2);
    c.stream = stream;
    return aggregate(c);
}

int lc_apply_update(float *theta, const uint64_t *vote_pos, const uint64_t *vote_nz, size_t n, float lr, float wd, float *m,
                    size_t m_stride_elems, const void *g, size_t g_stride_elems, int g_dtype, int n_m, float beta2,
                    void *stream)
{
    if (!theta || !vote_pos) return LC_ERR_NULL;
    if (!aligned(theta, 16) || !aligned(vote_pos, 8) || !aligned(vote_nz, 8)) return LC_ERR_ALIGN;
    if (n_m < 0 || n_m > LC_MAX_W || n > LC_MAX_N) return LC_ERR_SIZE;
    if (n_m > 0) {
        const int rc = check_mg(m, m_stride_elems, g, g_stride_elems, g_dtype, n_m);
        if (rc) return rc;
    }
    if (n == 0) return LC_OK;
    AggParams P{};
    P.W = 1;
    P.n = n;
    P.in_pos = vote_pos;
    P.in_nz = vote_nz;
    P.tie = -1;
    P.thresh = 0;
    P.tie_possible = 0;
    P.theta = theta;
    P.lr = lr;
    P.wd = wd;
    P.m = m;
    P.m_stride = m_stride_elems;
    P.g = g;
    P.g_stride = g_stride_elems;
    P.n_m = n_m;
    P.beta2 = beta2;
    P.omb2 = 1.0f - beta2;
    return from_hip(launch_aggregate(P, 0, true, false, n_m > 0 ? g_dtype : LC_F32, static_cast<hipStream_t>(stream)));
}

int lc_count_apply(const void *k_fields, int field_bits, size_t n, int total, uint64_t step, int tie_rule, float *theta,
                   float lr, float wd, float *m, size_t m_stride_elems, const void *g, size_t g_stride_elems, int g_dtype,
                   int n_m, float beta2, void *stream)
{
    if (field_bits != 2 && field_bits != 4 && field_bits != 8) return LC_ERR_MODE;
    if (tie_rule != LC_TIE_ZERO && tie_rule != LC_TIE_ALT) return LC_ERR_MODE;
    if (total < 1 || total > (1 << field_bits) - 1) return LC_ERR_RANGE;
    if (n > LC_MAX_N || n_m < 0 || n_m > LC_MAX_W) return LC_ERR_SIZE;
    if (!k_fields || !theta) return LC_ERR_NULL;
    if (!aligned(k_fields, 16) || !aligned(theta, 16)) return LC_ERR_ALIGN;
    if (n_m > 0) {
        const int rc = check_mg(m, m_stride_elems, g, g_stride_elems, g_dtype, n_m);
        if (rc) return rc;
    }
    if (n == 0) return LC_OK;
    AggParams P{};
    P.q = k_fields;
    P.W = 1;
    P.n = n;
    P.sum_bits = field_bits;
    P.tie = tie_code(tie_rule, step);
    P.thresh = total >> 1;           // 2 K > total  <=>  K > floor(total / 2)
    P.tie_possible = (total & 1) == 0;
    P.theta = theta;
    P.lr = lr;
    P.wd = wd;
    P.m = m;
    P.m_stride = m_stride_elems;
    P.g = g;
    P.g_stride = g_stride_elems;
    P.n_m = n_m;
    P.beta2 = beta2;
    P.omb2 = 1.0f - beta2;
    return from_hip(launch_aggregate(P, field_bits, true, false, n_m > 0 ? g_dtype : LC_F32, static_cast<hipStream_t>(stream)));
}

int lc_momentum_avg(float *m, size_t m_stride_elems, int W, size_t n, void *stream)
{
    if (W < 1 || W > LC_MAX_W || n > LC_MAX_N) return LC_ERR_SIZE;
    if (!m) return LC_ERR_NULL;
    if (!aligned(m, 16) || (W > 1 && (m_stride_elems * 4) % 16 != 0)) return LC_ERR_ALIGN;
    if (n == 0 || W == 1) return LC_OK;
    return from_hip(launch_momentum_avg(m, m_stride_elems, W, n, static_cast<hipStream_t>(stream)));
}

int lc_l1_mean_abs(const void *g, size_t g_stride_elems, int g_dtype, const float *m, size_t m_stride_elems, int W, size_t n,
                   float beta1, double *mean_abs, uint64_t *workspace, void *stream)
{
    if (W < 1 || W > LC_MAX_W || n > LC_MAX_N) return LC_ERR_SIZE;
    const int rc = check_mg(m, m_stride_elems, g, g_stride_elems, g_dtype, W);
    if (rc) return rc;
    if (!mean_abs || !workspace) return LC_ERR_NULL;
    if (!aligned(mean_abs, 8) || !aligned(workspace, 8)) return LC_ERR_ALIGN;
    return from_hip(launch_l1_mean_abs(g, g_stride_elems, g_dtype, m, m_stride_elems, W, n, beta1, mean_abs, workspace,
                                       L1Groups(), static_cast<hipStream_t>(stream)));
}

int lc_l1_mean_abs_static(const void *g, size_t g_stride_elems, int g_dtype, const float *m, size_t m_stride_elems, int W,
                          size_t n, float beta1, double *mean_abs, void *stream)
{
    if (W < 1 || W > LC_L1_STATIC_MAX_W || n > LC_MAX_N) return LC_ERR_SIZE;
    const int rc = check_mg(m, m_stride_elems, g, g_stride_elems, g_dtype, W);
    if (rc) return rc;
    if (!mean_abs) return LC_ERR_NULL;
    if (!aligned(mean_abs, 8)) return LC_ERR_ALIGN;
    return from_hip(launch_l1_mean_abs_static(g, g_stride_elems, g_dtype, m, m_stride_elems, W, n, beta1, mean_abs,
                                              static_cast<hipStream_t>(stream)));
}

size_t lc_l1_groups_workspace_words(int W, int n_groups)
{
    if (W < 1 || n_groups < 1) return 0;
    return static_cast<size_t>(W) * static_cast<size_t>(n_groups) * LC_L1_WORKSPACE_WORDS +
           (static_cast<size_t>(n_groups) + 2) / 2;
}

int lc_l1_mean_abs_groups(const void *g, size_t g_stride_elems, int g_dtype, const float *m, size_t m_stride_elems, int W,
                          size_t n, float beta1, const uint32_t *group_end64, const uint64_t *group_count, int n_groups,
                          double *mean_abs, uint64_t *workspace, void *stream)
{
    if (W < 1 || W > LC_MAX_W || n > kMaxGroupedN || n_groups < 1 || n_groups > LC_MAX_GROUPS) return LC_ERR_SIZE;
    const int rc = check_mg(m, m_stride_elems, g, g_stride_elems, g_dtype, W);
    if (rc) return rc;
    if (!mean_abs || !workspace || !group_end64) return LC_ERR_NULL;
    if (!aligned(mean_abs, 8) || !aligned(workspace, 8) || !aligned(group_end64, 4) || !aligned(group_count, 8))
        return LC_ERR_ALIGN;
    L1Groups grp;
    grp.end64 = group_end64;
    grp.count = group_count;
    grp.n = n_groups;
    return from_hip(launch_l1_mean_abs(g, g_stride_elems, g_dtype, m, m_stride_elems, W, n, beta1, mean_abs, workspace, grp,
                                       static_cast<hipStream_t>(stream)));
}

int lc_l1_quantize_pack(const void *g, size_t g_stride_elems, int g_dtype, float *m, size_t m_stride_elems, int W, size_t n,
                        float beta1, int update_m, float beta2, int levels, const double *mean_abs, uint8_t *q,
                        size_t q_stride_bytes, void *stream)
{
    if (W < 1 || W > LC_MAX_W || n > LC_MAX_N) return LC_ERR_SIZE;
    if (levels < 1 || levels > 127) return LC_ERR_RANGE;
    const int rc = check_mg(m, m_stride_elems, g, g_stride_elems, g_dtype, W);
    if (rc) return rc;
    if (!mean_abs || !q) return LC_ERR_NULL;
    if (!aligned(mean_abs, 8) || !aligned(q, 16) || (W > 1 && q_stride_bytes % 16 != 0)) return LC_ERR_ALIGN;
    if (n == 0) return LC_OK;
    return from_hip(launch_l1_quantize_pack(g, g_stride_elems, g_dtype, m, m_stride_elems, W, n, beta1, update_m != 0, beta2,
                                            levels, mean_abs, q, q_stride_bytes, L1Groups(), static_cast<hipStream_t>(stream)));
}

int lc_l1_quantize_pack_groups(const void *g, size_t g_stride_elems, int g_dtype, float *m, size_t m_stride_elems, int W,
                               size_t n, float beta1, int update_m, float beta2, int levels, const uint32_t *group_end64,
                               int n_groups, const double *mean_abs, uint8_t *q, size_t q_stride_bytes, void *stream)
{
    if (W < 1 || W > LC_MAX_W || n > kMaxGroupedN || n_groups < 1 || n_groups > LC_MAX_GROUPS) return LC_ERR_SIZE;
    if (levels < 1 || levels > 127) return LC_ERR_RANGE;
    const int rc = check_mg(m, m_stride_elems, g, g_stride_elems, g_dtype, W);
    if (rc) return rc;
    if (!mean_abs || !q || !group_end64) return LC_ERR_NULL;
    if (!aligned(mean_abs, 8) || !aligned(q, 16) || (W > 1 && q_stride_bytes % 16 != 0) || !aligned(group_end64, 4))
        return LC_ERR_ALIGN;
    if (n == 0) return LC_OK;
    L1Groups grp;
    grp.end64 = group_end64;
    grp.n = n_groups;
    return from_hip(launch_l1_quantize_pack(g, g_stride_elems, g_dtype, m, m_stride_elems, W, n, beta1, update_m != 0, beta2,
                                            levels, mean_abs, q, q_stride_bytes, grp, static_cast<hipStream_t>(stream)));
}

int lc_level_sum_sign(const uint8_t *q, size_t q_stride_bytes, int W, size_t n, int levels, uint8_t *sum_out,
                      uint64_t *vote_pos, uint64_t *vote_nz, uint64_t step, int tie_rule, void *stream)
{
    if (levels == 0) return LC_ERR_RANGE;
    AggCall c;
    c.q = q;
    c.q_stride_bytes = q_stride_bytes;
    c.in_bits = 8;
    c.W = W;
    c.n = n;
    c.levels = levels;
    c.sum_out = sum_out;
    c.vote_pos = vote_pos;
    c.vote_nz = vote_nz;
    c.step = step;
    c.tie_rule = tie_rule;
    c.stream = stream;
    return aggregate(c);
}

int lc_level_sum_apply(const uint8_t *q, size_t q_stride_bytes, int W, size_t n, int levels, uint8_t *sum_out, uint64_t step,
                       int tie_rule, float *theta, float lr, float wd, float *m, size_t m_stride_elems, const void *g,
                       size_t g_stride_elems, int g_dtype, int n_m, float beta2, void *stream)
{
    if (levels == 0) return LC_ERR_RANGE;
    AggCall c;
    c.q = q;
    c.q_stride_bytes = q_stride_bytes;
    c.in_bits = 8;
    c.W = W;
    c.n = n;
    c.levels = levels;
    c.sum_out = sum_out;
    c.step = step;
    c.tie_rule = tie_rule;
    c.apply = true;
    c.theta = theta;
    c.lr = lr;
    c.wd = wd;
    set_streams(c, m, m_stride_elems, g, g_stride_elems, g_dtype, n_m, beta2);
    c.stream = stream;
    return aggregate(c);
}

int lc_level_sum_apply_groups(const uint8_t *q, size_t q_stride_bytes, int W, size_t n, int levels, uint8_t *sum_out,
                              uint64_t step, int tie_rule, float *theta, const uint32_t *group_end64, const float *group_lr,
                              const float *group_wd, int n_groups, void *stream)
{
    if (levels == 0) return LC_ERR_RANGE;
    AggCall c;
    c.q = q;
    c.q_stride_bytes = q_stride_bytes;
    c.in_bits = 8;
    c.W = W;
    c.n = n;
    c.levels = levels;
    c.sum_out = sum_out;
    c.step = step;
    c.tie_rule = tie_rule;
    c.apply = true;
    c.theta = theta;
    set_groups(c, group_end64, group_lr, group_wd, n_groups);
    c.stream = stream;
    return aggregate(c);
}

int lc_local_update_pack_ternary(const void *g, size_t g_stride_elems, int g_dtype, float *m, size_t m_stride_elems, int W,
                                 size_t n, float beta1, int update_m, float beta2, uint64_t *pos, uint64_t *nz,
                                 size_t q_stride_words, void *stream)
{
    if (W < 1 || W > LC_MAX_W || n > LC_MAX_N) return LC_ERR_SIZE;
    const int rc = check_mg(m, m_stride_elems, g, g_stride_elems, g_dtype, W);
    if (rc) return rc;
    if (!pos || !nz) return LC_ERR_NULL;
    if (!aligned(pos, 8) || !aligned(nz, 8)) return LC_ERR_ALIGN;
    if (n == 0) return LC_OK;
    return from_hip(launch_local_update_pack_ternary(g, g_stride_elems, g_dtype, m, m_stride_elems, W, n, beta1,
                                                     update_m != 0, beta2, pos, nz, q_stride_words,
                                                     static_cast<hipStream_t>(stream)));
}

int lc_vote_ternary(const uint64_t *pos, const uint64_t *nz, size_t q_stride_words, int W, size_t n, uint64_t *vote_pos,
                    uint64_t *vote_nz, void *stream)
{
    AggCall c;
    c.q = pos;
    c.q2 = nz;
    c.q_stride_bytes = q_stride_words * 8;
    c.in_bits = 16;
    c.W = W;
    c.n = n;
    c.vote_pos = vote_pos;
    c.vote_nz = vote_nz;
    c.stream = stream;
    return aggregate(c);
}

int lc_vote_apply_ternary(const uint64_t *pos, const uint64_t *nz, size_t q_stride_words, int W, size_t n, float *theta,
                          float lr, float wd, float *m, size_t m_stride_elems, const void *g, size_t g_stride_elems,
                          int g_dtype, int n_m, float beta2, void *stream)
{
    AggCall c;
    c.q = pos;
    c.q2 = nz;
    c.q_stride_bytes = q_stride_words * 8;
    c.in_bits = 16;
    c.W = W;
    c.n = n;
    c.apply = true;
    c.theta = theta;
    c.lr = lr;
    c.wd = wd;
    set_streams(c, m, m_stride_elems, g, g_stride_elems, g_dtype, n_m, beta2);
    c.stream = stream;
    return aggregate(c);
}

int lc_momentum_divergence(const float *m, size_t m_stride_elems, int W, size_t n, double *max_std, void *stream)
{
    if (W < 1 || W > LC_MAX_W || n > LC_MAX_N) return LC_ERR_SIZE;
    if (!m || !max_std) return LC_ERR_NULL;
    if (!aligned(m, 16) || (W > 1 && (m_stride_elems * 4) % 16 != 0) || !aligned(max_std, 8)) return LC_ERR_ALIGN;
    return from_hip(launch_momentum_divergence(m, m_stride_elems, W, n, max_std, nullptr, 0, static_cast<hipStream_t>(stream)));
}

int lc_momentum_divergence_groups(const float *m, size_t m_stride_elems, int W, size_t n, const uint32_t *group_end64,
                                  int n_groups, double *max_std, void *stream)
{
    if (W < 1 || W > LC_MAX_W || n > kMaxGroupedN || n_groups < 1 || n_groups > LC_MAX_GROUPS) return LC_ERR_SIZE;
    if (!m || !max_std || !group_end64) return LC_ERR_NULL;
    if (!aligned(m, 16) || (W > 1 && (m_stride_elems * 4) % 16 != 0) || !aligned(max_std, 8) || !aligned(group_end64, 4))
        return LC_ERR_ALIGN;
    return from_hip(launch_momentum_divergence(m, m_stride_elems, W, n, max_std, group_end64, n_groups,
                                               static_cast<hipStream_t>(stream)));
}

int lc_momentum_sync_ranges(float *m, size_t m_stride_elems, int W, const size_t *offsets, const size_t *sizes, int n_ranges,
                            uint64_t step, uint64_t every, void *stream)
{
    if (W < 1 || W > LC_MAX_W || n_ranges < 0) return LC_ERR_SIZE;
    if (every == 0) return LC_ERR_MODE;
    if (!m || (n_ranges > 0 && (!offsets || !sizes))) return LC_ERR_NULL;
    if (!aligned(m, 16) || (W > 1 && (m_stride_elems * 4) % 16 != 0)) return LC_ERR_ALIGN;
    for (int r = 0; r < n_ranges; ++r) {
        if (offsets[r] % 4 != 0) return LC_ERR_ALIGN;
        if (sizes[r] > LC_MAX_N) return LC_ERR_SIZE;
    }
    if (step % every != 0 || W == 1) return LC_OK;  // not a synchronisation step
    return from_hip(launch_momentum_avg_ranges(m, m_stride_elems, W, offsets, sizes, n_ranges, static_cast<hipStream_t>(stream)));
}

int lc_vote_apply_1bit_groups(const uint64_t *q, size_t q_stride_words, int W, size_t n, uint64_t step, int tie_rule,
                              float *theta, const uint32_t *group_end64, const float *group_lr, const float *group_wd,
                              int n_groups, void *stream)
{
    AggCall c;
    c.q = q;
    c.q_stride_bytes = q_stride_words * 8;
    c.in_bits = 1;
    c.W = W;
    c.n = n;
    c.step = step;
    c.tie_rule = tie_rule;
    c.apply = true;
    c.theta = theta;
    set_groups(c, group_end64, group_lr, group_wd, n_groups);
    c.stream = stream;
    return aggregate(c);
}

int lc_pbit_sum_apply_groups(const void *q, size_t q_stride_bytes, int in_bits, int W, size_t n, int p, void *sum_out,
                             uint64_t step, int tie_rule, float *theta, const uint32_t *group_end64, const float *group_lr,
                             const float *group_wd, int n_groups, void *stream)
{
    if (p == 0) return LC_ERR_RANGE;
    AggCall c;
    c.q = q;
    c.q_stride_bytes = q_stride_bytes;
    c.in_bits = in_bits;
    c.W = W;
    c.n = n;
    c.p = p;
    c.sum_out = sum_out;
    c.step = step;
    c.tie_rule = tie_rule;
    c.apply = true;
    c.theta = theta;
    set_groups(c, group_end64, group_lr, group_wd, n_groups);
    c.stream = stream;
    return aggregate(c);
}

int lc_vote_apply_ternary_groups(const uint64_t *pos, const uint64_t *nz, size_t q_stride_words, int W, size_t n,
                                 float *theta, const uint32_t *group_end64, const float *group_lr, const float *group_wd,
                                 int n_groups, void *stream)
{
    AggCall c;
    c.q = pos;
    c.q2 = nz;
    c.q_stride_bytes = q_stride_words * 8;
    c.in_bits = 16;
    c.W = W;
    c.n = n;
    c.apply = true;
    c.theta = theta;
    set_groups(c, group_end64, group_lr, group_wd, n_groups);
    c.stream = stream;
    return aggregate(c);
}

int lc_container_bits(int p) { return container(p); }

const char *lc_status_string(int status)
{
    switch (status) {
    case LC_OK: return "LC_OK";
    case LC_ERR_NULL: return "LC_ERR_NULL: a required pointer is NULL";
    case LC_ERR_SIZE: return "LC_ERR_SIZE: worker, row, group or element count out of range";
    case LC_ERR_ALIGN: return "LC_ERR_ALIGN: pointer or row stride misaligned";
    case LC_ERR_RANGE: return "LC_ERR_RANGE: the sums would not fit their fields (p outside 1..8, W > 2^p - 1, 2 L W > 255 or total too large)";
    case LC_ERR_DTYPE: return "LC_ERR_DTYPE: unknown gradient dtype";
    case LC_ERR_MODE: return "LC_ERR_MODE: unknown rule or bit width";
    default: return status < 0 ? "HIP runtime error (status = -hipError_t)" : "unknown status";
    }
}

int lc_stream_probe(int kind, float *a, const float *b, size_t n, float s, void *stream)
{
    if (kind < LC_PROBE_READ || kind > LC_PROBE_RMW2) return LC_ERR_MODE;
    if (n > LC_MAX_N) return LC_ERR_SIZE;
    if (!a || ((kind == LC_PROBE_COPY || kind == LC_PROBE_RMW2) && !b)) return LC_ERR_NULL;
    if (!aligned(a, 16) || !aligned(b, 16)) return LC_ERR_ALIGN;
    if (n == 0) return LC_OK;
    return from_hip(launch_stream_probe(kind, a, b, n, s, static_cast<hipStream_t>(stream)));
}

int lc_version(void) { return 100; }

}  // extern "C"
