/*
 * lioncub.h -- C ABI of the MI355X (gfx950) library for the data-parallel hot path of
 * Lion Cub's compressed update step ("Lion Cub: Minimizing Communication Overhead for
 * Distributed Lion", arXiv 2411.16462; Algorithm 1 and Section 3).
 *
 * W simulated workers live on one GPU as W rows of gradient / momentum / packed-sign
 * buffers in device memory; the W-way aggregation is the local reduction that one
 * GPU performs on its share after the exchange of Section 3.
 *
 * Conventions that hold for every entry point
 *  - All data pointers are DEVICE pointers owned by the caller.  The library allocates
 *    nothing, keeps no state between calls (lc_l1_mean_abs_static alone uses a static
 *    device array of its own, see there), never frees or retains caller memory and
 *    never synchronises.  `stream` is a hipStream_t passed as void* (NULL = the null
 *    stream); every call only enqueues kernels on it and returns.
 *  - Row w of a per-worker buffer starts at base + w * stride.
 *  - theta and m are fp32.  g is fp32 (LC_F32) or bfloat16 (LC_BF16, widened exactly).
 *  - n counts the elements of one contiguous range (a flat arena, as the paper
 *    consolidates all gradients into one tensor, or one tensor of it).  n = 0 is a
 *    successful no-op.  A range handed to separate calls must start at an element
 *    offset that is a multiple of 64 so that packed words do not straddle calls.
 *  - 1-bit layout: element i is bit (i mod 64) of 64-bit word floor(i/64), least
 *    significant bit first -- the order of a wave64 lane mask.  ceil(n/64) words per
 *    row; bits past n in the last word are written as 0 and ignored on input.
 *  - p-bit layout (Appendix F.1: sub-byte entries are packed into a uint8 and the width
 *    must divide the container): a value of p bits sits in a field of C = 1, 2, 4 or 8
 *    bits, the smallest that holds p (p = 7 -> one byte).  Element i is field
 *    (i mod 8/C) of byte floor(i*C/8), low bits first; ceil(n*C/8) bytes per row; pad
 *    fields are written as 0.  Bytes past that count are neither read nor written.
 *  - Alignment: theta, m, g, field buffers and sum_out: base and every row 16-byte
 *    aligned.  1-bit buffers and vote planes: 8-byte aligned.  (Speed, not correctness:
 *    rows that start a large power of two apart -- a row stride of exactly 64 MiB, say --
 *    fall on the same memory channels; measured with 64 rows that costs a fifth of the
 *    bandwidth; pad the stride in that case.  And the float rows stream best when their
 *    stride is a multiple of 1 KiB, so that every 256-element tile of every row is aligned
 *    alike: measured 4 % on lc_momentum_avg with 16 rows.  So pad to a multiple of 1 KiB
 *    that is not a multiple of a large power of two.  1-bit rows: an odd number of 128-byte
 *    lines per row for up to 24 rows, an odd number of 64-byte units for 32 and more.)
 *  - `step` is the caller's 1-based iteration counter; only its parity is used, by the
 *    alternating rule of Appendix B.1 (zero -> +1 on odd iterations, -1 on even ones).
 *  - Buffers named in one call must not overlap each other.
 *  - Return value: LC_OK, or a positive LC_ERR_* found on the host before anything was
 *    launched (nothing was written), or -(hipError_t) if a launch failed.  The status is
 *    that of this call's own launches: an error that an earlier, unrelated HIP call of
 *    the host program left pending is neither reported here nor cleared.
 *  - Thread safety: re-entrant; calls on different streams may run concurrently as
 *    long as their buffers are disjoint.
 */
#ifndef LIONCUB_H
#define LIONCUB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LC_MAX_W 255 /* most workers one aggregation call accepts (counts fit 8 bits) */
#define LC_MAX_GROUPS (1 << 20) /* most parameter groups a *_groups call accepts */
#define LC_MAX_N ((size_t)1 << 38) /* most elements per row one call accepts */

enum {
    LC_OK = 0,
    LC_ERR_NULL = 1,  /* a required pointer is NULL                                      */
    LC_ERR_SIZE = 2,  /* W, n_m, n_groups or n (> LC_MAX_N) out of range                 */
    LC_ERR_ALIGN = 3, /* a base pointer or a row stride breaks the alignment rules       */
    LC_ERR_RANGE = 4, /* the sums would not fit their fields: p outside 1..8, W > 2^p - 1,
                         levels outside 1..127, 2 L W > 255, total > 2^field_bits - 1      */
    LC_ERR_DTYPE = 5, /* unknown gradient dtype                                          */
    LC_ERR_MODE = 6   /* unknown rule, out_bits / in_bits not one of the allowed widths  */
};
enum { LC_F32 = 0, LC_BF16 = 1 };
/* What an exact zero of sign(c) becomes when it has to fit one bit (Section 3 "forcing
 * 0 to be one or the other"; Appendix B.1 alternates by iteration parity). */
enum { LC_ZERO_ALT = 0, LC_ZERO_POS = 1, LC_ZERO_NEG = 2 };
/* What a tied vote becomes: 0 (the sign of a zero sum, Algorithm 1 line 5; needs the
 * nz plane), or the alternating sign of Appendix B.1 (fits one bit again). */
enum { LC_TIE_ZERO = 0, LC_TIE_ALT = 1 };

/* Algorithm 1 lines 3 and 6 plus the quantiser Q = sign, for all W workers in one
 * launch: c = beta1 * m_w + (1 - beta1) * g_w in fp32 as fma(beta1, m, fl((1-beta1)*g));
 * bit = 1 if c > 0, 0 if c < 0, the zero rule's bit if c == 0 (or NaN).
 *   out_bits = 1: q row w receives the 1-bit words.  out_bits = 2, 4, 8: the bit is
 *   stored as a 0/1 value in fields of that many bits ({-1,+1} -> {0,1}, Appendix F.1).
 *   q = NULL skips the packed output (then update_m must be set).
 *   update_m != 0: m_w <- beta2 * m_w + (1 - beta2) * g_w in place, from the same loads
 *   (line 6 reads the momentum line 3 read, so fusing changes no result).
 * g: rows of g_dtype, read only.  m: rows of fp32, read (and written if update_m). */
int lc_local_update_pack(const void *g, size_t g_stride_elems, int g_dtype,
                         float *m, size_t m_stride_elems, int W, size_t n, float beta1,
                         int update_m, float beta2, int out_bits, void *q,
                         size_t q_stride_bytes, uint64_t step, int zero_rule, void *stream);

/* Section 3, local part of the 1-bit compressed allreduce, and Appendix A.1: majority
 * vote over W 1-bit rows.  K_i = number of rows with bit i set, S_i = 2 K_i - W,
 * u_i = sign(S_i), a tie following tie_rule.  Output: two planes in the 1-bit layout,
 * vote_pos bit = (u > 0), vote_nz bit = (u != 0); either may be NULL. */
int lc_vote_1bit(const uint64_t *q, size_t q_stride_words, int W, size_t n,
                 uint64_t *vote_pos, uint64_t *vote_nz, uint64_t step, int tie_rule,
                 void *stream);

/* Section 3 "direct allreduce" / Appendix F.1: the p-bit sum of the workers' 0/1 signs,
 * then the sign of the sum of signs.  Requires 1 <= p <= 8 and W <= 2^p - 1.
 *   in_bits = container(p): q rows are p-bit field buffers; they are added field-wise.
 *   in_bits = 1:            q rows are 1-bit buffers (q_stride_bytes a multiple of 8).
 *   sum_out (may be NULL): K as container(p)-bit fields, ceil(n*C/8) bytes.
 *   vote_pos / vote_nz (may be NULL): as in lc_vote_1bit. */
int lc_pbit_sum_sign(const void *q, size_t q_stride_bytes, int in_bits, int W, size_t n,
                     int p, void *sum_out, uint64_t *vote_pos, uint64_t *vote_nz,
                     uint64_t step, int tie_rule, void *stream);

/* Algorithm 1 line 5 (read as Lion's decoupled weight decay) and line 6:
 *   theta <- theta - lr * (u + wd * theta), u from the planes (vote_nz = NULL: every
 *   element is non-zero, u = +1 where the pos bit is set and -1 elsewhere);
 *   for w < n_m: m_w <- beta2 * m_w + (1 - beta2) * g_w.  n_m = 0 leaves m and g unused
 *   (they may be NULL). */
int lc_apply_update(float *theta, const uint64_t *vote_pos, const uint64_t *vote_nz,
                    size_t n, float lr, float wd, float *m, size_t m_stride_elems,
                    const void *g, size_t g_stride_elems, int g_dtype, int n_m,
                    float beta2, void *stream);

/* The step after a SUMMING allreduce (Section 3 "direct allreduce"; Appendix F.1): the
 * fields were added across all workers by the collective, so one buffer of sums K arrives
 * (field layout as above, field_bits = 2, 4 or 8) together with the number they have to
 * be compared with: u = sign(2 K - total).  total = W for sums of 0/1 signs; total =
 * 2 W L for sums of L1 level bytes (S = K - W L).  Needs 1 <= total <= 2^field_bits - 1
 * (else LC_ERR_RANGE).  A tie (2 K = total) follows tie_rule.  Then theta, and the
 * momentum rows if n_m > 0, as in lc_apply_update. */
int lc_count_apply(const void *k_fields, int field_bits, size_t n, int total, uint64_t step,
                   int tie_rule, float *theta, float lr, float wd, float *m,
                   size_t m_stride_elems, const void *g, size_t g_stride_elems, int g_dtype,
                   int n_m, float beta2, void *stream);

/* Section 5, momentum synchronisation: every row becomes the mean of the W rows (what
 * an averaging allreduce leaves on every worker).  The W values of an element are summed
 * in fp32 (partial sums over interleaved subsets of the rows, then their sum), and the
 * total is multiplied once by 1/W; every row receives the same bits. */
int lc_momentum_avg(float *m, size_t m_stride_elems, int W, size_t n, void *stream);

/* Section 5.1, the quantity plotted per layer in Figure 6: the largest, over the n elements,
 * standard deviation of an element's W momentum values across workers (divisor W).
 * Evaluated in fp64, workers in order; *max_std (one double on the device) is written. */
int lc_momentum_divergence(const float *m, size_t m_stride_elems, int W, size_t n,
                           double *max_std, void *stream);

/* The same quantity for every parameter group in one launch (Figure 6 plots it per layer):
 * max_std[s] (n_groups doubles on the device) is the maximum over segment s of the group
 * table (as in lc_vote_apply_1bit_groups; device array); an empty segment gives 0. */
int lc_momentum_divergence_groups(const float *m, size_t m_stride_elems, int W, size_t n,
                                  const uint32_t *group_end64, int n_groups, double *max_std,
                                  void *stream);

/* Section 5 / 6.2, the policy the paper recommends: synchronise the momenta of selected
 * layers only, every `every` iterations (e.g. head and embedding, every 10).  If step is a
 * multiple of `every`, every range [offsets[r], offsets[r] + sizes[r]) of the rows receives
 * what lc_momentum_avg gives on it, bit for bit; otherwise nothing happens.  offsets and
 * sizes are HOST arrays of n_ranges entries (element units; offsets multiples of 4; sizes
 * may be 0), read before the call returns; every >= 1.  The ranges travel in the kernel
 * arguments, 32 to a launch, and must not overlap: ranges of one launch run side by side. */
int lc_momentum_sync_ranges(float *m, size_t m_stride_elems, int W, const size_t *offsets,
                            const size_t *sizes, int n_ranges, uint64_t step, uint64_t every,
                            void *stream);

/* Fused forms: lc_vote_1bit followed by lc_apply_update without writing the planes. */
int lc_vote_apply_1bit(const uint64_t *q, size_t q_stride_words, int W, size_t n,
                       uint64_t step, int tie_rule, float *theta, float lr, float wd,
                       float *m, size_t m_stride_elems, const void *g,
                       size_t g_stride_elems, int g_dtype, int n_m, float beta2,
                       void *stream);

/* lc_vote_apply_1bit with per-group learning rates and weight decays (Appendix F.3 scales
 * the rate of the head, embedding and scalar parameter groups) in ONE launch over the
 * whole arena: the range is cut into n_groups consecutive segments; segment s ends at
 * element 64 * group_end64[s] (ascending; the last end must reach n) and uses
 * group_lr[s], group_wd[s].  The three arrays live on the DEVICE (they are static for a
 * model: upload once).  No momentum streams (the signature has none: momenta are updated
 * by lc_local_update_pack, or by the forms without a group table).  One call per tensor
 * gives the same result but is launch-bound for small tensors.
 * Group tables in every *_groups call: n_groups in 1..LC_MAX_GROUPS, and n at most
 * 64 * (2^32 - 1) elements (ends are 32-bit), else LC_ERR_SIZE.  The table itself lives on
 * the device and is not validated.  Every kernel resolves it by one rule: a 64-element
 * block belongs to the first segment whose end lies beyond it, and to the last segment if
 * there is none -- so a last end short of n extends to n, and ends beyond n mean n.  A
 * table whose ends do not ascend is not detected; which segment an element then falls in
 * is unspecified (all accesses stay inside the caller's buffers). */
int lc_vote_apply_1bit_groups(const uint64_t *q, size_t q_stride_words, int W, size_t n,
                              uint64_t step, int tie_rule, float *theta,
                              const uint32_t *group_end64, const float *group_lr,
                              const float *group_wd, int n_groups, void *stream);

/* lc_pbit_sum_sign followed by lc_apply_update without writing the planes; sum_out as
 * in lc_pbit_sum_sign (may be NULL). */
int lc_pbit_sum_apply(const void *q, size_t q_stride_bytes, int in_bits, int W, size_t n,
                      int p, void *sum_out, uint64_t step, int tie_rule, float *theta,
                      float lr, float wd, float *m, size_t m_stride_elems, const void *g,
                      size_t g_stride_elems, int g_dtype, int n_m, float beta2,
                      void *stream);

/* lc_pbit_sum_apply with per-group learning rates and weight decays, group arrays as in
 * lc_vote_apply_1bit_groups; no momentum streams. */
int lc_pbit_sum_apply_groups(const void *q, size_t q_stride_bytes, int in_bits, int W, size_t n,
                             int p, void *sum_out, uint64_t step, int tie_rule, float *theta,
                             const uint32_t *group_end64, const float *group_lr,
                             const float *group_wd, int n_groups, void *stream);

/* ---- Ternary ("2-bit") wire format: exact zeros travel (Appendix B.1) ------------------
 * The worker's sign s = sign(c) in {-1, 0, +1} is sent unchanged as two 1-bit planes per
 * worker, pos (s > 0) and nz (s != 0), nothing is forced; the update is the sign of the
 * plain sum of the signs, S = K+ - K-, and a zero sum is 0.  Rows of pos and of nz share
 * one stride (in 64-bit words); 1-bit layout as above. */
int lc_local_update_pack_ternary(const void *g, size_t g_stride_elems, int g_dtype, float *m,
                                 size_t m_stride_elems, int W, size_t n, float beta1,
                                 int update_m, float beta2, uint64_t *pos, uint64_t *nz,
                                 size_t q_stride_words, void *stream);

/* K+ = rows with pos set, K- = rows with nz set and pos clear; u = sign(K+ - K-) as the
 * two planes vote_pos / vote_nz (either may be NULL).  A pos bit without its nz bit is
 * ignored. */
int lc_vote_ternary(const uint64_t *pos, const uint64_t *nz, size_t q_stride_words, int W,
                    size_t n, uint64_t *vote_pos, uint64_t *vote_nz, void *stream);

/* lc_vote_ternary followed by lc_apply_update without writing the planes. */
int lc_vote_apply_ternary(const uint64_t *pos, const uint64_t *nz, size_t q_stride_words, int W,
                          size_t n, float *theta, float lr, float wd, float *m,
                          size_t m_stride_elems, const void *g, size_t g_stride_elems,
                          int g_dtype, int n_m, float beta2, void *stream);

/* lc_vote_apply_ternary with per-group learning rates and weight decays, group arrays as
 * in lc_vote_apply_1bit_groups; no momentum streams. */
int lc_vote_apply_ternary_groups(const uint64_t *pos, const uint64_t *nz, size_t q_stride_words,
                                 int W, size_t n, float *theta, const uint32_t *group_end64,
                                 const float *group_lr, const float *group_wd, int n_groups,
                                 void *stream);

/* ---- L1-quantised updates (Section 4.2, Equation 1 with p = 1; Appendix F.1) ---------
 * Q_1(x)_i = clamp(round(L / (2 M_1(x)) * x_i), L) with M_1(x) = mean_j |x_j| and
 * L = 2^(bits-1) - 1 levels on each side of zero (the paper's 8-bit allreduce among 8
 * workers uses L = 15).  x is the worker's interpolation c of Algorithm 1 line 3, and
 * M_1 is taken over the n elements of the call (one call per tensor gives per-tensor
 * scales).  A level travels as the byte level + L in [0, 2L]; the W bytes of an element
 * are added as integers, which needs 2 L W <= 255 (else LC_ERR_RANGE); the update is the
 * sign of the summed levels, S = K - W L. */

#define LC_L1_WORKSPACE_WORDS 384 /* uint64 words of device workspace per worker */

/* First pass: mean_abs[w] = M_1(c_w), fp64.  The sum of |c| is formed without rounding
 * (as a long integer, whatever the order of the additions), rounded once to fp64 and
 * divided by n, so the result is reproducible bit for bit.  workspace: device buffer of
 * W * LC_L1_WORKSPACE_WORDS uint64, overwritten.  mean_abs: W doubles on the device.
 * n = 0 gives 0.  Inputs must be finite (a NaN or infinity makes mean_abs meaningless). */
int lc_l1_mean_abs(const void *g, size_t g_stride_elems, int g_dtype, const float *m,
                   size_t m_stride_elems, int W, size_t n, float beta1, double *mean_abs,
                   uint64_t *workspace, void *stream);

/* lc_l1_mean_abs for callers that cannot allocate device memory or bring a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * workspace is a static device array inside the library (LC_L1_STATIC_MAX_W *
 * LC_L1_WORKSPACE_WORDS uint64 = 192 KiB, held by every GPU the library runs on until the
 * process ends), so the call takes inputs and outputs only and calls no allocating
 * routine.  W > LC_L1_STATIC_MAX_W is refused with LC_ERR_SIZE; everything else, results
 * included, is as in lc_l1_mean_abs.  The first call on a device looks the array's address
 * up (make one call, n = 0 will do, before capturing a graph on that device); the
 * device that owns `stream` must be the current one.  All calls on one GPU share that
 * GPU's array: it is cleared at the start of every call, and two calls that overlap in
 * time on one GPU (different streams, or different host threads without ordering) race
 * and give wrong means -- order them on one stream or with events. */
#define LC_L1_STATIC_MAX_W 64
int lc_l1_mean_abs_static(const void *g, size_t g_stride_elems, int g_dtype, const float *m,
                          size_t m_stride_elems, int W, size_t n, float beta1, double *mean_abs,
                          void *stream);

/* Per-group scales in one call (a scale per parameter tensor, as when each tensor is
 * quantised on its own): the range is cut into n_groups consecutive segments as in
 * lc_vote_apply_1bit_groups (segment s ends at element 64 * group_end64[s], ascending, the
 * last end reaches n; a segment may be empty), and mean_abs[w * n_groups + s] receives
 * M_1 of worker w over segment s, formed exactly as in lc_l1_mean_abs.  group_count
 * (device, n_groups uint64, may be NULL): the number of elements that the sum of segment
 * s is divided by -- the tensor's true size when the arena pads tensors with zeros up to
 * a multiple of 64; NULL divides by the segment's length.  A count or length of 0 gives
 * 0.  workspace: lc_l1_groups_workspace_words(W, n_groups) uint64 on the device,
 * overwritten.  group_end64 and group_count live on the DEVICE. */
size_t lc_l1_groups_workspace_words(int W, int n_groups); /* utility, host only; 0 if an argument is < 1 */
int lc_l1_mean_abs_groups(const void *g, size_t g_stride_elems, int g_dtype, const float *m,
                          size_t m_stride_elems, int W, size_t n, float beta1,
                          const uint32_t *group_end64, const uint64_t *group_count,
                          int n_groups, double *mean_abs, uint64_t *workspace, void *stream);

/* Second pass: the scale L / (2 mean_abs[w]) is rounded to fp32, multiplied with c in
 * fp32, rounded to the nearest integer (ties to even), clamped to [-L, L] and stored as
 * the byte level + L: q row w receives n bytes.  mean_abs[w] = 0 (all of c is zero) gives
 * level 0 everywhere.  update_m as in lc_local_update_pack.  levels = L in 1..127. */
int lc_l1_quantize_pack(const void *g, size_t g_stride_elems, int g_dtype, float *m,
                        size_t m_stride_elems, int W, size_t n, float beta1, int update_m,
                        float beta2, int levels, const double *mean_abs, uint8_t *q,
                        size_t q_stride_bytes, void *stream);

/* lc_l1_quantize_pack with the scale of element i taken from mean_abs[w * n_groups + s]
 * for the segment s that holds i (mean_abs as lc_l1_mean_abs_groups wrote it). */
int lc_l1_quantize_pack_groups(const void *g, size_t g_stride_elems, int g_dtype, float *m,
                               size_t m_stride_elems, int W, size_t n, float beta1,
                               int update_m, float beta2, int levels,
                               const uint32_t *group_end64, int n_groups,
                               const double *mean_abs, uint8_t *q, size_t q_stride_bytes,
                               void *stream);

/* Sum of the W level bytes per element (sum_out, n bytes, may be NULL), and the sign of
 * the summed levels as vote planes; a zero sum follows tie_rule. */
int lc_level_sum_sign(const uint8_t *q, size_t q_stride_bytes, int W, size_t n, int levels,
                      uint8_t *sum_out, uint64_t *vote_pos, uint64_t *vote_nz, uint64_t step,
                      int tie_rule, void *stream);

/* lc_level_sum_sign followed by lc_apply_update without writing the planes. */
int lc_level_sum_apply(const uint8_t *q, size_t q_stride_bytes, int W, size_t n, int levels,
                       uint8_t *sum_out, uint64_t step, int tie_rule, float *theta, float lr,
                       float wd, float *m, size_t m_stride_elems, const void *g,
                       size_t g_stride_elems, int g_dtype, int n_m, float beta2, void *stream);

/* lc_level_sum_apply with per-group learning rates and weight decays, group arrays as in
 * lc_vote_apply_1bit_groups; no momentum streams. */
int lc_level_sum_apply_groups(const uint8_t *q, size_t q_stride_bytes, int W, size_t n,
                              int levels, uint8_t *sum_out, uint64_t step, int tie_rule,
                              float *theta, const uint32_t *group_end64,
                              const float *group_lr, const float *group_wd, int n_groups,
                              void *stream);

/* ---- Utilities (they follow no passage of the paper) -----------------------------------
 * lc_container_bits, lc_status_string, lc_version and lc_l1_groups_workspace_words above
 * touch no device memory and launch nothing; lc_stream_probe launches one bare streaming
 * kernel, a calibration aid for measurements. */

/* What this device reaches when a kernel only moves data, in the shape of the library's
 * streaming kernels (one wave per 256-element tile, 16-byte non-temporal accesses).  a and b
 * are device arrays of n floats, 16-byte aligned, not overlapping.  kind: */
#define LC_PROBE_READ 0   /* reads a, writes nothing                       4 n bytes */
#define LC_PROBE_WRITE 1  /* a[i] = s                                      4 n bytes */
#define LC_PROBE_COPY 2   /* a[i] = b[i]                                   8 n bytes */
#define LC_PROBE_SCALE 3  /* a[i] = a[i] * s, in place                     8 n bytes */
#define LC_PROBE_RMW2 4   /* a[i] = fma(s, a[i], fl(fl(1 - s) * b[i])): two streams read, one of
                             them written in place, update+pack without the packing  12 n bytes */
/* b may be NULL for READ, WRITE and SCALE.  Errors as for the other calls. */
int lc_stream_probe(int kind, float *a, const float *b, size_t n, float s, void *stream);

/* Smallest field width of 1, 2, 4, 8 bits that holds a p-bit value (the container rule of
 * the p-bit layout above); -1 if p is not in 1..8. */
int lc_container_bits(int p);

/* Static, human-readable name of a status code returned by the calls above. */
const char *lc_status_string(int status);

/* Library version as major * 10000 + minor * 100 + patch. */
int lc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LIONCUB_H */
