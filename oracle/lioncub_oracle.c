/*
 * lioncub_oracle.c -- plain CPU oracle for the Lion Cub compressed-update hot path.
 *
 * TEST INFRASTRUCTURE, NOT PRODUCT.  Only the test-suite, the smoke check and the
 * benchmark's "cpu_baseline" leg may build, load or call this file.  It shares no
 * code, header, table or helper with the HIP library and is never used as a fallback
 * for it.
 *
 * Every function is the paper's definition written out one element at a time:
 * no blocking, no bit tricks, no fusion, one loop per step, so that it can be
 * checked against the paper by eye.  Citations name the passage of
 * "Lion Cub: Minimizing Communication Overhead for Distributed Lion"
 * (arXiv 2411.16462) that each step follows.
 *
 * Precision.  The paper does not fix one.  Outputs that are real numbers (updated
 * parameters, momenta, averaged momenta) are evaluated in fp64 from the fp32 inputs.
 * The one place where floating point decides an integer -- the sign of the local
 * interpolation c (Algorithm 1, line 3) -- is taken in the precision the kernels work
 * in, fp32, with a fixed order of two roundings:
 *        t = fl32((1 - beta1) * g),   c = fl32(beta1 * m + t)   (a fused multiply-add)
 * where (1 - beta1) is itself formed in fp32.  orc_local_sign_exact() gives the sign
 * of the same expression without any rounding of products or sums, so that a test can
 * count how often the two differ.
 *
 * Build: gcc -O2 -ffp-contract=off -fPIC -shared (see oracle/build.py).  Contraction
 * is switched off so that the only fused operation is the one written as fmaf().
 *
 * Every function here is pinned by tests/test_oracle_*.py (hand-enumerated case,
 * exact rational arithmetic, closed forms, invariants, brute force).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

enum { ORC_OK = 0, ORC_ERR_RANGE = 4, ORC_ERR_ARG = 7 };
enum { ORC_F32 = 0, ORC_BF16 = 1 };
enum { ORC_ZERO_ALT = 0, ORC_ZERO_POS = 1, ORC_ZERO_NEG = 2 };
enum { ORC_TIE_ZERO = 0, ORC_TIE_ALT = 1 };

/* bfloat16 is the upper half of an IEEE binary32: widening it is exact. */
float orc_bf16_to_f32(uint16_t h)
{
    uint32_t bits = (uint32_t)h << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return f;
}

static float grad_at(const void *g, int g_dtype, size_t i)
{
    if (g_dtype == ORC_BF16)
        return orc_bf16_to_f32(((const uint16_t *)g)[i]);
    return ((const float *)g)[i];
}

/* The bit that stands for an exact zero on iteration `step` (1-based).
 * Appendix B.1 ("alternating sign"): zero becomes +1 on odd iterations and -1 on
 * even ones before the value is compressed to one bit.  Section 3 only says that
 * zero is forced to one side; POS / NEG are those fixed choices. */
static int zero_bit(uint64_t step, int rule)
{
    if (rule == ORC_ZERO_POS) return 1;
    if (rule == ORC_ZERO_NEG) return 0;
    return (step % 2u == 1u) ? 1 : 0;
}

/* ---- Algorithm 1, line 3, followed by the sign that Q applies ------------------
 * c_i = beta1 * m_i + (1 - beta1) * g_i ;  s_i = sign(c_i) in {-1, 0, +1}.
 * The sign is a comparison, not the sign bit: -0.0 and NaN give 0. */
void orc_local_sign(const float *m, const void *g, int g_dtype, size_t n,
                    float beta1, int8_t *s)
{
    const float omb1 = 1.0f - beta1;
    for (size_t i = 0; i < n; ++i) {
        const float gf = grad_at(g, g_dtype, i);
        const float t = omb1 * gf;
        const float c = fmaf(beta1, m[i], t);
        s[i] = (int8_t)((c > 0.0f) - (c < 0.0f));
    }
}

/* Same expression, same fp32 constants beta1 and fl32(1 - beta1), but with the
 * products and the sum carried without rounding error that could touch the sign:
 * a product of two binary32 values is exact in binary64, and the rounded sum of two
 * binary64 values has the sign of their exact sum.  Diagnostic only. */
void orc_local_sign_exact(const float *m, const void *g, int g_dtype, size_t n,
                          float beta1, int8_t *s)
{
    const float omb1 = 1.0f - beta1;
    for (size_t i = 0; i < n; ++i) {
        const double a = (double)beta1 * (double)m[i];
        const double b = (double)omb1 * (double)grad_at(g, g_dtype, i);
        const double c = a + b;
        s[i] = (int8_t)((c > 0.0) - (c < 0.0));
    }
}

/* ---- Section 3 / Appendix B.1: a ternary sign becomes one bit -------------------
 * {-1, +1} -> {0, 1} (Appendix F.1); an exact zero takes zero_bit(). */
void orc_zero_rule(const int8_t *s, size_t n, uint64_t step, int zero_rule, uint8_t *b)
{
    const int z = zero_bit(step, zero_rule);
    for (size_t i = 0; i < n; ++i) {
        if (s[i] > 0) b[i] = 1;
        else if (s[i] < 0) b[i] = 0;
        else b[i] = (uint8_t)z;
    }
}

/* ---- 1-bit representation (Section 3, "1-bit compressed allreduce") ------------
 * Element i is bit (i mod 64) of 64-bit word floor(i / 64), least significant bit
 * first.  Bits past n in the last word are zero.  (The paper does not give a bit
 * order; this one is the reading the library documents.) */
void orc_pack_1bit(const uint8_t *b, size_t n, uint64_t *words)
{
    const size_t nw = (n + 63) / 64;
    for (size_t j = 0; j < nw; ++j) words[j] = 0;
    for (size_t i = 0; i < n; ++i)
        if (b[i]) words[i / 64] |= (uint64_t)1 << (i % 64);
}

void orc_unpack_1bit(const uint64_t *words, size_t n, uint8_t *b)
{
    for (size_t i = 0; i < n; ++i)
        b[i] = (uint8_t)((words[i / 64] >> (i % 64)) & 1u);
}

/* ---- p-bit fields (Appendix F.1: entries are packed into a uint8 and
 * the bit width has to divide the size of the datatype) --------------------------
 * A p-bit value lives in the smallest container of 1, 2, 4 or 8 bits that holds p
 * bits (so p = 7 takes a whole byte).  Fields fill a byte from its low bits up. */
int orc_container_bits(int p)
{
    if (p < 1 || p > 8) return -1;
    if (p == 1) return 1;
    if (p == 2) return 2;
    if (p <= 4) return 4;
    return 8;
}

int orc_pack_fields(const uint8_t *v, size_t n, int p, uint8_t *bytes)
{
    const int C = orc_container_bits(p);
    if (C < 0) return ORC_ERR_RANGE;
    const size_t per = (size_t)(8 / C);
    const size_t nb = (n + per - 1) / per;
    for (size_t j = 0; j < nb; ++j) bytes[j] = 0;
    for (size_t i = 0; i < n; ++i) {
        if ((unsigned)v[i] >> C) return ORC_ERR_RANGE; /* value does not fit */
        bytes[i / per] |= (uint8_t)(v[i] << (C * (int)(i % per)));
    }
    return ORC_OK;
}

int orc_unpack_fields(const uint8_t *bytes, size_t n, int p, uint8_t *v)
{
    const int C = orc_container_bits(p);
    if (C < 0) return ORC_ERR_RANGE;
    const size_t per = (size_t)(8 / C);
    const unsigned mask = (1u << C) - 1u;
    for (size_t i = 0; i < n; ++i)
        v[i] = (uint8_t)((bytes[i / per] >> (C * (int)(i % per))) & mask);
    return ORC_OK;
}

/* ---- Algorithm 1, lines 4-5 with Q = sign: the W-way aggregation ----------------
 * b holds W rows of n bits (row w at b + w * n), each bit the {0,1} image of a
 * worker's sign.  K_i = sum_w b_{w,i} is what a summing allreduce over 0/1 values
 * leaves (Section 3, "direct allreduce": the sum lies between 0 and the number of
 * workers).  The sum of the signs themselves is S_i = 2 K_i - W, and the majority
 * vote is u_i = sign(S_i) (Appendix A.1).  A tie S_i = 0 stays 0 (what sign() gives
 * and what an allreduce that can carry zeros delivers) or, if the result must fit
 * one bit again, takes the alternating sign of Appendix B.1.
 * p > 0 asks for the range check of a p-bit sum: K can reach W, so W must not
 * exceed 2^p - 1 (four bits cannot serve sixteen workers).  p = 0: no check. */
int orc_count_sign(const uint8_t *b, int W, size_t n, int p, uint64_t step,
                   int tie_rule, int32_t *K, int32_t *S, int8_t *u)
{
    if (W < 1) return ORC_ERR_ARG;
    if (p != 0) {
        if (p < 1 || p > 8) return ORC_ERR_RANGE;
        if (W > (1 << p) - 1) return ORC_ERR_RANGE;
    }
    const int alt = (step % 2u == 1u) ? 1 : -1;
    for (size_t i = 0; i < n; ++i) {
        int32_t k = 0;
        for (int w = 0; w < W; ++w) k += b[(size_t)w * n + i];
        const int32_t sum = 2 * k - W;
        int v = (sum > 0) - (sum < 0);
        if (v == 0 && tie_rule == ORC_TIE_ALT) v = alt;
        if (K) K[i] = k;
        if (S) S[i] = sum;
        if (u) u[i] = (int8_t)v;
    }
    return ORC_OK;
}

/* A ternary update as two bit planes in the 1-bit layout above:
 * pos bit = (u > 0), nz bit = (u != 0). */
void orc_planes(const int8_t *u, size_t n, uint64_t *pos, uint64_t *nz)
{
    const size_t nw = (n + 63) / 64;
    for (size_t j = 0; j < nw; ++j) { pos[j] = 0; nz[j] = 0; }
    for (size_t i = 0; i < n; ++i) {
        if (u[i] > 0) pos[i / 64] |= (uint64_t)1 << (i % 64);
        if (u[i] != 0) nz[i / 64] |= (uint64_t)1 << (i % 64);
    }
}

void orc_unplanes(const uint64_t *pos, const uint64_t *nz, size_t n, int8_t *u)
{
    for (size_t i = 0; i < n; ++i) {
        const int p = (int)((pos[i / 64] >> (i % 64)) & 1u);
        const int z = (int)((nz[i / 64] >> (i % 64)) & 1u);
        u[i] = (int8_t)(z ? (p ? 1 : -1) : 0);
    }
}

/* ---- Algorithm 1, line 5: the parameter step -----------------------------------
 * The printed line has the decay term with the wrong sign and without the learning
 * rate; Lion's decoupled weight decay is meant:
 *      theta <- theta - eta * (u + lambda * theta).
 * fp64 from the fp32 inputs. */
void orc_apply(const float *theta, const int8_t *u, size_t n, float lr, float wd,
               double *theta_out)
{
    for (size_t i = 0; i < n; ++i) {
        const double th = (double)theta[i];
        theta_out[i] = th - (double)lr * ((double)u[i] + (double)wd * th);
    }
}

/* ---- Algorithm 1, line 6: each worker's own momentum ---------------------------
 * m <- beta2 * m + (1 - beta2) * g, from the momentum of the previous iteration
 * (the same m that line 3 read).  fp64 from the fp32 / bf16 inputs. */
void orc_momentum(const float *m, const void *g, int g_dtype, size_t n, float beta2,
                  double *m_out)
{
    const double b2 = (double)beta2;
    for (size_t i = 0; i < n; ++i)
        m_out[i] = b2 * (double)m[i] + (1.0 - b2) * (double)grad_at(g, g_dtype, i);
}

/* ---- Section 5, momentum synchronisation ---------------------------------------
 * What an averaging allreduce leaves on every worker: the mean over the W
 * momenta.  Row w starts at m + w * n.  fp64. */
void orc_momentum_avg(const float *m, int W, size_t n, double *mean_out)
{
    for (size_t i = 0; i < n; ++i) {
        double acc = 0.0;
        for (int w = 0; w < W; ++w) acc += (double)m[(size_t)w * n + i];
        mean_out[i] = acc / (double)W;
    }
}

/* ---- Appendix F.1: the p-bit allreduce is a plain integer sum over the packed
 * uint8 containers.  out[j] = sum_w bytes_w[j] (mod 256), row w at
 * bytes + w * nbytes.  When every field's total stays below 2^C no carry crosses a
 * field boundary and the result holds the per-field sums K. */
void orc_sum_bytes(const uint8_t *bytes, int W, size_t nbytes, uint8_t *out)
{
    for (size_t j = 0; j < nbytes; ++j) {
        unsigned acc = 0;
        for (int w = 0; w < W; ++w) acc += bytes[(size_t)w * nbytes + j];
        out[j] = (uint8_t)(acc & 0xFFu);
    }
}

/* ==== L1 quantisation (Section 4.2, Equation 1 with p = 1) ======================== */

/* The interpolation c of Algorithm 1 line 3 itself (same fp32 evaluation as above). */
void orc_local_c(const float *m, const void *g, int g_dtype, size_t n, float beta1, float *c)
{
    const float omb1 = 1.0f - beta1;
    for (size_t i = 0; i < n; ++i) {
        const float t = omb1 * grad_at(g, g_dtype, i);
        c[i] = fmaf(beta1, m[i], t);
    }
}

/* Sum of |x_i| without any rounding.  A finite binary32 is an integer M < 2^24 times
 * 2^(E-150) (E the biased exponent, denormals: E = 1 and no hidden bit), so the total of
 * the integers M per exponent is exact in 64 bits for any n < 2^40.  totals[E] receives
 * that integer; the caller forms sum_E totals[E] * 2^(E-150) with big integers.  Values
 * that are not finite are counted in totals[255] and make the mean undefined. */
void orc_abs_totals(const float *x, size_t n, uint64_t totals[256])
{
    for (int e = 0; e < 256; ++e) totals[e] = 0;
    for (size_t i = 0; i < n; ++i) {
        uint32_t bits;
        memcpy(&bits, &x[i], sizeof bits);
        const uint32_t e = (bits >> 23) & 0xFFu;
        const uint32_t frac = bits & 0x7FFFFFu;
        if (e == 255) totals[255] += 1;
        else if (e == 0) totals[1] += frac;
        else totals[e] += frac | 0x800000u;
    }
}

/* Equation 1 with p = 1:  Q_1(x)_i = clamp(round(L / (2 M_1) * x_i), L),  L = 2^(n-1) - 1,
 * M_1 = mean |x_j| (passed in, fp64).  The scale L / (2 M_1) is rounded once to fp32, the
 * product with x_i is one fp32 multiplication, and round() is round-half-to-even (the
 * paper does not say; it is what its PyTorch implementation's round does).  M_1 = 0 (all
 * entries zero) gives all levels 0. */
void orc_l1_levels(const float *x, size_t n, double mean_abs, int L, int8_t *level)
{
    const float scale = (mean_abs > 0.0) ? (float)((double)L / (2.0 * mean_abs)) : 0.0f;
    for (size_t i = 0; i < n; ++i) {
        float r = rintf(scale * x[i]);
        if (r > (float)L) r = (float)L;
        if (r < (float)-L) r = (float)-L;
        level[i] = (mean_abs > 0.0) ? (int8_t)r : 0;
    }
}

/* Appendix F.1: levels in [-L, L] travel as unsigned bytes level + L in [0, 2L], so that
 * a plain integer sum over W workers stays below 256 when 2 L W <= 255 (L = 15, 8 workers:
 * 240).  K = sum of the bytes, S = K - W L = sum of the levels, u = sign(S) (Algorithm 1
 * lines 4-5), ties as in orc_count_sign.  rows: W rows of n bytes. */
int orc_level_sum_sign(const uint8_t *rows, int W, size_t n, int L, uint64_t step, int tie_rule,
                       int32_t *K, int32_t *S, int8_t *u)
{
    if (W < 1 || L < 1 || L > 127) return ORC_ERR_ARG;
    if (2 * L * W > 255) return ORC_ERR_RANGE;
    const int alt = (step % 2u == 1u) ? 1 : -1;
    for (size_t i = 0; i < n; ++i) {
        int32_t k = 0;
        for (int w = 0; w < W; ++w) k += rows[(size_t)w * n + i];
        const int32_t sum = k - W * L;
        int v = (sum > 0) - (sum < 0);
        if (v == 0 && tie_rule == ORC_TIE_ALT) v = alt;
        if (K) K[i] = k;
        if (S) S[i] = sum;
        if (u) u[i] = (int8_t)v;
    }
    return ORC_OK;
}

/* ==== Ternary ("2-bit") wire format (Appendix B.1: an allreduce that transmits exact
 * zeros, the reference the alternating-sign rule is compared with) ==================
 * Every worker sends its sign s in {-1, 0, +1} unchanged; the update is the sign of the
 * plain sum of the signs (Algorithm 1 lines 4-5 with Q = sign and nothing forced).
 * s: W rows of n signs.  Kp / Kn: how many workers voted +1 / -1; S = Kp - Kn. */
int orc_ternary_vote(const int8_t *s, int W, size_t n, int32_t *Kp, int32_t *Kn, int32_t *S, int8_t *u)
{
    if (W < 1) return ORC_ERR_ARG;
    for (size_t i = 0; i < n; ++i) {
        int32_t kp = 0, kn = 0;
        for (int w = 0; w < W; ++w) {
            const int8_t v = s[(size_t)w * n + i];
            if (v > 0) ++kp;
            if (v < 0) ++kn;
        }
        const int32_t sum = kp - kn;
        if (Kp) Kp[i] = kp;
        if (Kn) Kn[i] = kn;
        if (S) S[i] = sum;
        if (u) u[i] = (int8_t)((sum > 0) - (sum < 0));
    }
    return ORC_OK;
}

/* ==== Divergence of the workers' momenta (Section 5.1, the quantity of Figure 6) =====
 * For every element the standard deviation of its W momentum values across workers
 * (population form, divisor W -- the paper does not say which), and the maximum of that
 * over the n elements of a layer.  Two-pass, fp64, workers in order. */
double orc_momentum_divergence(const float *m, int W, size_t n)
{
    double worst = 0.0;
    for (size_t i = 0; i < n; ++i) {
        double sum = 0.0;
        for (int w = 0; w < W; ++w) sum += (double)m[(size_t)w * n + i];
        const double mean = sum / (double)W;
        double ss = 0.0;
        for (int w = 0; w < W; ++w) {
            const double d = (double)m[(size_t)w * n + i] - mean;
            ss += d * d;
        }
        const double sd = sqrt(ss / (double)W);
        if (sd > worst) worst = sd;
    }
    return worst;
}
