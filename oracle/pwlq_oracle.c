/*
 * CPU oracle for the PWLQ breakpoint search and quantizer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, literal statement of what
 * the GPU library must compute.  It shares no code with the HIP path and must
 * never be called from it; only the tests, the smoke check and the benchmark's
 * cpu_baseline leg load it.
 *
 * What it follows (Fang et al., "Post-Training Piecewise Linear Quantization
 * for Deep Neural Networks"):
 *   - Eq.1 (Section 3.1): uniform quantizer  r_q = round((clamp(r) - z)/s),
 *     r_hat = s*r_q + z,  s = (r_u - r_l)/(N - 1).
 *   - Eq.3 (Section 3.2): the b-bit piecewise quantizer applies a (b-1)-bit
 *     uniform quantizer to |r| on [0,p] (offset 0) in the centre region
 *     R1 = [-p,p] and on [p,m] (offset p) in the tail region R2, then restores
 *     the sign; the error is  eps = pw(r) - r.
 *   - Eq.7 (Section 3.3): p* = argmin_p E(eps^2).  Here the expectation is the
 *     empirical sum of squared errors of the group, and the argmin runs over
 *     the uniform grid p_k = m*k/n, k = 1..n  (the numerical curve of Fig.1,
 *     right).
 *   - Section 4: one extra stored bit per weight names the region.
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   - each piece has N = 2^(b-1) levels, codes 0..L with L = 2^(b-1)-1 (the
 *     unsigned domain with z = r_l of Section 3.1), so s = range/L;
 *   - round is round-half-to-even;
 *   - the code is decided in IEEE binary32, by multiplying with the binary32
 *     reciprocal of the step, no fused operations;
 *   - the squared error is accumulated in binary64, in index order;
 *   - ties in the argmin go to the smallest k;
 *   - the top code of a piece decodes to the exact end point (p or m).
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { REF_OK = 0, REF_EINVAL = 1, REF_ENULL = 2 };
enum { REF_PER_CHANNEL = 0, REF_PER_TENSOR = 1 };

/* Parameters of the two pieces for one (m, p) pair.  Eq.1: s = Delta/(N-1). */
typedef struct {
    float p, m;
    float s1, s2; /* step of the centre piece [0,p] and of the tail piece [p,m] */
    float i1, i2; /* binary32 reciprocals of the steps (0 when the step is 0)   */
    float L;      /* highest code of a piece, 2^(b-1) - 1                        */
} pieces;

static pieces make_pieces(float m, float p, int bits)
{
    pieces q;
    q.m = m;
    q.p = p;
    q.L = (float)((1 << (bits - 1)) - 1);
    q.s1 = p / q.L;
    float width2 = m - p;
    q.s2 = width2 / q.L;
    q.i1 = (q.s1 > 0.0f) ? 1.0f / q.s1 : 0.0f;
    q.i2 = (q.s2 > 0.0f) ? 1.0f / q.s2 : 0.0f;
    return q;
}

/* Eq.3 on one magnitude a = |r|: which region, which code.  R1 is closed
 * (a <= p), R2 is (p, m].  Returns the code; *tail receives the region. */
static float piece_code(const pieces *q, float a, int *tail)
{
    float t;
    if (a > q->p) {
        *tail = 1;
        float x = a - q->p; /* clamp(r) - z with z = p */
        t = x * q->i2;
    } else {
        *tail = 0;
        t = a * q->i1;      /* z = 0 */
    }
    float code = rintf(t);  /* round half to even */
    if (code > q->L) code = q->L; /* saturation to the integer domain */
    return code;
}

/* eps = r_hat - r on the magnitude, in binary64 from the binary32 step,
 * offset, code and magnitude:  s*r_q + z - a. */
static double piece_error(const pieces *q, float a)
{
    int tail;
    float code = piece_code(q, a, &tail);
    double s = tail ? (double)q->s2 : (double)q->s1;
    double z = tail ? (double)q->p : 0.0;
    return (double)code * s + z - (double)a;
}

static float grid_point(float m, int k, int n)
{
    float ratio = (float)k / (float)n;
    return m * ratio;
}

static float group_absmax(const float *w, int64_t count)
{
    float m = 0.0f;
    for (int64_t i = 0; i < count; ++i) {
        float a = fabsf(w[i]);
        if (a > m || isnan(a)) m = a;
        if (isnan(m)) break;
    }
    return m;
}

/* One group: SSE[k-1] for k = 1..n written to curve (length n). */
static void group_curve_range(const float *w, int64_t count, float m, int bits,
                              int n, int k_lo, int k_hi, double *curve)
{
    for (int k = k_lo; k <= k_hi; ++k) {
        pieces q = make_pieces(m, grid_point(m, k, n), bits);
        double sse = 0.0;
        for (int64_t i = 0; i < count; ++i) {
            double e = piece_error(&q, fabsf(w[i]));
            sse += e * e;
        }
        curve[k - 1] = sse;
    }
}

static void group_pick(const double *curve, int n, float m, int64_t count,
                       float *p_star, int32_t *k_star, double *mse)
{
    int best = 1;
    for (int k = 2; k <= n; ++k)
        if (curve[k - 1] < curve[best - 1]) best = k; /* strict: smallest k wins ties */
    *k_star = best;
    *p_star = grid_point(m, best, n);
    *mse = curve[best - 1] / (double)count;
}

static int check_common(int64_t C, int64_t K, int bits, int mode)
{
    if (C < 1 || K < 1) return REF_EINVAL;
    if (bits < 2 || bits > 8) return REF_EINVAL;
    if (mode != REF_PER_CHANNEL && mode != REF_PER_TENSOR) return REF_EINVAL;
    return REF_OK;
}

/*
 * w: host [C,K] row-major binary32.  G = C groups (per-channel) or 1
 * (per-tensor).  Outputs are host arrays of length G; sse_curve (optional,
 * may be NULL) is [G, n_cand] binary64 and receives every candidate's SSE.
 * k_star is 1-based.  A group whose absmax is not finite gets k_star = -1 and
 * NaN for p_star and mse.
 */
int pwlq_ref_search(const float *w, int64_t C, int64_t K, int bits, int n_cand,
                    int mode, float *p_star, float *m_out, int32_t *k_star,
                    double *mse, double *sse_curve)
{
    if (!w || !p_star || !m_out || !k_star || !mse) return REF_ENULL;
    int rc = check_common(C, K, bits, mode);
    if (rc) return rc;
    if (n_cand < 1 || n_cand > 65535) return REF_EINVAL;

    if (mode == REF_PER_CHANNEL) {
        int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
        for (int64_t g = 0; g < C; ++g) {
            const float *row = w + g * K;
            float m = group_absmax(row, K);
            m_out[g] = m;
            double *curve = sse_curve ? sse_curve + g * (int64_t)n_cand
                                      : (double *)malloc(sizeof(double) * (size_t)n_cand);
            if (!curve) { failed = 1; continue; }
            if (!isfinite(m)) {
                k_star[g] = -1; p_star[g] = NAN; mse[g] = NAN;
                for (int k = 0; k < n_cand; ++k) curve[k] = NAN;
            } else {
                group_curve_range(row, K, m, bits, n_cand, 1, n_cand, curve);
                group_pick(curve, n_cand, m, K, &p_star[g], &k_star[g], &mse[g]);
            }
            if (!sse_curve) free(curve);
        }
        return failed ? REF_EINVAL : REF_OK;
    }

    /* per-tensor: one group of C*K elements; candidates are independent, so
     * the loop over them is the parallel one and every sum stays in index
     * order. */
    int64_t count = C * K;
    float m = group_absmax(w, count);
    m_out[0] = m;
    double *curve = sse_curve ? sse_curve : (double *)malloc(sizeof(double) * (size_t)n_cand);
    if (!curve) return REF_EINVAL;
    if (!isfinite(m)) {
        k_star[0] = -1; p_star[0] = NAN; mse[0] = NAN;
        for (int k = 0; k < n_cand; ++k) curve[k] = NAN;
    } else {
#pragma omp parallel for schedule(dynamic, 1)
        for (int k = 1; k <= n_cand; ++k)
            group_curve_range(w, count, m, bits, n_cand, k, k, curve);
        group_pick(curve, n_cand, m, count, &p_star[0], &k_star[0], &mse[0]);
    }
    if (!sse_curve) free(curve);
    return REF_OK;
}

/*
 * Quantize with given (m, p) per group.  codes: b-bit sign-magnitude in a
 * byte (sign in bit b-1, piece code in bits 0..b-2); flags: 0 centre, 1 tail
 * (Section 4's region bit); w_hat: sign * (s*code + z) in binary32, with the
 * top code of a piece decoding to the piece's end point.
 */
int pwlq_ref_quantize(const float *w, int64_t C, int64_t K, int bits, int mode,
                      const float *p_star, const float *m_in, uint8_t *codes,
                      uint8_t *flags, float *w_hat)
{
    if (!w || !p_star || !m_in || !codes || !flags || !w_hat) return REF_ENULL;
    int rc = check_common(C, K, bits, mode);
    if (rc) return rc;

#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < C; ++g) {
        int64_t gi = (mode == REF_PER_CHANNEL) ? g : 0;
        pieces q = make_pieces(m_in[gi], p_star[gi], bits);
        for (int64_t j = 0; j < K; ++j) {
            int64_t i = g * K + j;
            float r = w[i];
            int tail;
            float code = piece_code(&q, fabsf(r), &tail);
            float v;
            if (tail)
                v = (code == q.L) ? q.m : fmaf(code, q.s2, q.p);
            else
                v = (code == q.L) ? q.p : code * q.s1;
            int neg = (r < 0.0f) && (v > 0.0f);
            w_hat[i] = neg ? -v : v;
            flags[i] = (uint8_t)tail;
            codes[i] = (uint8_t)((int)code | (neg << (bits - 1)));
        }
    }
    return REF_OK;
}

/*
 * Storage format of Section 4 ("at most one extra bit per weight"): the b-bit
 * codes of a tensor as one little-endian bit stream, code i in bits
 * [i*b, (i+1)*b) counted from bit 0 of byte 0, and the region flags as a second
 * stream with flag i in bit i.  Unused bits of the last byte are 0.
 * packed_codes holds ceil(count*bits/8) bytes, packed_flags ceil(count/8).
 */
int pwlq_ref_pack(const uint8_t *codes, const uint8_t *flags, int64_t count, int bits,
                  uint8_t *packed_codes, uint8_t *packed_flags)
{
    if (!codes || !flags || !packed_codes || !packed_flags) return REF_ENULL;
    if (count < 0 || bits < 2 || bits > 8) return REF_EINVAL;
    int64_t code_bytes = (count * bits + 7) / 8, flag_bytes = (count + 7) / 8;
    for (int64_t i = 0; i < code_bytes; ++i) packed_codes[i] = 0;
    for (int64_t i = 0; i < flag_bytes; ++i) packed_flags[i] = 0;
    for (int64_t i = 0; i < count; ++i) {
        for (int bit = 0; bit < bits; ++bit) {
            if ((codes[i] >> bit) & 1) {
                int64_t pos = i * bits + bit;
                packed_codes[pos / 8] |= (uint8_t)(1u << (pos % 8));
            }
        }
        if (flags[i] & 1) packed_flags[i / 8] |= (uint8_t)(1u << (i % 8));
    }
    return REF_OK;
}

int pwlq_ref_unpack(const uint8_t *packed_codes, const uint8_t *packed_flags, int64_t count,
                    int bits, uint8_t *codes, uint8_t *flags)
{
    if (!codes || !flags || !packed_codes || !packed_flags) return REF_ENULL;
    if (count < 0 || bits < 2 || bits > 8) return REF_EINVAL;
    for (int64_t i = 0; i < count; ++i) {
        unsigned v = 0;
        for (int bit = 0; bit < bits; ++bit) {
            int64_t pos = i * bits + bit;
            v |= (unsigned)((packed_codes[pos / 8] >> (pos % 8)) & 1) << bit;
        }
        codes[i] = (uint8_t)v;
        flags[i] = (uint8_t)((packed_flags[i / 8] >> (i % 8)) & 1);
    }
    return REF_OK;
}

/*
 * The paper's own breakpoint selectors (Section 3.3 and Section 5.1).  They
 * assume the group follows a zero-mean Gaussian or Laplacian restricted to
 * [-m, m] and minimise the expected error of Eq.6; the minimiser satisfies the
 * stationarity condition of Eq.11,
 *     2 m F(p) = 2 m - p + m (m - 2 p) f(p),   0 < p < m/2,
 * with F, f the CDF and PDF on the bounded domain (F(-m) = 0, F(m) = 1).
 * selector 0: Section 5.1's closed form for a Gaussian, read with breakpoint
 *             and range in units of the standard deviation:
 *             p = sigma * ln(0.8614 m/sigma + 0.6079);
 * selector 1: Eq.11 solved for the truncated Gaussian;
 * selector 2: Eq.11 solved for the truncated Laplacian.
 * The scale is estimated about zero: sigma^2 = mean(w^2), beta = mean|w|.
 * All arithmetic in binary64; p is returned rounded to binary32.
 */
static double gauss_cdf(double x) { return 0.5 * erfc(-x * 0.70710678118654752440); }

/* Derivative of Eq.6 in p without its factor 2 C(b-1) (Eq.8):
 * p - 2m + 2m F(p) + m (2p - m) f(p); its root is Eq.11. */
static double stationarity(double p, double m, double scale, int laplace)
{
    double F, f;
    if (laplace) {
        double z = 1.0 - exp(-m / scale);           /* mass of |r| <= m          */
        F = 0.5 + 0.5 * (1.0 - exp(-p / scale)) / z; /* p > 0                     */
        f = exp(-p / scale) / (2.0 * scale) / z;
    } else {
        double z = 2.0 * gauss_cdf(m / scale) - 1.0;
        F = (gauss_cdf(p / scale) - gauss_cdf(-m / scale)) / z;
        f = exp(-0.5 * (p / scale) * (p / scale)) / (scale * 2.50662827463100050242) / z;
    }
    return p - 2.0 * m + 2.0 * m * F + m * (2.0 * p - m) * f;
}

static double solve_breakpoint(double m, double scale, int laplace)
{
    /* the expected error is convex on (0, m/2) (Lemma 1): bisection on its derivative */
    double lo = 0.0, hi = 0.5 * m;
    if (stationarity(hi, m, scale, laplace) <= 0.0) return hi;
    for (int it = 0; it < 200; ++it) {
        double mid = 0.5 * (lo + hi);
        if (stationarity(mid, m, scale, laplace) > 0.0) hi = mid; else lo = mid;
    }
    return 0.5 * (lo + hi);
}

int pwlq_ref_select_analytic(const float *w, int64_t C, int64_t K, int mode, int selector,
                             float *p_out, float *m_out)
{
    if (!w || !p_out || !m_out) return REF_ENULL;
    if (C < 1 || K < 1 || selector < 0 || selector > 2) return REF_EINVAL;
    if (mode != REF_PER_CHANNEL && mode != REF_PER_TENSOR) return REF_EINVAL;
    int64_t G = (mode == REF_PER_CHANNEL) ? C : 1;
    int64_t count = (mode == REF_PER_CHANNEL) ? K : C * K;
    for (int64_t g = 0; g < G; ++g) {
        const float *x = w + g * count;
        float m = group_absmax(x, count);
        m_out[g] = m;
        if (!isfinite(m)) { p_out[g] = NAN; continue; }
        if (m == 0.0f) { p_out[g] = 0.0f; continue; }
        double s2 = 0.0, s1 = 0.0;
        for (int64_t i = 0; i < count; ++i) {
            double v = (double)x[i];
            s2 += v * v;
            s1 += fabs(v);
        }
        double sigma = sqrt(s2 / (double)count), beta = s1 / (double)count;
        double p;
        if (selector == 0) p = sigma * log(0.8614 * ((double)m / sigma) + 0.6079);
        else if (selector == 1) p = solve_breakpoint((double)m, sigma, 0);
        else p = solve_breakpoint((double)m, beta, 1);
        if (p > (double)m) p = (double)m;
        if (p < 0.0) p = 0.0;
        p_out[g] = (float)p;
    }
    return REF_OK;
}

/* Mean squared error of Eq.3 for a given (m, p) per group, same arithmetic as
 * the search (binary32 code, binary64 error). */
int pwlq_ref_mse(const float *w, int64_t C, int64_t K, int bits, int mode, const float *p,
                 const float *m_in, double *mse)
{
    if (!w || !p || !m_in || !mse) return REF_ENULL;
    int rc = check_common(C, K, bits, mode);
    if (rc) return rc;
    int64_t G = (mode == REF_PER_CHANNEL) ? C : 1;
    int64_t count = (mode == REF_PER_CHANNEL) ? K : C * K;
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < G; ++g) {
        pieces q = make_pieces(m_in[g], p[g], bits);
        double sse = 0.0;
        for (int64_t i = 0; i < count; ++i) {
            double e = piece_error(&q, fabsf(w[g * count + i]));
            sse += e * e;
        }
        mse[g] = sse / (double)count;
    }
    return REF_OK;
}

/*
 * Section 4: inner products of uniformly quantized activations with PWLQ
 * weights on integer arithmetic.  Activations are X_hat = s_x X_q + z_x (Eq.1,
 * 8-bit, one scale and offset per call), weights are stored as b-bit
 * sign-magnitude codes plus the region bit.  With the signed code
 * w_q = sign * (piece code) and sigma = sign for a tail weight, the two paths
 * of Section 4 are
 *     P1 = C2 <X_q, W_q1>_R1 + C3,                       (centre, offset 0)
 *     P2 = C4 <X_q, W_q2>_R2 + C5 <X_q, sigma>_R2 + C6,  (tail, offset p)
 * with C2 = s_x s_1, C4 = s_x s_2, C5 = s_x p and the constants
 * C3 = z_x s_1 sum_R1 w_q,  C6 = z_x (s_2 sum_R2 w_q + p sum_R2 sigma).
 * (The paper writes <X_q, I>_R2 for magnitudes; on signed weights the offset p
 * carries the weight's sign, Eq.3.)  Three integer accumulators per output,
 * as Section 4 counts them.  s_1 = fl32(p/L), s_2 = fl32(fl32(m-p)/L) are the
 * quantizer's own binary32 steps; everything after the integer sums is
 * binary64.
 *
 * xq [M,K] int8; codes, flags [N,K] one byte each (as pwlq_ref_quantize writes
 * them); p, m per output channel n.  acc (optional) [3][M][N]: the integer
 * sums <X_q,W_q1>_R1, <X_q,W_q2>_R2, <X_q,sigma>_R2.  y [M][N] = P1 + P2.
 */
int pwlq_ref_linear(const int8_t *xq, int64_t M, int64_t K, float s_x, float z_x,
                    const uint8_t *codes, const uint8_t *flags, int64_t N, int bits,
                    const float *p, const float *m, int64_t *acc, double *y)
{
    if (!xq || !codes || !flags || !p || !m || !y) return REF_ENULL;
    if (M < 1 || K < 1 || N < 1 || bits < 2 || bits > 8) return REF_EINVAL;
    const int sign_bit = 1 << (bits - 1);
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        pieces q = make_pieces(m[n], p[n], bits);
        const uint8_t *c = codes + n * K, *f = flags + n * K;
        /* constants of the channel */
        int64_t sum1 = 0, sum2 = 0, sum3 = 0;
        for (int64_t k = 0; k < K; ++k) {
            int mag = c[k] & (sign_bit - 1);
            int sg = (c[k] & sign_bit) ? -1 : 1;
            if (f[k]) { sum2 += sg * mag; sum3 += sg; }
            else sum1 += sg * mag;
        }
        double C2 = (double)s_x * (double)q.s1, C4 = (double)s_x * (double)q.s2;
        double C5 = (double)s_x * (double)q.p;
        double C3 = (double)z_x * (double)q.s1 * (double)sum1;
        double C6 = (double)z_x * ((double)q.s2 * (double)sum2 + (double)q.p * (double)sum3);
        for (int64_t i = 0; i < M; ++i) {
            const int8_t *x = xq + i * K;
            int64_t a1 = 0, a2 = 0, a3 = 0;
            for (int64_t k = 0; k < K; ++k) {
                int mag = c[k] & (sign_bit - 1);
                int sg = (c[k] & sign_bit) ? -1 : 1;
                if (f[k]) { a2 += (int64_t)x[k] * (sg * mag); a3 += (int64_t)x[k] * sg; }
                else a1 += (int64_t)x[k] * (sg * mag);
            }
            if (acc) {
                acc[(0 * M + i) * N + n] = a1;
                acc[(1 * M + i) * N + n] = a2;
                acc[(2 * M + i) * N + n] = a3;
            }
            double P1 = C2 * (double)a1 + C3;
            double P2 = C4 * (double)a2 + C5 * (double)a3 + C6;
            y[i * N + n] = P1 + P2;
        }
    }
    return REF_OK;
}

int pwlq_ref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
