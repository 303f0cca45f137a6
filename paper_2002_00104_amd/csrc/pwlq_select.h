// k_stats, k_select: the paper's analytic breakpoint selectors (Section 3.3,
// Section 5.1).  k_mse_tile, k_mse_final: error of Eq.3 at a given (m, p).
#pragma once

#include "pwlq_tables.h"
#include "pwlq_refine.h"

namespace pwlq {

// Tensor of a per-lane index (lanes may ask for different tensors): largest i
// with prefix[i] <= x.
__device__ inline int find_tensor_lane(const int *__restrict__ prefix, int nt, int x)
{
    int lo = 0, hi = nt;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (prefix[mid] <= x) lo = mid;
        else hi = mid;
    }
    return lo;
}

// Sum over the workgroup in a fixed order, valid in thread 0.
__device__ inline double block_sum0(double v, double *lds)
{
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    double s = lds[0];
    for (int i = 1; i < kWaves; ++i) s += lds[i];
    return s;
}

// ------------------------------------------------------------------- stats
// Per tile: max|w| (NaN if any element is NaN), sum of w^2 and sum of |w| in
// binary64.  One workgroup per tile, every element read once.
__global__ __launch_bounds__(kWG) void k_stats(Tables tb, float *__restrict__ tile_max,
                                               double *__restrict__ tile_s2,
                                               double *__restrict__ tile_s1)
{
    __shared__ float red[kWaves];
    __shared__ int redbad[kWaves];
    __shared__ double lds2[kWaves], lds1[kWaves];
    int t;
    TensorRec r;
    TileInfo ti = tile_of(tb, blockIdx.x, r, t);
    float mx = 0.0f;
    int bad = 0;
    double s2 = 0.0, s1 = 0.0;
    for (int i = threadIdx.x; i < ti.len; i += kWG) {
        const float a = fabsf(ti.src[i]);
        bad |= (a != a);
        mx = fmaxf(mx, a);
        const double d = (double)a;
        s2 += d * d;
        s1 += d;
    }
    mx = wave_max(mx);
    bad = wave_or(bad);
    if ((threadIdx.x & 63) == 0) { red[threadIdx.x >> 6] = mx; redbad[threadIdx.x >> 6] = bad; }
    s2 = block_sum0(s2, lds2);
    s1 = block_sum0(s1, lds1);
    if (threadIdx.x == 0) {
        for (int i = 1; i < kWaves; ++i) { mx = fmaxf(mx, red[i]); bad |= redbad[i]; }
        tile_max[t] = bad ? __builtin_nanf("") : mx;
        tile_s2[t] = s2;
        tile_s1[t] = s1;
    }
}

// ------------------------------------------------------------------ select
// Density and distribution function of the assumed zero-mean law truncated to
// [-m, m] (F(-m) = 0, F(m) = 1), at 0 < p < m.
struct Law {
    double F, f, df;     // CDF, PDF, derivative of the PDF
};
__device__ inline double std_normal_cdf(double x)
{
    return 0.5 * erfc(-x * 0.70710678118654752440);
}
__device__ inline Law truncated_law(double p, double m, double scale, bool laplace)
{
    Law w;
    if (laplace) {
        const double z = 1.0 - exp(-m / scale);
        const double e = exp(-p / scale);
        w.F = 0.5 + 0.5 * (1.0 - e) / z;
        w.f = e / (2.0 * scale) / z;
        w.df = -w.f / scale;
    } else {
        const double z = 2.0 * std_normal_cdf(m / scale) - 1.0;
        const double x = p / scale;
        w.F = (std_normal_cdf(x) - std_normal_cdf(-m / scale)) / z;
        w.f = exp(-0.5 * x * x) / (scale * 2.50662827463100050242) / z;
        w.df = -x / scale * w.f;
    }
    return w;
}

// Minimiser of the expected error of Eq.6 over (0, m/2): root of its derivative
// (Eq.8; Eq.11 is that root written out).  The derivative is increasing there
// (Lemma 1: the second derivative, Eq.9, is positive), so Newton steps are kept
// inside a shrinking bracket and replaced by its midpoint when they leave it.
__device__ inline double solve_breakpoint(double m, double scale, bool laplace, double start)
{
    double lo = 0.0, hi = 0.5 * m;
    {
        const Law w = truncated_law(hi, m, scale, laplace);
        const double g = hi - 2.0 * m + 2.0 * m * w.F + m * (2.0 * hi - m) * w.f;
        if (g <= 0.0) return hi;
    }
    double p = (start > lo && start < hi) ? start : 0.5 * (lo + hi);
    for (int it = 0; it < 100; ++it) {
        const Law w = truncated_law(p, m, scale, laplace);
        const double g = p - 2.0 * m + 2.0 * m * w.F + m * (2.0 * p - m) * w.f;
        const double dg = 1.0 + 4.0 * m * w.f + m * (2.0 * p - m) * w.df;
        if (g > 0.0) hi = p;
        else lo = p;
        double next = p - g / dg;
        if (!(next > lo && next < hi)) next = 0.5 * (lo + hi);
        const double step = fabs(next - p);
        p = next;
        if (step <= 2.0e-16 * m || hi - lo <= 2.0e-16 * m) break;
    }
    return p;
}

// One thread per group: add the tiles' statistics in tile order, estimate the
// scale about zero (sigma^2 = mean w^2, beta = mean |w|) and select p.
// selector 0: Section 5.1's logarithmic fit, p = sigma ln(0.8614 m/sigma + 0.6079);
// selector 1: Eq.11 for the truncated Gaussian; 2: for the truncated Laplacian.
__global__ __launch_bounds__(kWG) void k_select(Tables tb, int n_groups, int selector,
                                                const float *__restrict__ tile_max,
                                                const double *__restrict__ tile_s2,
                                                const double *__restrict__ tile_s1,
                                                float *__restrict__ p_out,
                                                float *__restrict__ m_out)
{
    const int g = blockIdx.x * kWG + threadIdx.x;
    if (g >= n_groups) return;
    const int tensor = (tb.nt == 1) ? 0 : find_tensor_lane(tb.group_prefix, tb.nt, g);
    const TensorRec &r = (tb.nt == 1) ? tb.one : tb.recs[tensor];
    const int gl = g - r.group_base;
    const long long tile0 = r.tile_base + (long long)gl * r.tpg;
    float mf = 0.0f;
    int bad = 0;
    double s2 = 0.0, s1 = 0.0;
    for (int j = 0; j < r.tpg; ++j) {
        const float v = tile_max[tile0 + j];
        bad |= (v != v);
        mf = fmaxf(mf, v);
        s2 += tile_s2[tile0 + j];
        s1 += tile_s1[tile0 + j];
    }
    if (bad) mf = __builtin_nanf("");
    const long long og = r.out_group + gl;
    m_out[og] = mf;
    if (!(mf < __builtin_inff())) { p_out[og] = __builtin_nanf(""); return; }
    if (mf == 0.0f) { p_out[og] = 0.0f; return; }
    const double m = (double)mf;
    const double count = (double)r.gcount;
    const double sigma = sqrt(s2 / count), beta = s1 / count;
    const double fit = sigma * log(0.8614 * (m / sigma) + 0.6079);
    double p;
    if (selector == 0) p = fit;
    else if (selector == 1) p = solve_breakpoint(m, sigma, false, fit);
    else p = solve_breakpoint(m, beta, true, 0.25 * m);
    if (p > m) p = m;
    if (p < 0.0) p = 0.0;
    p_out[og] = (float)p;
}

// --------------------------------------------------------------------- mse
// Squared error of Eq.3 over one tile with the group's (m, p): canonical
// binary32 code, binary64 error, fixed summation order.
__global__ __launch_bounds__(kWG) void k_mse_tile(Tables tb, int bits,
                                                  const float *__restrict__ p_in,
                                                  const float *__restrict__ m_in,
                                                  double *__restrict__ tile_sse)
{
    __shared__ double lds[kWaves];
    int t;
    TensorRec r;
    TileInfo ti = tile_of(tb, blockIdx.x, r, t);
    const long long og = r.out_group + ti.group_local;
    const Pieces q = make_pieces(m_in[og], p_in[og], bits);
    double acc = 0.0;
    for (int i = threadIdx.x; i < ti.len; i += kWG) acc += exact_error_sq(q, fabsf(ti.src[i]));
    acc = block_sum0(acc, lds);
    if (threadIdx.x == 0) tile_sse[t] = acc;
}

__global__ __launch_bounds__(kWG) void k_mse_final(Tables tb, int n_groups,
                                                   const double *__restrict__ tile_sse,
                                                   double *__restrict__ mse)
{
    const int g = blockIdx.x * kWG + threadIdx.x;
    if (g >= n_groups) return;
    const int tensor = (tb.nt == 1) ? 0 : find_tensor_lane(tb.group_prefix, tb.nt, g);
    const TensorRec &r = (tb.nt == 1) ? tb.one : tb.recs[tensor];
    const int gl = g - r.group_base;
    const long long tile0 = r.tile_base + (long long)gl * r.tpg;
    double s = 0.0;
    for (int j = 0; j < r.tpg; ++j) s += tile_sse[tile0 + j];
    mse[r.out_group + gl] = s / (double)r.gcount;
}

} // namespace pwlq
