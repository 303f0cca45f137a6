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

// ------------------------------------------------------------------- stats
// Per tile: max|w| (NaN if any element is NaN), sum of w^2 and sum of |w| in
// binary64.  One wavefront per tile (most tiles are a few hundred elements: a
// workgroup per tile spends its time on the reductions and the barrier), every
// element read once, four loads in flight per lane with a partial sum each,
// added in a fixed order.
constexpr int kStatUnroll = 4;

__global__ __launch_bounds__(kWG) void k_stats(Tables tb, int n_tiles, float *__restrict__ tile_max,
                                               double *__restrict__ tile_s2,
                                               double *__restrict__ tile_s1)
{
    const int slot = uni((int)(blockIdx.x * kWaves + (threadIdx.x >> 6)));
    if (slot >= n_tiles) return;
    int t;
    TensorRec r;
    TileInfo ti = tile_of(tb, slot, r, t);
    const int lane = threadIdx.x & 63;
    float mx = 0.0f;
    int bad = 0;
    double s2[kStatUnroll], s1[kStatUnroll];
#pragma unroll
    for (int u = 0; u < kStatUnroll; ++u) s2[u] = s1[u] = 0.0;
    int i = lane;
    for (; i + 64 * (kStatUnroll - 1) < ti.len; i += 64 * kStatUnroll) {
        float a[kStatUnroll];
#pragma unroll
        for (int u = 0; u < kStatUnroll; ++u) a[u] = fabsf(ti.src[i + 64 * u]);
#pragma unroll
        for (int u = 0; u < kStatUnroll; ++u) {
            bad |= (a[u] != a[u]);
            mx = fmaxf(mx, a[u]);
            const double d = (double)a[u];
            s2[u] += d * d;
            s1[u] += d;
        }
    }
    for (; i < ti.len; i += 64) {
        const float a = fabsf(ti.src[i]);
        bad |= (a != a);
        mx = fmaxf(mx, a);
        const double d = (double)a;
        s2[0] += d * d;
        s1[0] += d;
    }
    const double t2 = wave_sum((s2[0] + s2[1]) + (s2[2] + s2[3]));
    const double t1 = wave_sum((s1[0] + s1[1]) + (s1[2] + s1[3]));
    mx = wave_max(mx);
    bad = wave_or(bad);
    if (lane == 0) {
        tile_max[t] = bad ? __builtin_nanf("") : mx;
        tile_s2[t] = t2;
        tile_s1[t] = t1;
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
constexpr int kSelectWG = 64;     // one wavefront per workgroup: a few ten thousand groups reach every CU

__global__ __launch_bounds__(kSelectWG) void k_select(Tables tb, int n_groups, int selector,
                                                const float *__restrict__ tile_max,
                                                const double *__restrict__ tile_s2,
                                                const double *__restrict__ tile_s1,
                                                float *__restrict__ p_out,
                                                float *__restrict__ m_out)
{
    const int g = blockIdx.x * kSelectWG + threadIdx.x;
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
// binary32 code, binary64 error, fixed summation order.  One wavefront per
// tile, as in k_stats.
__global__ __launch_bounds__(kWG) void k_mse_tile(Tables tb, int n_tiles, int bits,
                                                  const float *__restrict__ p_in,
                                                  const float *__restrict__ m_in,
                                                  double *__restrict__ tile_sse)
{
    const int slot = uni((int)(blockIdx.x * kWaves + (threadIdx.x >> 6)));
    if (slot >= n_tiles) return;
    int t;
    TensorRec r;
    TileInfo ti = tile_of(tb, slot, r, t);
    const long long og = r.out_group + ti.group_local;
    const Pieces q = make_pieces(m_in[og], p_in[og], bits);
    const int lane = threadIdx.x & 63;
    double acc[kStatUnroll];
#pragma unroll
    for (int u = 0; u < kStatUnroll; ++u) acc[u] = 0.0;
    int i = lane;
    for (; i + 64 * (kStatUnroll - 1) < ti.len; i += 64 * kStatUnroll) {
        float a[kStatUnroll];
#pragma unroll
        for (int u = 0; u < kStatUnroll; ++u) a[u] = fabsf(ti.src[i + 64 * u]);
#pragma unroll
        for (int u = 0; u < kStatUnroll; ++u) acc[u] += exact_error_sq(q, a[u]);
    }
    for (; i < ti.len; i += 64) acc[0] += exact_error_sq(q, fabsf(ti.src[i]));
    const double s = wave_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
    if (lane == 0) tile_sse[t] = s;
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
