// k_fast: candidate evaluation by bucketed prefix sums instead of one pass over
// the elements per candidate.  Same output as k_prep + k_search (the binary32
// filter value of every candidate of a tile, in candidate units), so the exact
// re-evaluation and the argmin that follow are shared.
//
// With u = |w|/m * n, candidate k quantizes the centre elements (u <= k) to the
// grid j*k/L and the tail elements to k + j*(n-k)/L, j = 0..L.  The elements
// that round to level j form a run of the sorted order whose ends are the
// half-way points (j +- 1/2) steps.  With cumulative counts N(b) and sums
// C(b) = sum of u over {u <= b}, summation by parts gives for a piece with
// step s, levels from offset z, and values v = u - z
//   sum (v - j s)^2 = S2 - 2 s (L C_L - sum_{j<L} C_j) + s^2 (L^2 N_L - sum_{j<L} (2j+1) N_j)
// where C_j, N_j are taken at the upper end of level j's run and S2 = sum v^2.
// So a candidate costs 2L+1 cumulative look-ups instead of a pass over the tile.
//
// A look-up needs no full sort: elements are grouped into T buckets that are
// monotone in u (one counting pass in LDS), bucket-level prefix sums of the
// count, of u and of u^2 are kept in binary64, and the look-up adds the part of
// the boundary's own bucket that lies at or below the boundary.
#pragma once

#include "pwlq_prep.h"
#include "pwlq_refine.h"
#include "pwlq_tables.h"

namespace pwlq {

constexpr int kFastWG = 512;                       // threads per workgroup
constexpr int kFastWaves = kFastWG / 64;
constexpr int kFastPer = kTileMax / kFastWG;       // elements of a tile held by one thread
constexpr int kFastTMax = 2048;                    // most buckets per tile
constexpr int kFastCrowd = 64;                     // fullest bucket the look-ups may walk: this or 1/16 of the tile

// Error of a tile's filter value from the binary64 prefix arithmetic: every
// cumulative sum is within (tile length + 64) * 2^-53 of its magnitude (at most
// n^2 K for the squares, n K for the sums), and about 32 such terms are
// combined with coefficients of at most n; kFastRelErr * n^2 * K bounds it and
// is added to the slack of the filter (keep_threshold).

// Bucket of a magnitude 0 <= u <= n: the top bits of its binary32 pattern
// (monotone in u), i.e. 2^(23-shift) buckets per octave over the 16 octaves
// below n; everything smaller shares bucket 0.  Weight distributions are dense
// near zero, so equal-width buckets would pile most elements into a few.
__device__ inline int fast_bucket(float u, int shift, int base)
{
    const int c = (__float_as_int(u) >> shift) - base;
    return c > 0 ? c : 0;
}

__device__ inline double wave_scan_incl_f64(double v)
{
    v += dpp_f64<0x111, 0xf>(0.0, v);
    v += dpp_f64<0x112, 0xf>(0.0, v);
    v += dpp_f64<0x114, 0xf>(0.0, v);
    v += dpp_f64<0x118, 0xf>(0.0, v);
    v += dpp_f64<0x142, 0xa>(0.0, v);
    v += dpp_f64<0x143, 0xc>(0.0, v);
    return v;
}

constexpr int kFastP2ShiftMin = 1, kFastP2ShiftMax = 3;   // 2, 4 or 8 buckets per entry of the prefix of squares:
                                                          // as fine as costs no workgroup per CU

struct FastLds {
    const unsigned short *start;   // [T+1] first element of each bucket
    const double *P1;              // [T+1] sum of u over the buckets before
    const double *P2;              // [(T >> p2_shift) + 1] sum of u^2 before every (1 << p2_shift)-th bucket
    const float *elems;            // grouped by bucket
    int shift, base;
    int p2_shift;
};

// Elements with u <= b: count and sum of u.  Every element of an earlier
// bucket is below b, every element of a later bucket above.  The boundary's own
// bucket is walked four elements at a time (the reads of a step are in flight
// together; the array has four spare words behind the tile, and what is read
// past the bucket's end is masked by position).
constexpr int kFastWalk = 2;          // elements per step of a bucket walk
constexpr int kFastWalkSq = 4;        // ... of the walk for the sum of squares, which spans several buckets

__device__ inline void fast_query(const FastLds &L, float b, int &count, double &s1)
{
    const int c = fast_bucket(b, L.shift, L.base);
    const int st = L.start[c], en = L.start[c + 1];
    int nn = st;
    double a1 = L.P1[c];
    for (int i = st; i < en; i += kFastWalk) {
        float u[kFastWalk];
#pragma unroll
        for (int x = 0; x < kFastWalk; ++x) u[x] = L.elems[i + x];
#pragma unroll
        for (int x = 0; x < kFastWalk; ++x) {
            const bool le = (i + x < en) && (u[x] <= b);
            nn += le ? 1 : 0;
            a1 += (double)(le ? u[x] : 0.0f);
        }
    }
    count = nn;
    s1 = a1;
}

// The same with the sum of squares, which is kept per 2, 4 or 8 buckets (it
// is needed once per candidate): the walk starts at that coarser boundary.
__device__ inline void fast_query_squares(const FastLds &L, float b, int &count, double &s1,
                                          double &s2)
{
    const int c = fast_bucket(b, L.shift, L.base);
    const int c0 = (c >> L.p2_shift) << L.p2_shift;
    const int st = L.start[c0], en = L.start[c + 1];
    int nn = st;
    double a1 = L.P1[c0];
    double a2 = L.P2[c0 >> L.p2_shift];
    for (int i = st; i < en; i += kFastWalkSq) {
        float u[kFastWalkSq];
#pragma unroll
        for (int x = 0; x < kFastWalkSq; ++x) u[x] = L.elems[i + x];
#pragma unroll
        for (int x = 0; x < kFastWalkSq; ++x) {
            const bool le = (i + x < en) && (u[x] <= b);
            const double d = (double)(le ? u[x] : 0.0f);
            nn += le ? 1 : 0;
            a1 += d;
            a2 += d * d;
        }
    }
    count = nn;
    s1 = a1;
    s2 = a2;
}

// Filter value of every candidate of the tile.
__device__ inline void fast_candidates(const FastLds &Q, int n, int len, int Li, double S1tot,
                                       double S2tot, float *__restrict__ row)
{
    const double Ld = (double)Li;
    for (int k = threadIdx.x + 1; k <= n; k += kFastWG) {
        const double kd = (double)k;
        // centre piece: offset 0, step k/L
        double sumC = 0.0;
        int sumN = 0;          // at most L^2 K < 2^31
        int cn;
        double c1;
        // half-way points in binary32: an element within a rounding of one is as far from
        // the level below as from the level above
        const float half_c = (float)(kd / (2.0 * Ld));
        for (int j = 0; j < Li; ++j) {
            fast_query(Q, (float)(2 * j + 1) * half_c, cn, c1);
            sumC += c1;
            sumN += __mul24(2 * j + 1, cn);
        }
        int nL;
        double cL, s2L;
        fast_query_squares(Q, (float)k, nL, cL, s2L);
        const double sc = kd / Ld;
        double sse = s2L - 2.0 * sc * (Ld * cL - sumC) +
                     sc * sc * (Ld * Ld * (double)nL - (double)sumN);
        if (k < n) {
            // tail piece: offset k, step (n-k)/L, values v = u - k
            const double wd = (double)(n - k);
            const float half_t = (float)(wd / (2.0 * Ld));
            const float kf = (float)k;
            double sumCt = 0.0;
            int sumNt = 0;
            for (int j = 0; j < Li; ++j) {
                fast_query(Q, __builtin_fmaf((float)(2 * j + 1), half_t, kf), cn, c1);
                const int nt = cn - nL;
                sumCt += (c1 - cL) - kd * (double)nt;
                sumNt += __mul24(2 * j + 1, nt);
            }
            const int ntL = len - nL;
            const double ctL = (S1tot - cL) - kd * (double)ntL;
            const double s2t = (S2tot - s2L) - 2.0 * kd * (S1tot - cL) + kd * kd * (double)ntL;
            const double st = wd / Ld;
            sse += s2t - 2.0 * st * (Ld * ctL - sumCt) +
                   st * st * (Ld * Ld * (double)ntL - (double)sumNt);
        }
        row[k - 1] = (float)(sse > 0.0 ? sse : 0.0);
    }
}

// A tile whose values crowd into a few buckets (many equal magnitudes: a bucket
// holding more than 1/16 of the tile) would make every look-up walk a long bucket; it is evaluated element by element
// instead, in binary32 with the chunked sums of the plain search kernel (all
// lanes read the same LDS word, which is a broadcast).
__device__ inline void fast_plain(const float *__restrict__ elems, int len, int n, int Li,
                                  float *__restrict__ row)
{
    const float Lf = (float)Li;
    for (int k = threadIdx.x + 1; k <= n; k += kFastWG) {
        const float kf = (float)k;
        const float nk = (float)(n - k);
        const float rc = Lf / kf;
        const float rt = (k < n) ? Lf / nk : 0.0f;
        const float ct = -kf * rt;
        const float stepc = kf / Lf, stept = nk / Lf;
        float outer = 0.0f;
        for (int cb = 0; cb < len; cb += kChunk) {
            const int ce = (cb + kChunk < len) ? cb + kChunk : len;
            float acc = 0.0f;
            for (int i = cb; i < ce; ++i) {
                const float u = elems[i];
                const bool tail = u > kf;
                const float t = tail ? __builtin_fmaf(u, rt, ct) : u * rc;
                const float err = (t - __builtin_rintf(t)) * (tail ? stept : stepc);
                acc = __builtin_fmaf(err, err, acc);
            }
            outer += acc;
        }
        row[k - 1] = outer;
    }
}

__global__ __launch_bounds__(kFastWG) void k_fast(Tables tb, int tile_begin, int n, int bits, int tcap, int p2_shift,
                                                  const float *__restrict__ tile_max,
                                                  float *__restrict__ gm,
                                                  float *__restrict__ sse32)
{
    // dynamic LDS: P1[tcap+1] (binary64; its space first serves as the histogram
    // and scatter cursor), P2[(tcap >> p2_shift) + 1], start[tcap+2] (16-bit), then
    // the grouped elements
    extern __shared__ double fast_lds[];
    __shared__ float redm[kFastWaves];
    __shared__ int redbad[kFastWaves];
    __shared__ int wsum[kFastWaves];
    __shared__ int wcrowd[kFastWaves];
    __shared__ double wsum1[kFastWaves], wsum2[kFastWaves];

    int t;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    TensorRec r;
    TileInfo ti = tile_of(tb, tile_begin + blockIdx.x, r, t);
    if (!r.fast) return;
    const int len = ti.len;

    double *P1 = fast_lds;
    double *P2 = fast_lds + (tcap + 1);
    int *cnt = reinterpret_cast<int *>(P1);
    unsigned short *start =
        reinterpret_cast<unsigned short *>(fast_lds + (tcap + 1) + ((tcap >> p2_shift) + 1));
    float *elems = reinterpret_cast<float *>(start + (tcap + 2));

    int T = 64;
    while (T < tcap && T <= 2 * len) T <<= 1;

    float a[kFastPer];
#pragma unroll
    for (int e = 0; e < kFastPer; ++e) {
        const int i = tid + e * kFastWG;
        a[e] = (i < len) ? fabsf(ti.src[i]) : 0.0f;
    }

    // group absmax: from the registers (single-tile group) or the tile maxima
    float m = 0.0f;
    int bad = 0;
    if (r.tpg == 1) {
#pragma unroll
        for (int e = 0; e < kFastPer; ++e) { bad |= (a[e] != a[e]); m = fmaxf(m, a[e]); }
    } else {
        const int tile0 = r.tile_base + ti.group_local * r.tpg;
        for (int j = tid; j < r.tpg; j += kFastWG) {
            const float v = tile_max[tile0 + j];
            bad |= (v != v);
            m = fmaxf(m, v);
        }
    }
    m = wave_max(m);
    bad = wave_or(bad);
    if (lane == 0) { redm[wave] = m; redbad[wave] = bad; }
    for (int i = tid; i < T; i += kFastWG) cnt[i] = 0;
    __syncthreads();
    m = redm[0];
    bad = redbad[0];
    for (int i = 1; i < kFastWaves; ++i) { m = fmaxf(m, redm[i]); bad |= redbad[i]; }
    if (bad) m = __builtin_nanf("");
    if (ti.tile_in_group == 0 && tid == 0) gm[ti.group] = m;

    const bool usable = (m > 0.0f) && (m < __builtin_inff());
    const float nf = (float)n;
    const float scale = usable ? nf / m : 0.0f;
    int shift = 16;                        // T = 2048: 128 buckets per octave
    for (int x = T; x < 2048; x <<= 1) ++shift;
    const int base = (__float_as_int(nf) >> shift) - (T - 1);

    // units and histogram
#pragma unroll
    for (int e = 0; e < kFastPer; ++e) {
        const int i = tid + e * kFastWG;
        if (i < len) {
            const float u = usable ? to_units(a[e], scale, nf) : 0.0f;
            a[e] = u;
            atomicAdd(&cnt[fast_bucket(u, shift, base)], 1);
        }
    }
    __syncthreads();

    // bucket starts (exclusive scan); the histogram becomes the scatter cursor
    const int per = (T + kFastWG - 1) / kFastWG;
    const int lo = tid * per < T ? tid * per : T;
    const int hi = lo + per < T ? lo + per : T;
    {
        // bucket 0 (zeros and near-zeros, e.g. pruned weights) only counts as
        // crowded if the lowest boundary, half a centre step of k = 1, can fall in it
        const float lowest = 0.5f / (float)((1 << (bits - 1)) - 1);
        const int first = (fast_bucket(lowest, shift, base) == 0) ? 0 : 1;
        int sum = 0, fullest = 0;
        for (int i = lo; i < hi; ++i) {
            sum += cnt[i];
            if (i >= first && cnt[i] > fullest) fullest = cnt[i];
        }
        const int incl = wave_scan_incl(sum);
        const int crowd = (len >> 4) > kFastCrowd ? (len >> 4) : kFastCrowd;
        fullest = (__ballot(fullest > crowd) != 0ull) ? 1 : 0;
        if (lane == 63) { wsum[wave] = incl; wcrowd[wave] = fullest; }
        __syncthreads();
        int run = incl - sum;
        for (int i = 0; i < wave; ++i) run += wsum[i];
        for (int i = lo; i < hi; ++i) {
            const int v = cnt[i];
            start[i] = (unsigned short)run;
            cnt[i] = 0;
            run += v;
        }
        if (tid == 0) start[T] = (unsigned short)len;
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < kFastPer; ++e) {
        const int i = tid + e * kFastWG;
        if (i < len) {
            const float u = a[e];
            const int c = fast_bucket(u, shift, base);
            elems[start[c] + atomicAdd(&cnt[c], 1)] = u;
        }
    }
    int crowded = 0;
    for (int i = 0; i < kFastWaves; ++i) crowded |= wcrowd[i];
    __syncthreads();
    if (crowded) {
        fast_plain(elems, len, n, (1 << (bits - 1)) - 1, sse32 + (long long)t * n);
        return;
    }

    // per-bucket sums and their exclusive prefix (binary64)
    {
        double b1[(kFastTMax + kFastWG - 1) / kFastWG], b2[(kFastTMax + kFastWG - 1) / kFastWG];
        double t1 = 0.0, t2 = 0.0;
#pragma unroll
        for (int x = 0; x < (kFastTMax + kFastWG - 1) / kFastWG; ++x) {
            const int c = lo + x;
            double s1 = 0.0, s2 = 0.0;
            if (c < hi) {
                for (int i = start[c]; i < start[c + 1]; ++i) {
                    const double d = (double)elems[i];
                    s1 += d;
                    s2 += d * d;
                }
            }
            b1[x] = t1;
            b2[x] = t2;
            t1 += s1;
            t2 += s2;
        }
        const double i1 = wave_scan_incl_f64(t1), i2 = wave_scan_incl_f64(t2);
        if (lane == 63) { wsum1[wave] = i1; wsum2[wave] = i2; }
        __syncthreads();           // also: every use of the cursor (aliases P1) is done
        double o1 = i1 - t1, o2 = i2 - t2;
        for (int i = 0; i < wave; ++i) { o1 += wsum1[i]; o2 += wsum2[i]; }
#pragma unroll
        for (int x = 0; x < (kFastTMax + kFastWG - 1) / kFastWG; ++x) {
            const int c = lo + x;
            if (c < hi) {
                P1[c] = o1 + b1[x];
                if ((c & ((1 << p2_shift) - 1)) == 0) P2[c >> p2_shift] = o2 + b2[x];
            }
        }
        if (tid == kFastWG - 1) { P1[T] = o1 + t1; P2[T >> p2_shift] = o2 + t2; }
    }
    __syncthreads();

    FastLds Q;
    Q.start = start;
    Q.P1 = P1;
    Q.P2 = P2;
    Q.elems = elems;
    Q.shift = shift;
    Q.base = base;
    Q.p2_shift = p2_shift;
    fast_candidates(Q, n, len, (1 << (bits - 1)) - 1, P1[T], P2[T >> p2_shift],
                    sse32 + (long long)t * n);
}

} // namespace pwlq
