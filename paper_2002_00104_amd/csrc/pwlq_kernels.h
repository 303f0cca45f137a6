// libpwlq kernels for gfx950.  Pipeline of one search call:
//
//   k_tile_absmax  max|w| of every tile                         (HBM read)
//   k_prep         group absmax; magnitudes rescaled to "candidate units"
//                  u = |w|/m * n and partitioned into one bucket per block of
//                  64 candidates                                (HBM read+write)
//   k_search       the hot loop: lane = candidate, elements arrive as
//                  wave-uniform scalar loads; binary32 squared error of every
//                  (element, candidate) pair                    (VALU bound)
//   k_flag         per group: candidates whose binary32 SSE is within the
//                  rounding slack of the minimum
//   k_exact        flagged candidates re-evaluated with the canonical binary32
//                  code and binary64 error; argmin for single-tile groups
//   k_final        argmin for groups spread over several tiles
//
// and of one quantize call:  k_emit (HBM bound).
#pragma once

#include "pwlq_device.h"

namespace pwlq {

typedef float float8 __attribute__((ext_vector_type(8)));

// A call with one tensor carries its record in the kernel arguments (`one`)
// and touches no table in memory; a model-level call reads `recs` and the
// prefix arrays from the head of the workspace.
struct Tables {
    const TensorRec *recs;
    const int *tile_prefix, *group_prefix, *unit_prefix, *mgroup_prefix;
    int nt;
    int n_units;
    TensorRec one;
};

// Every field of a record is the same in all lanes; passing it through
// readfirstlane tells the compiler so, which keeps loop bounds and addresses
// derived from it in scalar registers (and the loads they feed scalar loads).
__device__ inline int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ inline long long uni(long long v)
{
    unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(v & 0xffffffffLL));
    int hi = __builtin_amdgcn_readfirstlane((int)(v >> 32));
    return ((long long)hi << 32) | (long long)lo;
}
__device__ inline TensorRec rec_of(const Tables &tb, int i)
{
    TensorRec r = (tb.nt == 1) ? tb.one : tb.recs[i];
    r.w = reinterpret_cast<const float *>(uni((long long)reinterpret_cast<uintptr_t>(r.w)));
    r.gcount = uni(r.gcount);
    r.sorted_base = uni(r.sorted_base);
    r.out_elem = uni(r.out_elem);
    r.out_group = uni(r.out_group);
    r.tile_len = uni(r.tile_len);
    r.last_len = uni(r.last_len);
    r.tpg = uni(r.tpg);
    r.stride = uni(r.stride);
    r.tpu = uni(r.tpu);
    r.part_base = uni(r.part_base);
    r.tile_base = uni(r.tile_base);
    r.group_base = uni(r.group_base);
    r.unit_base = uni(r.unit_base);
    r.mgroup_base = uni(r.mgroup_base);
    r.ntiles = uni(r.ntiles);
    r.ngroups = uni(r.ngroups);
    return r;
}
__device__ inline TileInfo tile_of(const Tables &tb, int t, TensorRec &r)
{
    const int tensor = find_tensor(tb.tile_prefix, tb.nt, t);
    r = rec_of(tb, tensor);
    return tile_info(r, tensor, t);
}

// ------------------------------------------------------------------ absmax
// Only groups cut into several tiles need this pass; a single-tile group finds
// its absmax inside k_prep.
__global__ __launch_bounds__(kWG) void k_tile_absmax(Tables tb, float *__restrict__ tile_max)
{
    __shared__ float red[kWaves];
    __shared__ int redbad[kWaves];
    const int t = blockIdx.x;
    TensorRec r;
    TileInfo ti = tile_of(tb, t, r);
    if (r.tpg == 1) return;
    float mx = 0.0f;
    int bad = 0;
    for (int i = threadIdx.x; i < ti.len; i += kWG) {
        float a = fabsf(ti.src[i]);
        bad |= (a != a);
        mx = fmaxf(mx, a);
    }
    mx = wave_max(mx);
    bad = wave_or(bad);
    if ((threadIdx.x & 63) == 0) { red[threadIdx.x >> 6] = mx; redbad[threadIdx.x >> 6] = bad; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < kWaves; ++i) { mx = fmaxf(mx, red[i]); bad |= redbad[i]; }
        tile_max[t] = bad ? __builtin_nanf("") : mx;
    }
}

// -------------------------------------------------------------------- prep
// Magnitude in candidate units: u = |w|/m * n in [0, n]; candidate k has its
// breakpoint at u = k.  Bucket j holds the elements whose region differs among
// the candidates 64j+1 .. 64j+64; every earlier bucket is centre for all of
// them, every later bucket is tail for all of them.
__device__ inline float to_units(float a, float m, float nf)
{
    float u = (a / m) * nf;
    return fminf(fmaxf(u, 0.0f), nf);     // also maps a NaN to 0
}
__device__ inline int bucket_of(float u)
{
    int kc = (int)ceilf(u);          // smallest candidate with u <= k
    kc = kc < 1 ? 1 : kc;
    return (kc - 1) >> 6;
}

// inclusive prefix sum over the 64 lanes of a wavefront
__device__ inline int wave_scan_incl(int v)
{
    const int lane = threadIdx.x & 63;
    for (int off = 1; off < 64; off <<= 1) {
        int o = __shfl_up(v, off, 64);
        if (lane >= off) v += o;
    }
    return v;
}

// Sorted layout of one tile: [pad zeros][bucket 0][bucket 1]...[one vector of
// slack]; the padded length is a multiple of kVec and off[j] is the start of
// bucket j.  The tile's elements stay in registers between the passes, so the
// weights are read from memory once.  kPrivate (at most 32 buckets): every
// thread counts into its own histogram column and positions are assigned in
// (bucket, thread, element) order, so the layout is repeatable; otherwise LDS
// integer atomics assign positions inside a bucket in arrival order.
template <bool kPrivate>
__global__ __launch_bounds__(kWG) void k_prep(Tables tb, int n, int nblk,
                                               const float *__restrict__ tile_max,
                                               float *__restrict__ gm,
                                               int *__restrict__ offsets,
                                               float *__restrict__ sorted)
{
    extern __shared__ int hist[];     // kPrivate: [nblk][kWG], else [nblk]
    __shared__ float redm[kWaves];
    __shared__ int redbad[kWaves];
    __shared__ int wtot[32 * kWaves];
    __shared__ int scan_lds[kWaves];
    const int t = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    TensorRec r;
    TileInfo ti = tile_of(tb, t, r);
    const int len = ti.len;

    float a[kPerThread];
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
        const int i = tid + e * kWG;
        a[e] = (i < len) ? fabsf(ti.src[i]) : 0.0f;
    }

    // group absmax: from the registers (single-tile group) or the tile maxima
    float m = 0.0f;
    int bad = 0;
    if (r.tpg == 1) {
#pragma unroll
        for (int e = 0; e < kPerThread; ++e) { bad |= (a[e] != a[e]); m = fmaxf(m, a[e]); }
    } else {
        const int tile0 = r.tile_base + ti.group_local * r.tpg;
        for (int j = tid; j < r.tpg; j += kWG) {
            float v = tile_max[tile0 + j];
            bad |= (v != v);
            m = fmaxf(m, v);
        }
    }
    m = wave_max(m);
    bad = wave_or(bad);
    if (lane == 0) { redm[wave] = m; redbad[wave] = bad; }
    if (!kPrivate) for (int i = tid; i < nblk; i += kWG) hist[i] = 0;
    __syncthreads();
    m = redm[0];
    bad = redbad[0];
    for (int i = 1; i < kWaves; ++i) { m = fmaxf(m, redm[i]); bad |= redbad[i]; }
    if (bad) m = __builtin_nanf("");
    if (ti.tile_in_group == 0 && tid == 0) gm[ti.group] = m;

    const bool usable = (m > 0.0f) && (m < __builtin_inff());
    const float nf = (float)n;
    const int padded = (len + kVec - 1) / kVec * kVec;
    const int pad = padded - len;
    float *out = sorted + ti.sorted_off;
    int *off = offsets + (long long)t * (nblk + 1);

    // pass A: units and histogram
    if (kPrivate) for (int b = 0; b < nblk; ++b) hist[b * kWG + tid] = 0;
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
        const int i = tid + e * kWG;
        if (i < len) {
            const float u = usable ? to_units(a[e], m, nf) : 0.0f;
            a[e] = u;
            const int b = bucket_of(u);
            if (kPrivate) hist[b * kWG + tid] += 1;
            else atomicAdd(&hist[b], 1);
        }
    }

    // exclusive positions
    if (kPrivate) {
        for (int b = 0; b < nblk; ++b) {
            const int c = hist[b * kWG + tid];
            const int incl = wave_scan_incl(c);
            hist[b * kWG + tid] = incl - c;                 // exclusive inside the wavefront
            if (lane == 63) wtot[b * kWaves + wave] = incl;
        }
        __syncthreads();
        if (wave == 0) {
            int w[kWaves];
            int tot = 0;
#pragma unroll
            for (int i = 0; i < kWaves; ++i) {
                w[i] = (lane < nblk) ? wtot[lane * kWaves + i] : 0;
                tot += w[i];
            }
            int run = wave_scan_incl(tot) - tot;            // first position of bucket `lane`
            if (lane < nblk) {
                off[lane] = pad + run;
#pragma unroll
                for (int i = 0; i < kWaves; ++i) { wtot[lane * kWaves + i] = run; run += w[i]; }
            }
            if (lane == 0) off[nblk] = pad + len;
        }
    } else {
        __syncthreads();
        const int per = (nblk + kWG - 1) / kWG;
        const int lo = tid * per;
        int hi = lo + per;
        if (hi > nblk) hi = nblk;
        int sum = 0;
        for (int i = lo; i < hi; ++i) sum += hist[i];
        const int incl = wave_scan_incl(sum);
        if (lane == 63) scan_lds[wave] = incl;
        __syncthreads();
        int run = incl - sum;
        for (int i = 0; i < wave; ++i) run += scan_lds[i];
        for (int i = lo; i < hi; ++i) { int v = hist[i]; hist[i] = run; off[i] = pad + run; run += v; }
        if (tid == 0) off[nblk] = pad + len;
    }
    for (int i = tid; i < pad + kVec; i += kWG) {
        if (i < pad) out[i] = 0.0f;
        else out[padded + (i - pad)] = 0.0f;      // one vector of slack for the prefetch
    }
    __syncthreads();

    // pass B: scatter
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
        const int i = tid + e * kWG;
        if (i < len) {
            const float u = a[e];
            const int b = bucket_of(u);
            int pos;
            if (kPrivate) {
                pos = wtot[b * kWaves + wave] + hist[b * kWG + tid];
                hist[b * kWG + tid] += 1;
            } else {
                pos = atomicAdd(&hist[b], 1);
            }
            out[pad + pos] = u;
        }
    }
}

// ------------------------------------------------------------------ search
// One wavefront = one block of 64 candidates of one tile.  In candidate units
// the centre piece of candidate k has step k/L and the tail piece (n-k)/L, so
// the position of u in steps is  t = u*(L/k)  or  t = (u-k)*(L/(n-k)), and the
// error in steps is f = t - rne(t).  Sum f^2 per region, scale by step^2 at the
// end.  None of this depends on the group's absmax.
__device__ inline float8 load8(const float *__restrict__ p)
{
    return *reinterpret_cast<const float8 *>(__builtin_assume_aligned(p, 32));
}

template <bool kTail>
__device__ inline float zone_one_region(const float *__restrict__ us, int begin, int end,
                                        float r, float c)
{
    float outer = 0.0f;
    for (int cb = begin; cb < end; cb += kChunk) {
        const int ce = (cb + kChunk < end) ? cb + kChunk : end;
        float acc0 = 0.0f, acc1 = 0.0f;
        float8 cur = load8(us + cb);
        for (int i = cb; i < ce; i += kVec) {
            float8 nxt = load8(us + i + kVec);        // slack vector keeps this in bounds
#pragma unroll
            for (int e = 0; e < kVec; e += 2) {
                float t0 = kTail ? __builtin_fmaf(cur[e], r, c) : cur[e] * r;
                float t1 = kTail ? __builtin_fmaf(cur[e + 1], r, c) : cur[e + 1] * r;
                float f0 = t0 - __builtin_rintf(t0);
                float f1 = t1 - __builtin_rintf(t1);
                acc0 = __builtin_fmaf(f0, f0, acc0);
                acc1 = __builtin_fmaf(f1, f1, acc1);
            }
            cur = nxt;
        }
        outer += acc0 + acc1;
    }
    return outer;
}

__device__ inline float zone_mixed(const float *__restrict__ us, int begin, int end, float kf,
                                   float rc, float rt, float ct, float stepc, float stept)
{
    float outer = 0.0f;
    for (int cb = begin; cb < end; cb += kChunk) {
        const int ce = (cb + kChunk < end) ? cb + kChunk : end;
        float acc = 0.0f;
        for (int i = cb; i < ce; i += kVec) {
            float8 cur = load8(us + i);
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                const float u = cur[e];
                const bool tail = u > kf;
                const float r = tail ? rt : rc;
                const float c = tail ? ct : 0.0f;
                const float st = tail ? stept : stepc;
                float t = __builtin_fmaf(u, r, c);
                float err = (t - __builtin_rintf(t)) * st;
                acc = __builtin_fmaf(err, err, acc);
            }
        }
        outer += acc;
    }
    return outer;
}

__global__ __launch_bounds__(kWG) void k_search(Tables tb, int n, int nblk, int bits,
                                                int units_padded, int ny,
                                                const int *__restrict__ offsets,
                                                const float *__restrict__ sorted,
                                                float *__restrict__ sse32)
{
    // Workgroup ids are dealt round-robin to the 8 XCDs.  Keep the ny
    // workgroups of one unit (same tiles, different candidate blocks) on one
    // XCD so its L2 serves their reads, and deal units round-robin.
    const int wg = blockIdx.x;
    const int xcd = wg & 7;
    const int slot = wg >> 3;
    const int unit = (slot / ny) * 8 + xcd;
    const int jy = slot % ny;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = jy * kWaves + wave;
    if (unit >= tb.n_units || j >= nblk) return;

    const int tensor = find_tensor(tb.unit_prefix, tb.nt, unit);
    const TensorRec r = rec_of(tb, tensor);
    const int first = r.tile_base + (unit - r.unit_base) * r.tpu;
    int last = first + r.tpu;
    if (last > r.tile_base + r.ntiles) last = r.tile_base + r.ntiles;

    const int lane = threadIdx.x & 63;
    int k = j * kBlk + lane + 1;
    const bool live = k <= n;
    if (!live) k = n;
    const float Lf = (float)((1 << (bits - 1)) - 1);
    const float kf = (float)k;
    const float nk = (float)(n - k);
    const float rc = Lf / kf;
    const float rt = (k < n) ? Lf / nk : 0.0f;
    const float ct = -kf * rt;
    const float stepc = kf / Lf;
    const float stept = nk / Lf;

    for (int t = first; t < last; ++t) {
        const int local = t - r.tile_base;
        const int tig = local % r.tpg;
        const int len = (tig == r.tpg - 1) ? r.last_len : r.tile_len;
        const int padded = (len + kVec - 1) / kVec * kVec;
        const float *us = sorted + (r.sorted_base + (long long)local * r.stride);
        const int *off = offsets + (long long)t * (nblk + 1);
        const int lo = off[j] & ~(kVec - 1);
        const int hi = (off[j + 1] + kVec - 1) & ~(kVec - 1);
        const float sc = zone_one_region<false>(us, 0, lo, rc, 0.0f);
        const float sm = zone_mixed(us, lo, hi, kf, rc, rt, ct, stepc, stept);
        const float st = zone_one_region<true>(us, hi, padded, rt, ct);
        if (live)
            sse32[(long long)t * n + (k - 1)] = (stepc * stepc) * sc + (stept * stept) * st + sm;
    }
}

// -------------------------------------------------------------------- flag
// The binary32 SSE of k_search (candidate units) is only a filter: every
// candidate within the rounding slack of the minimum is kept and re-evaluated
// exactly.  The slack bounds twice the error of k_search: eps = 2^-21 n per
// element error (candidate units) and 3e-5 relative for the binary32 sums.
__device__ inline double keep_threshold(double mn, double count, int n)
{
    const double eps = (double)n * 4.76837158203125e-07;   // 2^-21 n
    return mn + 2.0 * (3e-5 * mn + 2.0 * eps * sqrt(count * mn) + count * eps * eps);
}

__device__ inline double group_sse(const float *__restrict__ sse32, long long tile0, int tpg,
                                   int n, int k0)
{
    double v = 0.0;
    for (int j = 0; j < tpg; ++j) v += (double)sse32[(tile0 + j) * n + k0];
    return v;
}

// Groups spread over several tiles: tile sums added in binary64, kept
// candidates written as a bit mask (bit k-1 of the group's row).
__global__ __launch_bounds__(kWG) void k_flag(Tables tb, int n, int nwords,
                                              const float *__restrict__ gm,
                                              const float *__restrict__ sse32,
                                              uint32_t *__restrict__ mask)
{
    __shared__ double lds[kWaves];
    const int mg = blockIdx.x;
    const int tid = threadIdx.x;
    const int tensor = find_tensor(tb.mgroup_prefix, tb.nt, mg);
    const TensorRec r = rec_of(tb, tensor);
    const int gl = mg - r.mgroup_base;
    const int g = r.group_base + gl;
    const long long tile0 = r.tile_base + (long long)gl * r.tpg;
    uint32_t *gmask = mask + (long long)g * nwords;
    const float m = gm[g];
    if (!(m > 0.0f) || !(m < __builtin_inff())) {
        // all-zero group: every candidate has zero error, the first wins.
        // non-finite group: nothing to evaluate.
        for (int wi = tid; wi < nwords; wi += kWG)
            gmask[wi] = (wi == 0 && m == 0.0f) ? 1u : 0u;
        return;
    }
    double mn = __builtin_inf();
    for (int k0 = tid; k0 < n; k0 += kWG) mn = fmin(mn, group_sse(sse32, tile0, r.tpg, n, k0));
    mn = block_min(mn, lds);
    const double thr = keep_threshold(mn, (double)r.gcount, n);
    for (int wi = tid; wi < nwords; wi += kWG) {
        uint32_t word = 0;
        for (int b = 0; b < 32; ++b) {
            int k0 = wi * 32 + b;
            if (k0 < n && group_sse(sse32, tile0, r.tpg, n, k0) <= thr) word |= (1u << b);
        }
        gmask[wi] = word;
    }
}

// ------------------------------------------------------------------- exact
// Canonical evaluation of the kept candidates over one tile: binary32 code
// (Eq.3), binary64 error  s*code + z - |w|, summed per thread in index order and
// then over the workgroup in a fixed tree.  The tile's magnitudes stay in
// registers and up to kBatch candidates share one pass.  A single-tile group
// does its own filtering (mask in LDS) and its own argmin.
struct BitCursor {
    const uint32_t *words;
    int nwords, wi;
    uint32_t word;
};
__device__ inline int next_candidate(BitCursor &c)
{
    while (c.word == 0) {
        if (++c.wi >= c.nwords) return -1;
        c.word = c.words[c.wi];
    }
    const int b = __builtin_ctz(c.word);
    c.word &= c.word - 1;
    return c.wi * 32 + b + 1;
}

__device__ inline double exact_error_sq(const Pieces &q, float a)
{
    bool tail;
    const float code = piece_code(q, a, tail);
    const double s = tail ? (double)q.s2 : (double)q.s1;
    const double z = tail ? (double)q.p : 0.0;
    const double e = (double)code * s + z - (double)a;
    return e * e;
}

struct ExactState {
    double best;
    int best_k;
    int slot;
};

// Evaluates every kept candidate over a tile whose threads hold kEpt elements
// each.  Candidates are taken one or two at a time (there are rarely more).
template <int kEpt>
__device__ inline void exact_tile(const float *__restrict__ src, int len, float m, int n, int bits,
                                  BitCursor &cur, bool single, double *__restrict__ part,
                                  double *lds, ExactState &st)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    // kEpt > 0: the thread's elements stay in registers; kEpt == 0 (long
    // tiles): they are re-read for every pass (they sit in L2)
    float a[kEpt > 0 ? kEpt : 1];
    if (kEpt > 0) {
#pragma unroll
        for (int e = 0; e < kEpt; ++e) {
            const int i = tid + e * kWG;
            a[e] = (i < len) ? fabsf(src[i]) : 0.0f;
        }
    }
    for (;;) {
        const int k0 = next_candidate(cur);
        if (k0 < 0) break;
        const int k1 = next_candidate(cur);
        const Pieces q0 = make_pieces(m, grid_point(m, k0, n), bits);
        double acc0 = 0.0, acc1 = 0.0;
        if (k1 < 0) {
            if (kEpt > 0) {
#pragma unroll
                for (int e = 0; e < kEpt; ++e)
                    if (tid + e * kWG < len) acc0 += exact_error_sq(q0, a[e]);
            } else {
                for (int i = tid; i < len; i += kWG) acc0 += exact_error_sq(q0, fabsf(src[i]));
            }
        } else {
            const Pieces q1 = make_pieces(m, grid_point(m, k1, n), bits);
            if (kEpt > 0) {
#pragma unroll
                for (int e = 0; e < kEpt; ++e) {
                    if (tid + e * kWG < len) {
                        acc0 += exact_error_sq(q0, a[e]);
                        acc1 += exact_error_sq(q1, a[e]);
                    }
                }
            } else {
                for (int i = tid; i < len; i += kWG) {
                    const float av = fabsf(src[i]);
                    acc0 += exact_error_sq(q0, av);
                    acc1 += exact_error_sq(q1, av);
                }
            }
        }
        acc0 = wave_sum(acc0);
        acc1 = wave_sum(acc1);
        __syncthreads();
        if (lane == 0) { lds[wave * 2] = acc0; lds[wave * 2 + 1] = acc1; }
        __syncthreads();
        double s0 = lds[0], s1 = lds[1];
        for (int w = 1; w < kWaves; ++w) { s0 += lds[w * 2]; s1 += lds[w * 2 + 1]; }
        if (single) {
            if (st.best_k < 0 || s0 < st.best) { st.best = s0; st.best_k = k0; }
            if (k1 >= 0 && s1 < st.best) { st.best = s1; st.best_k = k1; }
        } else if (tid == 0) {
            part[st.slot] = s0;
            if (k1 >= 0) part[st.slot + 1] = s1;
        }
        st.slot += (k1 >= 0) ? 2 : 1;
    }
}

__global__ __launch_bounds__(kWG) void k_exact(Tables tb, int n, int nwords, int bits,
                                               const float *__restrict__ gm,
                                               const float *__restrict__ sse32,
                                               const uint32_t *__restrict__ mask,
                                               double *__restrict__ part64,
                                               float *__restrict__ p_star,
                                               float *__restrict__ m_out,
                                               int32_t *__restrict__ k_star,
                                               double *__restrict__ mse)
{
    extern __shared__ uint32_t lmask[];          // single-tile groups: ceil(n/256)*8 words
    __shared__ double lds[kWaves * 2];
    const int t = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    TensorRec r;
    TileInfo ti = tile_of(tb, t, r);
    const bool single = r.tpg == 1;
    const float m = gm[ti.group];
    const long long og = r.out_group + ti.group_local;
    const bool usable = (m > 0.0f) && (m < __builtin_inff());

    BitCursor cur;
    cur.wi = -1;
    cur.word = 0;
    if (single) {
        const int lwords = (n + kWG - 1) / kWG * 8;
        if (!usable) {
            for (int wi = tid; wi < lwords; wi += kWG) lmask[wi] = (wi == 0 && m == 0.0f) ? 1u : 0u;
        } else {
            const float *row = sse32 + (long long)t * n;
            double mn = __builtin_inf();
            for (int k0 = tid; k0 < n; k0 += kWG) mn = fmin(mn, (double)row[k0]);
            mn = block_min(mn, lds);
            const double thr = keep_threshold(mn, (double)r.gcount, n);
            for (int base = 0; base < n; base += kWG) {
                const int k0 = base + tid;
                const bool keep = (k0 < n) && ((double)row[k0] <= thr);
                const unsigned long long bal = __ballot(keep);
                if (lane == 0) {
                    lmask[(base >> 5) + wave * 2] = (uint32_t)bal;
                    lmask[(base >> 5) + wave * 2 + 1] = (uint32_t)(bal >> 32);
                }
            }
        }
        __syncthreads();
        cur.words = lmask;
        cur.nwords = lwords;
    } else {
        cur.words = mask + (long long)ti.group * nwords;
        cur.nwords = nwords;
    }

    double *part = single ? nullptr
                          : part64 + (long long)(r.part_base + ti.local_tile) * n;
    ExactState st;
    st.best = 0.0;
    st.best_k = -1;
    st.slot = 0;
    if (ti.len <= kWG)
        exact_tile<1>(ti.src, ti.len, m, n, bits, cur, single, part, lds, st);
    else if (ti.len <= 4 * kWG)
        exact_tile<4>(ti.src, ti.len, m, n, bits, cur, single, part, lds, st);
    else if (ti.len <= 10 * kWG)
        exact_tile<10>(ti.src, ti.len, m, n, bits, cur, single, part, lds, st);
    else
        exact_tile<0>(ti.src, ti.len, m, n, bits, cur, single, part, lds, st);

    if (single && tid == 0) {
        m_out[og] = m;
        if (st.best_k < 0) {
            k_star[og] = -1;
            p_star[og] = __builtin_nanf("");
            mse[og] = __builtin_nan("");
        } else {
            k_star[og] = st.best_k;
            p_star[og] = grid_point(m, st.best_k, n);
            mse[og] = st.best / (double)r.gcount;
        }
    }
}

// ------------------------------------------------------------------- final
// Groups spread over several tiles: add the tiles' partial sums in tile order,
// then take the smallest sum, lowest candidate first.
__global__ __launch_bounds__(kWG) void k_final(Tables tb, int n, int nwords,
                                               const float *__restrict__ gm,
                                               const uint32_t *__restrict__ mask,
                                               const double *__restrict__ part64,
                                               float *__restrict__ p_star,
                                               float *__restrict__ m_out,
                                               int32_t *__restrict__ k_star,
                                               double *__restrict__ mse)
{
    __shared__ double lds[kWaves];
    __shared__ int slot_lds[kWaves];
    const int mg = blockIdx.x;
    const int tid = threadIdx.x;
    const int tensor = find_tensor(tb.mgroup_prefix, tb.nt, mg);
    const TensorRec r = rec_of(tb, tensor);
    const int gl = mg - r.mgroup_base;
    const int g = r.group_base + gl;
    const long long og = r.out_group + gl;
    const float m = gm[g];
    const uint32_t *gmask = mask + (long long)g * nwords;
    int nflag = 0;
    for (int wi = 0; wi < nwords; ++wi) nflag += __builtin_popcount(gmask[wi]);
    const double *part = part64 + (long long)(r.part_base + gl * r.tpg) * n;

    double best = __builtin_inf();
    int best_slot = 0x7fffffff;
    for (int s = tid; s < nflag; s += kWG) {
        double v = 0.0;
        for (int j = 0; j < r.tpg; ++j) v += part[(long long)j * n + s];
        if (v < best) { best = v; best_slot = s; }
    }
    // lexicographic (sum, slot) minimum over the workgroup
    const double wbest = block_min(best, lds);
    int cand = (best == wbest) ? best_slot : 0x7fffffff;
    for (int off = 32; off > 0; off >>= 1) {
        int o = __shfl_xor(cand, off, 64);
        cand = o < cand ? o : cand;
    }
    __syncthreads();
    if ((tid & 63) == 0) slot_lds[tid >> 6] = cand;
    __syncthreads();
    if (tid == 0) {
        for (int i = 1; i < kWaves; ++i) cand = slot_lds[i] < cand ? slot_lds[i] : cand;
        m_out[og] = m;
        if (nflag == 0 || cand == 0x7fffffff) {
            k_star[og] = -1;
            p_star[og] = __builtin_nanf("");
            mse[og] = __builtin_nan("");
        } else {
            int k = -1, seen = 0;
            for (int wi = 0; wi < nwords && k < 0; ++wi) {
                uint32_t word = gmask[wi];
                int c = __builtin_popcount(word);
                if (seen + c > cand) {
                    for (int i = 0; i < cand - seen; ++i) word &= word - 1;
                    k = wi * 32 + __builtin_ctz(word) + 1;
                }
                seen += c;
            }
            k_star[og] = k;
            p_star[og] = grid_point(m, k, n);
            mse[og] = wbest / (double)r.gcount;
        }
    }
}

// -------------------------------------------------------------------- emit
// Eq.3 with given (m, p): code, region flag and dequantized value per weight.
__device__ inline void emit_one(const Pieces &q, int bits, float w, uint8_t &code_out,
                                uint8_t &flag_out, float &hat_out)
{
    bool tail;
    const float code = piece_code(q, fabsf(w), tail);
    float v;
    if (tail) v = (code == q.L) ? q.m : __builtin_fmaf(code, q.s2, q.p);
    else v = (code == q.L) ? q.p : code * q.s1;
    const bool neg = (w < 0.0f) && (v > 0.0f);
    hat_out = neg ? -v : v;
    flag_out = tail ? 1 : 0;
    code_out = (uint8_t)((int)code | ((neg ? 1 : 0) << (bits - 1)));
}

__global__ __launch_bounds__(kWG) void k_emit(Tables tb, int bits,
                                              const float *__restrict__ p_star,
                                              const float *__restrict__ m_in,
                                              uint8_t *__restrict__ codes,
                                              uint8_t *__restrict__ flags,
                                              float *__restrict__ w_hat)
{
    const int t = blockIdx.x;
    TensorRec r;
    TileInfo ti = tile_of(tb, t, r);
    const long long og = r.out_group + ti.group_local;
    const Pieces q = make_pieces(m_in[og], p_star[og], bits);
    const long long base = r.out_elem + ti.elem_off;
    const float *src = ti.src;
    uint8_t *co = codes + base;
    uint8_t *fo = flags + base;
    float *ho = w_hat + base;
    const bool vec_ok = ((((uintptr_t)src) | ((uintptr_t)ho)) & 15) == 0 &&
                        ((((uintptr_t)co) | ((uintptr_t)fo)) & 3) == 0;
    int done = 0;
    if (vec_ok) {
        const int nvec = ti.len >> 2;
        for (int v = threadIdx.x; v < nvec; v += kWG) {
            const float4 w4 = reinterpret_cast<const float4 *>(src)[v];
            uchar4 c4, f4;
            float4 h4;
            emit_one(q, bits, w4.x, c4.x, f4.x, h4.x);
            emit_one(q, bits, w4.y, c4.y, f4.y, h4.y);
            emit_one(q, bits, w4.z, c4.z, f4.z, h4.z);
            emit_one(q, bits, w4.w, c4.w, f4.w, h4.w);
            reinterpret_cast<uchar4 *>(co)[v] = c4;
            reinterpret_cast<uchar4 *>(fo)[v] = f4;
            reinterpret_cast<float4 *>(ho)[v] = h4;
        }
        done = nvec << 2;
    }
    for (int i = done + threadIdx.x; i < ti.len; i += kWG)
        emit_one(q, bits, src[i], co[i], fo[i], ho[i]);
}

} // namespace pwlq
