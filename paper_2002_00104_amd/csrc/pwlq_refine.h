// k_group_sum, k_flag, k_exact, k_final: filter by the binary32 SSE, exact
// binary64 re-evaluation of the kept candidates, argmin.
#pragma once

#include "pwlq_tables.h"

namespace pwlq {

// -------------------------------------------------------------------- flag
// The binary32 SSE of k_search (candidate units) is only a filter: every
// candidate within the rounding slack of the minimum is kept and re-evaluated
// exactly.  The slack bounds twice the error of k_search: eps = 2^-21 n per
// element error (candidate units) and 3e-5 relative for the binary32 sums.
// Tiles evaluated by prefix sums add the bound of that arithmetic
// (kFastRelErr n^2 per element).
constexpr double kFastRelErr = 3.0e-11;
__device__ inline double keep_threshold(double mn, double count, int n, bool fast)
{
    const double eps = (double)n * 4.76837158203125e-07;   // 2^-21 n
    const double extra = fast ? kFastRelErr * (double)n * (double)n * count : 0.0;
    return mn + 2.0 * (3e-5 * mn + 2.0 * eps * sqrt(count * mn) + count * eps * eps + extra);
}

// Groups spread over several tiles, step 1: add the tiles' binary32 sums in
// binary64.  A workgroup takes 32 candidates of one group; thread (c, ph) adds
// the tiles ph, ph+8, ph+16, ... of candidate c in that order, and the 8 partial
// sums are added in phase order, so the result is repeatable.  (One thread per
// candidate walking all tiles left a group of 2048 tiles to four workgroups.)
constexpr int kSumCand = 32, kSumPhases = kWG / kSumCand;
__global__ __launch_bounds__(kWG) void k_group_sum(Tables tb, int n,
                                                   const float *__restrict__ sse32,
                                                   double *__restrict__ gsum)
{
    __shared__ double part[kSumPhases][kSumCand];
    const int nbx = (n + kSumCand - 1) / kSumCand;             // workgroups per group
    const int mg = blockIdx.x / nbx;
    const int c = threadIdx.x & (kSumCand - 1), ph = threadIdx.x / kSumCand;
    const int k0 = (blockIdx.x - mg * nbx) * kSumCand + c;
    const int tensor = find_tensor(tb.mgroup_prefix, tb.nt, mg);
    const TensorRec r = rec_of(tb, tensor);
    const int gl = mg - r.mgroup_base;
    const long long tile0 = r.tile_base + (long long)gl * r.tpg;
    double v = 0.0;
    if (k0 < n) {
        int j = ph;
        for (; j + 3 * kSumPhases < r.tpg; j += 4 * kSumPhases) {     // four loads in flight, added in the same order
            const float x0 = sse32[(tile0 + j) * n + k0], x1 = sse32[(tile0 + j + kSumPhases) * n + k0],
                        x2 = sse32[(tile0 + j + 2 * kSumPhases) * n + k0],
                        x3 = sse32[(tile0 + j + 3 * kSumPhases) * n + k0];
            v += (double)x0;
            v += (double)x1;
            v += (double)x2;
            v += (double)x3;
        }
        for (; j < r.tpg; j += kSumPhases) v += (double)sse32[(tile0 + j) * n + k0];
    }
    part[ph][c] = v;
    __syncthreads();
    if (ph == 0 && k0 < n) {
        double s = part[0][c];
        for (int i = 1; i < kSumPhases; ++i) s += part[i][c];
        gsum[(long long)mg * n + k0] = s;
    }
}

// Step 2: the group's minimum and the ascending list of kept candidates:
// klist[mg][0] = count, klist[mg][1..count] = candidates (1-based).
__global__ __launch_bounds__(kWG) void k_flag(Tables tb, int n,
                                              const float *__restrict__ gm,
                                              const double *__restrict__ gsum,
                                              int *__restrict__ klist)
{
    __shared__ double lds[kWaves];
    __shared__ int wcount[kWaves];
    const int mg = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int tensor = find_tensor(tb.mgroup_prefix, tb.nt, mg);
    const TensorRec r = rec_of(tb, tensor);
    const int g = r.group_base + (mg - r.mgroup_base);
    int *list = klist + (long long)mg * (n + 1);
    const double *row = gsum + (long long)mg * n;
    const float m = gm[g];
    if (!(m > 0.0f) || !(m < __builtin_inff())) {
        // all-zero group: every candidate has zero error, the first wins.
        // non-finite group: nothing to evaluate.
        if (tid == 0) {
            list[0] = (m == 0.0f) ? 1 : 0;
            list[1] = 1;
        }
        return;
    }
    double mn = __builtin_inf();
    for (int k0 = tid; k0 < n; k0 += kWG) mn = fmin(mn, row[k0]);
    mn = block_min(mn, lds);
    const double thr = keep_threshold(mn, (double)r.gcount, n, r.fast != 0);
    int total = 0;
    for (int base = 0; base < n; base += kWG) {
        const int k0 = base + tid;
        const bool keep = (k0 < n) && (row[k0] <= thr);
        const unsigned long long bal = __ballot(keep);
        __syncthreads();
        if (lane == 0) wcount[wave] = __builtin_popcountll(bal);
        __syncthreads();
        int before = total;
        for (int w = 0; w < wave; ++w) before += wcount[w];
        if (keep) list[1 + before + __builtin_popcountll(bal & ((1ull << lane) - 1ull))] = k0 + 1;
        for (int w = 0; w < kWaves; ++w) total += wcount[w];
    }
    if (tid == 0) list[0] = total;
}

// ------------------------------------------------------------------- exact
// Canonical evaluation of the kept candidates over one tile: binary32 code
// (Eq.3), binary64 error  s*code + z - |w|, summed per thread in index order and
// then over the workgroup in a fixed order.
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
};

// Evaluates list[0..count) over a tile whose threads hold kEpt elements each
// (kEpt == 0: long tile, re-read from memory for every pass).  Candidates are
// taken one or two at a time (there are rarely more).  Single-tile groups keep
// the lexicographic (sum, k) minimum, so the order of the list does not matter;
// tiles of longer groups store the sums in list order.
template <int kEpt, int kT>
__device__ inline void load_tile(const float *__restrict__ src, int len,
                                 float (&a)[kEpt > 0 ? kEpt : 1])
{
    if (kEpt > 0) {
#pragma unroll
        for (int e = 0; e < kEpt; ++e) {
            const int i = threadIdx.x + e * kT;
            a[e] = (i < len) ? fabsf(src[i]) : 0.0f;
        }
    }
}

template <int kEpt, int kT>
__device__ inline void exact_tile(const float *__restrict__ src, int len,
                                  const float (&a)[kEpt > 0 ? kEpt : 1], float m, int n, int bits,
                                  const int *list, int count, bool single,
                                  double *__restrict__ part, double *lds, ExactState &st)
{
    constexpr int kW = kT / 64;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    for (int c = 0; c < count; c += 2) {
        const int k0 = list[c];
        const int k1 = (c + 1 < count) ? list[c + 1] : -1;
        const Pieces q0 = make_pieces(m, grid_point(m, k0, n), bits);
        double acc0 = 0.0, acc1 = 0.0;
        if (k1 < 0) {
            if (kEpt > 0) {
#pragma unroll
                for (int e = 0; e < kEpt; ++e)
                    if (tid + e * kT < len) acc0 += exact_error_sq(q0, a[e]);
            } else {
                // eight, then four loads in flight per thread: the pass is bound by their latency
                int i = tid;
                for (; i + 7 * kT < len; i += 8 * kT) {
                    float av[8];
#pragma unroll
                    for (int x = 0; x < 8; ++x) av[x] = fabsf(src[i + x * kT]);
#pragma unroll
                    for (int x = 0; x < 8; ++x) acc0 += exact_error_sq(q0, av[x]);
                }
                for (; i + 3 * kT < len; i += 4 * kT) {
                    const float a0 = fabsf(src[i]), a1 = fabsf(src[i + kT]),
                                a2 = fabsf(src[i + 2 * kT]), a3 = fabsf(src[i + 3 * kT]);
                    acc0 += exact_error_sq(q0, a0);
                    acc0 += exact_error_sq(q0, a1);
                    acc0 += exact_error_sq(q0, a2);
                    acc0 += exact_error_sq(q0, a3);
                }
                for (; i < len; i += kT) acc0 += exact_error_sq(q0, fabsf(src[i]));
            }
        } else {
            const Pieces q1 = make_pieces(m, grid_point(m, k1, n), bits);
            if (kEpt > 0) {
#pragma unroll
                for (int e = 0; e < kEpt; ++e) {
                    if (tid + e * kT < len) {
                        acc0 += exact_error_sq(q0, a[e]);
                        acc1 += exact_error_sq(q1, a[e]);
                    }
                }
            } else {
                int i = tid;
                for (; i + 7 * kT < len; i += 8 * kT) {
                    float av[8];
#pragma unroll
                    for (int x = 0; x < 8; ++x) av[x] = fabsf(src[i + x * kT]);
#pragma unroll
                    for (int x = 0; x < 8; ++x) {
                        acc0 += exact_error_sq(q0, av[x]);
                        acc1 += exact_error_sq(q1, av[x]);
                    }
                }
                for (; i + 3 * kT < len; i += 4 * kT) {
                    const float a0 = fabsf(src[i]), a1 = fabsf(src[i + kT]),
                                a2 = fabsf(src[i + 2 * kT]), a3 = fabsf(src[i + 3 * kT]);
                    acc0 += exact_error_sq(q0, a0);
                    acc1 += exact_error_sq(q1, a0);
                    acc0 += exact_error_sq(q0, a1);
                    acc1 += exact_error_sq(q1, a1);
                    acc0 += exact_error_sq(q0, a2);
                    acc1 += exact_error_sq(q1, a2);
                    acc0 += exact_error_sq(q0, a3);
                    acc1 += exact_error_sq(q1, a3);
                }
                for (; i < len; i += kT) {
                    const float av = fabsf(src[i]);
                    acc0 += exact_error_sq(q0, av);
                    acc1 += exact_error_sq(q1, av);
                }
            }
        }
        acc0 = wave_sum(acc0);
        acc1 = wave_sum(acc1);
        double s0 = acc0, s1 = acc1;
        if (kW > 1) {
            __syncthreads();
            if (lane == 0) { lds[wave * 2] = acc0; lds[wave * 2 + 1] = acc1; }
            __syncthreads();
            s0 = lds[0];
            s1 = lds[1];
            for (int w = 1; w < kW; ++w) { s0 += lds[w * 2]; s1 += lds[w * 2 + 1]; }
        }
        if (single) {
            if (st.best_k < 0 || s0 < st.best || (s0 == st.best && k0 < st.best_k)) {
                st.best = s0;
                st.best_k = k0;
            }
            if (k1 >= 0 && (s1 < st.best || (s1 == st.best && k1 < st.best_k))) {
                st.best = s1;
                st.best_k = k1;
            }
        } else if (tid == 0) {
            part[c] = s0;
            if (k1 >= 0) part[c + 1] = s1;
        }
    }
}

constexpr int kListCap = 2048;   // kept candidates of a single-tile group, per round (256-thread workgroups)
constexpr int kListCapSmall = 1024;   // ... of a one-wavefront workgroup
template <int kT> struct RowRegs { static constexpr int value = 1024 / kT; };   // 1024 candidates either way

// The thread's elements are loaded first, so that their memory latency
// overlaps the filtering that follows.
template <int kEpt, int kT, int kCap>
__device__ inline void exact_body(const TensorRec &r, const TileInfo &ti, int t, int n, int bits,
                                  const float *__restrict__ gm, const float *__restrict__ sse32,
                                  const int *__restrict__ klist, double *__restrict__ part64,
                                  float *__restrict__ p_star, float *__restrict__ m_out,
                                  int32_t *__restrict__ k_star, double *__restrict__ mse,
                                  int *llist, int *lcount, double *lds)
{
    const int tid = threadIdx.x;
    float a[kEpt > 0 ? kEpt : 1];
    load_tile<kEpt, kT>(ti.src, ti.len, a);
    const bool single = r.tpg == 1;
    // Up to kRowRegs * kT candidates: a single-tile group's row of filter sums stays in
    // registers between the two passes over it (minimum, then selection).  Its loads are
    // issued here, together with the elements' and before anything waits for the group's
    // absmax: the kernel is bound by the latency of its loads, not by their volume.
    constexpr int kRowRegs = RowRegs<kT>::value;
    const bool in_regs = n <= kRowRegs * kT;
    const float *row = sse32 + (long long)t * n;
    float rv[kRowRegs];
    if (single && in_regs) {
#pragma unroll
        for (int x = 0; x < kRowRegs; ++x) {
            const int k0 = tid + x * kT;
            rv[x] = (k0 < n) ? row[k0] : __builtin_inff();
        }
    }
    const float m = gm[ti.group];
    const long long og = r.out_group + ti.group_local;
    const bool usable = (m > 0.0f) && (m < __builtin_inff());
    ExactState st;
    st.best = 0.0;
    st.best_k = -1;

    if (!single) {
        // the group's list was built by k_flag; sums go to this tile's row
        const int mg = r.mgroup_base + ti.group_local;
        const int *list = klist + (long long)mg * (n + 1);
        const int count = uni(list[0]);
        double *part = part64 + (long long)(r.part_base + ti.local_tile) * n;
        exact_tile<kEpt, kT>(ti.src, ti.len, a, m, n, bits, list + 1, count, false, part, lds, st);
        return;
    }

    // single-tile group: filter here, a round of at most kCap candidates at a time
    if (m == 0.0f) {
        if (tid == 0) llist[0] = 1;
        __syncthreads();
        exact_tile<kEpt, kT>(ti.src, ti.len, a, m, n, bits, llist, 1, true, nullptr, lds, st);
    } else if (usable) {
        float mnf = __builtin_inff();
        if (in_regs) {
#pragma unroll
            for (int x = 0; x < kRowRegs; ++x) mnf = fminf(mnf, rv[x]);
        } else {
            int k0 = tid;
            for (; k0 + 3 * kT < n; k0 += 4 * kT) {
                const float v0 = row[k0], v1 = row[k0 + kT], v2 = row[k0 + 2 * kT], v3 = row[k0 + 3 * kT];
                mnf = fminf(fminf(mnf, fminf(v0, v1)), fminf(v2, v3));
            }
            for (; k0 < n; k0 += kT) mnf = fminf(mnf, row[k0]);
        }
        const double mn = block_min<kT / 64>((double)mnf, lds);
        const double thr = keep_threshold(mn, (double)r.gcount, n, r.fast != 0);
        // the sums are binary32: v <= thr exactly when v <= the largest binary32 value not above thr
        float thrf = (float)thr;
        if ((double)thrf > thr) thrf = __int_as_float(__float_as_int(thrf) - 1);   // thr >= 0: the value below
        for (int rbase = 0; rbase < n; rbase += kCap) {
            __syncthreads();
            if (tid == 0) *lcount = 0;
            __syncthreads();
            const int rend = (rbase + kCap < n) ? rbase + kCap : n;
            if (in_regs) {
#pragma unroll
                for (int x = 0; x < kRowRegs; ++x) {
                    const int k0 = tid + x * kT;
                    if (k0 >= rbase && k0 < rend && rv[x] <= thrf) llist[atomicAdd(lcount, 1)] = k0 + 1;
                }
            } else {
                for (int k0 = rbase + tid; k0 < rend; k0 += kT)
                    if (row[k0] <= thrf) llist[atomicAdd(lcount, 1)] = k0 + 1;
            }
            __syncthreads();
            const int count = uni(*lcount);
            exact_tile<kEpt, kT>(ti.src, ti.len, a, m, n, bits, llist, count, true, nullptr, lds, st);
        }
    }
    if (tid == 0) {
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

// The kernel waits on chains of dependent loads (table, tile, filter row,
// elements), so wavefronts in flight are what it runs on: the 128-thread
// variant fits 78 registers, six wavefronts per SIMD, without spilling (the
// one-wavefront variant spills below 111 and measured slower there).
// kMaxPer (one-wavefront variant): the most elements a thread holds, 16 for tiles up to 1024
// elements, 8 when the launch only sees tiles up to 512 (then 6 wavefronts per SIMD too).
template <int kT, int kMaxPer = 16>
__global__ __launch_bounds__(kT, (kT == 128 || (kT == 64 && kMaxPer == 8)) ? 6 : 1) void k_exact(Tables tb, int tile_begin, int n, int bits,
                                              const float *__restrict__ gm,
                                              const float *__restrict__ sse32,
                                              const int *__restrict__ klist,
                                              double *__restrict__ part64,
                                              float *__restrict__ p_star,
                                              float *__restrict__ m_out,
                                              int32_t *__restrict__ k_star,
                                              double *__restrict__ mse)
{
    constexpr int kCap = (kT == 64) ? kListCapSmall : kListCap;
    __shared__ int llist[kCap];
    __shared__ int lcount;
    __shared__ double lds[(kT / 64) * 2];
    int t;
    TensorRec r;
    TileInfo ti = tile_of(tb, tile_begin + blockIdx.x, r, t);
#define PWLQ_EXACT(E)                                                                              \
    exact_body<E, kT, kCap>(r, ti, t, n, bits, gm, sse32, klist, part64, p_star, m_out, k_star,    \
                            mse, llist, &lcount, lds)
    if (kT == 64) {                    // one wavefront per tile of at most kSmallTile elements
        if (ti.len <= 64) PWLQ_EXACT(1);
        else if (ti.len <= 128) PWLQ_EXACT(2);
        else if (ti.len <= 256) PWLQ_EXACT(4);
        else if (ti.len <= 512 || kMaxPer == 8) PWLQ_EXACT(8);
        else if (ti.len <= 640) PWLQ_EXACT(10);
        else PWLQ_EXACT(kSmallPer);
    } else {
        if (ti.len <= kT) PWLQ_EXACT(1);
        else if (ti.len <= 4 * kT) PWLQ_EXACT(4);
        else if (ti.len <= 10 * kT) PWLQ_EXACT(10);
        else PWLQ_EXACT(0);     // longer tiles are re-read per pass: holding 16 per thread measured 15 % slower
    }
#undef PWLQ_EXACT
}

// ------------------------------------------------------------------- final
// Groups spread over several tiles: add the tiles' partial sums in tile order,
// then take the smallest sum, lowest candidate first (the list is ascending).
__global__ __launch_bounds__(kWG) void k_final(Tables tb, int n,
                                               const float *__restrict__ gm,
                                               const int *__restrict__ klist,
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
    const int *list = klist + (long long)mg * (n + 1);
    const int count = list[0];
    const double *part = part64 + (long long)(r.part_base + gl * r.tpg) * n;

    // Kept candidates are few and a group can have hundreds of tiles: one
    // wavefront per candidate, lanes over the tiles (lane l adds tiles l, l+64, ...
    // in order, then the 64 partial sums are added in lane order), so the order of
    // the additions is fixed.
    double best = __builtin_inf();
    int best_slot = 0x7fffffff;
    const int lane = tid & 63, wave = tid >> 6;
    for (int s = wave; s < count; s += kWaves) {
        double v = 0.0;
        for (int j = lane; j < r.tpg; j += 64) v += part[(long long)j * n + s];
        v = wave_sum(v);
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
        if (count == 0 || cand == 0x7fffffff) {
            k_star[og] = -1;
            p_star[og] = __builtin_nanf("");
            mse[og] = __builtin_nan("");
        } else {
            const int k = list[1 + cand];
            k_star[og] = k;
            p_star[og] = grid_point(m, k, n);
            mse[og] = wbest / (double)r.gcount;
        }
    }
}

} // namespace pwlq
