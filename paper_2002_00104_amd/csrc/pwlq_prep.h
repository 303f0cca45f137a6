// k_tile_absmax and k_prep: group absmax, rescaling to candidate units, partition by candidate block.
#pragma once

#include "pwlq_tables.h"

namespace pwlq {

// ------------------------------------------------------------------ absmax
// Only groups cut into several tiles need this pass; a single-tile group finds
// its absmax inside k_prep.
__global__ __launch_bounds__(kWG) void k_tile_absmax(Tables tb, float *__restrict__ tile_max)
{
    __shared__ float red[kWaves];
    __shared__ int redbad[kWaves];
    int t;
    TensorRec r;
    TileInfo ti = tile_of(tb, blockIdx.x, r, t);
    if (r.tpg == 1) return;
    float mx = 0.0f;
    int bad = 0;
    int i = threadIdx.x;
    for (; i + 3 * kWG < ti.len; i += 4 * kWG) {       // four loads in flight per thread
        const float a0 = fabsf(ti.src[i]), a1 = fabsf(ti.src[i + kWG]), a2 = fabsf(ti.src[i + 2 * kWG]),
                    a3 = fabsf(ti.src[i + 3 * kWG]);
        bad |= (a0 != a0) | (a1 != a1) | (a2 != a2) | (a3 != a3);
        mx = fmaxf(fmaxf(mx, fmaxf(a0, a1)), fmaxf(a2, a3));
    }
    for (; i < ti.len; i += kWG) {
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
// `scale` = n/m rounded once: two roundings per element, as many as (a/m)*n has,
// and no division per element.
__device__ inline float to_units(float a, float scale, float nf)
{
    float u = a * scale;
    return fminf(fmaxf(u, 0.0f), nf);     // also maps a NaN to 0
}
// smallest candidate with u <= k, 0-based
__device__ inline int candidate_bin(float u, int n)
{
    int kc = (int)ceilf(u);
    kc = kc < 1 ? 1 : kc;
    return (kc > n ? n : kc) - 1;
}
__device__ inline int bucket_of(float u)
{
    int kc = (int)ceilf(u);          // smallest candidate with u <= k
    kc = kc < 1 ? 1 : kc;
    return (kc - 1) >> 6;
}

// Sorted layout of one tile: [pad zeros][bucket 0][bucket 1]...; the padded
// length is a multiple of kVec and off[j] is the start of bucket j.  The tile's
// elements stay in registers between the passes, so the weights are read from
// memory once.  A workgroup has kT threads holding kPer elements each (256 x 32
// for any tile, 64 x 16 for tiles of at most kSmallTile elements: one wavefront
// per tile, so that four times as many short tiles are in flight and no barrier
// waits on another wavefront).  kPrivate (at most 32 buckets): every
// thread counts into its own histogram column and positions are assigned in
// (bucket, thread, element) order, so the layout is repeatable; otherwise LDS
// integer atomics assign positions inside a bucket in arrival order.  kFine: the
// tile is ordered by ceil(u), i.e. by the first candidate for which the element
// is a centre element (one bin per candidate), and the position at which every
// candidate switches from centre to tail is written as well; the search kernel
// then knows the region of a whole vector of elements without comparing values.
template <bool kPrivate, bool kFine, int kT, int kPer>
__global__ __launch_bounds__(kT) void k_prep(Tables tb, int tile_begin, int n, int nblk,
                                               const float *__restrict__ tile_max,
                                               float *__restrict__ gm,
                                               int *__restrict__ offsets,
                                               unsigned short *__restrict__ fine,
                                               float *__restrict__ sorted)
{
    static_assert(!(kPrivate && kFine), "the fine order uses shared counters");
    extern __shared__ int hist[];     // kPrivate: [ceil(nblk/2)][kT] packed pairs, else [bins]
    constexpr int kW = kT / 64;
    __shared__ float redm[kW];
    __shared__ int redbad[kW];
    __shared__ int wtot[32 * kW];
    __shared__ int wpair[16 * kW];
    __shared__ int scan_lds[kW];
    int t;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    TensorRec r;
    TileInfo ti = tile_of(tb, tile_begin + blockIdx.x, r, t);
    if (r.fast) return;               // evaluated by k_fast
    const int len = ti.len;

    float a[kPer];
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
        const int i = tid + e * kT;
        a[e] = (i < len) ? fabsf(ti.src[i]) : 0.0f;
    }

    // group absmax: from the registers (single-tile group) or the tile maxima
    float m = 0.0f;
    int bad = 0;
    if (r.tpg == 1) {
#pragma unroll
        for (int e = 0; e < kPer; ++e) { bad |= (a[e] != a[e]); m = fmaxf(m, a[e]); }
    } else {
        const int tile0 = r.tile_base + ti.group_local * r.tpg;
        for (int j = tid; j < r.tpg; j += kT) {
            float v = tile_max[tile0 + j];
            bad |= (v != v);
            m = fmaxf(m, v);
        }
    }
    m = wave_max(m);
    bad = wave_or(bad);
    if (lane == 0) { redm[wave] = m; redbad[wave] = bad; }
    const int bins = kFine ? n : nblk;     // kFine: one bin per candidate (ceil(u) = 1..n)
    if (!kPrivate) for (int i = tid; i < bins; i += kT) hist[i] = 0;
    __syncthreads();
    m = redm[0];
    bad = redbad[0];
    for (int i = 1; i < kW; ++i) { m = fmaxf(m, redm[i]); bad |= redbad[i]; }
    if (bad) m = __builtin_nanf("");
    if (ti.tile_in_group == 0 && tid == 0) gm[ti.group] = m;

    const bool usable = (m > 0.0f) && (m < __builtin_inff());
    const float nf = (float)n;
    const float scale = usable ? nf / m : 0.0f;
    const int padded = (len + kVec - 1) / kVec * kVec;
    const int pad = padded - len;
    float *out = sorted + ti.sorted_off;
    int *off = offsets + (long long)t * (nblk + 1);

    // pass A: units and histogram
    // kPrivate: a thread's counts of buckets 2w and 2w+1 share one word (16 bits
    // each: a thread holds at most 32 elements and a wavefront 2048, so neither
    // the counts nor their prefix sums carry into the other half)
    const int nb2 = (nblk + 1) >> 1;
    if (kPrivate) for (int w = 0; w < nb2; ++w) hist[w * kT + tid] = 0;
    // shared counters: the value the add returns is the element's rank inside its bin (in
    // arrival order), kept for pass B, which then needs no second round of atomics
    int rank[kPrivate ? 1 : kPer];
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
        const int i = tid + e * kT;
        if (i < len) {
            const float u = usable ? to_units(a[e], scale, nf) : 0.0f;
            a[e] = u;
            const int b = kFine ? candidate_bin(u, n) : bucket_of(u);
            // private column: fire-and-forget LDS add; the atomic form only keeps the
            // updates pipelined instead of read-modify-write round trips
            if (kPrivate) atomicAdd(&hist[(b >> 1) * kT + tid], 1 << (16 * (b & 1)));
            else rank[e] = atomicAdd(&hist[b], 1);
        }
    }

    // exclusive positions
    if (kPrivate) {
        for (int w = 0; w < nb2; ++w) {
            const int c = hist[w * kT + tid];
            const int incl = wave_scan_incl(c);             // both halves at once
            hist[w * kT + tid] = incl - c;                 // exclusive inside the wavefront
            if (lane == 63) wpair[w * kW + wave] = incl;
        }
        __syncthreads();
        if (wave == 0) {
            int w[kW];
            int tot = 0;
#pragma unroll
            for (int i = 0; i < kW; ++i) {
                w[i] = (lane < nblk)
                           ? (wpair[(lane >> 1) * kW + i] >> (16 * (lane & 1))) & 0xffff
                           : 0;
                tot += w[i];
            }
            int run = wave_scan_incl(tot) - tot;            // first position of bucket `lane`
            if (lane < nblk) {
                off[lane] = pad + run;
#pragma unroll
                for (int i = 0; i < kW; ++i) { wtot[lane * kW + i] = run; run += w[i]; }
            }
            if (lane == 0) off[nblk] = pad + len;
        }
    } else {
        __syncthreads();
        const int per = (bins + kT - 1) / kT;
        const int lo = tid * per;
        int hi = lo + per;
        if (hi > bins) hi = bins;
        int sum = 0;
        for (int i = lo; i < hi; ++i) sum += hist[i];
        const int incl = wave_scan_incl(sum);
        if (lane == 63) scan_lds[wave] = incl;
        __syncthreads();
        int run = incl - sum;
        for (int i = 0; i < wave; ++i) run += scan_lds[i];
        unsigned short *fo = kFine ? fine + (long long)t * (n + 1) : nullptr;
        for (int i = lo; i < hi; ++i) {
            const int v = hist[i];
            hist[i] = run;
            if (kFine) {
                // position of the first element whose ceil(u) exceeds i: where candidate i
                // (1-based; entry 0 is the start) switches from centre to tail
                fo[i] = (unsigned short)(pad + run);
                if ((i & (kBlk - 1)) == 0) off[i >> 6] = pad + run;
            } else {
                off[i] = pad + run;
            }
            run += v;
        }
        if (tid == 0) {
            off[nblk] = pad + len;
            if (kFine) fo[n] = (unsigned short)(pad + len);
        }
    }
    // pass B: scatter into the LDS image of the sorted tile, then write it out
    // with full-width coalesced stores (scattered 4-byte stores to memory cost
    // one transaction each)
    float *stage = reinterpret_cast<float *>(hist + (kPrivate ? nb2 * kT : bins));
    for (int i = tid; i < pad; i += kT) stage[i] = 0.0f;
    __syncthreads();
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
        const int i = tid + e * kT;
        if (i < len) {
            const float u = a[e];
            const int b = kFine ? candidate_bin(u, n) : bucket_of(u);
            int pos;
            if (kPrivate) {
                const int sh = 16 * (b & 1);
                const int old = atomicAdd(&hist[(b >> 1) * kT + tid], 1 << sh);
                pos = wtot[b * kW + wave] + ((old >> sh) & 0xffff);
            }
            else {
                pos = hist[b] + rank[e];          // hist now holds the first position of each bin
            }
            stage[pad + pos] = u;
        }
    }
    __syncthreads();
    for (int i = tid * 4; i < padded; i += kT * 4)
        *reinterpret_cast<float4 *>(out + i) = *reinterpret_cast<const float4 *>(stage + i);
}

} // namespace pwlq
