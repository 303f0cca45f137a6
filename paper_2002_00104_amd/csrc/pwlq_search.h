// k_search: the candidate-evaluation kernel (dominant).
#pragma once

#include "pwlq_tables.h"

namespace pwlq {

// One wavefront = one block of 64 candidates of one tile; lane = candidate;
// the 16 wavefronts of a workgroup take 16 consecutive blocks of the same tile,
// so they stream the same cache lines through one scalar cache.
//
// In candidate units the centre piece of candidate k has step k/L and the tail
// piece (n-k)/L, so the position of u in steps is  t = u*(L/k)  or
// t = (u-k)*(L/(n-k)), and the error in steps is f = t - rne(t).  Sum f^2 per
// region, scale by step^2 at the end.  None of this depends on the group's
// absmax.  Elements arrive as wave-uniform scalar loads (SGPR operands).
__device__ inline float8 load8(const float *__restrict__ p)
{
    return *reinterpret_cast<const float8 *>(__builtin_assume_aligned(p, 32));
}

template <bool kTail>
__device__ inline void eval8(const float8 &x, float r, float c, float &acc0, float &acc1)
{
#pragma unroll
    for (int e = 0; e < kVec; e += 2) {
        const float t0 = kTail ? __builtin_fmaf(x[e], r, c) : x[e] * r;
        const float t1 = kTail ? __builtin_fmaf(x[e + 1], r, c) : x[e + 1] * r;
        const float f0 = t0 - __builtin_rintf(t0);
        const float f1 = t1 - __builtin_rintf(t1);
        acc0 = __builtin_fmaf(f0, f0, acc0);
        acc1 = __builtin_fmaf(f1, f1, acc1);
    }
}

// All 64 candidates see every element of us[begin, end) in the same region.
template <bool kTail>
__device__ inline float zone_one_region(const float *__restrict__ us, int begin, int end,
                                        float r, float c)
{
    float outer = 0.0f;
    for (int cb = begin; cb < end; cb += kChunk) {
        const int ce = (cb + kChunk < end) ? cb + kChunk : end;
        float acc0 = 0.0f, acc1 = 0.0f;
        for (int i = cb; i < ce; i += kVec) {
            const float8 x = load8(us + i);
            eval8<kTail>(x, r, c, acc0, acc1);
        }
        outer += acc0 + acc1;
    }
    return outer;
}

// The wavefront's own bucket: the region differs from lane to lane.  Both
// positions are computed and selected per lane (compare, two selects); masking
// the two regions one after the other costs more, because every change of the
// execution mask waits for the comparison.  The error is summed in candidate
// units.
__device__ inline float zone_mixed(const float *__restrict__ us, int begin, int end, float kf,
                                   float rc, float rt, float ct, float stepc, float stept)
{
    float outer = 0.0f;
    for (int cb = begin; cb < end; cb += kChunk) {
        const int ce = (cb + kChunk < end) ? cb + kChunk : end;
        float acc = 0.0f;
        for (int i = cb; i < ce; i += kVec) {
            const float8 cur = load8(us + i);
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                const float u = cur[e];
                const bool tail = u > kf;
                const float tc = u * rc;
                const float tt = __builtin_fmaf(u, rt, ct);
                const float t = tail ? tt : tc;
                const float step = tail ? stept : stepc;
                const float err = (t - __builtin_rintf(t)) * step;
                acc = __builtin_fmaf(err, err, acc);
            }
        }
        outer += acc;
    }
    return outer;
}

// One vector of 8 elements in the per-lane form (see zone_mixed).
__device__ inline void mixed8(const float8 &cur, float kf, float rc, float rt, float ct,
                              float stepc, float stept, float &acc)
{
#pragma unroll
    for (int e = 0; e < kVec; ++e) {
        const float u = cur[e];
        const bool tail = u > kf;
        const float tc = u * rc;
        const float tt = __builtin_fmaf(u, rt, ct);
        const float t = tail ? tt : tc;
        const float step = tail ? stept : stepc;
        const float err = (t - __builtin_rintf(t)) * step;
        acc = __builtin_fmaf(err, err, acc);
    }
}

// The same bucket when the tile is ordered by ceil(u) and `sw` is the position at
// which this lane's candidate switches from centre to tail.  A vector of 8
// elements that lies on one side of the lane's switch is evaluated with the
// lane's own multiplier and offset, selected once per vector: no per-element
// compare, no branch.  The one vector that holds the lane's switch contributes
// nothing in that loop; every lane evaluates its own switch vector afterwards,
// element by element (a per-lane load of 32 bytes, once per tile).
__device__ inline void zone_mixed_fine(const float *__restrict__ us, int begin, int end, int sw,
                                       float kf, float rc, float rt, float ct, float &sum_c,
                                       float &sum_t)
{
    for (int cb = begin; cb < end; cb += kChunk) {
        const int ce = (cb + kChunk < end) ? cb + kChunk : end;
        float acc_c = 0.0f, acc_t = 0.0f;
        for (int i = cb; i < ce; i += kVec) {
            const float8 cur = load8(us + i);
            const bool cen = sw >= i + kVec;
            const bool tl = sw <= i;
            const float R = cen ? rc : rt, C = cen ? 0.0f : ct;
            float s0 = 0.0f, s1 = 0.0f;
#pragma unroll
            for (int e = 0; e < kVec; e += 2) {
                const float t0 = __builtin_fmaf(cur[e], R, C);
                const float t1 = __builtin_fmaf(cur[e + 1], R, C);
                const float f0 = t0 - __builtin_rintf(t0);
                const float f1 = t1 - __builtin_rintf(t1);
                s0 = __builtin_fmaf(f0, f0, s0);
                s1 = __builtin_fmaf(f1, f1, s1);
            }
            const float sv = s0 + s1;
            acc_c += cen ? sv : 0.0f;
            acc_t += tl ? sv : 0.0f;
        }
        sum_c += acc_c;
        sum_t += acc_t;
    }
    // the lane's own switch vector (none if the switch falls between two vectors)
    const bool has = (sw & (kVec - 1)) != 0;
    const int i0 = has ? (sw & ~(kVec - 1)) : begin;
    const float4 v0 = *reinterpret_cast<const float4 *>(us + i0);
    const float4 v1 = *reinterpret_cast<const float4 *>(us + i0 + 4);
    const float own[kVec] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
    float oc = 0.0f, ot = 0.0f;
#pragma unroll
    for (int e = 0; e < kVec; ++e) {
        const float u = own[e];
        const bool tail = u > kf;
        const float t = tail ? __builtin_fmaf(u, rt, ct) : u * rc;
        const float f = t - __builtin_rintf(t);
        const float g = f * f;
        oc += tail ? 0.0f : g;
        ot += tail ? g : 0.0f;
    }
    sum_c += has ? oc : 0.0f;
    sum_t += has ? ot : 0.0f;
}

__global__ __launch_bounds__(kSearchWaves * 64) void k_search(Tables tb, int n, int nblk, int bits,
                                                              int ny, int upw, int bpw_log2,
                                                              const int *__restrict__ offsets,
                                                              const float *__restrict__ sorted,
                                                              const unsigned short *__restrict__ fine,
                                                              int fine_tiles,
                                                              float *__restrict__ sse32)
{
    // Workgroup ids are dealt round-robin to the 8 XCDs.  The ny workgroups of
    // one unit (same tiles, different candidate blocks) stay on one XCD so its L2
    // serves their reads.  Unit groups are dealt to the XCDs with a rotation per
    // row of 8, so that a pattern in the tile order (a long group cut into a full
    // and a short tile alternates the two) does not always meet the same XCDs.
    // With fewer than 16 candidate blocks a workgroup's wavefronts are shared by
    // upw = 16 / bpw units (bpw: blocks rounded up to a power of two).
    const int wg = blockIdx.x;
    const int xcd = wg & 7;
    const int slot = wg >> 3;
    const int q = slot / ny;
    const int jy = slot - q * ny;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int ug = q * 8 + ((xcd + q) & 7);
    const int unit = ug * upw + (wave >> bpw_log2);
    const int j = jy * kSearchWaves + (wave & ((1 << bpw_log2) - 1));
    if (unit >= tb.n_units || j >= nblk) return;

    const int tensor = find_tensor(tb.unit_prefix, tb.nt, unit);
    const TensorRec r = rec_of(tb, tensor);
    if (r.fast) return;               // evaluated by k_fast
    int first = r.tile_base + (unit - r.unit_base) * r.tpu;
    int last = first + r.tpu;
    if (last > r.tile_base + r.ntiles) last = r.tile_base + r.ntiles;
    if (r.tpg > 1) {        // one tile per unit; full tiles first (see slot_to_tile)
        first = slot_to_tile(r, first);
        last = first + 1;
    }

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

    // Tiles of at most kTinyTile elements (depthwise 3x3 filters: 9) are two vectors.  A
    // wavefront would spend its time waiting for the bucket offsets and then for the
    // elements of tile after tile; instead every element is evaluated in the per-lane
    // form (no offsets: the order inside the tile does not matter, the zero padding adds
    // nothing), and the next tile's vectors are loaded while this one is evaluated.
    if (r.tile_len <= kTinyTile && r.tpg == 1) {
        const bool two = r.tile_len > kVec;                 // the second vector holds elements
        const float *us = sorted + (r.sorted_base + (long long)(first - r.tile_base) * r.stride);
        float8 c0 = load8(us), c1 = load8(us + kVec);       // the spare vector of a tile, if not its second
        for (int t = first; t < last; ++t) {
            // the tile after the tensor's last one does not exist: read this one again
            const float *nx = (t + 1 < last) ? us + r.stride : us;
            const float8 n0 = load8(nx), n1 = load8(nx + kVec);
            float acc0 = 0.0f, acc1 = 0.0f;
            mixed8(c0, kf, rc, rt, ct, stepc, stept, acc0);
            if (two) mixed8(c1, kf, rc, rt, ct, stepc, stept, acc1);
            if (live) sse32[(long long)t * n + (k - 1)] = acc0 + acc1;
            c0 = n0;
            c1 = n1;
            us = nx;
        }
        return;
    }

    for (int t = first; t < last; ++t) {
        const int local = t - r.tile_base;
        const int tig = local % r.tpg;
        const int len = (tig == r.tpg - 1) ? r.last_len : r.tile_len;
        const int padded = (len + kVec - 1) / kVec * kVec;
        const float *us = sorted + (r.sorted_base + (long long)local * r.stride);
        const int *off = offsets + (long long)t * (nblk + 1);
        const int lo = off[j] & ~(kVec - 1);
        const int hi = (off[j + 1] + kVec - 1) & ~(kVec - 1);
        float sc = zone_one_region<false>(us, 0, lo, rc, 0.0f);
        float st = zone_one_region<true>(us, hi, padded, rt, ct);
        float sm = 0.0f;
        // tiles before fine_tiles are ordered by candidate; that evaluation pays from
        // about 64 elements in the bucket
        if (t < fine_tiles && hi - lo >= kFineMin) zone_mixed_fine(us, lo, hi, fine[(long long)t * (n + 1) + k], kf, rc, rt, ct, sc, st);
        else sm = zone_mixed(us, lo, hi, kf, rc, rt, ct, stepc, stept);
        if (live)
            sse32[(long long)t * n + (k - 1)] = (stepc * stepc) * sc + (stept * stept) * st + sm;
    }
}

} // namespace pwlq
