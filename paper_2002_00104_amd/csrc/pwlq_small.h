// k_small: the whole search of a group inside one workgroup, for calls that are
// too small to fill the chip.
//
// A call with a few hundred short groups (one conv layer) is bound by the
// latency of its launches, not by arithmetic: partition, evaluation and exact
// stage as three dependent launches leave most of the chip idle three times.
// Here one workgroup of 16 wavefronts takes one group of at most 1024 elements
// and does everything: the weights are loaded once (one per thread), the absmax
// is reduced in LDS, the magnitudes are rescaled to candidate units and staged
// in LDS, the wavefronts take the candidate blocks (lane = candidate) and read
// the elements as LDS broadcasts, the filter sums meet in LDS, and the same
// workgroup selects the candidates within the slack of the minimum and
// re-evaluates them exactly (exact_tile, as k_exact does).  Nothing goes
// through the workspace.  Without the partition every element is evaluated in
// the per-lane form (both positions, select): 20 cycles per evaluation instead
// of 8, which does not matter where the launch latency is the cost.  With fewer
// than 16 candidate blocks the spare wavefronts split the elements of a block
// into slices whose partial sums are added in a fixed order.
#pragma once

#include "pwlq_prep.h"
#include "pwlq_refine.h"
#include "pwlq_search.h"
#include "pwlq_tables.h"

namespace pwlq {

constexpr int kSmallWG = 1024;                 // threads: one element each, 16 wavefronts
constexpr int kSmallWaves = kSmallWG / 64;
constexpr int kSmallLen = kSmallWG;            // longest group
constexpr int kSmallCand = kSmallWaves * kBlk; // most candidates: one block per wavefront

__global__ __launch_bounds__(kSmallWG) void k_small(Tables tb, int n, int nblk, int bits,
                                                    float *__restrict__ p_star,
                                                    float *__restrict__ m_out,
                                                    int32_t *__restrict__ k_star,
                                                    double *__restrict__ mse)
{
    __shared__ __attribute__((aligned(16))) float units[kSmallLen + kVec];
    __shared__ float part[kSmallWaves][kBlk];   // partial filter sums: [slice * blocks + block][lane]
    __shared__ float filt[kSmallCand];          // filter sum of every candidate
    __shared__ float redm[kSmallWaves];
    __shared__ int redbad[kSmallWaves];
    __shared__ int llist[kSmallCand];
    __shared__ int lcount;
    __shared__ double lds[kSmallWaves * 2];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = uni(tid >> 6);
    int t;
    TensorRec r;
    const TileInfo ti = tile_of(tb, blockIdx.x, r, t);      // one tile per group here
    const int len = ti.len;
    const long long og = r.out_group + ti.group_local;

    // ---- the group's elements, its absmax, candidate units
    float a[1];
    a[0] = (tid < len) ? fabsf(ti.src[tid]) : 0.0f;
    float m = wave_max(a[0]);
    int bad = wave_or(a[0] != a[0]);
    if (lane == 0) { redm[wave] = m; redbad[wave] = bad; }
    if (tid == 0) lcount = 0;
    __syncthreads();
    m = redm[0];
    bad = redbad[0];
    for (int i = 1; i < kSmallWaves; ++i) { m = fmaxf(m, redm[i]); bad |= redbad[i]; }
    if (bad) m = __builtin_nanf("");
    const bool usable = (m > 0.0f) && (m < __builtin_inff());
    const float nf = (float)n;
    const float scale = usable ? nf / m : 0.0f;
    const int padded = (len + kVec - 1) / kVec * kVec;
    units[tid] = (usable && tid < len) ? to_units(a[0], scale, nf) : 0.0f;
    if (tid < kVec) units[kSmallLen + tid] = 0.0f;
    __syncthreads();

    // ---- filter sums: wavefront = (slice of the elements, block of 64 candidates)
    int blocks_log2 = 0;                         // candidate blocks rounded up to a power of two
    while ((1 << blocks_log2) < nblk) ++blocks_log2;
    const int slices = kSmallWaves >> blocks_log2;
    const int j = wave & ((1 << blocks_log2) - 1);
    const int slice = wave >> blocks_log2;
    if (j < nblk && usable) {
        int k = j * kBlk + lane + 1;
        if (k > n) k = n;
        const float Lf = (float)((1 << (bits - 1)) - 1);
        const float kf = (float)k;
        const float nk = (float)(n - k);
        const float rc = Lf / kf;
        const float rt = (k < n) ? Lf / nk : 0.0f;
        const float ct = -kf * rt;
        const float stepc = kf / Lf;
        const float stept = nk / Lf;
        const int per = ((padded + slices - 1) / slices + kVec - 1) / kVec * kVec;   // elements per slice
        const int begin = slice * per;
        const int end = (begin + per < padded) ? begin + per : padded;
        float outer = 0.0f;
        for (int cb = begin; cb < end; cb += kChunk) {
            const int ce = (cb + kChunk < end) ? cb + kChunk : end;
            float acc = 0.0f;
            for (int i = cb; i < ce; i += kVec) {
                // every lane reads the same two 16-byte words: an LDS broadcast
                const float4 x0 = *reinterpret_cast<const float4 *>(units + i);
                const float4 x1 = *reinterpret_cast<const float4 *>(units + i + 4);
                float8 cur;
                cur[0] = x0.x; cur[1] = x0.y; cur[2] = x0.z; cur[3] = x0.w;
                cur[4] = x1.x; cur[5] = x1.y; cur[6] = x1.z; cur[7] = x1.w;
                mixed8(cur, kf, rc, rt, ct, stepc, stept, acc);
            }
            outer += acc;
        }
        part[wave][lane] = outer;
    }
    __syncthreads();
    if (tid < nblk * kBlk) {                     // slices added in slice order
        float s = 0.0f;
        if (usable)
            for (int x = 0; x < slices; ++x) s += part[(x << blocks_log2) + (tid >> 6)][tid & 63];
        filt[tid] = s;
    }
    __syncthreads();

    // ---- candidates within the slack of the minimum, exact stage, result
    ExactState st;
    st.best = 0.0;
    st.best_k = -1;
    if (m == 0.0f) {
        if (tid == 0) llist[0] = 1;
        __syncthreads();
        exact_tile<1, kSmallWG>(ti.src, len, a, m, n, bits, llist, 1, true, nullptr, lds, st);
    } else if (usable) {
        const float mine = (tid < n) ? filt[tid] : __builtin_inff();     // n <= 1024: one per thread
        const double mn = block_min<kSmallWaves>((double)mine, lds);
        const double thr = keep_threshold(mn, (double)r.gcount, n, false);
        float thrf = (float)thr;
        if ((double)thrf > thr) thrf = __int_as_float(__float_as_int(thrf) - 1);
        if (mine <= thrf) llist[atomicAdd(&lcount, 1)] = tid + 1;
        __syncthreads();
        const int count = uni(lcount);
        exact_tile<1, kSmallWG>(ti.src, len, a, m, n, bits, llist, count, true, nullptr, lds, st);
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

} // namespace pwlq
