// k_linear: inner products of 8-bit activations with bit-packed PWLQ weights on
// the integer matrix cores (Section 4).  k_linear_wsum: the per-channel constants.
//
// For output channel n with steps s1 = p/L, s2 = (m-p)/L and activations
// X_hat = s_x X_q + z_x, Section 4 splits the inner product by region:
//   P1 = C2 <X_q, W_q1>_R1 + C3,   P2 = C4 <X_q, W_q2>_R2 + C5 <X_q, sigma>_R2 + C6,
// three integer accumulators per output (sigma: the sign of a tail weight, which
// the offset p carries).  On the matrix cores these are three int8 products of the
// same activation tile with three operand planes decoded from the packed codes:
//   plane 0: signed code where the region bit is 0, else 0
//   plane 1: signed code where the region bit is 1, else 0
//   plane 2: sign (+1 / -1) where the region bit is 1, else 0
// The planes exist only in LDS; memory holds b + 1 bits per weight.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pwlq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kLinBM = 128;       // activation rows per workgroup
constexpr int kLinBN = 64;        // output channels per workgroup
constexpr int kLinBK = 64;        // reduction elements per step
constexpr int kLinStride = 80;    // bytes per LDS row: 64 + 16 keeps 16-byte reads off the same banks
constexpr int kLinWG = 256;       // 4 wavefronts, 2 (rows) x 2 (channels), each 64 x 32 outputs

// 16 consecutive b-bit codes of a stream (sign-magnitude: bit b-1 is the sign)
// starting at element index e0 (a multiple of 16), returned as 16 bytes, one
// code per byte, in order.  The 2b bytes start 2-byte aligned.
__device__ inline void load_codes16(const uint8_t *__restrict__ stream, long long e0, int bits,
                                    uint32_t (&out)[4])
{
    const uint8_t *src = stream + (e0 >> 4) * (2 * bits);
    if (bits == 4) {
        const uint2 v = *reinterpret_cast<const uint2 *>(src);      // 8-byte aligned
        const uint32_t w[2] = {v.x, v.y};
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t ev = w[h] & 0x0f0f0f0fu;          // elements 0,2,4,6 of this half
            const uint32_t od = (w[h] >> 4) & 0x0f0f0f0fu;   // elements 1,3,5,7
            // interleave bytes: (e0,o0,e1,o1) and (e2,o2,e3,o3)
            out[2 * h] = __builtin_amdgcn_perm(od, ev, 0x05010400u);
            out[2 * h + 1] = __builtin_amdgcn_perm(od, ev, 0x07030602u);
        }
        return;
    }
    if (bits == 8) {
        const uint4 v = *reinterpret_cast<const uint4 *>(src);      // 16-byte aligned
        out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
        return;
    }
    // any other width: gather the 2b bytes into a 128-bit window, then shift
    unsigned long long lo = 0, hi = 0;
    const uint16_t *s16 = reinterpret_cast<const uint16_t *>(src);
    for (int i = 0; i < bits; ++i) {
        const unsigned long long h = s16[i];
        if (i < 4) lo |= h << (16 * i);
        else hi |= h << (16 * (i - 4));
    }
    const uint32_t mask = (1u << bits) - 1u;
#pragma unroll
    for (int wd = 0; wd < 4; ++wd) {
        uint32_t word = 0;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int pos = (wd * 4 + x) * bits;
            unsigned long long v;
            if (pos >= 64) v = hi >> (pos - 64);
            else if (pos == 0) v = lo;
            else v = (lo >> pos) | (hi << (64 - pos));
            word |= ((uint32_t)v & mask) << (8 * x);
        }
        out[wd] = word;
    }
}

// Four sign-magnitude codes (one per byte) and their four region bits (low
// nibble of f) -> the three operand planes, four int8 each.
__device__ inline void planes4(uint32_t codes, uint32_t f, int bits, uint32_t &w1, uint32_t &w2,
                               uint32_t &w3)
{
    const uint32_t magmask = ((1u << (bits - 1)) - 1u) * 0x01010101u;
    const uint32_t mag = codes & magmask;
    const uint32_t sgn = (codes >> (bits - 1)) & 0x01010101u;
    const uint32_t smask = sgn * 0xffu;                                 // 0xff in bytes of negative codes
    const uint32_t neg = (0x80808080u - mag) ^ 0x80808080u;            // -mag per byte (mag <= 127)
    const uint32_t val = (neg & smask) | (mag & ~smask);
    const uint32_t fm = (((f & 0xfu) * 0x00204081u) & 0x01010101u) * 0xffu;   // 0xff in tail bytes
    w1 = val & ~fm;
    w2 = val & fm;
    w3 = (smask | 0x01010101u) & fm;
}

// ---------------------------------------------------------------- constants
// wconst[n] = s1 * sum_R1 w_q + s2 * sum_R2 w_q + p * sum_R2 sigma (binary64,
// rounded to binary32): multiplied by z_x it is C3 + C6 of Section 4.  One
// wavefront per channel.
__device__ inline int sum_bytes(uint32_t w)
{
    return (int)(int8_t)(w & 0xff) + (int)(int8_t)((w >> 8) & 0xff) +
           (int)(int8_t)((w >> 16) & 0xff) + (int)(int8_t)(w >> 24);
}

__global__ __launch_bounds__(kLinWG) void k_linear_wsum(const uint8_t *__restrict__ pcodes,
                                                        const uint8_t *__restrict__ pflags,
                                                        long long N, long long K, int bits,
                                                        const float *__restrict__ p,
                                                        const float *__restrict__ m,
                                                        float *__restrict__ wconst)
{
    const long long n = (long long)blockIdx.x * (kLinWG / 64) + (threadIdx.x >> 6);
    if (n >= N) return;
    const int lane = threadIdx.x & 63;
    int b1 = 0, b2 = 0, b3 = 0;
    for (long long k0 = 16LL * lane; k0 < K; k0 += 16 * 64) {
        const long long e0 = n * K + k0;
        uint32_t c[4];
        load_codes16(pcodes, e0, bits, c);
        const uint32_t f = *reinterpret_cast<const uint16_t *>(pflags + (e0 >> 3));
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            uint32_t w1, w2, w3;
            planes4(c[x], f >> (4 * x), bits, w1, w2, w3);
            b1 += sum_bytes(w1);
            b2 += sum_bytes(w2);
            b3 += sum_bytes(w3);
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        b1 += __shfl_xor(b1, off, 64);
        b2 += __shfl_xor(b2, off, 64);
        b3 += __shfl_xor(b3, off, 64);
    }
    if (lane == 0) {
        const float Lf = (float)((1 << (bits - 1)) - 1);
        const float pn = p[n], mn = m[n];
        const float s1 = pn / Lf;
        const float width = mn - pn;
        const float s2 = width / Lf;
        wconst[n] = (float)((double)s1 * (double)b1 + (double)s2 * (double)b2 + (double)pn * (double)b3);
    }
}

// -------------------------------------------------------------------- linear
struct LinStage {
    v4i a0, a1;            // 32 activation bytes of one row
    uint32_t codes[4];     // 16 weight codes, one per byte
    uint32_t flags;        // their 16 region bits
};

__device__ inline void lin_load(LinStage &st, const int8_t *__restrict__ xq, long long M,
                                long long K, const uint8_t *__restrict__ pcodes,
                                const uint8_t *__restrict__ pflags, long long N, int bits,
                                long long row0, long long col0, long long k0)
{
    const int t = threadIdx.x;
    const long long r = row0 + (t >> 1);
    if (r < M) {
        const v4i *src = reinterpret_cast<const v4i *>(xq + r * K + k0 + (t & 1) * 32);
        st.a0 = src[0];
        st.a1 = src[1];
    } else {
        st.a0 = v4i{0, 0, 0, 0};
        st.a1 = v4i{0, 0, 0, 0};
    }
    const long long n = col0 + (t >> 2);
    if (n < N) {
        const long long e0 = n * K + k0 + (t & 3) * 16;
        load_codes16(pcodes, e0, bits, st.codes);
        st.flags = *reinterpret_cast<const uint16_t *>(pflags + (e0 >> 3));
    } else {
        st.codes[0] = st.codes[1] = st.codes[2] = st.codes[3] = 0;
        st.flags = 0;
    }
}

__device__ inline void lin_store(const LinStage &st, int bits, int8_t *__restrict__ sA,
                                 int8_t *__restrict__ sB)
{
    const int t = threadIdx.x;
    v4i *da = reinterpret_cast<v4i *>(sA + (t >> 1) * kLinStride + (t & 1) * 32);
    da[0] = st.a0;
    da[1] = st.a1;
    v4i w1, w2, w3;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        uint32_t a, b, c;
        planes4(st.codes[x], st.flags >> (4 * x), bits, a, b, c);
        w1[x] = (int)a;
        w2[x] = (int)b;
        w3[x] = (int)c;
    }
    const int off = (t >> 2) * kLinStride + (t & 3) * 16;
    *reinterpret_cast<v4i *>(sB + off) = w1;
    *reinterpret_cast<v4i *>(sB + kLinBN * kLinStride + off) = w2;
    *reinterpret_cast<v4i *>(sB + 2 * kLinBN * kLinStride + off) = w3;
}

// Workgroup ids are dealt round-robin to the 8 XCDs.  Each XCD takes a
// contiguous eighth of the channel tiles and walks all row tiles of one channel
// tile before the next, so the packed weights of its channels stay in its L2
// while the activations stream through.
__global__ __launch_bounds__(kLinWG) void k_linear(const int8_t *__restrict__ xq, long long M,
                                                   long long K, float s_x, float z_x,
                                                   const uint8_t *__restrict__ pcodes,
                                                   const uint8_t *__restrict__ pflags,
                                                   long long N, int bits,
                                                   const float *__restrict__ p,
                                                   const float *__restrict__ m,
                                                   const float *__restrict__ wconst,
                                                   float *__restrict__ y, int *__restrict__ acc_out,
                                                   int tiles_m, int tiles_n, int tn_per_xcd)
{
    __shared__ __attribute__((aligned(16))) int8_t sA[2][kLinBM * kLinStride];
    __shared__ __attribute__((aligned(16))) int8_t sB[2][3 * kLinBN * kLinStride];

    const int xcd = blockIdx.x & 7;
    const int slot = blockIdx.x >> 3;
    const int bn = xcd * tn_per_xcd + slot / tiles_m;
    const int bm = slot % tiles_m;
    if (slot / tiles_m >= tn_per_xcd || bn >= tiles_n) return;
    const long long row0 = (long long)bm * kLinBM, col0 = (long long)bn * kLinBN;

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    v16i acc[2][3];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 3; ++b)
#pragma unroll
            for (int c = 0; c < 16; ++c) acc[a][b][c] = 0;

    LinStage st;
    lin_load(st, xq, M, K, pcodes, pflags, N, bits, row0, col0, 0);
    lin_store(st, bits, sA[0], sB[0]);
    __syncthreads();
    const int steps = (int)(K / kLinBK);
    for (int kt = 0; kt < steps; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < steps)
            lin_load(st, xq, M, K, pcodes, pflags, N, bits, row0, col0, (long long)(kt + 1) * kLinBK);
        const int8_t *a_base = sA[buf] + (wm * 64 + (lane & 31)) * kLinStride + 16 * (lane >> 5);
        const int8_t *b_base = sB[buf] + (wn * 32 + (lane & 31)) * kLinStride + 16 * (lane >> 5);
#pragma unroll
        for (int ks = 0; ks < kLinBK / 32; ++ks) {
            v4i bf[3];
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
                bf[pl] = *reinterpret_cast<const v4i *>(b_base + pl * kLinBN * kLinStride + ks * 32);
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const v4i af =
                    *reinterpret_cast<const v4i *>(a_base + mt * 32 * kLinStride + ks * 32);
#pragma unroll
                for (int pl = 0; pl < 3; ++pl)
                    acc[mt][pl] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af, bf[pl], acc[mt][pl], 0, 0, 0);
            }
        }
        if (kt + 1 < steps) lin_store(st, bits, sA[buf ^ 1], sB[buf ^ 1]);
        __syncthreads();
    }

    // epilogue: C2 A1 + C4 A2 + C5 A3 + (C3 + C6), per output channel
    const long long n = col0 + wn * 32 + (lane & 31);
    if (n >= N) return;
    const float Lf = (float)((1 << (bits - 1)) - 1);
    const float pn = p[n], mn = m[n];
    const float s1 = pn / Lf;
    const float width = mn - pn;
    const float s2 = width / Lf;
    const float cst = z_x * wconst[n];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const long long row = row0 + wm * 64 + mt * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
            if (row < M) {
                const int a1 = acc[mt][0][r], a2 = acc[mt][1][r], a3 = acc[mt][2][r];
                float t = s1 * (float)a1;
                t = __builtin_fmaf(s2, (float)a2, t);
                t = __builtin_fmaf(pn, (float)a3, t);
                y[row * N + n] = __builtin_fmaf(s_x, t, cst);
                if (acc_out) {
                    acc_out[(0 * M + row) * N + n] = a1;
                    acc_out[(1 * M + row) * N + n] = a2;
                    acc_out[(2 * M + row) * N + n] = a3;
                }
            }
        }
    }
}

} // namespace pwlq
