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
//
// A caller that wants y alone does not need the second and third sum apart:
// C5 = C2 L (the offset p is L steps of the centre), so
//   C2 A1 + C5 A3 = C2 (A1 + L A3),
// and L sigma fits an int8 like any code.  The folded form keeps two planes,
//   plane 0: signed code where the region bit is 0, else L sigma
//   plane 1: signed code where the region bit is 1, else 0
// two matrix products per weight instead of three, with the same bound on the
// integer sums (|entry| <= L in both planes).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pwlq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kLinWM = 2;          // wavefronts along the rows; 2 along the channels
constexpr int kLinBN = 64;        // output channels per workgroup
constexpr int kLinBK = 64;        // reduction elements per step
constexpr int kLinStride = 64;    // bytes per LDS row; the four 16-byte chunks of a row are swizzled
constexpr int kLinWG = 128 * kLinWM;   // wavefronts kLinWM (rows) x 2 (channels), each 32*kMT x 32 outputs

// kMT: 32-row tiles per wavefront.  The accumulators of a wavefront are
// kMT * planes * 16 registers: 3 tiles with three planes (1, 2, 4 measured
// slower), 4 tiles with two.
constexpr int lin_mt(int planes) { return planes == 3 ? 3 : 4; }
constexpr int lin_bm(int planes) { return kLinWM * 32 * lin_mt(planes); }   // activation rows per workgroup
constexpr int lin_avec(int planes) { return lin_bm(planes) * kLinBK / 16 / kLinWG; }   // 16-byte activation loads per thread

// LDS rows hold 64 reduction bytes as four 16-byte chunks; chunk c of row r is
// stored at position c ^ swz(r), swz(r) = (r >> 3) & 3.  A 16-byte LDS read of a
// wavefront is served 16 lanes per cycle over 64 banks, and the lanes of a cycle
// are not consecutive: measured on this chip, lanes 0-3, 12-15, 20-23 and 24-27
// go together (of the eight groups of four lanes in each half of the wavefront,
// those whose index has even parity, then those with odd parity).  The fragment
// reads of the matrix cores (lane = row, same chunk) therefore need the four
// groups {0, 3, 5, 6} and {1, 2, 4, 7} of four rows on different chunk
// positions, which r >> 3 gives; a swizzle that spreads consecutive rows
// instead costs 6.9 cycles per read against 3.6.  The 16-byte writes of the
// staging threads (four lanes = the four chunks of one row) are indifferent to it.
__device__ inline int lin_swz(int row) { return (row >> 3) & 3; }

// 16 consecutive b-bit codes of a stream (sign-magnitude: bit b-1 is the sign)
// starting at element index e0 (a multiple of 16) occupy 2b bytes that start
// 2-byte aligned (4-byte aligned for even b, 8 for b = 4, 16 for b = 8).
// load_raw16 only issues the loads; unpack16 turns the raw bytes into 16 bytes,
// one code per byte, in order.  Keeping the two apart lets the loads of a later
// step fly while the matrix cores work on the current one.
template <int kBits>
struct RawCodes {
    uint32_t w[(2 * kBits + 3) / 4];
};

template <int kBits>
__device__ inline void load_raw16(const uint8_t *__restrict__ stream, long long e0,
                                  RawCodes<kBits> &raw)
{
    const uint8_t *src = stream + (e0 >> 4) * (2 * kBits);
    if (kBits == 4) {
        const uint2 v = *reinterpret_cast<const uint2 *>(src);
        raw.w[0] = v.x;
        raw.w[1] = v.y;
    } else if (kBits == 8) {
        const uint4 v = *reinterpret_cast<const uint4 *>(src);
        raw.w[0] = v.x; raw.w[1] = v.y; raw.w[2] = v.z; raw.w[3] = v.w;
    } else if (kBits % 2 == 0) {
#pragma unroll
        for (int i = 0; i < kBits / 2; ++i) raw.w[i] = reinterpret_cast<const uint32_t *>(src)[i];
    } else {
        const uint16_t *s16 = reinterpret_cast<const uint16_t *>(src);
#pragma unroll
        for (int i = 0; i < (2 * kBits + 3) / 4; ++i) raw.w[i] = 0;
#pragma unroll
        for (int i = 0; i < kBits; ++i) raw.w[i / 2] |= (uint32_t)s16[i] << (16 * (i & 1));
    }
}

template <int kBits>
__device__ inline void zero_raw16(RawCodes<kBits> &raw)
{
#pragma unroll
    for (int i = 0; i < (2 * kBits + 3) / 4; ++i) raw.w[i] = 0;
}

template <int kBits>
__device__ inline void unpack16(const RawCodes<kBits> &raw, uint32_t (&out)[4])
{
    if (kBits == 4) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t ev = raw.w[h] & 0x0f0f0f0fu;          // elements 0,2,4,6 of this half
            const uint32_t od = (raw.w[h] >> 4) & 0x0f0f0f0fu;   // elements 1,3,5,7
            // interleave bytes: (e0,o0,e1,o1) and (e2,o2,e3,o3)
            out[2 * h] = __builtin_amdgcn_perm(od, ev, 0x05010400u);
            out[2 * h + 1] = __builtin_amdgcn_perm(od, ev, 0x07030602u);
        }
    } else if (kBits == 8) {
#pragma unroll
        for (int i = 0; i < 4; ++i) out[i] = raw.w[i];
    } else {
        constexpr uint32_t mask = (1u << kBits) - 1u;
#pragma unroll
        for (int wd = 0; wd < 4; ++wd) {
            uint32_t word = 0;
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int pos = (wd * 4 + x) * kBits;       // compile-time after unrolling
                const int wi = pos >> 5, sh = pos & 31;
                uint32_t v = raw.w[wi] >> sh;
                if (sh + kBits > 32) v |= raw.w[wi + 1] << (32 - sh);
                word |= (v & mask) << (8 * x);
            }
            out[wd] = word;
        }
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
    // 0xff in the bytes that hold 1 (written so that it stays two full-rate
    // instructions: x * 0xff would be a quarter-rate 32-bit multiply)
    const uint32_t smask = (0x80808080u - sgn) ^ 0x80808080u;          // negative codes
    const uint32_t neg = (0x80808080u - mag) ^ 0x80808080u;            // -mag per byte (mag <= 127)
    const uint32_t val = (neg & smask) | (mag & ~smask);
    const uint32_t f01 = __umul24(f & 0xfu, 0x00204081u) & 0x01010101u;   // region bit of each byte (24-bit multiply: full rate)
    const uint32_t fm = (0x80808080u - f01) ^ 0x80808080u;             // tail bytes
    w1 = val & ~fm;
    w2 = val & fm;
    w3 = (smask | 0x01010101u) & fm;
}

// The folded form: plane 0 holds L sigma in the tail bytes, plane 1 as above.
__device__ inline void planes4_folded(uint32_t codes, uint32_t f, int bits, uint32_t &w1, uint32_t &w2)
{
    const uint32_t magmask = ((1u << (bits - 1)) - 1u) * 0x01010101u;      // L in every byte
    const uint32_t mag = codes & magmask;
    const uint32_t sgn = (codes >> (bits - 1)) & 0x01010101u;
    const uint32_t smask = (0x80808080u - sgn) ^ 0x80808080u;
    const uint32_t f01 = __umul24(f & 0xfu, 0x00204081u) & 0x01010101u;
    const uint32_t fm = (0x80808080u - f01) ^ 0x80808080u;
    const uint32_t neg = (0x80808080u - mag) ^ 0x80808080u;
    const uint32_t val = (neg & smask) | (mag & ~smask);                   // signed code
    const uint32_t negl = (0x80808080u - magmask) ^ 0x80808080u;           // -L in every byte
    const uint32_t lsig = (negl & smask) | (magmask & ~smask);             // L sigma
    w1 = (lsig & fm) | (val & ~fm);
    w2 = val & fm;
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

template <int kBits>
__global__ __launch_bounds__(kLinWG) void k_linear_wsum(const uint8_t *__restrict__ pcodes,
                                                        const uint8_t *__restrict__ pflags,
                                                        long long N, long long K,
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
        RawCodes<kBits> raw;
        uint32_t c[4];
        load_raw16<kBits>(pcodes, e0, raw);
        unpack16<kBits>(raw, c);
        const uint32_t f = *reinterpret_cast<const uint16_t *>(pflags + (e0 >> 3));
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            uint32_t w1, w2, w3;
            planes4(c[x], f >> (4 * x), kBits, w1, w2, w3);
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
        const float Lf = (float)((1 << (kBits - 1)) - 1);
        const float pn = p[n], mn = m[n];
        const float s1 = pn / Lf;
        const float width = mn - pn;
        const float s2 = width / Lf;
        wconst[n] = (float)((double)s1 * (double)b1 + (double)s2 * (double)b2 + (double)pn * (double)b3);
    }
}

// -------------------------------------------------------------------- linear
template <int kBits, int kAVec>
struct LinStage {
    v4i a[kAVec];       // activation bytes: vector v of thread t is piece t + v*kLinWG of the tile
    RawCodes<kBits> codes; // 16 packed weight codes
    uint32_t flags;        // their 16 region bits
};

// Issues the loads of one reduction step and nothing else.  Rows past M and
// channels past N read the last valid row / channel instead (their products are
// never written), so no load sits under a branch and the compiler can count the
// outstanding loads exactly.
// kvalid: how many of the step's four 16-element pieces lie below K (4 except in
// the last step when K is not a multiple of 64); the others read the step's first
// piece instead and are zeroed when the step is written to LDS.
template <int kBits, int kAVec>
__device__ inline void lin_load(LinStage<kBits, kAVec> &st, const int8_t *__restrict__ xq, long long M,
                                long long K, const uint8_t *__restrict__ pcodes,
                                const uint8_t *__restrict__ pflags, long long N, long long row0,
                                long long col0, long long k0, int kvalid)
{
    static_assert(kLinWG == 4 * kLinBN, "every thread carries 16 weights of the tile");
    const int t = threadIdx.x;
    const int c = ((t & 3) < kvalid) ? (t & 3) : 0;     // piece & 3 == t & 3: kLinWG is a multiple of 4
#pragma unroll
    for (int v = 0; v < kAVec; ++v) {
        const int piece = t + v * kLinWG;              // 4 pieces of 16 bytes per row
        long long r = row0 + (piece >> 2);
        r = r < M ? r : M - 1;
        st.a[v] = *reinterpret_cast<const v4i *>(xq + r * K + k0 + c * 16);
    }
    long long n = col0 + (t >> 2);
    n = n < N ? n : N - 1;
    const long long e0 = n * K + k0 + c * 16;
    load_raw16<kBits>(pcodes, e0, st.codes);
    st.flags = *reinterpret_cast<const uint16_t *>(pflags + (e0 >> 3));
}

// The same loads for a step that lies wholly below K, from addresses split into
// a base that is the same in every lane and changes from step to step (scalar
// arithmetic) and a 32-bit offset per thread that never changes (computed once,
// before the loop): no vector address arithmetic per step.
template <int kBits, int kAVec>
struct LinOffsets {
    unsigned a[kAVec];      // from xq + row0*K + k0
    unsigned codes, flags;     // from the streams at element col0*K + k0
};

template <int kBits, int kAVec>
__device__ inline LinOffsets<kBits, kAVec> lin_offsets(long long M, long long K, long long N,
                                                long long row0, long long col0)
{
    LinOffsets<kBits, kAVec> o;
    const int t = threadIdx.x;
#pragma unroll
    for (int v = 0; v < kAVec; ++v) {
        const int piece = t + v * kLinWG;
        long long r = row0 + (piece >> 2);
        r = r < M ? r : M - 1;
        o.a[v] = (unsigned)((r - row0) * K) + (unsigned)((t & 3) * 16);     // < 256 * 2^22 + 64
    }
    long long n = col0 + (t >> 2);
    n = n < N ? n : N - 1;
    const unsigned piece16 = (unsigned)((n - col0) * (K >> 4)) + (unsigned)(t & 3);   // in runs of 16 elements
    o.codes = piece16 * (2 * kBits);
    o.flags = piece16 * 2;
    return o;
}

template <int kBits, int kAVec>
__device__ inline void lin_load_whole(LinStage<kBits, kAVec> &st, const LinOffsets<kBits, kAVec> &o,
                                      const int8_t *__restrict__ a_base,
                                      const uint8_t *__restrict__ code_base,
                                      const uint8_t *__restrict__ flag_base)
{
#pragma unroll
    for (int v = 0; v < kAVec; ++v)
        st.a[v] = *reinterpret_cast<const v4i *>(a_base + o.a[v]);
    load_raw16<kBits>(code_base + o.codes, 0, st.codes);
    st.flags = *reinterpret_cast<const uint16_t *>(flag_base + o.flags);
}

// Writes one step into LDS: activations as they are, weights decoded into the
// operand planes (three, or two in the folded form).
template <int kBits, int kPlanes>
__device__ inline void lin_store(const LinStage<kBits, lin_avec(kPlanes)> &st, int8_t *__restrict__ sA,
                                 int8_t *__restrict__ sB, int kvalid)
{
    const int t = threadIdx.x;
    const int keep = ((t & 3) < kvalid) ? -1 : 0;       // all ones for a piece below K
#pragma unroll
    for (int v = 0; v < lin_avec(kPlanes); ++v) {
        const int piece = t + v * kLinWG;
        v4i a = st.a[v];
        a[0] &= keep; a[1] &= keep; a[2] &= keep; a[3] &= keep;
        *reinterpret_cast<v4i *>(sA + (piece >> 2) * kLinStride +
                                 (((piece & 3) ^ lin_swz(piece >> 2)) * 16)) = a;
    }
    uint32_t c[4];
    unpack16<kBits>(st.codes, c);
    v4i w1, w2, w3;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        uint32_t a, b, d = 0;
        if (kPlanes == 3)
            planes4(c[x], st.flags >> (4 * x), kBits, a, b, d);
        else
            planes4_folded(c[x], st.flags >> (4 * x), kBits, a, b);
        w1[x] = (int)a & keep;
        w2[x] = (int)b & keep;
        w3[x] = (int)d & keep;
    }
    const int off = (t >> 2) * kLinStride + (((t & 3) ^ lin_swz(t >> 2)) * 16);
    *reinterpret_cast<v4i *>(sB + off) = w1;
    *reinterpret_cast<v4i *>(sB + kLinBN * kLinStride + off) = w2;
    if (kPlanes == 3) *reinterpret_cast<v4i *>(sB + 2 * kLinBN * kLinStride + off) = w3;
}

// One reduction step of a wavefront: fragments of LDS buffer `buf`, the next
// step decoded into the other buffer (kStore), 2 * kMT * kPlanes matrix
// instructions, one barrier.
template <int kBits, int kPlanes, bool kStore>
__device__ inline void lin_step(v16i (&acc)[lin_mt(kPlanes)][kPlanes],
                                const LinStage<kBits, lin_avec(kPlanes)> &next, int kvalid_next,
                                const int8_t *a_lane, const int8_t *b_lane, int swz, int half,
                                int8_t *sA0, int8_t *sB0, int buf)
{
    constexpr int kMT = lin_mt(kPlanes);
    constexpr int kABuf = lin_bm(kPlanes) * kLinStride, kBBuf = kPlanes * kLinBN * kLinStride;
    const int8_t *a_base = a_lane + buf * kABuf;
    const int8_t *b_base = b_lane + buf * kBBuf;
    v4i bf[kLinBK / 32][kPlanes], af[kLinBK / 32][kMT];
#pragma unroll
    for (int ks = 0; ks < kLinBK / 32; ++ks) {
        const int chunk = ((2 * ks + half) ^ swz) * 16;
#pragma unroll
        for (int pl = 0; pl < kPlanes; ++pl)
            bf[ks][pl] = *reinterpret_cast<const v4i *>(b_base + pl * kLinBN * kLinStride + chunk);
#pragma unroll
        for (int mt = 0; mt < kMT; ++mt)
            af[ks][mt] = *reinterpret_cast<const v4i *>(a_base + mt * 32 * kLinStride + chunk);
    }
    if (kStore)
        lin_store<kBits, kPlanes>(next, sA0 + (buf ^ 1) * kABuf, sB0 + (buf ^ 1) * kBBuf, kvalid_next);
#pragma unroll
    for (int ks = 0; ks < kLinBK / 32; ++ks)
#pragma unroll
        for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
            for (int pl = 0; pl < kPlanes; ++pl)
                acc[mt][pl] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[ks][mt], bf[ks][pl],
                                                                    acc[mt][pl], 0, 0, 0);
    __syncthreads();
}

// Workgroup ids are dealt round-robin to the 8 XCDs.  Each XCD takes a
// contiguous eighth of the channel tiles (their packed weights, about 1 MB,
// stay in its L2) and walks them for one row tile before the next row tile, so
// that the workgroups in flight on an XCD share a few activation tiles: every
// XCD then reads the activations once instead of once per channel tile.
//
// Pipeline of a step kt: the loads of step kt+2 are issued, the fragments of
// step kt are read from LDS buffer kt&1, step kt+1 (loaded one step ago) is
// decoded into the other buffer, the matrix cores run, one barrier.
//
// kPlanes = 3: the three sums of Section 4 apart (acc_out may receive them);
// kPlanes = 2: the folded form, y only.
template <int kBits, int kPlanes>
__global__ __launch_bounds__(kLinWG, 2) void k_linear(const int8_t *__restrict__ xq, long long M,
                                                   long long K, float s_x, float z_x,
                                                   const uint8_t *__restrict__ pcodes,
                                                   const uint8_t *__restrict__ pflags,
                                                   long long N,
                                                   const float *__restrict__ p,
                                                   const float *__restrict__ m,
                                                   const float *__restrict__ wconst,
                                                   float *__restrict__ y, int *__restrict__ acc_out,
                                                   int tiles_m, int tiles_n, int tn_per_xcd)
{
    constexpr int kMT = lin_mt(kPlanes), kBM = lin_bm(kPlanes), kAVec = lin_avec(kPlanes);
    __shared__ __attribute__((aligned(16))) int8_t sA[2][kBM * kLinStride];
    __shared__ __attribute__((aligned(16))) int8_t sB[2][kPlanes * kLinBN * kLinStride];

    const int xcd = blockIdx.x & 7;
    const int slot = blockIdx.x >> 3;
    const int bn = xcd * tn_per_xcd + slot % tn_per_xcd;
    const int bm = slot / tn_per_xcd;
    if (bm >= tiles_m || bn >= tiles_n) return;
    const long long row0 = (long long)bm * kBM, col0 = (long long)bn * kLinBN;

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;        // wm in [0, kLinWM)

    v16i acc[kMT][kPlanes];
#pragma unroll
    for (int a = 0; a < kMT; ++a)
#pragma unroll
        for (int b = 0; b < kPlanes; ++b)
#pragma unroll
            for (int c = 0; c < 16; ++c) acc[a][b][c] = 0;

    // K is a multiple of 16; the last step holds 1 to 4 pieces of 16 elements
    const int steps = (int)((K + kLinBK - 1) / kLinBK);
    const int last_valid = (int)((K - (long long)(steps - 1) * kLinBK) / 16);
    auto valid = [&](int step) { return step == steps - 1 ? last_valid : 4; };
    LinStage<kBits, kAVec> near, far;
    lin_load<kBits, kAVec>(near, xq, M, K, pcodes, pflags, N, row0, col0, 0, valid(0));
    lin_store<kBits, kPlanes>(near, sA[0], sB[0], valid(0));
    if (steps > 1) lin_load<kBits, kAVec>(near, xq, M, K, pcodes, pflags, N, row0, col0, kLinBK, valid(1));
    __syncthreads();
    // row of this lane's fragments (every 32-row tile of a wavefront has the same
    // swizzle: tiles start at multiples of 32 rows) and its chunk swizzle
    const int8_t *a_lane = sA[0] + (wm * 32 * kMT + (lane & 31)) * kLinStride;
    const int8_t *b_lane = sB[0] + (wn * 32 + (lane & 31)) * kLinStride;
    const int swz = lin_swz(lane & 31), half = lane >> 5;
    // the last two steps have nothing left to load / to decode: peeled, so that
    // the steady-state body is free of branches
    int kt = 0;
    // Steady state, two steps per trip so that the two register stages swap roles
    // instead of being copied; every step loaded here lies wholly below K.
    const LinOffsets<kBits, kAVec> offs = lin_offsets<kBits, kAVec>(M, K, N, row0, col0);
    const int8_t *a_base = xq + row0 * K;                                   // + k0
    const uint8_t *code_base = pcodes + ((col0 * K) >> 4) * (2 * kBits);    // + (k0 / 16) * 2b
    const uint8_t *flag_base = pflags + ((col0 * K) >> 3);                  // + k0 / 8
    for (; kt + 4 < steps; kt += 2) {
        const long long k2 = (long long)(kt + 2) * kLinBK, k3 = k2 + kLinBK;
        lin_load_whole<kBits, kAVec>(far, offs, a_base + k2, code_base + (k2 >> 4) * (2 * kBits), flag_base + (k2 >> 3));
        lin_step<kBits, kPlanes, true>(acc, near, 4, a_lane, b_lane, swz, half, sA[0], sB[0], 0);
        lin_load_whole<kBits, kAVec>(near, offs, a_base + k3, code_base + (k3 >> 4) * (2 * kBits), flag_base + (k3 >> 3));
        lin_step<kBits, kPlanes, true>(acc, far, 4, a_lane, b_lane, swz, half, sA[0], sB[0], 1);
    }
    for (; kt + 2 < steps; ++kt) {
        lin_load<kBits, kAVec>(far, xq, M, K, pcodes, pflags, N, row0, col0, (long long)(kt + 2) * kLinBK,
                               valid(kt + 2));
        lin_step<kBits, kPlanes, true>(acc, near, valid(kt + 1), a_lane, b_lane, swz, half, sA[0], sB[0], kt & 1);
        near = far;
    }
    if (kt + 1 < steps) {
        lin_step<kBits, kPlanes, true>(acc, near, valid(kt + 1), a_lane, b_lane, swz, half, sA[0], sB[0], kt & 1);
        ++kt;
    }
    lin_step<kBits, kPlanes, false>(acc, near, 4, a_lane, b_lane, swz, half, sA[0], sB[0], kt & 1);

    // epilogue: C2 A1 + C4 A2 + C5 A3 + (C3 + C6), per output channel
    const long long n = col0 + wn * 32 + (lane & 31);
    if (n >= N) return;
    const float Lf = (float)((1 << (kBits - 1)) - 1);
    const float pn = p[n], mn = m[n];
    const float s1 = pn / Lf;
    const float width = mn - pn;
    const float s2 = width / Lf;
    const float cst = z_x * wconst[n];
#pragma unroll
    for (int mt = 0; mt < kMT; ++mt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const long long row = row0 + wm * 32 * kMT + mt * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
            if (row < M) {
                if (kPlanes == 3) {
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
                } else {
                    // acc[mt][0] = A1 + L A3
                    float t = s1 * (float)acc[mt][0][r];
                    t = __builtin_fmaf(s2, (float)acc[mt][1][r], t);
                    y[row * N + n] = __builtin_fmaf(s_x, t, cst);
                }
            }
        }
    }
}

} // namespace pwlq
