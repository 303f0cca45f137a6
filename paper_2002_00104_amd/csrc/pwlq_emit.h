// k_emit: the quantizer (codes, flags, dequantized weights).
#pragma once

#include "pwlq_tables.h"

namespace pwlq {

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

// group of row-major element e; 32-bit division when the tensor allows it
__device__ inline long long group_of(long long e, long long gcount, bool small)
{
    if (small) return (long long)((unsigned)e / (unsigned)gcount);
    return e / gcount;
}

__device__ inline Pieces group_pieces(const float *__restrict__ p_star,
                                      const float *__restrict__ m_in, long long og, int bits)
{
    return make_pieces(m_in[og], p_star[og], bits);
}

// A workgroup streams one chunk of kEmitChunk consecutive elements of one
// tensor: 16 bytes in, 4 + 4 + 16 bytes out per lane and access, four accesses
// in flight per thread.  The group of an element is its row-major index
// divided by the group length; a vector of four that stays inside one group
// shares one set of parameters.
__global__ __launch_bounds__(kWG) void k_emit(Tables tb, int bits,
                                              const float *__restrict__ p_star,
                                              const float *__restrict__ m_in,
                                              uint8_t *__restrict__ codes,
                                              uint8_t *__restrict__ flags,
                                              float *__restrict__ w_hat)
{
    const int chunk = blockIdx.x;
    const int tensor = find_tensor(tb.emit_prefix, tb.nt, chunk);
    const TensorRec r = rec_of(tb, tensor);
    const long long total = (long long)r.ngroups * r.gcount;
    const long long e0 = (long long)(chunk - r.emit_base) * kEmitChunk;
    const float *src = r.w;
    uint8_t *co = codes + r.out_elem;
    uint8_t *fo = flags + r.out_elem;
    float *ho = w_hat + r.out_elem;
    const bool aligned = ((((uintptr_t)src) | ((uintptr_t)ho)) & 15) == 0 &&
                         ((((uintptr_t)co) | ((uintptr_t)fo)) & 3) == 0;
    constexpr int kPer = kEmitChunk / (4 * kWG);          // vectors per thread
    const bool small = total < 0x7fffffffLL;

    if (aligned) {
        float4 w4[kPer];
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const long long e = e0 + 4 * (long long)(i * kWG + threadIdx.x);
            if (e + 3 < total) w4[i] = *reinterpret_cast<const float4 *>(src + e);
        }
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            const long long e = e0 + 4 * (long long)(i * kWG + threadIdx.x);
            if (e + 3 < total) {
                const long long g = group_of(e, r.gcount, small);
                const long long in_row = e - g * r.gcount;
                uchar4 c4, f4;
                float4 h4;
                if (in_row + 3 < r.gcount) {
                    const Pieces q = group_pieces(p_star, m_in, r.out_group + g, bits);
                    emit_one(q, bits, w4[i].x, c4.x, f4.x, h4.x);
                    emit_one(q, bits, w4[i].y, c4.y, f4.y, h4.y);
                    emit_one(q, bits, w4[i].z, c4.z, f4.z, h4.z);
                    emit_one(q, bits, w4[i].w, c4.w, f4.w, h4.w);
                } else {
                    // the vector straddles a group boundary
                    const float wv[4] = {w4[i].x, w4[i].y, w4[i].z, w4[i].w};
                    uint8_t cv[4], fv[4];
                    float hv[4];
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        const Pieces q =
                            group_pieces(p_star, m_in, r.out_group + group_of(e + x, r.gcount, small), bits);
                        emit_one(q, bits, wv[x], cv[x], fv[x], hv[x]);
                    }
                    c4 = make_uchar4(cv[0], cv[1], cv[2], cv[3]);
                    f4 = make_uchar4(fv[0], fv[1], fv[2], fv[3]);
                    h4 = make_float4(hv[0], hv[1], hv[2], hv[3]);
                }
                *reinterpret_cast<uchar4 *>(co + e) = c4;
                *reinterpret_cast<uchar4 *>(fo + e) = f4;
                *reinterpret_cast<float4 *>(ho + e) = h4;
            } else {
                for (long long x = e; x < total && x < e + 4; ++x) {
                    const Pieces q =
                        group_pieces(p_star, m_in, r.out_group + group_of(x, r.gcount, small), bits);
                    emit_one(q, bits, src[x], co[x], fo[x], ho[x]);
                }
            }
        }
    } else {
        for (int i = threadIdx.x; i < kEmitChunk; i += kWG) {
            const long long x = e0 + i;
            if (x < total) {
                const Pieces q =
                        group_pieces(p_star, m_in, r.out_group + group_of(x, r.gcount, small), bits);
                emit_one(q, bits, src[x], co[x], fo[x], ho[x]);
            }
        }
    }
}

} // namespace pwlq
