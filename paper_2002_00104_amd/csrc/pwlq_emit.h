// k_emit: the quantizer (codes, flags, dequantized weights).
#pragma once

#include "pwlq_tables.h"

namespace pwlq {

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
