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

// What the quantize kernels need to know of a tensor.  A model-level call of up
// to kEmitArgTensors tensors carries these fields inside the kernel arguments
// (EmitArgs), so that it launches nothing but the kernel itself; a longer table
// is read from the workspace like every other kernel's.
constexpr int kEmitArgTensors = 56;
struct EmitArgs {
    long long w[kEmitArgTensors];               // device address of the weights
    long long gcount[kEmitArgTensors], out_elem[kEmitArgTensors], out_group[kEmitArgTensors];
    long long out_code_byte[kEmitArgTensors], out_flag_byte[kEmitArgTensors];
    int ngroups[kEmitArgTensors];
    int emit_prefix[kEmitArgTensors + 1];       // first chunk of each tensor, then the total
    int nt;                                     // 0: not used, the table is in the workspace
};
struct EmitRec {
    const float *w;
    long long gcount, out_elem, out_group, out_code_byte, out_flag_byte;
    int ngroups, emit_base;
};
__device__ inline EmitRec emit_rec(const Tables &tb, const EmitArgs &ea, int chunk)
{
    EmitRec e;
    if (ea.nt > 0) {
        const int i = find_tensor(ea.emit_prefix, ea.nt, chunk);
        e.w = reinterpret_cast<const float *>(uni(ea.w[i]));
        e.gcount = uni(ea.gcount[i]);
        e.out_elem = uni(ea.out_elem[i]);
        e.out_group = uni(ea.out_group[i]);
        e.out_code_byte = uni(ea.out_code_byte[i]);
        e.out_flag_byte = uni(ea.out_flag_byte[i]);
        e.ngroups = uni(ea.ngroups[i]);
        e.emit_base = uni(ea.emit_prefix[i]);
    } else {
        const TensorRec r = rec_of(tb, find_tensor(tb.emit_prefix, tb.nt, chunk));
        e.w = r.w;
        e.gcount = r.gcount;
        e.out_elem = r.out_elem;
        e.out_group = r.out_group;
        e.out_code_byte = r.out_code_byte;
        e.out_flag_byte = r.out_flag_byte;
        e.ngroups = r.ngroups;
        e.emit_base = r.emit_base;
    }
    return e;
}

// A workgroup streams one chunk of kEmitChunk consecutive elements of one
// tensor: 16 bytes in, 4 + 4 + 16 bytes out per lane and access, four accesses
// in flight per thread.  The group of an element is its row-major index
// divided by the group length; a vector of four that stays inside one group
// shares one set of parameters.
__global__ __launch_bounds__(kWG) void k_emit(Tables tb, EmitArgs ea, int bits,
                                              const float *__restrict__ p_star,
                                              const float *__restrict__ m_in,
                                              uint8_t *__restrict__ codes,
                                              uint8_t *__restrict__ flags,
                                              float *__restrict__ w_hat)
{
    const int chunk = blockIdx.x;
    const EmitRec r = emit_rec(tb, ea, chunk);
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

// Bit-packed variant: a thread takes 8 consecutive elements, i.e. exactly
// `bits` bytes of the code stream and one byte of the flag stream.  The
// workgroup assembles its 256*bits code bytes and 256 flag bytes in LDS and
// writes them out as whole words; w_hat is optional.
constexpr int kPackPass = 8 * kWG;      // elements per pass of a workgroup
static_assert(kEmitChunk % kPackPass == 0 && kEmitChunk % (4 * kWG) == 0, "a chunk is a whole number of passes");

__global__ __launch_bounds__(kWG) void k_emit_packed(Tables tb, EmitArgs ea, int bits,
                                                     const float *__restrict__ p_star,
                                                     const float *__restrict__ m_in,
                                                     uint8_t *__restrict__ packed_codes,
                                                     uint8_t *__restrict__ packed_flags,
                                                     float *__restrict__ w_hat)
{
    __shared__ uint32_t code_stage[kWG * 8 / 4];
    __shared__ uint32_t flag_stage[kWG / 4];
    uint8_t *code_bytes = reinterpret_cast<uint8_t *>(code_stage);
    uint8_t *flag_bytes = reinterpret_cast<uint8_t *>(flag_stage);
    const int tid = threadIdx.x;
    const int chunk = blockIdx.x;
    const EmitRec r = emit_rec(tb, ea, chunk);
    const long long total = (long long)r.ngroups * r.gcount;
    const float *src = r.w;
    uint8_t *co = packed_codes + r.out_code_byte;
    uint8_t *fo = packed_flags + r.out_flag_byte;
    float *ho = w_hat ? w_hat + r.out_elem : nullptr;
    const bool small = total < 0x7fffffffLL;
    const bool in_aligned = (((uintptr_t)src) & 15) == 0;
    const bool hat_aligned = ho && (((uintptr_t)ho) & 15) == 0;
    const bool words_ok = ((((uintptr_t)co) | ((uintptr_t)fo)) & 3) == 0;

    for (int pass = 0; pass < kEmitChunk / kPackPass; ++pass) {
        const long long base = (long long)(chunk - r.emit_base) * kEmitChunk + (long long)pass * kPackPass;
        if (base >= total) break;
        const long long e = base + 8LL * tid;
        float wv[8];
        if (in_aligned && e + 7 < total) {
            const float4 a = *reinterpret_cast<const float4 *>(src + e);
            const float4 b = *reinterpret_cast<const float4 *>(src + e + 4);
            wv[0] = a.x; wv[1] = a.y; wv[2] = a.z; wv[3] = a.w;
            wv[4] = b.x; wv[5] = b.y; wv[6] = b.z; wv[7] = b.w;
        } else {
#pragma unroll
            for (int x = 0; x < 8; ++x) wv[x] = (e + x < total) ? src[e + x] : 0.0f;
        }
        unsigned long long word = 0;
        unsigned fbyte = 0;
        float hv[8];
        if (e < total) {
            const long long g = group_of(e, r.gcount, small);
            const bool one_group = (e - g * r.gcount) + 7 < r.gcount;
            Pieces q = group_pieces(p_star, m_in, r.out_group + g, bits);
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                if (e + x < total) {
                    if (!one_group)
                        q = group_pieces(p_star, m_in,
                                         r.out_group + group_of(e + x, r.gcount, small), bits);
                    uint8_t c, f;
                    emit_one(q, bits, wv[x], c, f, hv[x]);
                    word |= (unsigned long long)c << (x * bits);
                    fbyte |= (unsigned)f << x;
                }
            }
        }
        for (int x = 0; x < bits; ++x) code_bytes[tid * bits + x] = (uint8_t)(word >> (8 * x));
        flag_bytes[tid] = (uint8_t)fbyte;
        if (ho && e < total) {
            if (hat_aligned && e + 7 < total) {
                *reinterpret_cast<float4 *>(ho + e) = make_float4(hv[0], hv[1], hv[2], hv[3]);
                *reinterpret_cast<float4 *>(ho + e + 4) = make_float4(hv[4], hv[5], hv[6], hv[7]);
            } else {
#pragma unroll
                for (int x = 0; x < 8; ++x)
                    if (e + x < total) ho[e + x] = hv[x];
            }
        }
        __syncthreads();
        // bytes of this pass that exist in the streams
        long long left = total - base;
        if (left > kPackPass) left = kPackPass;
        const int nflag = (int)((left + 7) / 8);
        const int ncode = (int)((left * bits + 7) / 8);
        const long long code_at = base / 8 * bits;
        const long long flag_at = base / 8;
        if (words_ok) {
            for (int i = tid; i < ncode / 4; i += kWG)
                reinterpret_cast<uint32_t *>(co + code_at)[i] = code_stage[i];
            for (int i = (ncode & ~3) + tid; i < ncode; i += kWG) co[code_at + i] = code_bytes[i];
            for (int i = tid; i < nflag / 4; i += kWG)
                reinterpret_cast<uint32_t *>(fo + flag_at)[i] = flag_stage[i];
            for (int i = (nflag & ~3) + tid; i < nflag; i += kWG) fo[flag_at + i] = flag_bytes[i];
        } else {
            for (int i = tid; i < ncode; i += kWG) co[code_at + i] = code_bytes[i];
            for (int i = tid; i < nflag; i += kWG) fo[flag_at + i] = flag_bytes[i];
        }
        __syncthreads();
    }
}

} // namespace pwlq
