// k_emit: the quantizer (codes, flags, dequantized weights).
#pragma once

#include "pwlq_tables.h"

namespace pwlq {

// Eq.3 with given (m, p): code, region flag and dequantized value per weight.
// Same arithmetic as piece_code (t = a*i1 in the centre, (a-p)*i2 in the tail,
// half-to-even, saturated) with the piece's parameters selected once per
// element instead of two evaluations selected afterwards; the centre value
// code*s1 is written fma(code, s1, +0), which rounds the same product.
// kHat = false: the dequantized value is not wanted.  The sign bit of a code is set for a
// negative weight whose value is not zero, and the value step*code + offset is zero exactly
// when the code is 0 and the offset (0 in the centre, p in the tail) is 0, so the code and
// the flag do not need the value at all.
template <bool kHat = true>
__device__ inline void emit_one(const Pieces &q, int bits, float w, uint8_t &code_out,
                                uint8_t &flag_out, float &hat_out)
{
    const float a = fabsf(w);
    const bool tail = a > q.p;
    const float z = tail ? q.p : 0.0f;
    const float x = a - z;                      // a - 0 is a
    const float inv = tail ? q.i2 : q.i1;
    float code = rintf(x * inv);
    code = (code > q.L) ? q.L : code;
    bool neg;
    if (kHat) {
        const float s = tail ? q.s2 : q.s1;
        const float top = tail ? q.m : q.p;
        float v = __builtin_fmaf(code, s, z);
        v = (code == q.L) ? top : v;
        neg = (w < 0.0f) && (v > 0.0f);
        hat_out = neg ? -v : v;
    } else {
        neg = (w < 0.0f) && (code > 0.0f || (tail && q.p > 0.0f));
    }
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

// Bit-packed variant: a thread takes kPackPer = 8 or 16 consecutive elements,
// i.e. whole bytes of the code stream and one or two bytes of the flag stream.
// Without w_hat the kernel is bound by its instructions, and 16 per thread pay
// the group's parameters (four correctly rounded divisions) and the index
// division once per 16 elements; with w_hat it is bound by the stores, and 8
// per thread keep a wavefront's 16-byte stores closer together (16 per thread
// measured 40 % slower there).  With 2, 4 or 8 bits a thread's codes are whole
// 32-bit words (16 bits for 8 elements of 2): it stores them itself, and
// neighbouring lanes combine their flag bytes into one word through DPP;
// nothing goes through LDS and nothing waits on another wavefront.  Other
// widths (and streams that are not word-aligned) assemble the workgroup's code
// and flag bytes in LDS and write them out as whole words.
template <int kBits, int kPackPer>
__global__ __launch_bounds__(kEmitChunk / kPackPer) void k_emit_packed(Tables tb, EmitArgs ea,
                                                        const float *__restrict__ p_star,
                                                        const float *__restrict__ m_in,
                                                        uint8_t *__restrict__ packed_codes,
                                                        uint8_t *__restrict__ packed_flags,
                                                        float *__restrict__ w_hat)
{
    static_assert(kPackPer == 8 || kPackPer == 16, "one or two flag bytes per thread");
    constexpr int kPackT = kEmitChunk / kPackPer;              // one chunk per workgroup
    constexpr int bits = kBits;
    constexpr bool kWordsPerThread = kBits == 2 || kBits == 4 || kBits == 8;
    constexpr int kCodeBytes = kPackPer * kBits / 8;           // per thread
    constexpr int kFlagBytes = kPackPer / 8;
    __shared__ uint32_t code_stage[kPackT * kCodeBytes / 4];
    __shared__ uint32_t flag_stage[kPackT * kFlagBytes / 4];
    uint8_t *code_bytes = reinterpret_cast<uint8_t *>(code_stage);
    uint8_t *flag_bytes = reinterpret_cast<uint8_t *>(flag_stage);
    const int tid = threadIdx.x;
    const int chunk = blockIdx.x;
    const EmitRec r = emit_rec(tb, ea, chunk);
    const long long total = (long long)r.ngroups * r.gcount;
    const long long last = total - 1;
    const float *src = r.w;
    uint8_t *co = packed_codes + r.out_code_byte;
    uint8_t *fo = packed_flags + r.out_flag_byte;
    float *ho = w_hat ? w_hat + r.out_elem : nullptr;
    const bool small = total < 0x7fffffffLL;
    const bool in_aligned = (((uintptr_t)src) & 15) == 0;
    const bool hat_aligned = ho && (((uintptr_t)ho) & 15) == 0;
    const bool words_ok = ((((uintptr_t)co) | ((uintptr_t)fo)) & 3) == 0;
    const bool direct = kWordsPerThread && words_ok;

    const long long base = (long long)(chunk - r.emit_base) * kEmitChunk;
    const long long e = base + (long long)kPackPer * tid;
    const bool full = e + (kPackPer - 1) <= last;
    float wv[kPackPer];
    if (in_aligned && full) {
#pragma unroll
        for (int v = 0; v < kPackPer / 4; ++v) {
            const float4 a = *reinterpret_cast<const float4 *>(src + e + 4 * v);
            wv[4 * v] = a.x; wv[4 * v + 1] = a.y; wv[4 * v + 2] = a.z; wv[4 * v + 3] = a.w;
        }
    } else {
#pragma unroll
        for (int x = 0; x < kPackPer; ++x) wv[x] = (e + x <= last) ? src[e + x] : 0.0f;
    }
    // codes of elements 0-7 in cw[0], of 8-15 in cw[1] (kBits bytes each); flags in fbits
    unsigned long long cw[2] = {0, 0};          // cw[1] stays 0 with 8 elements per thread
    unsigned fbits = 0;
    float hv[kPackPer];
    if (e <= last) {
        const long long g = group_of(e, r.gcount, small);
        const bool one_group = (e - g * r.gcount) + (kPackPer - 1) < r.gcount;
        Pieces q = group_pieces(p_star, m_in, r.out_group + g, bits);
        if (full && one_group) {
#pragma unroll
            for (int x = 0; x < kPackPer; ++x) {
                uint8_t c, f;
                if (kPackPer == 16) emit_one<false>(q, bits, wv[x], c, f, hv[x]);     // launched without w_hat
                else emit_one<true>(q, bits, wv[x], c, f, hv[x]);
                cw[x >> 3] |= (unsigned long long)c << ((x & 7) * bits);
                fbits |= (unsigned)f << x;
            }
        } else {
#pragma unroll
            for (int x = 0; x < kPackPer; ++x) {
                if (e + x <= last) {
                    if (!one_group)
                        q = group_pieces(p_star, m_in,
                                         r.out_group + group_of(e + x, r.gcount, small), bits);
                    uint8_t c, f;
                    emit_one(q, bits, wv[x], c, f, hv[x]);
                    cw[x >> 3] |= (unsigned long long)c << ((x & 7) * bits);
                    fbits |= (unsigned)f << x;
                }
            }
        }
    }
    if (ho && e <= last) {
        if (hat_aligned && full) {
#pragma unroll
            for (int v = 0; v < kPackPer / 4; ++v)
                *reinterpret_cast<float4 *>(ho + e + 4 * v) =
                    make_float4(hv[4 * v], hv[4 * v + 1], hv[4 * v + 2], hv[4 * v + 3]);
        } else {
#pragma unroll
            for (int x = 0; x < kPackPer; ++x)
                if (e + x <= last) ho[e + x] = hv[x];
        }
    }
    const long long code_at = base / 8 * bits;          // first byte of this workgroup in the streams
    const long long flag_at = base / 8;
    if (direct) {
        // the thread's code bytes as 32-bit words (8 elements of 2 bits: one 16-bit word)
        uint32_t words[4] = {0, 0, 0, 0};
        if (kBits == 2) words[0] = (uint32_t)cw[0] | ((uint32_t)cw[1] << 16);
        else if (kBits == 4) { words[0] = (uint32_t)cw[0]; words[1] = (uint32_t)cw[1]; }
        else { words[0] = (uint32_t)cw[0]; words[1] = (uint32_t)(cw[0] >> 32);
               words[2] = (uint32_t)cw[1]; words[3] = (uint32_t)(cw[1] >> 32); }
        uint8_t *mine = co + code_at + (long long)kCodeBytes * tid;
        if (full) {
            if (kCodeBytes == 2) *reinterpret_cast<uint16_t *>(mine) = (uint16_t)words[0];
#pragma unroll
            for (int x = 0; x < kCodeBytes / 4; ++x) reinterpret_cast<uint32_t *>(mine)[x] = words[x];
        } else if (e <= last) {                          // the stream ends inside this thread's bytes
            const int nb = (int)(((last - e + 1) * kBits + 7) / 8);
            for (int x = 0; x < nb; ++x) mine[x] = (uint8_t)(words[x >> 2] >> (8 * (x & 3)));
        }
        // the flag bytes of 4 / kFlagBytes neighbouring lanes into the first one's word
        unsigned fw;
        if (kFlagBytes == 2) {              // quad_perm 1,1,3,3: the next lane's half-word
            fw = fbits | ((unsigned)__builtin_amdgcn_mov_dpp((int)fbits, 0xF5, 0xf, 0xf, true) << 16);
        } else {                            // quad_perm 1,2,3,3: the next lane's byte, then 2,3,2,3
            fw = fbits | ((unsigned)__builtin_amdgcn_mov_dpp((int)fbits, 0xF9, 0xf, 0xf, true) << 8);
            fw = (fw & 0xffffu) | ((unsigned)__builtin_amdgcn_mov_dpp((int)fw, 0xEE, 0xf, 0xf, true) << 16);
        }
        constexpr int kLanes = 4 / kFlagBytes;              // lanes per flag word
        const long long e_first = e - (long long)kPackPer * (tid & (kLanes - 1));
        if (e_first + 31 <= last) {
            if ((tid & (kLanes - 1)) == 0) *reinterpret_cast<uint32_t *>(fo + flag_at + kFlagBytes * tid) = fw;
        } else if (e <= last) {
            const int nb = (int)((last - e + 8) / 8);     // flag bytes of this thread that exist
            for (int x = 0; x < nb && x < kFlagBytes; ++x)
                fo[flag_at + kFlagBytes * tid + x] = (uint8_t)(fbits >> (8 * x));
        }
        return;
    }
    for (int x = 0; x < bits; ++x) {
        code_bytes[tid * kCodeBytes + x] = (uint8_t)(cw[0] >> (8 * x));
        if (kPackPer == 16) code_bytes[tid * kCodeBytes + bits + x] = (uint8_t)(cw[1] >> (8 * x));
    }
    flag_bytes[kFlagBytes * tid] = (uint8_t)fbits;
    if (kFlagBytes == 2) flag_bytes[2 * tid + 1] = (uint8_t)(fbits >> 8);
    __syncthreads();
    // bytes of this chunk that exist in the streams
    long long left = total - base;
    if (left > kEmitChunk) left = kEmitChunk;
    const int nflag = (int)((left + 7) / 8);
    const int ncode = (int)((left * bits + 7) / 8);
    if (words_ok) {
        for (int i = tid; i < ncode / 4; i += kPackT)
            reinterpret_cast<uint32_t *>(co + code_at)[i] = code_stage[i];
        for (int i = (ncode & ~3) + tid; i < ncode; i += kPackT) co[code_at + i] = code_bytes[i];
        for (int i = tid; i < nflag / 4; i += kPackT)
            reinterpret_cast<uint32_t *>(fo + flag_at)[i] = flag_stage[i];
        for (int i = (nflag & ~3) + tid; i < nflag; i += kPackT) fo[flag_at + i] = flag_bytes[i];
    } else {
        for (int i = tid; i < ncode; i += kPackT) co[code_at + i] = code_bytes[i];
        for (int i = tid; i < nflag; i += kPackT) fo[flag_at + i] = flag_bytes[i];
    }
}

} // namespace pwlq
