// Device-side tables and helpers shared by the libpwlq kernels (gfx950).
//
// A call describes its tensors with a small table of TensorRec (one per
// tensor, sorted by tile length, longest first).  Kernels turn a tile, group
// or unit index into a tensor with a binary search over a prefix array and
// derive everything else arithmetically, so no per-tile table is uploaded.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pwlq {

constexpr int kWG = 256;          // threads per workgroup (4 wavefronts of 64)
constexpr int kWaves = kWG / 64;
constexpr int kBlk = 64;          // candidates per wavefront: lane = candidate
constexpr int kSearchWaves = 16;  // wavefronts (candidate blocks) per search workgroup (4 and 8 measured slower)
constexpr int kTileMax = 8192;    // longest run of a group handled by one workgroup
constexpr int kPerThread = kTileMax / kWG;  // elements of a tile held by one thread
constexpr int kFineMax = 2048;    // most candidates for which long tiles are ordered by candidate
constexpr int kFineMin = 64;      // shortest own bucket evaluated in candidate order (32 and 128 measured the same)
constexpr int kSmallTile = 1024;  // tiles up to this length get one wavefront each in k_prep and k_exact
constexpr int kSmallPer = kSmallTile / 64;
constexpr int kTinyTile = 16;     // tiles up to this length are two vectors: evaluated without offsets, loads one tile ahead
constexpr int kTinyUnit = 32;     // ... and batched up to this many per unit
constexpr int kSmallCallTiles = 256;    // a search of at most this many short single-tile groups (one per CU) ...
constexpr long long kSmallCallEvals = 50000000;   // ... and evaluations is one fused launch (measured crossover)
constexpr int kUnitElems = 4096;  // small tiles are batched up to about this many elements
constexpr int kMinUnits = 4096;   // ... unless that would leave fewer search units than this
constexpr int kEmitChunk = 2048;  // elements per workgroup of the quantize kernel (4096 and 8192: 12-45 % slower on a 25 M-element model)
constexpr int kVec = 8;           // elements per scalar vector load in the search loop
constexpr int kChunk = 128;       // elements per inner fp32 accumulation chunk

struct TensorRec {
    const float *w;        // device [C, K]
    long long gcount;      // elements per group
    long long sorted_base; // first element of this tensor's region in the sorted array
    long long out_elem;    // caller's elem_offset
    long long out_group;   // caller's group_offset
    long long out_code_byte, out_flag_byte;   // packed quantizer: start of this tensor's streams
    int tile_len;          // full tile length
    int last_len;          // length of the last tile of a group
    int tpg;               // tiles per group
    int stride;            // padded tile length in the sorted array
    int tpu;               // tiles per search unit
    int part_base;         // first partial-sum row (multi-tile groups), else -1
    int tile_base, group_base, unit_base, mgroup_base;
    int emit_base;         // first chunk of this tensor in the quantize kernel's grid
    int ntiles, ngroups;
    int fast;              // tiles evaluated by the prefix-sum kernel instead of prep + search
};

struct TileInfo {
    const float *src;
    long long sorted_off;
    long long elem_off;   // row-major index of the tile's first element in its tensor
    int len, group, tensor, local_tile, group_local, tile_in_group;
};

// largest i in [0, nt) with prefix[i] <= x; prefix[nt] > x is required
// prefix is non-decreasing with prefix[0] = 0, and x is the same in every lane.
// Every lane tests one entry and a ballot counts how many are <= x, so the
// lookup costs one memory round trip per 64 tensors instead of one per halving
// step.  Must be called with all 64 lanes of the wavefront active.
__device__ inline int find_tensor(const int *__restrict__ prefix, int nt, int x)
{
    if (nt == 1) return 0;
    const int lane = threadIdx.x & 63;
    int count = 0;
    for (int base = 0; base < nt; base += 64) {
        const int i = base + lane;
        const bool le = (i < nt) && (prefix[i] <= x);
        const unsigned long long bal = __ballot(le);
        count += __builtin_popcountll(bal);
        if (bal != ~0ull) break;
    }
    return __builtin_amdgcn_readfirstlane(count - 1);
}

__device__ inline TileInfo tile_info(const TensorRec &r, int tensor, int t)
{
    TileInfo ti;
    ti.tensor = tensor;
    ti.local_tile = t - r.tile_base;
    ti.group_local = ti.local_tile / r.tpg;
    ti.tile_in_group = ti.local_tile - ti.group_local * r.tpg;
    ti.elem_off = (long long)ti.group_local * r.gcount + (long long)ti.tile_in_group * r.tile_len;
    ti.src = r.w + ti.elem_off;
    ti.len = (ti.tile_in_group == r.tpg - 1) ? r.last_len : r.tile_len;
    ti.group = r.group_base + ti.group_local;
    ti.sorted_off = r.sorted_base + (long long)ti.local_tile * r.stride;
    return ti;
}

// ---- wavefront / workgroup reductions (fixed order, so results are repeatable)
// Built on DPP row shifts and row broadcasts: four shift-and-combine steps scan
// each row of 16 lanes, row_bcast:15 carries a row's total into the next row
// (rows 1 and 3), row_bcast:31 carries lane 31 into rows 2 and 3.  After the six
// steps lane i holds the combination of lanes 0..i, so lane 63 holds the total.
// A lane with no source keeps `old`.
template <int kCtrl, int kRows>
__device__ inline int dpp_i32(int old, int v)
{
    return __builtin_amdgcn_update_dpp(old, v, kCtrl, kRows, 0xf, false);
}
template <int kCtrl, int kRows>
__device__ inline float dpp_f32(float old, float v)
{
    return __int_as_float(dpp_i32<kCtrl, kRows>(__float_as_int(old), __float_as_int(v)));
}
template <int kCtrl, int kRows>
__device__ inline double dpp_f64(double old, double v)
{
    const int lo = dpp_i32<kCtrl, kRows>(__double2loint(old), __double2loint(v));
    const int hi = dpp_i32<kCtrl, kRows>(__double2hiint(old), __double2hiint(v));
    return __hiloint2double(hi, lo);
}
__device__ inline double lane63(double v)
{
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), 63),
                            __builtin_amdgcn_readlane(__double2loint(v), 63));
}

// inclusive prefix sum over the 64 lanes of a wavefront
__device__ inline int wave_scan_incl(int v)
{
    v += dpp_i32<0x111, 0xf>(0, v);
    v += dpp_i32<0x112, 0xf>(0, v);
    v += dpp_i32<0x114, 0xf>(0, v);
    v += dpp_i32<0x118, 0xf>(0, v);
    v += dpp_i32<0x142, 0xa>(0, v);
    v += dpp_i32<0x143, 0xc>(0, v);
    return v;
}
__device__ inline float wave_max(float v)
{
    v = fmaxf(v, dpp_f32<0x111, 0xf>(v, v));
    v = fmaxf(v, dpp_f32<0x112, 0xf>(v, v));
    v = fmaxf(v, dpp_f32<0x114, 0xf>(v, v));
    v = fmaxf(v, dpp_f32<0x118, 0xf>(v, v));
    v = fmaxf(v, dpp_f32<0x142, 0xa>(v, v));
    v = fmaxf(v, dpp_f32<0x143, 0xc>(v, v));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ inline double wave_sum(double v)
{
    v += dpp_f64<0x111, 0xf>(0.0, v);
    v += dpp_f64<0x112, 0xf>(0.0, v);
    v += dpp_f64<0x114, 0xf>(0.0, v);
    v += dpp_f64<0x118, 0xf>(0.0, v);
    v += dpp_f64<0x142, 0xa>(0.0, v);
    v += dpp_f64<0x143, 0xc>(0.0, v);
    return lane63(v);
}
__device__ inline double wave_min(double v)
{
    v = fmin(v, dpp_f64<0x111, 0xf>(v, v));
    v = fmin(v, dpp_f64<0x112, 0xf>(v, v));
    v = fmin(v, dpp_f64<0x114, 0xf>(v, v));
    v = fmin(v, dpp_f64<0x118, 0xf>(v, v));
    v = fmin(v, dpp_f64<0x142, 0xa>(v, v));
    v = fmin(v, dpp_f64<0x143, 0xc>(v, v));
    return lane63(v);
}
__device__ inline int wave_or(int v)
{
    return __ballot(v != 0) != 0ull;
}

// Sum / minimum over a workgroup of kW wavefronts, returned to every thread.
// `lds` holds kW doubles.
template <int kW = kWaves>
__device__ inline double block_sum(double v, double *lds)
{
    v = wave_sum(v);
    if (kW == 1) return v;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    double s = lds[0];
    for (int i = 1; i < kW; ++i) s += lds[i];
    return s;
}
template <int kW = kWaves>
__device__ inline double block_min(double v, double *lds)
{
    v = wave_min(v);
    if (kW == 1) return v;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    double s = lds[0];
    for (int i = 1; i < kW; ++i) s = fmin(s, lds[i]);
    return s;
}

// ---- the canonical binary32 arithmetic of one (m, p) pair: Eq.1 steps of the
// centre piece [0,p] and the tail piece [p,m], each with L = 2^(b-1)-1 steps.
struct Pieces {
    float p, m, s1, s2, i1, i2, L;
};

__device__ inline float grid_point(float m, int k, int n)
{
    float ratio = (float)k / (float)n;
    return m * ratio;
}

__device__ inline Pieces make_pieces(float m, float p, int bits)
{
    Pieces q;
    q.m = m;
    q.p = p;
    q.L = (float)((1 << (bits - 1)) - 1);
    q.s1 = p / q.L;
    float width = m - p;
    q.s2 = width / q.L;
    q.i1 = (q.s1 > 0.0f) ? 1.0f / q.s1 : 0.0f;
    q.i2 = (q.s2 > 0.0f) ? 1.0f / q.s2 : 0.0f;
    return q;
}

// Eq.3 on a magnitude: region (closed centre) and saturated, half-to-even code.
__device__ inline float piece_code(const Pieces &q, float a, bool &tail)
{
    tail = a > q.p;
    float x = a - q.p;
    float t = tail ? x * q.i2 : a * q.i1;
    float code = rintf(t);
    return (code > q.L) ? q.L : code;
}

} // namespace pwlq
