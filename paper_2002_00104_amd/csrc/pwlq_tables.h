// Per-call tensor table as the kernels see it.
#pragma once

#include "pwlq_device.h"

namespace pwlq {

typedef float float8 __attribute__((ext_vector_type(8)));

// A call with one tensor carries its record in the kernel arguments (`one`)
// and touches no table in memory; a model-level call reads `recs` and the
// prefix arrays from the head of the workspace.
struct Tables {
    const TensorRec *recs;
    const int *tile_prefix, *group_prefix, *unit_prefix, *mgroup_prefix, *emit_prefix;
    int nt;
    int n_units;
    TensorRec one;
};

// Every field of a record is the same in all lanes; passing it through
// readfirstlane tells the compiler so, which keeps loop bounds and addresses
// derived from it in scalar registers (and the loads they feed scalar loads).
__device__ inline int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ inline long long uni(long long v)
{
    unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(v & 0xffffffffLL));
    int hi = __builtin_amdgcn_readfirstlane((int)(v >> 32));
    return ((long long)hi << 32) | (long long)lo;
}
__device__ inline TensorRec rec_of(const Tables &tb, int i)
{
    TensorRec r = (tb.nt == 1) ? tb.one : tb.recs[i];
    r.w = reinterpret_cast<const float *>(uni((long long)reinterpret_cast<uintptr_t>(r.w)));
    r.gcount = uni(r.gcount);
    r.sorted_base = uni(r.sorted_base);
    r.out_elem = uni(r.out_elem);
    r.out_group = uni(r.out_group);
    r.out_code_byte = uni(r.out_code_byte);
    r.out_flag_byte = uni(r.out_flag_byte);
    r.tile_len = uni(r.tile_len);
    r.last_len = uni(r.last_len);
    r.tpg = uni(r.tpg);
    r.stride = uni(r.stride);
    r.tpu = uni(r.tpu);
    r.part_base = uni(r.part_base);
    r.tile_base = uni(r.tile_base);
    r.group_base = uni(r.group_base);
    r.unit_base = uni(r.unit_base);
    r.mgroup_base = uni(r.mgroup_base);
    r.emit_base = uni(r.emit_base);
    r.ntiles = uni(r.ntiles);
    r.ngroups = uni(r.ngroups);
    r.fast = uni(r.fast);
    return r;
}
// Tile taken by the workgroup with index `slot`, returned in t.  For tensors
// whose groups are cut into several tiles the slots of the tensor take all full
// tiles first and the groups' last, shorter tiles afterwards: in tile order the
// two alternate, and because workgroups are placed on the CUs in turn every
// other CU would get only the short ones.
__device__ inline int slot_to_tile(const TensorRec &r, int slot)
{
    if (r.tpg == 1) return slot;
    const int ls = slot - r.tile_base;
    const int nfull = r.ngroups * (r.tpg - 1);
    const int g = ls < nfull ? ls / (r.tpg - 1) : ls - nfull;
    const int tig = ls < nfull ? ls - g * (r.tpg - 1) : r.tpg - 1;
    return r.tile_base + g * r.tpg + tig;
}
__device__ inline TileInfo tile_of(const Tables &tb, int slot, TensorRec &r, int &t)
{
    const int tensor = find_tensor(tb.tile_prefix, tb.nt, slot);
    r = rec_of(tb, tensor);
    t = slot_to_tile(r, slot);
    return tile_info(r, tensor, t);
}

// The per-call tables reach the device inside kernel arguments: no host memory
// has to outlive the call, the copy is ordered on the stream like any launch and
// it can be recorded into a graph.  One launch carries kUploadWords 32-bit words.
constexpr int kUploadWords = 1016;          // 4064 bytes of the 4 KB a launch may pass
struct UploadChunk {
    unsigned int words[kUploadWords];
};
__global__ __launch_bounds__(kWG) void k_upload(UploadChunk c, unsigned int *__restrict__ dst,
                                                int nwords)
{
    for (int i = threadIdx.x; i < nwords; i += kWG) dst[i] = c.words[i];
}

} // namespace pwlq
