// Host side of libpwlq: argument checks, the per-call tensor table, workspace
// layout and kernel launches.  See include/pwlq.h for the contract.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <atomic>
#include <mutex>
#include <numeric>
#include <vector>

#include "../../include/pwlq.h"
#include "../../include/pwlq_bench.h"
#include "pwlq_kernels.h"

// Scratch of pwlq_search_static: one copy per GPU, resident until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress; the
// device address it yields is what kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[PWLQ_STATIC_SCRATCH_BYTES];

namespace {

using namespace pwlq;

thread_local char g_error[512] = "";
thread_local long long g_last_tiles = 0, g_last_groups = 0, g_last_units = 0;
thread_local const char *g_last_search_kernel = "k_search";

int fail(int status, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return status;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Everything a call needs to know about its tensors, built on the host.
struct Plan {
    std::vector<TensorRec> recs;
    std::vector<int> tile_prefix, group_prefix, unit_prefix, mgroup_prefix, emit_prefix;
    int nt = 0;
    long long n_tiles = 0, n_groups = 0, n_units = 0, n_mgroups = 0, n_chunks = 0;
    int n = 0, nblk = 0;
    // workspace offsets in bytes
    size_t off_recs = 0, off_prefix = 0, off_tile_max = 0, off_gm = 0, off_offsets = 0,
           off_sorted = 0, off_sse32 = 0, off_mask = 0, off_part = 0, off_gsum = 0,
           off_stat_max = 0, off_stat_s2 = 0, off_stat_s1 = 0, off_fine = 0, total = 0;
    bool fine = false;     // tiles ordered by candidate, with per-candidate switch positions
};

// per-tile scratch beyond the tensor table
enum Aux { kAuxNone = 0, kAuxStats = 1, kAuxMse = 2 };

int check_common(int bits, int mode)
{
    if (bits < 2 || bits > 8) return fail(PWLQ_EINVAL, "bits=%d outside [2,8]", bits);
    if (mode != PWLQ_PER_CHANNEL && mode != PWLQ_PER_TENSOR)
        return fail(PWLQ_EINVAL, "mode=%d is neither PWLQ_PER_CHANNEL nor PWLQ_PER_TENSOR", mode);
    return PWLQ_OK;
}

// n_cand == 0 builds a plan without search scratch (quantizer, selectors, error).
int build_plan(Plan &pl, const pwlq_tensor_desc *desc, int n_tensors, int n_cand, int mode,
               bool need_pointers, const int64_t *code_byte_offset = nullptr,
               const int64_t *flag_byte_offset = nullptr, Aux aux = kAuxNone,
               int fast_min_len = 0)
{
    if (!desc) return fail(PWLQ_ENULL, "tensor descriptor table is NULL");
    if (n_tensors < 1) return fail(PWLQ_EINVAL, "n_tensors=%d must be >= 1", n_tensors);
    pl.nt = n_tensors;
    pl.n = n_cand;
    pl.nblk = (n_cand + kBlk - 1) / kBlk;

    struct Item { int idx; int tile_len; };
    std::vector<Item> order(n_tensors);
    std::vector<TensorRec> tmp(n_tensors);
    for (int i = 0; i < n_tensors; ++i) {
        const pwlq_tensor_desc &d = desc[i];
        if (need_pointers && !d.w) return fail(PWLQ_ENULL, "desc[%d].w is NULL", i);
        if (d.C < 1 || d.K < 1) return fail(PWLQ_EINVAL, "desc[%d]: C=%lld K=%lld must be >= 1", i,
                                            (long long)d.C, (long long)d.K);
        if (d.group_offset < 0 || d.elem_offset < 0)
            return fail(PWLQ_EINVAL, "desc[%d]: negative offset", i);
        if (d.C > (1LL << 40) / d.K) return fail(PWLQ_EINVAL, "desc[%d]: tensor too large", i);
        TensorRec r;
        memset(&r, 0, sizeof(r));
        r.w = d.w;
        const long long groups = (mode == PWLQ_PER_CHANNEL) ? d.C : 1;
        r.gcount = (mode == PWLQ_PER_CHANNEL) ? d.K : d.C * d.K;
        r.out_elem = d.elem_offset;
        r.out_group = d.group_offset;
        r.out_code_byte = code_byte_offset ? code_byte_offset[i] : 0;
        r.out_flag_byte = flag_byte_offset ? flag_byte_offset[i] : 0;
        if (r.out_code_byte < 0 || r.out_flag_byte < 0)
            return fail(PWLQ_EINVAL, "desc[%d]: negative byte offset", i);
        const long long tpg = (r.gcount + kTileMax - 1) / kTileMax;
        r.tile_len = (tpg == 1) ? (int)r.gcount : kTileMax;
        r.last_len = (int)(r.gcount - (tpg - 1) * (long long)r.tile_len);
        if (groups * tpg > 0x3fffffffLL) return fail(PWLQ_EINVAL, "desc[%d]: too many tiles", i);
        r.tpg = (int)tpg;
        r.ngroups = (int)groups;
        r.ntiles = (int)(groups * tpg);
        r.stride = (r.tile_len + kVec - 1) / kVec * kVec + kVec;   // one spare vector: loads may run one ahead
        r.tpu = std::max(1, kUnitElems / r.tile_len);
        r.fast = (fast_min_len > 0 && r.tile_len >= fast_min_len) ? 1 : 0;
        tmp[i] = r;
        order[i] = {i, r.tile_len};
    }
    // a search workgroup walks tpu tiles one after the other; keep enough
    // workgroups to fill the chip when the call is small
    {
        long long total_tiles = 0;
        for (const TensorRec &r : tmp) total_tiles += r.ntiles;
        const int cap = (int)std::max(1LL, total_tiles / kMinUnits);
        // tiles of at most kTinyTile elements cost a unit little each (no offsets, loads one
        // tile ahead): up to kTinyUnit per unit while they still make about a thousand units
        long long tiny_tiles = 0;
        for (const TensorRec &r : tmp) if (r.tile_len <= kTinyTile && r.tpg == 1) tiny_tiles += r.ntiles;
        const int tiny_cap = (int)std::min((long long)kTinyUnit, std::max((long long)cap, tiny_tiles / 1024));
        for (TensorRec &r : tmp)
            r.tpu = std::min(r.tpu, (r.tile_len <= kTinyTile && r.tpg == 1) ? tiny_cap : cap);
    }
    // longest tiles first: the search kernel's workgroups are dispatched in
    // index order, so the big items start early and the small ones fill gaps
    std::stable_sort(order.begin(), order.end(),
                     [](const Item &a, const Item &b) { return a.tile_len > b.tile_len; });
    pl.recs.resize(n_tensors);
    pl.tile_prefix.assign(n_tensors + 1, 0);
    pl.group_prefix.assign(n_tensors + 1, 0);
    pl.unit_prefix.assign(n_tensors + 1, 0);
    pl.mgroup_prefix.assign(n_tensors + 1, 0);
    pl.emit_prefix.assign(n_tensors + 1, 0);
    long long tiles = 0, groups = 0, units = 0, mgroups = 0, parts = 0, sorted = 0, chunks = 0;
    for (int s = 0; s < n_tensors; ++s) {
        TensorRec r = tmp[order[s].idx];
        r.tile_base = (int)tiles;
        r.group_base = (int)groups;
        r.unit_base = (int)units;
        r.mgroup_base = (int)mgroups;
        r.sorted_base = sorted;
        r.part_base = (r.tpg > 1) ? (int)parts : -1;
        pl.tile_prefix[s] = (int)tiles;
        pl.group_prefix[s] = (int)groups;
        pl.unit_prefix[s] = (int)units;
        pl.mgroup_prefix[s] = (int)mgroups;
        pl.emit_prefix[s] = (int)chunks;
        r.emit_base = (int)chunks;
        chunks += ((long long)r.ngroups * r.gcount + kEmitChunk - 1) / kEmitChunk;
        tiles += r.ntiles;
        groups += r.ngroups;
        units += (r.ntiles + r.tpu - 1) / r.tpu;
        if (r.tpg > 1) { mgroups += r.ngroups; parts += r.ntiles; }
        if (!r.fast) sorted += (long long)r.ntiles * r.stride;
        if (tiles > 0x3fffffffLL || units > 0x3fffffffLL || chunks > 0x3fffffffLL)
            return fail(PWLQ_EINVAL, "call has too many tiles");
        pl.recs[s] = r;
    }
    pl.tile_prefix[n_tensors] = (int)tiles;
    pl.group_prefix[n_tensors] = (int)groups;
    pl.unit_prefix[n_tensors] = (int)units;
    pl.mgroup_prefix[n_tensors] = (int)mgroups;
    pl.emit_prefix[n_tensors] = (int)chunks;
    pl.n_chunks = chunks;
    pl.n_tiles = tiles;
    pl.n_groups = groups;
    pl.n_units = units;
    pl.n_mgroups = mgroups;

    size_t off = 0;
    auto take = [&](size_t bytes) { size_t at = off; off = align_up(off + bytes, 256); return at; };
    pl.off_recs = take(sizeof(TensorRec) * (size_t)n_tensors);
    pl.off_prefix = take(sizeof(int) * 5 * (size_t)(n_tensors + 1));
    if (n_cand > 0) {
        pl.off_tile_max = take(sizeof(float) * (size_t)tiles);
        pl.off_gm = take(sizeof(float) * (size_t)groups);
        pl.off_offsets = take(sizeof(int) * (size_t)tiles * (size_t)(pl.nblk + 1));
        pl.off_sorted = take(sizeof(float) * (size_t)sorted);
        pl.off_sse32 = take(sizeof(float) * (size_t)tiles * (size_t)n_cand);
        pl.fine = n_cand <= kFineMax;
        if (pl.fine) pl.off_fine = take(sizeof(unsigned short) * (size_t)tiles * (size_t)(n_cand + 1));
        pl.off_mask = take(sizeof(int) * (size_t)mgroups * (size_t)(n_cand + 1));
        pl.off_part = take(sizeof(double) * (size_t)parts * (size_t)n_cand);
        pl.off_gsum = take(sizeof(double) * (size_t)mgroups * (size_t)n_cand);
    }
    if (aux == kAuxStats) {
        pl.off_stat_max = take(sizeof(float) * (size_t)tiles);
        pl.off_stat_s2 = take(sizeof(double) * (size_t)tiles);
        pl.off_stat_s1 = take(sizeof(double) * (size_t)tiles);
    } else if (aux == kAuxMse) {
        pl.off_stat_s2 = take(sizeof(double) * (size_t)tiles);
    }
    pl.total = off;
    return PWLQ_OK;
}

int check_workspace(const Plan &pl, const void *workspace, size_t bytes)
{
    if (!workspace) return fail(PWLQ_EWORKSPACE, "workspace is NULL (%zu bytes needed)", pl.total);
    if (((uintptr_t)workspace & 255) != 0)
        return fail(PWLQ_EWORKSPACE, "workspace is not 256-byte aligned");
    if (bytes < pl.total)
        return fail(PWLQ_EWORKSPACE, "workspace holds %zu bytes, %zu needed", bytes, pl.total);
    return PWLQ_OK;
}

// Writes the tensor table into the head of the workspace and returns the
// device-side view.  Tables of up to kUploadMaxBytes travel in the arguments of
// k_upload launches (asynchronous, nothing on the host has to outlive the call,
// recordable into a graph); longer ones are copied from a host image that lives
// only for this call, so the call waits for the copy, and cannot be recorded.
constexpr size_t kUploadMaxBytes = 16 * sizeof(UploadChunk);

int upload_tables(const Plan &pl, char *ws, hipStream_t stream, Tables &tb)
{
    memset(&tb, 0, sizeof(tb));
    tb.nt = pl.nt;
    tb.n_units = (int)pl.n_units;
    if (pl.nt == 1) {            // the record travels in the kernel arguments
        tb.one = pl.recs[0];
        return PWLQ_OK;
    }
    // host image of [off_recs, off_prefix + prefix bytes): records, padding, the five prefix arrays
    static_assert(sizeof(TensorRec) % 4 == 0, "the table is copied in 32-bit words");
    const size_t prefix_bytes = sizeof(int) * 5 * (size_t)(pl.nt + 1);
    const size_t bytes = pl.off_prefix - pl.off_recs + prefix_bytes;
    std::vector<unsigned int> image(bytes / 4, 0u);
    memcpy(image.data(), pl.recs.data(), sizeof(TensorRec) * (size_t)pl.nt);
    int *prefix = reinterpret_cast<int *>(image.data() + (pl.off_prefix - pl.off_recs) / 4);
    const std::vector<int> *parts[5] = {&pl.tile_prefix, &pl.group_prefix, &pl.unit_prefix,
                                        &pl.mgroup_prefix, &pl.emit_prefix};
    for (int i = 0; i < 5; ++i)
        memcpy(prefix + (size_t)i * (pl.nt + 1), parts[i]->data(), sizeof(int) * (size_t)(pl.nt + 1));
    if (bytes <= kUploadMaxBytes) {
        UploadChunk chunk;
        for (size_t w0 = 0; w0 < image.size(); w0 += kUploadWords) {
            const size_t nw = std::min((size_t)kUploadWords, image.size() - w0);
            memcpy(chunk.words, image.data() + w0, nw * 4);
            k_upload<<<1, kWG, 0, stream>>>(chunk, reinterpret_cast<unsigned int *>(ws + pl.off_recs) + w0,
                                            (int)nw);
        }
        if (hipGetLastError() != hipSuccess) return fail(PWLQ_EHIP, "table upload launch failed");
    } else {
        // this copy reads host memory that is gone when the call returns: a graph that
        // recorded it would read freed memory at every replay
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(stream, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone)
            return fail(PWLQ_EINVAL, "a call with this many tensors copies its table from host memory "
                                     "and cannot be recorded into a graph");
        hipError_t e = hipMemcpyAsync(ws + pl.off_recs, image.data(), bytes, hipMemcpyHostToDevice, stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);    // `image` is gone when this function returns
        if (e != hipSuccess) return fail(PWLQ_EHIP, "table upload: %s", hipGetErrorString(e));
    }
    tb.recs = reinterpret_cast<const TensorRec *>(ws + pl.off_recs);
    const int *p = reinterpret_cast<const int *>(ws + pl.off_prefix);
    tb.tile_prefix = p;
    tb.group_prefix = p + (pl.nt + 1);
    tb.unit_prefix = p + 2 * (pl.nt + 1);
    tb.mgroup_prefix = p + 3 * (pl.nt + 1);
    tb.emit_prefix = p + 4 * (pl.nt + 1);
    return PWLQ_OK;
}

// The quantize kernels' view of a small tensor table, for the kernel arguments.
bool fill_emit_args(const Plan &pl, EmitArgs &ea)
{
    memset(&ea, 0, sizeof(ea));
    if (pl.nt < 2 || pl.nt > kEmitArgTensors) return false;
    for (int i = 0; i < pl.nt; ++i) {
        const TensorRec &r = pl.recs[i];
        ea.w[i] = (long long)reinterpret_cast<uintptr_t>(r.w);
        ea.gcount[i] = r.gcount;
        ea.out_elem[i] = r.out_elem;
        ea.out_group[i] = r.out_group;
        ea.out_code_byte[i] = r.out_code_byte;
        ea.out_flag_byte[i] = r.out_flag_byte;
        ea.ngroups[i] = r.ngroups;
        ea.emit_prefix[i] = pl.emit_prefix[i];
    }
    ea.emit_prefix[pl.nt] = pl.emit_prefix[pl.nt];
    ea.nt = pl.nt;
    return true;
}

int launch_status(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(PWLQ_EHIP, "%s: %s", what, hipGetErrorString(e));
    return PWLQ_OK;
}

// Optional event timing of the dominant kernels (benchmarks only).
// A ring of the last kProfRing recorded launches per role, so that a benchmark
// can time a run of calls without waiting inside it.
constexpr int kProfRoles = 4, kProfRing = 64;
unsigned g_profile = 0;         // bit r: events are recorded around the kernel of role r
hipEvent_t g_ev[kProfRoles][kProfRing][2];
bool g_ev_made = false;
long long g_ev_count[kProfRoles] = {0, 0, 0, 0};     // launches recorded so far

// idx = 2*role for the event before the kernel, 2*role+1 for the one after it
void profile_mark(int idx, hipStream_t stream)
{
    if (!((g_profile >> (idx >> 1)) & 1u) || !g_ev_made) return;
    const int role = idx >> 1;
    (void)hipEventRecord(g_ev[role][g_ev_count[role] % kProfRing][idx & 1], stream);
    if (idx & 1) ++g_ev_count[role];
}

// Shortest tile handed to the prefix-sum evaluator by the fast search: its
// cost per candidate grows with the number of levels (2L+1 look-ups) and does
// not depend on the tile length, the plain evaluation costs one pass over the
// tile.
int fast_min_len(int bits)
{
    const int L = (1 << (bits - 1)) - 1;
    return 16 * (2 * L + 1) + 64;
}

// Largest number of groups a search call may have and still run as one fused launch
// (PWLQ_SMALL_CALL_TILES overrides the default once; pwlq_set_small_call_tiles at any time).
std::atomic<int> &small_call_tiles()
{
    static std::atomic<int> v([] {
        const char *e = getenv("PWLQ_SMALL_CALL_TILES");
        return e ? atoi(e) : kSmallCallTiles;
    }());
    return v;
}

int run_search(const pwlq_tensor_desc *desc, int n_tensors, int bits, int n_cand, int mode,
               float *p_star, float *m_out, int32_t *k_star, double *mse, void *workspace,
               size_t workspace_bytes, void *stream_v, bool fast = false)
{
    int rc = check_common(bits, mode);
    if (rc) return rc;
    if (n_cand < 1 || n_cand > 65535) return fail(PWLQ_EINVAL, "n_cand=%d outside [1,65535]", n_cand);
    if (!p_star || !m_out || !k_star || !mse) return fail(PWLQ_ENULL, "an output pointer is NULL");
    Plan pl;
    rc = build_plan(pl, desc, n_tensors, n_cand, mode, true, nullptr, nullptr, kAuxNone,
                    fast ? fast_min_len(bits) : 0);
    if (rc) return rc;
    rc = check_workspace(pl, workspace, workspace_bytes);
    if (rc) return rc;
    // every limit is checked before the first launch: a failing call enqueues nothing
    const int ny = (pl.nblk + kSearchWaves - 1) / kSearchWaves;
    int bpw_log2 = 0;                      // candidate blocks per unit in a workgroup, as a power of two
    while ((1 << bpw_log2) < std::min(pl.nblk, kSearchWaves)) ++bpw_log2;
    // ... but a small call keeps one unit per workgroup rather than a handful of workgroups
    while (bpw_log2 < 4 && pl.n_units / (kSearchWaves >> bpw_log2) < 2048) ++bpw_log2;
    const int upw = kSearchWaves >> bpw_log2;       // units per workgroup
    const long long unit_groups = (pl.n_units + upw - 1) / upw;
    const long long wgs = (unit_groups + 7) / 8 * 8 * ny;
    if (wgs > 0x7fffffffLL) return fail(PWLQ_EINVAL, "search grid too large");
    const long long group_sum_wgs = pl.n_mgroups * (long long)((n_cand + kSumCand - 1) / kSumCand);
    if (group_sum_wgs > 0x7fffffffLL) return fail(PWLQ_EINVAL, "too many groups longer than one tile");

    hipStream_t stream = (hipStream_t)stream_v;
    char *ws = (char *)workspace;
    Tables tb;
    rc = upload_tables(pl, ws, stream, tb);
    if (rc) return rc;
    float *tile_max = (float *)(ws + pl.off_tile_max);
    float *gm = (float *)(ws + pl.off_gm);
    int *offsets = (int *)(ws + pl.off_offsets);
    float *sorted = (float *)(ws + pl.off_sorted);
    float *sse32 = (float *)(ws + pl.off_sse32);
    unsigned short *fine = pl.fine ? (unsigned short *)(ws + pl.off_fine) : nullptr;
    int *klist = (int *)(ws + pl.off_mask);
    double *part64 = (double *)(ws + pl.off_part);
    double *gsum = (double *)(ws + pl.off_gsum);

    const int NT = (int)pl.n_tiles;
    // A call too small to fill the chip: everything for a group in one workgroup, one launch.
    {
        int longest_any = 0;
        long long evals = 0;
        for (const TensorRec &r : pl.recs) {
            longest_any = std::max(longest_any, r.tile_len);
            evals += (long long)r.ntiles * r.tile_len * n_cand;
        }
        // (also for a fast search: at this size the fused exhaustive launch is the faster way
        // to the same result)
        if (pl.n_mgroups == 0 && NT <= small_call_tiles().load() && evals <= kSmallCallEvals &&
            longest_any <= kSmallLen && n_cand <= kSmallCand) {
            profile_mark(fast ? 4 : 0, stream);
            k_small<<<NT, kSmallWG, 0, stream>>>(tb, n_cand, pl.nblk, bits, p_star, m_out, k_star, mse);
            profile_mark(fast ? 5 : 1, stream);
            g_last_tiles = pl.n_tiles;
            g_last_groups = pl.n_groups;
            g_last_units = pl.n_tiles;
            g_last_search_kernel = "k_small";
            return launch_status("search launch");
        }
    }
    g_last_search_kernel = fast ? "k_fast" : "k_search";
    if (pl.n_mgroups > 0) k_tile_absmax<<<NT, kWG, 0, stream>>>(tb, tile_max);
    int longest = 0, longest_fast = 0, fast_tiles = 0;
    for (const TensorRec &r : pl.recs) {
        if (r.fast) { longest_fast = std::max(longest_fast, r.tile_len); fast_tiles += r.ntiles; }
        else longest = std::max(longest, r.tile_len);
    }
    if (fast_tiles > 0) {
        // tensors are ordered longest tile first, so the fast tiles are 0 .. fast_tiles-1
        static_assert(sizeof(double) * (kFastTMax + 1 + (kFastTMax >> kFastP2ShiftMax) + 1) +
                          sizeof(unsigned short) * (kFastTMax + 2) + sizeof(float) * (kTileMax + kFastWalkSq) <=
                      64 * 1024, "k_fast must fit the LDS a launch gets without asking for more");
        auto tcap_of = [](int longest_len) {
            int tcap = 64;
            while (tcap < kFastTMax && tcap <= 2 * longest_len) tcap <<= 1;
            return tcap;
        };
        auto lds_bytes = [&](int longest_len, int p2_shift) {
            const int tcap = tcap_of(longest_len);
            return sizeof(double) * (size_t)(tcap + 1 + (tcap >> p2_shift) + 1) +
                   sizeof(unsigned short) * (size_t)(tcap + 2) +
                   sizeof(float) * (size_t)(longest_len + kFastWalkSq);
        };
        // workgroups of a launch per CU: 160 KB of LDS (256 bytes of it static per workgroup),
        // 32 wavefront slots
        auto per_cu = [](size_t bytes) {
            return std::min((size_t)(32 / kFastWaves), (size_t)(160 * 1024) / (bytes + 256));
        };
        // A launch's LDS is sized for its longest tile.  When the longest tiles keep the others
        // from a fourth workgroup per CU, they get a launch of their own.
        int split = 0;          // tiles of the first launch; 0: one launch
        {
            int seen = 0, first_full = -1;
            for (const TensorRec &r : pl.recs) {
                if (!r.fast) break;
                if (first_full < 0 && per_cu(lds_bytes(r.tile_len, kFastP2ShiftMax)) >
                                          per_cu(lds_bytes(longest_fast, kFastP2ShiftMax)))
                    first_full = seen;
                seen += r.ntiles;
            }
            if (first_full >= 1024 && fast_tiles - first_full >= 1024) split = first_full;
        }
        profile_mark(4, stream);
        for (int part = 0; part < (split ? 2 : 1); ++part) {
            const int begin = part ? split : 0;
            const int count = split ? (part ? fast_tiles - split : split) : fast_tiles;
            int part_longest = 0, seen = 0;
            for (const TensorRec &r : pl.recs) {
                if (!r.fast) break;
                if (seen >= begin && seen < begin + count) part_longest = std::max(part_longest, r.tile_len);
                seen += r.ntiles;
            }
            // the finer prefix of squares shortens a walk; taken unless it costs a workgroup per CU
            int p2_shift = kFastP2ShiftMax;
            while (p2_shift > kFastP2ShiftMin && lds_bytes(part_longest, p2_shift - 1) <= 64 * 1024 &&
                   per_cu(lds_bytes(part_longest, p2_shift - 1)) == per_cu(lds_bytes(part_longest, kFastP2ShiftMax)))
                --p2_shift;
            k_fast<<<count, kFastWG, lds_bytes(part_longest, p2_shift), stream>>>(
                tb, begin, n_cand, bits, tcap_of(part_longest), p2_shift, tile_max, gm, sse32);
        }
        profile_mark(5, stream);
    }
    // tiles of at most kSmallTile elements (a suffix of the tile order) get one wavefront each
    int nt_large = 0, longest_small = 0;
    for (const TensorRec &r : pl.recs) {
        if (r.tile_len > kSmallTile) nt_large += r.ntiles;
        else if (!r.fast) longest_small = std::max(longest_small, r.tile_len);
    }
    if (NT - nt_large < 1024) nt_large = NT;     // too few short tiles to pay for launches of their own
    const int nt_small = NT - nt_large;
    if (fast_tiles < NT) {
        auto stage_bytes = [](int len) { return sizeof(float) * (size_t)((len + kVec - 1) / kVec * kVec); };
        const int nb2 = (pl.nblk + 1) / 2;
        const bool large = nt_large > 0 && (longest > kSmallTile || nt_small == 0);
        const bool small = nt_small > 0 && longest_small > 0;
        // long tiles are ordered by candidate (one bin per candidate and the switch
        // positions written out: worth it only where buckets can be long), short
        // ones by block of 64 candidates
        if (pl.fine) {
            if (large) {    // 512 threads x 16 elements: 256 x 32 measured 7-27 % slower, 1024 x 8 slower still
                if (longest <= 256 * 16)    // tiles of at most 4096 elements: smaller workgroups, twice as many in flight
                    k_prep<false, true, 256, 16><<<nt_large, 256, sizeof(int) * n_cand + stage_bytes(longest), stream>>>(
                        tb, 0, n_cand, pl.nblk, tile_max, gm, offsets, fine, sorted);
                else
                    k_prep<false, true, 512, 16><<<nt_large, 512, sizeof(int) * n_cand + stage_bytes(longest), stream>>>(
                        tb, 0, n_cand, pl.nblk, tile_max, gm, offsets, fine, sorted);
            }
            if (small)
                k_prep<true, false, 64, kSmallPer><<<nt_small, 64, sizeof(int) * nb2 * 64 + stage_bytes(longest_small), stream>>>(
                    tb, nt_large, n_cand, pl.nblk, tile_max, gm, offsets, fine, sorted);
        } else if (pl.nblk <= 32) {
            if (large)
                k_prep<true, false, kWG, kPerThread><<<nt_large, kWG, sizeof(int) * nb2 * kWG + stage_bytes(longest), stream>>>(
                    tb, 0, n_cand, pl.nblk, tile_max, gm, offsets, fine, sorted);
            if (small)
                k_prep<true, false, 64, kSmallPer><<<nt_small, 64, sizeof(int) * nb2 * 64 + stage_bytes(longest_small), stream>>>(
                    tb, nt_large, n_cand, pl.nblk, tile_max, gm, offsets, fine, sorted);
        } else {
            if (large)
                k_prep<false, false, kWG, kPerThread><<<nt_large, kWG, sizeof(int) * pl.nblk + stage_bytes(longest), stream>>>(
                    tb, 0, n_cand, pl.nblk, tile_max, gm, offsets, fine, sorted);
            if (small)
                k_prep<false, false, 64, kSmallPer><<<nt_small, 64, sizeof(int) * pl.nblk + stage_bytes(longest_small), stream>>>(
                    tb, nt_large, n_cand, pl.nblk, tile_max, gm, offsets, fine, sorted);
        }
        profile_mark(0, stream);
        k_search<<<(unsigned)wgs, kSearchWaves * 64, 0, stream>>>(tb, n_cand, pl.nblk, bits, ny, upw, bpw_log2,
                                                    offsets, sorted, fine, pl.fine ? nt_large : 0, sse32);
        profile_mark(1, stream);
    }
    if (pl.n_mgroups > 0) {
        k_group_sum<<<(unsigned)group_sum_wgs, kWG, 0, stream>>>(tb, n_cand, sse32, gsum);
        k_flag<<<(int)pl.n_mgroups, kWG, 0, stream>>>(tb, n_cand, gm, gsum, klist);
    }
    // Single-tile groups only: the short tiles above 512 elements (next in the tile order) join
    // the two-wavefront launch, so that the one-wavefront launch holds 8 elements per thread
    // instead of 16 and fits six wavefronts per SIMD like the other.
    int nt_mid = 0;
    if (pl.n_mgroups == 0 && nt_large > 0 && nt_small > 0)
        for (const TensorRec &r : pl.recs)
            if (r.tile_len <= kSmallTile && r.tile_len > 512) nt_mid += r.ntiles;
    if (nt_large > 0) {
        // single-tile groups only: workgroups of two wavefronts, twice as many in flight (the
        // stage is bound by latency); with groups spread over tiles, where a tile's threads
        // share the evaluation of the group's whole list, four wavefronts measured faster
        if (pl.n_mgroups == 0)
            k_exact<128><<<nt_large + nt_mid, 128, 0, stream>>>(tb, 0, n_cand, bits, gm, sse32, klist, part64,
                                                                p_star, m_out, k_star, mse);
        else
            k_exact<kWG><<<nt_large, kWG, 0, stream>>>(tb, 0, n_cand, bits, gm, sse32, klist, part64, p_star,
                                                       m_out, k_star, mse);
    }
    if (nt_small > 0) {
        if (nt_mid > 0) {
            if (nt_small > nt_mid)
                k_exact<64, 8><<<nt_small - nt_mid, 64, 0, stream>>>(tb, nt_large + nt_mid, n_cand, bits, gm, sse32,
                                                                      klist, part64, p_star, m_out, k_star, mse);
        } else {
            k_exact<64><<<nt_small, 64, 0, stream>>>(tb, nt_large, n_cand, bits, gm, sse32, klist, part64,
                                                     p_star, m_out, k_star, mse);
        }
    }
    if (pl.n_mgroups > 0)
        k_final<<<(int)pl.n_mgroups, kWG, 0, stream>>>(tb, n_cand, gm, klist, part64, p_star, m_out,
                                                       k_star, mse);
    g_last_tiles = pl.n_tiles;
    g_last_groups = pl.n_groups;
    g_last_units = pl.n_units;
    return launch_status("search launch");
}

int run_quantize(const pwlq_tensor_desc *desc, int n_tensors, int bits, int mode,
                 const float *p_star, const float *m, uint8_t *codes, uint8_t *flags, float *w_hat,
                 void *workspace, size_t workspace_bytes, void *stream_v)
{
    int rc = check_common(bits, mode);
    if (rc) return rc;
    if (!p_star || !m || !codes || !flags || !w_hat)
        return fail(PWLQ_ENULL, "an input or output pointer is NULL");
    Plan pl;
    rc = build_plan(pl, desc, n_tensors, 0, mode, true);
    if (rc) return rc;
    if (pl.nt > 1) {
        rc = check_workspace(pl, workspace, workspace_bytes);
        if (rc) return rc;
    }
    hipStream_t stream = (hipStream_t)stream_v;
    Tables tb;
    static_assert(sizeof(Tables) + sizeof(EmitArgs) + 64 <= 4096, "a launch passes at most 4 KB");
    EmitArgs ea;
    if (fill_emit_args(pl, ea)) {          // the table travels with the launch
        memset(&tb, 0, sizeof(tb));
        tb.nt = pl.nt;
    } else {
        rc = upload_tables(pl, (char *)workspace, stream, tb);
        if (rc) return rc;
    }
    profile_mark(2, stream);
    k_emit<<<(int)pl.n_chunks, kWG, 0, stream>>>(tb, ea, bits, p_star, m, codes, flags, w_hat);
    profile_mark(3, stream);
    return launch_status("quantize launch");
}

int run_quantize_packed(const pwlq_tensor_desc *desc, int n_tensors, int bits, int mode,
                        const float *p_star, const float *m, uint8_t *packed_codes,
                        const int64_t *code_byte_offset, uint8_t *packed_flags,
                        const int64_t *flag_byte_offset, float *w_hat, void *workspace,
                        size_t workspace_bytes, void *stream_v)
{
    int rc = check_common(bits, mode);
    if (rc) return rc;
    if (!p_star || !m || !packed_codes || !packed_flags)
        return fail(PWLQ_ENULL, "an input or output pointer is NULL");
    if (n_tensors > 1 && (!code_byte_offset || !flag_byte_offset))
        return fail(PWLQ_ENULL, "byte offset tables are NULL");
    Plan pl;
    rc = build_plan(pl, desc, n_tensors, 0, mode, true, code_byte_offset, flag_byte_offset);
    if (rc) return rc;
    if (pl.nt > 1) {
        rc = check_workspace(pl, workspace, workspace_bytes);
        if (rc) return rc;
    }
    hipStream_t stream = (hipStream_t)stream_v;
    Tables tb;
    EmitArgs ea;
    if (fill_emit_args(pl, ea)) {
        memset(&tb, 0, sizeof(tb));
        tb.nt = pl.nt;
    } else {
        rc = upload_tables(pl, (char *)workspace, stream, tb);
        if (rc) return rc;
    }
#define PWLQ_PACKED_CASE(B)                                                                        \
    case B:                                                                                        \
        if (w_hat)                                                                                 \
            k_emit_packed<B, 8><<<(int)pl.n_chunks, kEmitChunk / 8, 0, stream>>>(                  \
                tb, ea, p_star, m, packed_codes, packed_flags, w_hat);                             \
        else                                                                                       \
            k_emit_packed<B, 16><<<(int)pl.n_chunks, kEmitChunk / 16, 0, stream>>>(                \
                tb, ea, p_star, m, packed_codes, packed_flags, w_hat);                             \
        break;
    switch (bits) {
        PWLQ_PACKED_CASE(2)
        PWLQ_PACKED_CASE(3)
        PWLQ_PACKED_CASE(4)
        PWLQ_PACKED_CASE(5)
        PWLQ_PACKED_CASE(6)
        PWLQ_PACKED_CASE(7)
        PWLQ_PACKED_CASE(8)
    }
#undef PWLQ_PACKED_CASE
    return launch_status("packed quantize launch");
}

int run_select(const pwlq_tensor_desc *desc, int n_tensors, int mode, int selector, float *p_out,
               float *m_out, void *workspace, size_t workspace_bytes, void *stream_v)
{
    int rc = check_common(2, mode);
    if (rc) return rc;
    if (selector < PWLQ_SELECT_GAUSS_FIT || selector > PWLQ_SELECT_LAPLACE_SOLVE)
        return fail(PWLQ_EINVAL, "selector=%d is not a pwlq_selector", selector);
    if (!p_out || !m_out) return fail(PWLQ_ENULL, "an output pointer is NULL");
    Plan pl;
    rc = build_plan(pl, desc, n_tensors, 0, mode, true, nullptr, nullptr, kAuxStats);
    if (rc) return rc;
    rc = check_workspace(pl, workspace, workspace_bytes);
    if (rc) return rc;
    hipStream_t stream = (hipStream_t)stream_v;
    char *ws = (char *)workspace;
    Tables tb;
    rc = upload_tables(pl, ws, stream, tb);
    if (rc) return rc;
    float *tile_max = (float *)(ws + pl.off_stat_max);
    double *tile_s2 = (double *)(ws + pl.off_stat_s2);
    double *tile_s1 = (double *)(ws + pl.off_stat_s1);
    k_stats<<<(int)((pl.n_tiles + kWaves - 1) / kWaves), kWG, 0, stream>>>(tb, (int)pl.n_tiles, tile_max, tile_s2,
                                                                      tile_s1);
    k_select<<<(int)((pl.n_groups + kSelectWG - 1) / kSelectWG), kSelectWG, 0, stream>>>(
        tb, (int)pl.n_groups, selector, tile_max, tile_s2, tile_s1, p_out, m_out);
    return launch_status("select launch");
}

int run_mse(const pwlq_tensor_desc *desc, int n_tensors, int bits, int mode, const float *p,
            const float *m, double *mse, void *workspace, size_t workspace_bytes, void *stream_v)
{
    int rc = check_common(bits, mode);
    if (rc) return rc;
    if (!p || !m || !mse) return fail(PWLQ_ENULL, "an input or output pointer is NULL");
    Plan pl;
    rc = build_plan(pl, desc, n_tensors, 0, mode, true, nullptr, nullptr, kAuxMse);
    if (rc) return rc;
    rc = check_workspace(pl, workspace, workspace_bytes);
    if (rc) return rc;
    hipStream_t stream = (hipStream_t)stream_v;
    char *ws = (char *)workspace;
    Tables tb;
    rc = upload_tables(pl, ws, stream, tb);
    if (rc) return rc;
    double *tile_sse = (double *)(ws + pl.off_stat_s2);
    k_mse_tile<<<(int)((pl.n_tiles + kWaves - 1) / kWaves), kWG, 0, stream>>>(tb, (int)pl.n_tiles, bits, p, m,
                                                                         tile_sse);
    k_mse_final<<<(int)((pl.n_groups + kWG - 1) / kWG), kWG, 0, stream>>>(tb, (int)pl.n_groups,
                                                                        tile_sse, mse);
    return launch_status("mse launch");
}

int run_linear(const int8_t *xq, int64_t M, int64_t K, float s_x, float z_x,
               const uint8_t *packed_codes, const uint8_t *packed_flags, int64_t N, int bits,
               const float *p, const float *m, float *y, int32_t *acc, void *workspace,
               size_t workspace_bytes, void *stream_v)
{
    int rc = check_common(bits, PWLQ_PER_CHANNEL);
    if (rc) return rc;
    if (!xq || !packed_codes || !packed_flags || !p || !m || !y)
        return fail(PWLQ_ENULL, "an input or output pointer is NULL");
    if (M < 1 || N < 1 || K < 1) return fail(PWLQ_EINVAL, "M=%lld N=%lld K=%lld must be >= 1",
                                             (long long)M, (long long)N, (long long)K);
    if (K % 16 != 0) return fail(PWLQ_EINVAL, "K=%lld is not a multiple of 16", (long long)K);
    if (M > (1LL << 31) / 4 || N > (1LL << 31) / 4 || K > (1LL << 22))
        return fail(PWLQ_EINVAL, "matrix too large");
    if ((((uintptr_t)xq) | ((uintptr_t)packed_codes)) & 15)
        return fail(PWLQ_EINVAL, "xq and packed_codes must be 16-byte aligned");
    if (((uintptr_t)packed_flags) & 1) return fail(PWLQ_EINVAL, "packed_flags must be 2-byte aligned");
    const size_t need = align_up(sizeof(float) * (size_t)N, 256);
    if (!workspace) return fail(PWLQ_EWORKSPACE, "workspace is NULL (%zu bytes needed)", need);
    if (((uintptr_t)workspace & 255) != 0) return fail(PWLQ_EWORKSPACE, "workspace is not 256-byte aligned");
    if (workspace_bytes < need)
        return fail(PWLQ_EWORKSPACE, "workspace holds %zu bytes, %zu needed", workspace_bytes, need);
    // the three sums apart only when the caller asks for them; else the folded form
    const int planes = acc ? 3 : 2;
    const long long tiles_m = (M + lin_bm(planes) - 1) / lin_bm(planes), tiles_n = (N + kLinBN - 1) / kLinBN;
    const long long tn_per_xcd = (tiles_n + 7) / 8;
    const long long wgs = 8 * tn_per_xcd * tiles_m;
    if (wgs > 0x7fffffffLL) return fail(PWLQ_EINVAL, "grid too large");
    hipStream_t stream = (hipStream_t)stream_v;
    float *wconst = (float *)workspace;
    const unsigned wsum_wgs = (unsigned)((N + kLinWG / 64 - 1) / (kLinWG / 64));
#define PWLQ_LINEAR_CASE(B)                                                                       \
    case B:                                                                                        \
        k_linear_wsum<B><<<wsum_wgs, kLinWG, 0, stream>>>(packed_codes, packed_flags, N, K, p, m,  \
                                                          wconst);                                 \
        profile_mark(6, stream);                                                                   \
        if (planes == 3)                                                                           \
            k_linear<B, 3><<<(unsigned)wgs, kLinWG, 0, stream>>>(                                  \
                xq, M, K, s_x, z_x, packed_codes, packed_flags, N, p, m, wconst, y, acc,           \
                (int)tiles_m, (int)tiles_n, (int)tn_per_xcd);                                      \
        else                                                                                       \
            k_linear<B, 2><<<(unsigned)wgs, kLinWG, 0, stream>>>(                                  \
                xq, M, K, s_x, z_x, packed_codes, packed_flags, N, p, m, wconst, y, nullptr,       \
                (int)tiles_m, (int)tiles_n, (int)tn_per_xcd);                                      \
        profile_mark(7, stream);                                                                   \
        break;
    switch (bits) {
        PWLQ_LINEAR_CASE(2)
        PWLQ_LINEAR_CASE(3)
        PWLQ_LINEAR_CASE(4)
        PWLQ_LINEAR_CASE(5)
        PWLQ_LINEAR_CASE(6)
        PWLQ_LINEAR_CASE(7)
        PWLQ_LINEAR_CASE(8)
    }
#undef PWLQ_LINEAR_CASE
    return launch_status("linear launch");
}

// Device address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(PWLQ_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(PWLQ_EHIP, "device index %d not supported", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(PWLQ_EHIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev,
                        hipGetErrorString(e));
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return PWLQ_OK;
}

} // namespace

extern "C" {

int pwlq_search_static(const float *w, int64_t C, int64_t K, int bits, int n_cand, int mode,
                       float *p_star, float *m_out, int32_t *k_star, double *mse, void *stream)
{
    if (!w) return fail(PWLQ_ENULL, "w is NULL");
    int rc = check_common(bits, mode);
    if (rc) return rc;
    if (n_cand < 1 || n_cand > 65535) return fail(PWLQ_EINVAL, "n_cand=%d outside [1,65535]", n_cand);
    pwlq_tensor_desc d = {w, C, K, 0, 0};
    Plan pl;
    rc = build_plan(pl, &d, 1, n_cand, mode, true);
    if (rc) return rc;
    if (pl.total > (size_t)PWLQ_STATIC_SCRATCH_BYTES)
        return fail(PWLQ_EWORKSPACE,
                    "this search needs %zu bytes of scratch, the library's static buffer holds %zu: "
                    "call pwlq_search with a workspace of the caller's",
                    pl.total, (size_t)PWLQ_STATIC_SCRATCH_BYTES);
    void *ptr = nullptr;
    rc = static_scratch(&ptr);
    if (rc) return rc;
    return run_search(&d, 1, bits, n_cand, mode, p_star, m_out, k_star, mse, ptr,
                      (size_t)PWLQ_STATIC_SCRATCH_BYTES, stream);
}

size_t pwlq_linear_workspace_bytes(int64_t N)
{
    if (N < 1) return 0;
    return align_up(sizeof(float) * (size_t)N, 256);
}

int pwlq_linear_i8(const int8_t *xq, int64_t M, int64_t K, float s_x, float z_x,
                   const uint8_t *packed_codes, const uint8_t *packed_flags, int64_t N, int bits,
                   const float *p, const float *m, float *y, int32_t *acc, void *workspace,
                   size_t workspace_bytes, void *stream)
{
    return run_linear(xq, M, K, s_x, z_x, packed_codes, packed_flags, N, bits, p, m, y, acc,
                      workspace, workspace_bytes, stream);
}

size_t pwlq_select_list_workspace_bytes(const pwlq_tensor_desc *desc, int n_tensors, int mode)
{
    if (check_common(2, mode)) return 0;
    Plan pl;
    if (build_plan(pl, desc, n_tensors, 0, mode, false, nullptr, nullptr, kAuxStats)) return 0;
    return pl.total;
}

size_t pwlq_select_workspace_bytes(int64_t C, int64_t K, int mode)
{
    pwlq_tensor_desc d = {nullptr, C, K, 0, 0};
    return pwlq_select_list_workspace_bytes(&d, 1, mode);
}

int pwlq_select_analytic_list(const pwlq_tensor_desc *desc, int n_tensors, int mode, int selector,
                              float *p_out, float *m_out, void *workspace, size_t workspace_bytes,
                              void *stream)
{
    return run_select(desc, n_tensors, mode, selector, p_out, m_out, workspace, workspace_bytes,
                      stream);
}

int pwlq_select_analytic(const float *w, int64_t C, int64_t K, int mode, int selector,
                         float *p_out, float *m_out, void *workspace, size_t workspace_bytes,
                         void *stream)
{
    if (!w) return fail(PWLQ_ENULL, "w is NULL");
    pwlq_tensor_desc d = {w, C, K, 0, 0};
    return run_select(&d, 1, mode, selector, p_out, m_out, workspace, workspace_bytes, stream);
}

size_t pwlq_mse_list_workspace_bytes(const pwlq_tensor_desc *desc, int n_tensors, int mode)
{
    if (check_common(2, mode)) return 0;
    Plan pl;
    if (build_plan(pl, desc, n_tensors, 0, mode, false, nullptr, nullptr, kAuxMse)) return 0;
    return pl.total;
}

size_t pwlq_mse_workspace_bytes(int64_t C, int64_t K, int mode)
{
    pwlq_tensor_desc d = {nullptr, C, K, 0, 0};
    return pwlq_mse_list_workspace_bytes(&d, 1, mode);
}

int pwlq_mse_list(const pwlq_tensor_desc *desc, int n_tensors, int bits, int mode, const float *p,
                  const float *m, double *mse, void *workspace, size_t workspace_bytes,
                  void *stream)
{
    return run_mse(desc, n_tensors, bits, mode, p, m, mse, workspace, workspace_bytes, stream);
}

int pwlq_mse(const float *w, int64_t C, int64_t K, int bits, int mode, const float *p,
             const float *m, double *mse, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!w) return fail(PWLQ_ENULL, "w is NULL");
    pwlq_tensor_desc d = {w, C, K, 0, 0};
    return run_mse(&d, 1, bits, mode, p, m, mse, workspace, workspace_bytes, stream);
}

size_t pwlq_search_list_workspace_bytes(const pwlq_tensor_desc *desc, int n_tensors, int bits,
                                        int n_cand, int mode)
{
    if (check_common(bits, mode) || n_cand < 1 || n_cand > 65535) return 0;
    Plan pl;
    if (build_plan(pl, desc, n_tensors, n_cand, mode, false)) return 0;
    return pl.total;
}

size_t pwlq_search_workspace_bytes(int64_t C, int64_t K, int bits, int n_cand, int mode)
{
    pwlq_tensor_desc d = {nullptr, C, K, 0, 0};
    return pwlq_search_list_workspace_bytes(&d, 1, bits, n_cand, mode);
}

int pwlq_search_list(const pwlq_tensor_desc *desc, int n_tensors, int bits, int n_cand, int mode,
                     float *p_star, float *m_out, int32_t *k_star, double *mse, void *workspace,
                     size_t workspace_bytes, void *stream)
{
    return run_search(desc, n_tensors, bits, n_cand, mode, p_star, m_out, k_star, mse, workspace,
                      workspace_bytes, stream);
}

int pwlq_search(const float *w, int64_t C, int64_t K, int bits, int n_cand, int mode,
                float *p_star, float *m_out, int32_t *k_star, double *mse, void *workspace,
                size_t workspace_bytes, void *stream)
{
    if (!w) return fail(PWLQ_ENULL, "w is NULL");
    pwlq_tensor_desc d = {w, C, K, 0, 0};
    return run_search(&d, 1, bits, n_cand, mode, p_star, m_out, k_star, mse, workspace,
                      workspace_bytes, stream);
}

int pwlq_search_fast_list(const pwlq_tensor_desc *desc, int n_tensors, int bits, int n_cand,
                          int mode, float *p_star, float *m_out, int32_t *k_star, double *mse,
                          void *workspace, size_t workspace_bytes, void *stream)
{
    return run_search(desc, n_tensors, bits, n_cand, mode, p_star, m_out, k_star, mse, workspace,
                      workspace_bytes, stream, true);
}

int pwlq_search_fast(const float *w, int64_t C, int64_t K, int bits, int n_cand, int mode,
                     float *p_star, float *m_out, int32_t *k_star, double *mse, void *workspace,
                     size_t workspace_bytes, void *stream)
{
    if (!w) return fail(PWLQ_ENULL, "w is NULL");
    pwlq_tensor_desc d = {w, C, K, 0, 0};
    return run_search(&d, 1, bits, n_cand, mode, p_star, m_out, k_star, mse, workspace,
                      workspace_bytes, stream, true);
}

size_t pwlq_quantize_list_workspace_bytes(const pwlq_tensor_desc *desc, int n_tensors, int bits,
                                          int mode)
{
    if (check_common(bits, mode)) return 0;
    Plan pl;
    if (build_plan(pl, desc, n_tensors, 0, mode, false)) return 0;
    return pl.total;
}

int pwlq_quantize_list(const pwlq_tensor_desc *desc, int n_tensors, int bits, int mode,
                       const float *p_star, const float *m, uint8_t *codes, uint8_t *flags,
                       float *w_hat, void *workspace, size_t workspace_bytes, void *stream)
{
    return run_quantize(desc, n_tensors, bits, mode, p_star, m, codes, flags, w_hat, workspace,
                        workspace_bytes, stream);
}

int pwlq_quantize(const float *w, int64_t C, int64_t K, int bits, int mode, const float *p_star,
                  const float *m, uint8_t *codes, uint8_t *flags, float *w_hat, void *stream)
{
    if (!w) return fail(PWLQ_ENULL, "w is NULL");
    pwlq_tensor_desc d = {w, C, K, 0, 0};
    return run_quantize(&d, 1, bits, mode, p_star, m, codes, flags, w_hat, nullptr, 0, stream);
}

size_t pwlq_packed_code_bytes(int64_t count, int bits)
{
    if (count < 0 || bits < 2 || bits > 8) return 0;
    return (size_t)((count * bits + 7) / 8);
}

size_t pwlq_packed_flag_bytes(int64_t count) { return count < 0 ? 0 : (size_t)((count + 7) / 8); }

int pwlq_quantize_packed(const float *w, int64_t C, int64_t K, int bits, int mode,
                         const float *p_star, const float *m, uint8_t *packed_codes,
                         uint8_t *packed_flags, float *w_hat, void *stream)
{
    if (!w) return fail(PWLQ_ENULL, "w is NULL");
    pwlq_tensor_desc d = {w, C, K, 0, 0};
    return run_quantize_packed(&d, 1, bits, mode, p_star, m, packed_codes, nullptr, packed_flags,
                               nullptr, w_hat, nullptr, 0, stream);
}

int pwlq_quantize_packed_list(const pwlq_tensor_desc *desc, int n_tensors, int bits, int mode,
                              const float *p_star, const float *m, uint8_t *packed_codes,
                              const int64_t *code_byte_offset, uint8_t *packed_flags,
                              const int64_t *flag_byte_offset, float *w_hat, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    return run_quantize_packed(desc, n_tensors, bits, mode, p_star, m, packed_codes,
                               code_byte_offset, packed_flags, flag_byte_offset, w_hat, workspace,
                               workspace_bytes, stream);
}

const char *pwlq_last_error(void) { return g_error; }

void pwlq_profile_enable(int roles)
{
    // the events are made here, on the first call that enables anything, so that no
    // call that launches kernels pays for them
    if (roles && !g_ev_made) {
        for (auto &role : g_ev)
            for (auto &slot : role)
                for (auto &ev : slot) (void)hipEventCreate(&ev);
        g_ev_made = true;
    }
    g_profile = (unsigned)roles & ((1u << kProfRoles) - 1u);
}

double pwlq_profile_ms(int role, int back)
{
    if (role < 0 || role >= kProfRoles || !g_ev_made) return -1.0;
    if (back < 0 || back >= kProfRing || back >= g_ev_count[role]) return -1.0;
    hipEvent_t *pair = g_ev[role][(g_ev_count[role] - 1 - back) % kProfRing];
    float ms = -1.0f;
    if (hipEventSynchronize(pair[1]) != hipSuccess) return -1.0;
    if (hipEventElapsedTime(&ms, pair[0], pair[1]) != hipSuccess) return -1.0;
    return (double)ms;
}

double pwlq_profile_last_ms(int role) { return pwlq_profile_ms(role, 0); }

void pwlq_last_search_shape(int64_t *n_tiles, int64_t *n_groups, int64_t *n_units)
{
    if (n_tiles) *n_tiles = g_last_tiles;
    if (n_groups) *n_groups = g_last_groups;
    if (n_units) *n_units = g_last_units;
}

int pwlq_set_small_call_tiles(int tiles)
{
    return small_call_tiles().exchange(tiles < 0 ? kSmallCallTiles : tiles);
}

const char *pwlq_last_search_kernel(void) { return g_last_search_kernel; }

const char *pwlq_kernel_name(int role)
{
    if (role == 0) return "k_search";
    if (role == 1) return "k_emit";
    if (role == 2) return "k_fast";
    if (role == 3) return "k_linear";
    return nullptr;
}

} // extern "C"
