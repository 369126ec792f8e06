// Pieces shared by the 32-bit planner kernels: the LDS row entry, the per-stage constants, scalar
// helpers, the LDS-only barrier, and the workspace layout the pre-pass and the DP kernels agree on.
#pragma once

#include "harp_internal.h"

namespace harp {
namespace fastdp {

constexpr uint32_t kInf32 = 0xFFFFFFFFu;
constexpr int kPad = 4;
constexpr int kFastThreads = 256;
constexpr uint32_t kRowMask = (1u << 27) - 1u;
constexpr uint32_t kDeadStatusShift = 30;   // dead-list entry: candidate | status << 30

struct alignas(8) Pair {
    uint32_t d;   // previous DP row
    uint32_t p;   // fused time row of the stage's slot
};

// Workgroup barrier that orders LDS traffic only.  Global loads and stores stay in flight across
// it (the stage loop never communicates through global memory), which keeps the round trips of the
// back-pointer stores and of the next stage's table rows off the per-stage critical path.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ uint32_t umax3(uint32_t a, uint32_t b, uint32_t c) {
    uint32_t m = a > b ? a : b;
    return m > c ? m : c;
}

// A value every lane of the wave holds, moved to a scalar register.
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int64_t uniform64(int64_t v) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}
template <typename T>
__device__ __forceinline__ const T *uniform_ptr(const T *p) {
    return reinterpret_cast<const T *>(uniform64(reinterpret_cast<int64_t>(p)));
}

// Per-slot constants of the candidate in flight, computed once per candidate so that the stage
// loop starts from LDS and never waits on a chain of dependent global loads.
// Rows are named by element offsets from the table bases, not by pointers: a pointer read back
// from LDS has no known address space and would turn every table access into a flat load.
struct alignas(16) StageConst {
    int64_t cap;            // tp * device memory of the slot's GPU type
    uint32_t p_row;         // element offset of the slot's fused time row in P32
    uint32_t cm_row_shift;  // element offset of the link's cut-time row in CM (low 27 bits) | log2 tp << 27
};
static_assert(sizeof(StageConst) == 16, "one 16-byte LDS read per stage");
static_assert(kFastCutTableLimit / 4 <= (size_t(1) << 27), "cut-table offsets must fit 27 bits");

__device__ __forceinline__ int band_lo(uint32_t w) { return int(w & 0xFFFFu); }
__device__ __forceinline__ int band_hi(uint32_t w) { return int(w >> 16); }

__device__ __forceinline__ int tp_index(const TablesDev &tb, int tp) {
    int k = -1;
    for (int q = 0; q < tb.n_tp; ++q)
        if (tb.tp[q] == tp) k = q;
    return k;
}

inline int fast_row_len(int L) { return (L + 1 + kPad + 7) / 8 * 8; }

inline size_t fast_lds_bytes(int L, int S_max) {
    size_t b = size_t(fast_row_len(L)) * 32 + size_t(S_max) * sizeof(StageConst) +
               size_t(S_max + 2) * 4 + size_t(S_max) * 3;
    return (b + 15) & ~size_t(15);
}

// Back-pointer slice of one wavefront (k2_fast) or workgroup (the kernels built on it): a 16-bit
// entry per DP cell, followed by the one-byte entries k2_fast uses for cells whose back-pointers
// leave LDS (distance to the previous cut; the 16-bit entry holds the cut itself when the distance
// does not fit a byte).
inline size_t fast_arg_u16_bytes(int L, int S_max) {
    size_t b = size_t(S_max) * fast_row_len(L) * sizeof(uint16_t);
    return (b + 255) & ~size_t(255);
}
inline size_t fast_arg_per_group(int L, int S_max) {
    size_t b = size_t(S_max) * fast_row_len(L);
    return fast_arg_u16_bytes(L, S_max) + ((b + 255) & ~size_t(255));
}

// Rows of the feasibility index (see k2_fast.hip): one per in-flight count n = 1 .. n_max, GPU type and
// degree index.  Two tables of that many rows, one after the other: entry i of a row of the first
// is the lowest previous cut j such that operators [j, i) fit, entry j of a row of the second the
// highest cut i such that they do.
inline int lo_n_max(int L, int S_max, int M) {
    int n = S_max < M ? S_max : M;
    return n < L ? n : L;
}
inline size_t lo_pitch(int L) { return (size_t(L) + 1 + 31) & ~size_t(31); }
inline size_t lo_table_bytes(int L, int S_max, int M, int T, int n_tp) {
    return 2 * size_t(lo_n_max(L, S_max, M)) * size_t(T) * size_t(n_tp) * lo_pitch(L) * sizeof(uint16_t);
}

// Workspace: counters | live list [C] | dead list [C] | bands [C][S_max+1] | feasibility index |
// back-pointer slices (one per resident wavefront of k2_fast, one per workgroup of the other kernels).
struct FastWorkspace {
    int *counts;
    int32_t *live_list;
    uint32_t *dead_list;
    uint32_t *bands;
    uint16_t *lo_tab;
    unsigned char *arg;
    size_t total;
};

struct FastShape {
    int L, S_max, C, M, T, n_tp;
};

inline FastShape fast_shape(const TablesDev &tb, const CandDev &cd) {
    return FastShape{tb.L, cd.S_max, cd.C, tb.M, tb.T, tb.n_tp};
}

inline FastWorkspace carve(void *ws, const FastShape &f, int n_slices) {
    auto up = [](size_t x) { return (x + 255) & ~size_t(255); };
    unsigned char *base = static_cast<unsigned char *>(ws);
    FastWorkspace w;
    size_t off = 0;
    w.counts = reinterpret_cast<int *>(base + off); off += 256;
    w.live_list = reinterpret_cast<int32_t *>(base + off); off += up(size_t(f.C) * 4);
    w.dead_list = reinterpret_cast<uint32_t *>(base + off); off += up(size_t(f.C) * 4);
    w.bands = reinterpret_cast<uint32_t *>(base + off); off += up(size_t(f.C) * (f.S_max + 1) * 4);
    w.lo_tab = reinterpret_cast<uint16_t *>(base + off); off += up(lo_table_bytes(f.L, f.S_max, f.M, f.T, f.n_tp));
    w.arg = base + off; off += size_t(n_slices) * fast_arg_per_group(f.L, f.S_max);
    w.total = off;
    return w;
}

}  // namespace fastdp
}  // namespace harp
