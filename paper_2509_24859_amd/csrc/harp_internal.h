// Internal declarations shared by the host layer and the gfx950 kernels.  Not part of the ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "harp.h"

namespace harp {

constexpr int kMaxTp = HARP_MAX_TP_DEGREES;
constexpr int kMaxStages = 256;        // S_max accepted by plan/score
constexpr int kFastMaxL = 4096;        // 32-bit tables, the min-max planner and the exact search on them
constexpr int kFastRowsMaxL = 1024;    // 32-bit kernels that keep whole rows of several arrays in LDS: H-1F1B, submesh
constexpr size_t kFastCutTableLimit = size_t(256) << 20;
constexpr int64_t kInf = INT64_MAX;
constexpr int64_t kTimeLimit = int64_t(1) << 47;

// Device-side verdict of the table build, first bytes of the table buffer.
struct BuildHeader {
    unsigned int bad_arg;        // nonzero: malformed values
    unsigned int overflow;       // nonzero: magnitudes out of range
    unsigned int fast32;         // 1: 32-bit rows and cut table are valid
    unsigned int pad;
    unsigned long long max_act;  // largest act_bytes entry
    long long worst_time;        // largest stage or transfer time any plan can see
    long long total_devices;     // sum of group_ndev
    long long reserved[3];
};

// Everything a kernel needs to read the tables; passed by value.
struct TablesDev {
    int32_t L, T, G, M, n_tp, ar_count;
    int32_t tp[kMaxTp];
    int32_t tp_shift[kMaxTp];    // log2(tp) when tp is a power of two, else -1
    int64_t pitch;               // elements between int64 rows
    int64_t pitch32;             // elements between uint32 rows
    BuildHeader *header;
    int64_t *rows;               // PF rows, PP, PS, PR rows, consecutive
    int64_t *chunk_sums;         // scan scratch, [n_rows][n_chunks]
    int32_t *group_base;         // [G] first global device id of each group
    uint32_t *P32;               // [G*n_tp][pitch32]  PF[type g][i] + tp * PR[g][k][i]
    uint32_t *CM;                // [G*G][pitch32]     ceil(act_bytes[i-1] / bw[g][h]), 0 at i = 0
    const int64_t *fwd_us, *bwd_us, *param_bytes, *stash_bytes, *act_bytes;
    const int64_t *type_mem, *bw;
    const int32_t *group_type, *group_ndev;

    __host__ __device__ const int64_t *PF(int t) const { return rows + int64_t(t) * pitch; }
    __host__ __device__ const int64_t *PP() const { return rows + int64_t(T) * pitch; }
    __host__ __device__ const int64_t *PS() const { return rows + int64_t(T + 1) * pitch; }
    __host__ __device__ const int64_t *PR(int g, int k) const {
        return rows + (int64_t(T + 2) + int64_t(g) * n_tp + k) * pitch;
    }
    __host__ __device__ int n_rows() const { return T + 2 + G * n_tp; }
};

struct CandDev {
    int32_t C, S_max;
    const int32_t *cand_S, *cand_group, *cand_tp;
};

struct PlansDev {
    int32_t *splits, *dev_first;
    int64_t *bottleneck, *iter_time;
    int32_t *status;
};

// limits derived on the host for the magnitude guard (products that must stay inside int64; sums are
// checked where they are formed)
struct BuildLimits {
    int64_t act_max;    // act_bytes bound so that the all-reduce numerator fits
    int64_t bw_max;     // bandwidth bound so that tp * bw fits
    int64_t mem_max;    // device memory bound so that tp * mem fits
    int32_t want_fast;  // 1: the buffer has room for the 32-bit rows and the cut table
};

constexpr int kScanThreads = 256;
constexpr int kScanItems = 4;
constexpr int kScanChunk = kScanThreads * kScanItems;
constexpr int kLongL = 1 << 18;        // from here on the table build runs chunk-major, 256 operators per wavefront

void launch_build(const TablesDev &tb, const BuildLimits &lim, hipStream_t st);
void launch_plan_generic(const TablesDev &tb, const CandDev &cd, const PlansDev &out, void *ws,
                         int n_groups, bool banded, hipStream_t st);
void launch_plan_generic_exact(const TablesDev &tb, const CandDev &cd, const PlansDev &out, int32_t *n_passes,
                               void *ws, int n_groups, bool banded, hipStream_t st);
size_t plan_generic_ws_per_group(int L, int S_max);
void launch_plan_fast(const TablesDev &tb, const CandDev &cd, const PlansDev &out, void *ws,
                      int n_slices, int n_cu, unsigned long long *work, hipStream_t st);
void launch_plan_prepass(const TablesDev &tb, const CandDev &cd, void *ws, int n_groups, hipStream_t st);
void launch_plan_h1f1b(const TablesDev &tb, const CandDev &cd, const int64_t *t_max, const PlansDev &out,
                       int32_t *warmup, void *ws, int n_groups, int n_slices, int n_cu, hipStream_t st);
void launch_plan_generic_h1f1b(const TablesDev &tb, const CandDev &cd, const int64_t *t_max, const PlansDev &out,
                               int32_t *warmup, void *ws, int n_groups, bool banded, hipStream_t st);
size_t plan_generic_h1f1b_ws_per_group(int L, int S_max);
void launch_score_h1f1b(const TablesDev &tb, const CandDev &cd, const int32_t *splits, const int64_t *t_max,
                        int32_t *warmup, int64_t *bottleneck, int64_t *iter_time, int32_t *status,
                        hipStream_t st);
struct OrdDev {
    int32_t C, G_max, S_max;
    const int32_t *ord_S, *ord_G, *ord_group;
};
constexpr int kMaxOrderGroups = 1024;   // groups one ordering may list (their offsets sit in LDS)
void launch_plan_mesh(const TablesDev &tb, const OrdDev &od, const PlansDev &out, int32_t *stage_group,
                      int32_t *stage_tp, int32_t *n_passes, bool exact, bool fast32, void *ws, int n_groups,
                      int threads, int64_t total_devices, hipStream_t st);
void launch_plan_mesh_h1f1b(const TablesDev &tb, const OrdDev &od, const int64_t *t_max, const PlansDev &out,
                            int32_t *stage_group, int32_t *stage_tp, int32_t *warmup, bool fast32, void *ws,
                            int n_groups, int threads, int64_t total_devices, hipStream_t st);
void launch_plan_mesh_h1f1b_sweep(const TablesDev &tb, const OrdDev &od, const int32_t *cand_group,
                                  const int32_t *cand_tp, int max_caps, const PlansDev &out,
                                  int32_t *stage_group, int32_t *stage_tp, int32_t *warmup, int64_t *t_max_out,
                                  int32_t *n_caps, bool fast32, void *ws, int n_groups, int threads, int W_climb,
                                  int W, int64_t total_devices, hipStream_t st);
size_t plan_mesh_sweep_slot_bytes(int S_max);
size_t plan_mesh_ws_per_group(int L, int S_max, int64_t total_devices);
int plan_mesh_threads(int L, int64_t total_devices, int C, int n_cu);
size_t plan_fast_ws_bytes(const TablesDev &tb, int S_max, int C, int n_slices);
void launch_clear_work(unsigned long long *work, hipStream_t st);
size_t plan_fast_index_bytes(const TablesDev &tb, int S_max);
int plan_fast_groups(int L, int S_max, int n_cu);
int plan_fast_waves(int L, int S_max, int n_cu);
constexpr int kFastWaves = 4;           // wavefronts per workgroup of k2_fast; they share nothing
constexpr size_t kFastIndexLimit = size_t(256) << 20;   // feasibility index of the pre-pass
constexpr int kIndexMaxL = 16383;       // its build keeps one 8-byte sum per cut in LDS (128 KB)
void launch_plan_exact(const TablesDev &tb, const CandDev &cd, const PlansDev &out, int32_t *n_passes,
                       void *ws, int n_groups, int n_slices, int n_cu, hipStream_t st);
void launch_score(const TablesDev &tb, const CandDev &cd, const int32_t *splits,
                  int64_t *bottleneck, int64_t *iter_time, int32_t *status, bool fast32, int n_cu,
                  hipStream_t st);
void launch_valu_int32(int blocks, int iters, uint32_t *sink, hipStream_t st);
void launch_argmin(int32_t C, const int64_t *iter_time, const int32_t *status, int64_t *best_time,
                   int32_t *best_index, hipStream_t st);

}  // namespace harp
