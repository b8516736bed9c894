// Internal layout of a plan: host arrays written by the planner (plan.cpp) and the
// device copies read by the kernels (kernels.hip).  Not part of the public ABI.
#pragma once

#include <cstdint>
#include <vector>

#include "libra.h"

namespace libra {

// Device-side pointers of one sub-plan (all inside the caller's buffer).
struct SubPlanDev {
    const libra_task_t *tasks = nullptr;
    const int32_t *win_blkptr = nullptr;
    const int32_t *blk_cols = nullptr;
    const uint64_t *blk_bitmap = nullptr;
    const int32_t *blk_valptr = nullptr;
    void *dense_val = nullptr;
    const int32_t *dense_perm = nullptr;
    const int32_t *res_rowptr = nullptr;
    const int32_t *res_row = nullptr;
    const int32_t *res_col = nullptr;
    void *res_val = nullptr;
    const int32_t *res_perm = nullptr;
    const int32_t *zero_rows = nullptr;
};

struct SubPlan {
    std::vector<int32_t> win_blkptr, blk_cols, blk_valptr, dense_perm;
    std::vector<uint64_t> blk_bitmap;
    std::vector<uint8_t> dense_val, res_val;        // raw bytes, value dtype
    std::vector<int32_t> res_rowptr, res_row, res_col, res_perm, zero_rows;
    std::vector<libra_task_t> tasks;
    int64_t n_window_tasks = 0, n_chunk_tasks = 0;
    int64_t dense_vectors = 0, pad_slots = 0;
    int64_t short_rows = 0, long_rows = 0, split_rows = 0;
    SubPlanDev dev;
    int64_t n_blocks() const { return (int64_t)blk_valptr.size() - 1; }
};

struct Resolved {
    int mode, W, KB, tau_spmm, tau_sddmm, Ts, Cs, short_len, sddmm_Cs, threads;
    bool fill, build_spmm, build_sddmm, heavy_first;
};

}  // namespace libra

struct libra_plan_s {
    int64_t M = 0, Kc = 0, nnz = 0;
    int vdt = LIBRA_F16;
    int vsize = 2;
    libra::Resolved o{};
    std::vector<int32_t> rowptr;
    libra::SubPlan spmm, sddmm;
    libra_stats_t stats{};
    // device copy
    void *dev_base = nullptr;
    size_t dev_bytes = 0;
    const int32_t *d_rowptr = nullptr;
};
