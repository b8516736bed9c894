// Internal layout of a plan: host arrays written by the planner (plan.cpp) and the
// device copies read by the kernels (kernels.hip).  Not part of the public ABI.
#pragma once

#include <cstdint>
#include <functional>
#include <vector>

#include "libra.h"

#ifdef __HIPCC__
#define LIBRA_HD __host__ __device__
#else
#define LIBRA_HD
#endif

#define LIBRA_SOFTMAX_LONG_ROW 2048
#define LIBRA_XCDS 8                 // accelerator dies of an MI355X; workgroup k runs on die k mod 8
#define LIBRA_LOCALITY_WINDOWS 4     // neighbouring windows whose tasks are kept on one die (XCD-aware order)
#define LIBRA_LOCALITY_SEGMENTS 8    // consecutive SDDMM residual segments kept on one die
#define LIBRA_SHARE_THRESHOLD 0.67   // die-aware order when 4 neighbouring windows together have at most this share of their separate columns

namespace libra {

// Task record as the kernels read it (32 bytes).  SpMM: a decomposed-row segment is stored
// as a window task without blocks whose only output row is the atomic one.
struct DevTask {
    int32_t id;                 // window index
    int32_t blk_begin, blk_end; // dense blocks
    int32_t res_begin, res_end; // residual entries
    uint32_t masks;             // SpMM: atomic_mask | store_mask << 16
    uint32_t kind;
    int32_t val_begin;          // first packed value of block blk_begin
};

// Residual entries of the SpMM sub-plan: blocks of RES_BLOCK entries, each block RES_BLOCK 32-bit words (column in the
// low RES_ROW_SHIFT bits, row inside the window above them) followed by RES_BLOCK values of the storage type: 384 bytes
// with 16-bit values, 512 with fp32.  Entry i is slot i % RES_BLOCK of block i / RES_BLOCK, so a task's entries are
// addressed from their index alone, a task reads words and values from neighbouring lines, and new values overwrite
// whole 128-byte runs.  A plan on the device is therefore limited to 2^27 columns.
constexpr int RES_BLOCK = 64;
constexpr int RES_ROW_SHIFT = 27;                               // windows of up to 32 rows
constexpr uint32_t RES_COL_MASK = (1u << RES_ROW_SHIFT) - 1u;
inline size_t res_block_bytes(size_t value_bytes) { return RES_BLOCK * (4 + value_bytes); }
inline size_t res_blocked_bytes(size_t n, size_t value_bytes) { return (n + RES_BLOCK - 1) / RES_BLOCK * res_block_bytes(value_bytes); }
// Residual entry of the SDDMM sub-plan: 16 bytes.
struct SdEnt {
    int32_t row, col, perm;
    uint32_t val;               // fp16 bits in the low half, or fp32 bits
};

// Packed dense nonzero of the SDDMM sub-plan: where the result goes and the value that scales it.
struct SdPv {
    int32_t perm;
    uint32_t val;               // fp16 bits in the low half
};

// Device-side pointers of one sub-plan (all inside the caller's buffer).
struct SubPlanDev {
    const DevTask *tasks = nullptr;
    const int32_t *blk_cols = nullptr;
    const uint64_t *blk_bitmap = nullptr;
    const int32_t *blk_valptr = nullptr;
    void *dense_val = nullptr;          // SpMM: packed values in bit order
    void *dense_pv = nullptr;           // SDDMM: SdPv per packed value
    const int32_t *dense_perm = nullptr;
    void *res_ent = nullptr;            // SpMM: blocked words and values (see RES_BLOCK); SDDMM: SdEnt per entry
    const int32_t *res_perm = nullptr;
    const int32_t *zero_rows = nullptr;
};

// Sizes of a sub-plan's arrays.  Set by finish_plan from the host vectors, or by the device planner when the
// arrays only exist in device memory.
struct Counts {
    int64_t blocks = 0, col_slots = 0, bitmap_words = 0, dense = 0, res = 0, zero_rows = 0, tasks = 0;
};

// Where the device planner left a sub-plan's arrays (host planner's format, device memory).
struct DeviceSource {
    const int32_t *blk_cols, *blk_valptr, *dense_perm, *res_perm, *res_row, *res_col, *zero_rows;
    const uint64_t *blk_bitmap;
    const void *dense_val, *res_val;
};

struct SubPlan {
    Counts n;
    std::vector<int32_t> win_blkptr, blk_cols, blk_valptr, dense_perm;
    std::vector<uint64_t> blk_bitmap;
    std::vector<uint8_t> dense_val, res_val;        // raw bytes, value dtype
    std::vector<int32_t> win_resptr, res_row, res_col, res_perm, zero_rows;
    std::vector<libra_task_t> tasks;
    std::vector<int32_t> task_col;      // SpMM, until the tables are ordered: first column of a row segment's entries, -1 for other tasks
    std::vector<int32_t> seg_col;       // SDDMM, until the tables are ordered: per flat residual segment, its first column if all its
                                        // nonzeros lie in one row, else -1 (the device planner fills it; the host planner derives it)
    int64_t n_window_tasks = 0, n_chunk_tasks = 0;
    int64_t dense_vectors = 0, pad_slots = 0;
    int64_t short_rows = 0, long_rows = 0, split_rows = 0;
    SubPlanDev dev;
    int64_t n_blocks() const { return (int64_t)blk_valptr.size() - 1; }     // while the host planner appends
    void count_host_arrays() {
        n.blocks = blk_valptr.empty() ? 0 : (int64_t)blk_valptr.size() - 1;
        n.col_slots = (int64_t)blk_cols.size();
        n.bitmap_words = (int64_t)blk_bitmap.size();
        n.dense = (int64_t)dense_perm.size();
        n.res = (int64_t)res_perm.size();
        n.zero_rows = (int64_t)zero_rows.size();
    }
};

struct Resolved {
    int mode, W, KB, tau_spmm, tau_sddmm, Ts, Cs, short_len, sddmm_Cs, sddmm_Ts, threads;
    int sddmm_min_dense_pct = 0;        // 0: off
    bool fill, build_spmm, build_sddmm, heavy_first, segments_by_column, two_kernels;
    int xcd_order;       // 1 on, 0 off, -1 decide from the matrix
};

// The whole-matrix form of the utilisation rule for the SDDMM sub-plan (hybrid mode only): its dense blocks are kept only
// if they hold at least sddmm_min_dense_pct percent of the nonzeros.
inline bool share_rule_fires(const Resolved &o, int64_t dense_nnz, int64_t nnz) {
    return o.mode == LIBRA_MODE_HYBRID && o.sddmm_min_dense_pct > 0 && 100 * dense_nnz < (int64_t)o.sddmm_min_dense_pct * nnz;
}

}  // namespace libra

struct libra_plan_s {
    int64_t M = 0, Kc = 0, nnz = 0;
    int vdt = LIBRA_F16;
    int vsize = 2;
    libra::Resolved o{};
    std::vector<int32_t> rowptr;
    std::vector<int32_t> long_rows;     // rows with more than LIBRA_SOFTMAX_LONG_ROW nonzeros (edge softmax)
    std::vector<int32_t> medium_rows;   // rows with 65 .. LIBRA_SOFTMAX_LONG_ROW nonzeros
    libra::SubPlan spmm, sddmm;
    bool host_arrays = true;            // false: built on the device without a host copy (nothing to export or upload)
    libra_stats_t stats{};
    // device copy
    void *dev_base = nullptr;
    size_t dev_bytes = 0;
    const int32_t *d_rowptr = nullptr;
    const int32_t *d_long_rows = nullptr;
    const int32_t *d_medium_rows = nullptr;
};

namespace libra {
// Host pointer to the column indices of CSR positions [p0, p1).
typedef std::function<const int32_t *(int64_t p0, int64_t p1)> ColumnFetch;
int resolve_options(const libra_plan_opts_t *in, int value_dtype, Resolved &out);
// Shared tail of the host and the device planner (segments of the SDDMM residual list, task order, statistics).
// `share` (optional): the two sums of the sampled column-sharing statistic {together, apart} if the caller has
// already counted them; otherwise they are counted from `cols`.
void finish_plan(libra_plan_s *plan, const ColumnFetch &cols, const int64_t *share = nullptr);
// The sample of that statistic: group k of `nsample` is sampled_group(k, ...) out of `ngroups` groups of
// LIBRA_LOCALITY_WINDOWS windows.
LIBRA_HD inline int64_t share_samples(int64_t ngroups) { return ngroups < 256 ? ngroups : 256; }
LIBRA_HD inline int64_t sampled_group(int64_t k, int64_t ngroups, int64_t nsample) { return k * ngroups / nsample; }
// Lay the plan out in `dev_buf` taking the big arrays from device memory (device planner) instead of the host vectors.
int adopt_device_arrays(libra_plan_s *plan, const DeviceSource &spmm, const DeviceSource &sddmm, void *dev_buf, size_t bytes, void *stream);
// Bytes libra_plan_upload / adopt_device_arrays need for a plan with these array sizes.
size_t plan_buffer_bytes(const libra_plan_s *plan);
}  // namespace libra
