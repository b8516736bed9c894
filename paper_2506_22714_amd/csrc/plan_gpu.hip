// Device planner: the preprocessing of Section 4.5 (Algorithm 1) on the GPU.
//
// Builds the same plan as the host planner (plan.cpp), bit for bit, from a CSR matrix that is
// already in device memory.  The window-by-window loops of the host code become flat passes
// over arrays plus prefix sums:
//
//   1. every nonzero gets the key (column, row inside the window); a segmented sort (segments =
//      windows) puts the nonzeros of each column vector next to each other (the "census");
//   2. head flags + a prefix sum number the vectors; a second segmented sort orders the vectors
//      of a window by (NNZ descending, column ascending) - the order of the SDDMM blocks and of
//      the vectors that fill the padding of the last SpMM block;
//   3. per window: how many vectors reach the SpMM threshold, how many fill padding, how many
//      SDDMM blocks reach the block threshold (their NNZ never increases along the order, so a
//      binary search finds the cut); prefix sums give block offsets;
//   4. vectors are scattered to their slots, blocks build bitmaps by ballots, packed values go
//      to the position given by the popcount of the bits below theirs;
//   5. nonzeros outside the dense vectors are flagged in CSR order; prefix sums give residual
//      positions; per window the load-balancing rule of Section 4.3 emits the task records.
//
// Sorting and prefix sums are rocPRIM device primitives; everything else is written here.
// The arrays are produced in the host planner's format in the caller's workspace, copied to the
// plan's host vectors, and the shared tail (task order, statistics) runs on the host.
#include <hip/hip_runtime.h>

#include <mutex>

#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include <rocprim/rocprim.hpp>

#include "plan_internal.h"

using namespace libra;

namespace {

constexpr int W = 16, KB = 16;
typedef unsigned long long u64;

enum Counter { C_NV = 0, C_NNZ1, C_SHORT, C_LONG, C_SPLIT, C_DV_A, C_PAD_A, C_DV_D, C_PAD_D, C_ERR, C_TOGETHER, C_APART, C_DNNZ_D, C_COUNT };

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Bump allocator over the workspace (base == nullptr: size pass).
struct Arena {
    char *base;
    size_t off = 0;
    template <class T> T *take(size_t n) {
        off = align256(off);
        T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
        off += n * sizeof(T) + 64;
        return p;
    }
};

struct Sizes {
    int64_t M, n;
    int64_t nw, nbmax, tasks_a_max, tasks_d_max, segs_d_max;
};

Sizes make_sizes(int64_t M, int64_t n, const Resolved &o) {
    Sizes z;
    z.M = M; z.n = n;
    z.nw = (M + W - 1) / W;
    z.nbmax = n / KB + z.nw + 1;
    z.tasks_a_max = z.nbmax / o.Ts + 2 * z.nw + 2 * (n / o.Cs) + 8;
    z.tasks_d_max = z.nbmax / o.sddmm_Ts + z.nw + 8;
    z.segs_d_max = n / o.sddmm_Cs + 2;
    return z;
}

struct SubOut {      // one sub-plan in the host planner's format
    int32_t *slotvec, *blk_cols, *blknnz, *blk_valptr, *blkmask, *blkncols, *dense_perm;
    u64 *bitmap;
    uint8_t *dense_val, *res_val, *dflag;
    int32_t *resf, *rescan, *res_perm, *res_row, *res_col;
    int32_t *nb, *ndv, *blkptr, *ntasks, *tbase;
    libra_task_t *tasks;
};

struct Layout {
    int32_t *win_ptr, *spos, *hflag, *vid, *einfo, *ewin, *row_of, *rowbase;
    u64 *key_in, *key_out, *key2_in, *key2_out, *ctr;
    int32_t *vfirst, *vinfo, *vcol, *vwin, *sv, *srank, *scnt, *cum, *tflag, *taud, *win_vptr;
    int32_t *ntau, *nzero, *zbase, *nres, *resptr, *zero_rows, *task_col, *seg_col;
    SubOut a, d;
    void *tmp;
    size_t tmp_bytes;
    size_t total;
};

size_t rocprim_temp_bytes(const Sizes &z) {
    size_t best = 0, sz = 0;
    const unsigned n = (unsigned)z.n, nw = (unsigned)z.nw;
    (void)rocprim::segmented_radix_sort_pairs(nullptr, sz, (u64 *)nullptr, (u64 *)nullptr, rocprim::counting_iterator<int32_t>(0),
                                        (int32_t *)nullptr, n, nw, (int32_t *)nullptr, (int32_t *)nullptr, 0, 64);
    best = std::max(best, sz);
    sz = 0;
    (void)rocprim::exclusive_scan(nullptr, sz, (int32_t *)nullptr, (int32_t *)nullptr, (int32_t)0, (size_t)(z.n + z.nw + 2),
                            rocprim::plus<int32_t>());
    best = std::max(best, sz);
    return best + 4096;
}

Layout make_layout(const Sizes &z, int vsize, void *base) {
    Layout L{};
    Arena A{(char *)base};
    const size_t n = (size_t)z.n, nw = (size_t)z.nw, nb = (size_t)z.nbmax;
    L.ctr = A.take<u64>(C_COUNT);
    L.win_ptr = A.take<int32_t>(nw + 1);
    L.key_in = A.take<u64>(n);
    L.key_out = A.take<u64>(n);
    L.spos = A.take<int32_t>(n);
    L.hflag = A.take<int32_t>(n + 1);
    L.vid = A.take<int32_t>(n + 1);
    L.einfo = A.take<int32_t>(n);
    L.ewin = A.take<int32_t>(n);
    L.row_of = A.take<int32_t>(n);
    L.rowbase = A.take<int32_t>((size_t)z.M + 1);
    L.vfirst = A.take<int32_t>(n);
    L.vinfo = A.take<int32_t>(n);
    L.vcol = A.take<int32_t>(n);
    L.vwin = A.take<int32_t>(n);
    L.key2_in = A.take<u64>(n);
    L.key2_out = A.take<u64>(n);
    L.sv = A.take<int32_t>(n);
    L.srank = A.take<int32_t>(n);
    L.scnt = A.take<int32_t>(n + 1);
    L.cum = A.take<int32_t>(n + 1);
    L.tflag = A.take<int32_t>(n + 1);
    L.taud = A.take<int32_t>(n + 1);
    L.win_vptr = A.take<int32_t>(nw + 1);
    L.ntau = A.take<int32_t>(nw);
    L.nzero = A.take<int32_t>(nw + 1);
    L.zbase = A.take<int32_t>(nw + 1);
    L.nres = A.take<int32_t>(nw + 1);
    L.resptr = A.take<int32_t>(nw + 1);
    L.zero_rows = A.take<int32_t>((size_t)z.M);
    L.task_col = A.take<int32_t>((size_t)z.tasks_a_max);
    L.seg_col = A.take<int32_t>((size_t)z.segs_d_max);
    for (SubOut *s : {&L.a, &L.d}) {
        s->slotvec = A.take<int32_t>(nb * KB);
        s->blk_cols = A.take<int32_t>(nb * KB);
        s->bitmap = A.take<u64>(nb * 4);
        s->blknnz = A.take<int32_t>(nb + 1);
        s->blk_valptr = A.take<int32_t>(nb + 1);
        s->blkmask = A.take<int32_t>(nb);
        s->blkncols = A.take<int32_t>(nb);
        s->dense_perm = A.take<int32_t>(n);
        s->dense_val = A.take<uint8_t>(n * vsize);
        s->dflag = A.take<uint8_t>(n);
        s->resf = A.take<int32_t>(n + 1);
        s->rescan = A.take<int32_t>(n + 1);
        s->res_perm = A.take<int32_t>(n);
        s->res_row = A.take<int32_t>(n);
        s->res_col = A.take<int32_t>(n);
        s->res_val = A.take<uint8_t>(n * vsize);
        s->nb = A.take<int32_t>(nw + 1);
        s->ndv = A.take<int32_t>(nw);
        s->blkptr = A.take<int32_t>(nw + 1);
        s->ntasks = A.take<int32_t>(nw + 1);
        s->tbase = A.take<int32_t>(nw + 1);
        s->tasks = A.take<libra_task_t>((size_t)(s == &L.a ? z.tasks_a_max : z.tasks_d_max));
    }
    L.tmp_bytes = rocprim_temp_bytes(z);
    L.tmp = A.take<uint8_t>(L.tmp_bytes);
    L.total = align256(A.off) + 256;
    return L;
}

// ------------------------------------------------------------------------------------------
// kernels
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_win_ptr(const int32_t *rowptr, int64_t M, int nw, int32_t *win_ptr) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t <= nw) win_ptr[t] = rowptr[min((int64_t)M, t * W)];
}

// Per nonzero (CSR order): its row (bisection over rowptr; rows without nonzeros are skipped over), the sort key
// (column, row in window), and the checks the host planner makes.
__global__ __launch_bounds__(256) void k_keys(const int32_t *rowptr, const int32_t *col, int64_t M, int64_t Kc, int n,
                                              u64 *key_in, int32_t *row_of, u64 *ctr) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n) return;
    int64_t lo = 0, hi = M;                 // rowptr[lo] <= p < rowptr[hi]
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (rowptr[mid] <= p) lo = mid; else hi = mid;
    }
    const int c = col[p];
    unsigned bad = 0;
    if (c < 0 || c >= Kc) bad = 1u;
    else if (p > rowptr[lo] && col[p - 1] >= c) bad = 2u;
    key_in[p] = ((u64)(uint32_t)c << 4) | (u64)(lo & (W - 1));
    row_of[p] = (int32_t)lo;
    if (bad) atomicOr(&ctr[C_ERR], (u64)bad);
}

// largest w in [0, nw) with win_ptr[w] <= e   (win_ptr[0] = 0 <= e < win_ptr[nw])
__device__ inline int window_of(const int32_t *win_ptr, int nw, int e) {
    int lo = 0, hi = nw;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (win_ptr[mid] <= e) lo = mid; else hi = mid;
    }
    return lo;
}

// Per sorted nonzero: is it the first of its column vector; if so, the vector's NNZ and row mask.
__global__ __launch_bounds__(256) void k_census(const u64 *skey, const int32_t *win_ptr, int nw, int n,
                                                int32_t *hflag, int32_t *einfo, int32_t *ewin) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n) return;
    const u64 key = skey[e];
    const u64 c = key >> 4;
    const int w = window_of(win_ptr, nw, e);
    const int ws = win_ptr[w], we = win_ptr[w + 1];
    const bool head = e == ws || (skey[e - 1] >> 4) != c;
    int info = 0;
    if (head) {
        int cnt = 1;
        unsigned mask = 1u << (unsigned)(key & 15);
        for (int k = 1; k < W; ++k) {
            if (e + k >= we) break;
            const u64 kk = skey[e + k];
            if ((kk >> 4) != c) break;
            ++cnt;
            mask |= 1u << (unsigned)(kk & 15);
        }
        info = cnt | (int)(mask << 8);
    }
    hflag[e] = head ? 1 : 0;
    einfo[e] = info;
    ewin[e] = w;
}

__global__ __launch_bounds__(256) void k_vectors(const u64 *skey, const int32_t *hflag, const int32_t *vid, const int32_t *einfo,
                                                 const int32_t *ewin, int n, int tau_a, int colbits,
                                                 int32_t *vfirst, int32_t *vinfo, int32_t *vcol, int32_t *vwin, int32_t *tflag,
                                                 u64 *key2, u64 *ctr) {
    __shared__ int ones;
    if (threadIdx.x == 0) ones = 0;
    __syncthreads();
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n && hflag[e]) {
        const int v = vid[e];
        const int info = einfo[e];
        const int cnt = info & 0xff;
        const int c = (int)(skey[e] >> 4);
        vfirst[v] = e;
        vinfo[v] = info;
        vcol[v] = c;
        vwin[v] = ewin[e];
        tflag[v] = cnt >= tau_a ? 1 : 0;
        key2[v] = ((u64)(W - cnt) << colbits) | (u64)(uint32_t)c;
        if (cnt == 1) atomicAdd(&ones, 1);
    }
    if (e == n - 1) ctr[C_NV] = (u64)(vid[e] + hflag[e]);
    __syncthreads();
    if (threadIdx.x == 0 && ones) atomicAdd(&ctr[C_NNZ1], (u64)ones);
}

__global__ __launch_bounds__(256) void k_win_vptr(const int32_t *win_ptr, const int32_t *vid, int nw, int n, const u64 *ctr, int32_t *win_vptr) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t > nw) return;
    const int p = win_ptr[t];
    win_vptr[t] = p < n ? vid[p] : (int)ctr[C_NV];
}

// Per position of the (NNZ desc, column asc) order: the vector's NNZ; per vector: its rank in its window.
__global__ __launch_bounds__(256) void k_sorted(const int32_t *sv, const int32_t *vinfo, const int32_t *vwin, const int32_t *win_vptr,
                                                int nv, int32_t *scnt, int32_t *srank) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= nv) return;
    const int v = sv[k];
    scnt[k] = vinfo[v] & 0xff;
    srank[v] = k - win_vptr[vwin[v]];
}

// The sampled column-sharing statistic (one workgroup per sampled group of LIBRA_LOCALITY_WINDOWS windows): how
// many distinct columns the windows have together (a vector counts unless an earlier window of the group has its
// column) and one by one.
__global__ __launch_bounds__(256) void k_share(const int32_t *win_vptr, const int32_t *vcol, int nw, int64_t ngroups, int64_t nsample, u64 *ctr) {
    __shared__ int together;
    if (threadIdx.x == 0) together = 0;
    __syncthreads();
    const int64_t g = sampled_group(blockIdx.x, ngroups, nsample);
    const int w0 = (int)(g * LIBRA_LOCALITY_WINDOWS), w1 = (int)min((int64_t)nw, (g + 1) * LIBRA_LOCALITY_WINDOWS);
    const int v0 = win_vptr[w0], v1 = win_vptr[w1];
    int mine = 0;
    // the group's vectors are dealt to the gridDim.y workgroups of the group
    for (int v = v0 + (int)(blockIdx.y * blockDim.x + threadIdx.x); v < v1; v += (int)(blockDim.x * gridDim.y)) {
        const int c = vcol[v];
        bool seen = false;
        for (int w = w0; w < w1 && !seen; ++w) {
            const int a = win_vptr[w], b = win_vptr[w + 1];
            if (b > v) break;                     // only the windows before the vector's own
            int lo = a, hi = b;                   // first position with column >= c
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (vcol[mid] < c) lo = mid + 1; else hi = mid;
            }
            seen = lo < b && vcol[lo] == c;
        }
        mine += seen ? 0 : 1;
    }
    if (mine) atomicAdd(&together, mine);
    __syncthreads();
    if (threadIdx.x == 0) {
        if (together) atomicAdd(&ctr[C_TOGETHER], (u64)together);
        if (blockIdx.y == 0) atomicAdd(&ctr[C_APART], (u64)(v1 - v0));
    }
}

struct Rule {
    int mode, fill, tau_d, Ts, Cs, short_len, build_a, build_d, Ts_d;
};

// Per window: dense vectors and blocks of both sub-plans (Section 4.2).
__global__ __launch_bounds__(256) void k_window_counts(const int32_t *win_vptr, const int32_t *taud, const int32_t *cum, int nw, Rule R,
                                                       int32_t *ntau_o, int32_t *ndv_a, int32_t *nb_a, int32_t *ndv_d, int32_t *nb_d, u64 *ctr) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= nw) return;
    const int base = win_vptr[t], nvw = win_vptr[t + 1] - base;
    int ntau = 0, ndv = 0, nb = 0;
    if (R.build_a) {
        ntau = taud[base + nvw] - taud[base];
        int nprom = 0;
        if (R.fill && ntau > 0 && ntau % KB) nprom = min(KB - ntau % KB, nvw - ntau);
        ndv = ntau + nprom;
        nb = (ndv + KB - 1) / KB;
    }
    ntau_o[t] = ntau;
    ndv_a[t] = ndv;
    nb_a[t] = nb;
    int nbd = 0;
    if (R.build_d && R.mode != LIBRA_MODE_SCALAR_ONLY) {
        const int nblk = (nvw + KB - 1) / KB;
        if (R.mode == LIBRA_MODE_DENSE_ONLY) {
            nbd = nblk;
        } else {
            // block NNZ never increases along the order: first block below the threshold by bisection
            int lo = 0, hi = nblk;          // blocks [0, lo) pass, blocks [hi, nblk) fail
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                const int nnzb = cum[base + min(nvw, mid * KB + KB)] - cum[base + mid * KB];
                if (nnzb >= R.tau_d) lo = mid + 1; else hi = mid;
            }
            nbd = lo;
        }
    }
    const int ndvd = min(nvw, nbd * KB);
    ndv_d[t] = ndvd;
    nb_d[t] = nbd;
    if (ndv) { atomicAdd(&ctr[C_DV_A], (u64)ndv); }
    if (nb * KB - ndv) atomicAdd(&ctr[C_PAD_A], (u64)(nb * KB - ndv));
    if (ndvd) atomicAdd(&ctr[C_DV_D], (u64)ndvd);
    if (ndvd) atomicAdd(&ctr[C_DNNZ_D], (u64)(cum[base + ndvd] - cum[base]));       // nonzeros in the window's dense SDDMM blocks
    if (nbd * KB - ndvd) atomicAdd(&ctr[C_PAD_D], (u64)(nbd * KB - ndvd));
}

// Per vector: its slot in the SpMM blocks (threshold vectors in column order, then the fillers in sorted order)
// and in the SDDMM blocks (sorted order).
__global__ __launch_bounds__(256) void k_slots(const int32_t *vwin, const int32_t *win_vptr, const int32_t *srank, const int32_t *taud,
                                               const int32_t *ntau, const int32_t *ndv_a, const int32_t *blkptr_a,
                                               const int32_t *ndv_d, const int32_t *blkptr_d, int nv, Rule R,
                                               int32_t *slotvec_a, uint8_t *dflag_a, int32_t *slotvec_d, uint8_t *dflag_d) {
    const int v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= nv) return;
    const int w = vwin[v];
    const int base = win_vptr[w];
    const int k = srank[v];
    if (R.build_a && k < ndv_a[w]) {
        const int slot = k < ntau[w] ? taud[v] - taud[base] : k;
        slotvec_a[(int64_t)blkptr_a[w] * KB + slot] = v;
        dflag_a[v] = 1;
    }
    if (R.build_d && k < ndv_d[w]) {
        slotvec_d[(int64_t)blkptr_d[w] * KB + k] = v;
        dflag_d[v] = 1;
    }
}

// 16 lanes per block: column ids, the bitmap (bit r*16+s) by ballots, NNZ, touched rows, real columns.
__global__ __launch_bounds__(256) void k_blocks(const int32_t *slotvec, const int32_t *vcol, const int32_t *vinfo, int nb,
                                                int32_t *blk_cols, u64 *bitmap, int32_t *blknnz, int32_t *blkmask, int32_t *blkncols) {
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int b = (int)(gid >> 4), s = (int)(gid & 15);
    const int grp = (threadIdx.x & 63) >> 4;
    const bool live = b < nb;
    const int v = live ? slotvec[(int64_t)b * KB + s] : -1;
    const unsigned mask = v >= 0 ? ((unsigned)vinfo[v] >> 8) & 0xffffu : 0u;
    if (live) blk_cols[(int64_t)b * KB + s] = v >= 0 ? vcol[v] : -1;
    u64 word = 0;           // lane s < 4 builds word s (rows 4s .. 4s+3)
    int nnz = 0;
    unsigned touched = 0;
    for (int r = 0; r < W; ++r) {
        const u64 bal = __ballot((mask >> r) & 1u);
        const u64 rb = (bal >> (16 * grp)) & 0xffffull;
        nnz += __popcll(rb);
        if (rb) touched |= 1u << r;
        if ((r >> 2) == s) word |= rb << (16 * (r & 3));
    }
    const u64 balc = __ballot(v >= 0);
    const int ncols = __popcll((balc >> (16 * grp)) & 0xffffull);
    if (live && s < 4) bitmap[(int64_t)b * 4 + s] = word;
    if (live && s == 0) {
        blknnz[b] = nnz;
        blkmask[b] = (int)touched;
        blkncols[b] = ncols;
    }
}

// 16 lanes per block: CSR position and value of every packed nonzero, at popcount(bits below its bit).
__global__ __launch_bounds__(256) void k_block_values(const int32_t *slotvec, const int32_t *vfirst, const int32_t *vinfo, const u64 *bitmap,
                                                      const int32_t *blk_valptr, const int32_t *spos, const uint8_t *val, int vsize, int nb,
                                                      int32_t *dense_perm, uint8_t *dense_val) {
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int b = (int)(gid >> 4), s = (int)(gid & 15);
    if (b >= nb) return;
    const int v = slotvec[(int64_t)b * KB + s];
    if (v < 0) return;
    const unsigned mask = ((unsigned)vinfo[v] >> 8) & 0xffffu;
    const u64 w0 = bitmap[(int64_t)b * 4], w1 = bitmap[(int64_t)b * 4 + 1], w2 = bitmap[(int64_t)b * 4 + 2], w3 = bitmap[(int64_t)b * 4 + 3];
    const int c0 = __popcll(w0), c1 = __popcll(w1), c2 = __popcll(w2);
    const int vbase = blk_valptr[b];
    int e = vfirst[v];
    for (int r = 0; r < W; ++r) {
        if (!((mask >> r) & 1u)) continue;
        const int q = r >> 2;
        const u64 word = q == 0 ? w0 : q == 1 ? w1 : q == 2 ? w2 : w3;
        const int below = (q > 0 ? c0 : 0) + (q > 1 ? c1 : 0) + (q > 2 ? c2 : 0) + __popcll(word & ((1ull << ((r & 3) * 16 + s)) - 1ull));
        const int dst = vbase + below;
        const int p = spos[e];
        dense_perm[dst] = p;
        if (vsize == 2) reinterpret_cast<uint16_t *>(dense_val)[dst] = reinterpret_cast<const uint16_t *>(val)[p];
        else reinterpret_cast<uint32_t *>(dense_val)[dst] = reinterpret_cast<const uint32_t *>(val)[p];
        ++e;
    }
}

// Per sorted nonzero: residual flags of both sub-plans, written at the nonzero's CSR position.
__global__ __launch_bounds__(256) void k_entry_flags(const int32_t *hflag, const int32_t *vid, const int32_t *spos, const uint8_t *dflag_a,
                                                     const uint8_t *dflag_d, int n, Rule R, int32_t *resf_a, int32_t *resf_d) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n) return;
    const int v = vid[e] + hflag[e] - 1;
    const int p = spos[e];
    resf_a[p] = R.build_a && !dflag_a[v] ? 1 : 0;
    resf_d[p] = R.build_d && !dflag_d[v] ? 1 : 0;
}

struct WinRows {
    int nr;
    int rlen[W];
    unsigned valid, split, scalar;
    int q_unsplit, q_split;
};

__device__ inline WinRows window_rows(const int32_t *rowptr, const int32_t *rescan, int64_t M, int t, const Rule &R, int *n_short, int *n_long) {
    WinRows z;
    const int64_t r0 = (int64_t)t * W;
    z.nr = (int)min((int64_t)W, M - r0);
    z.valid = z.split = z.scalar = 0;
    z.q_unsplit = z.q_split = 0;
    *n_short = *n_long = 0;
    for (int r = 0; r < W; ++r) {
        z.rlen[r] = 0;
        if (r >= z.nr) continue;
        const int len = rescan[rowptr[r0 + r + 1]] - rescan[rowptr[r0 + r]];
        z.rlen[r] = len;
        z.valid |= 1u << r;
        if (len == 0) continue;
        if (len < R.short_len) {
            ++*n_short;
        } else {
            ++*n_long;
            if (len > R.Cs) z.split |= 1u << r;
        }
        if (!((z.split >> r) & 1u)) { z.scalar |= 1u << r; z.q_unsplit += len; } else z.q_split += len;
    }
    return z;
}

__device__ inline void put_task(libra_task_t *t, int kind, int id, int b0, int b1, int q0, int q1, unsigned sc, unsigned at, unsigned st, unsigned cost) {
    t->kind = kind; t->id = id; t->blk_begin = b0; t->blk_end = b1; t->res_begin = q0; t->res_end = q1;
    t->scalar_mask = sc; t->atomic_mask = at; t->store_mask = st; t->cost = cost;
}

// Per window: the hybrid load-balancing rule (Section 4.3).  FILL = false counts tasks, rows to clear and
// residual nonzeros; FILL = true writes them at the offsets the prefix sums gave.
template <bool FILL>
__global__ __launch_bounds__(128) void k_window_tasks(const int32_t *rowptr, const int32_t *rescan_a, int64_t M, int nw, Rule R,
                                                      const int32_t *blkptr_a, const int32_t *blkmask_a, const int32_t *blkncols_a,
                                                      const int32_t *blkptr_d, const int32_t *blkncols_d,
                                                      int32_t *ntasks_a, int32_t *nzero, int32_t *nres, int32_t *ntasks_d, u64 *ctr,
                                                      const int32_t *tbase_a, const int32_t *zbase, const int32_t *resptr, const int32_t *tbase_d,
                                                      libra_task_t *tasks_a, int32_t *zero_rows, libra_task_t *tasks_d) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= nw) return;
    const int64_t r0 = (int64_t)t * W;
    if (R.build_a) {
        int n_short, n_long;
        const WinRows z = window_rows(rowptr, rescan_a, M, t, R, &n_short, &n_long);
        const int b0 = blkptr_a[t], b1 = blkptr_a[t + 1];
        const bool many = b1 - b0 > R.Ts;
        int nchunks = 0;
        for (int r = 0; r < z.nr; ++r)
            if ((z.split >> r) & 1u) nchunks += (z.rlen[r] + R.Cs - 1) / R.Cs;
        if (!FILL) {
            const int nwt = many ? (b1 - b0 + R.Ts - 1) / R.Ts + (z.scalar ? 1 : 0) : 1;
            ntasks_a[t] = nwt + nchunks;
            nzero[t] = many ? z.nr : __popc(z.split);
            nres[t] = z.q_unsplit + z.q_split;
            if (n_short) atomicAdd(&ctr[C_SHORT], (u64)n_short);
            if (n_long) atomicAdd(&ctr[C_LONG], (u64)n_long);
            if (z.split) atomicAdd(&ctr[C_SPLIT], (u64)__popc(z.split));
        } else {
            libra_task_t *out = tasks_a + tbase_a[t];
            int32_t *zr = zero_rows + zbase[t];
            const int q0 = resptr[t], q1 = q0 + z.q_unsplit;
            auto touched = [&](int g0, int g1) { unsigned m = 0; for (int b = g0; b < g1; ++b) m |= (unsigned)blkmask_a[b]; return m; };
            auto cols_in = [&](int g0, int g1) { unsigned c = 0; for (int b = g0; b < g1; ++b) c += (unsigned)blkncols_a[b]; return c; };
            if (many) {
                for (int g0 = b0; g0 < b1; g0 += R.Ts) {
                    const int g1 = min(b1, g0 + R.Ts);
                    put_task(out++, LIBRA_TASK_WINDOW, t, g0, g1, q0, q0, 0u, touched(g0, g1), 0u, cols_in(g0, g1));
                }
                if (z.scalar) put_task(out++, LIBRA_TASK_WINDOW, t, b1, b1, q0, q1, z.scalar, z.scalar, 0u, (unsigned)(q1 - q0));
                for (int r = 0; r < z.nr; ++r) *zr++ = (int32_t)(r0 + r);
            } else {
                put_task(out++, LIBRA_TASK_WINDOW, t, b0, b1, q0, q1, z.scalar, z.split & touched(b0, b1), z.valid & ~z.split,
                         cols_in(b0, b1) + (unsigned)(q1 - q0));
                for (int r = 0; r < z.nr; ++r)
                    if ((z.split >> r) & 1u) *zr++ = (int32_t)(r0 + r);
            }
            int q = q1;
            for (int r = 0; r < z.nr; ++r) {
                if (!((z.split >> r) & 1u)) continue;
                const int e = q + z.rlen[r];
                for (; q < e; q += R.Cs) {
                    const int qe = min(e, q + R.Cs);
                    put_task(out++, LIBRA_TASK_CHUNK, (int)(r0 + r), 0, 0, q, qe, 0u, 0u, 0u, (unsigned)(qe - q));
                }
                q = e;
            }
        }
    } else if (!FILL) {
        ntasks_a[t] = 0; nzero[t] = 0; nres[t] = 0;
    }
    if (R.build_d) {
        const int b0 = blkptr_d[t], b1 = blkptr_d[t + 1];
        if (!FILL) {
            ntasks_d[t] = (b1 - b0 + R.Ts_d - 1) / R.Ts_d;
        } else {
            libra_task_t *out = tasks_d + tbase_d[t];
            for (int g0 = b0; g0 < b1; g0 += R.Ts_d) {
                const int g1 = min(b1, g0 + R.Ts_d);
                unsigned c = 0;
                for (int b = g0; b < g1; ++b) c += (unsigned)blkncols_d[b];
                put_task(out++, LIBRA_TASK_WINDOW, t, g0, g1, 0, 0, 0u, 0u, 0u, c + (unsigned)W);
            }
        }
    } else if (!FILL) {
        ntasks_d[t] = 0;
    }
}

// Per window: where each row's residual nonzeros start in the SpMM residual array (rows that are not decomposed
// first, in row order, then the decomposed rows), minus the row's own prefix so that a nonzero only adds its scan value.
__global__ __launch_bounds__(128) void k_row_bases(const int32_t *rowptr, const int32_t *rescan_a, const int32_t *resptr, int64_t M, int nw, Rule R,
                                                   int32_t *rowbase) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= nw) return;
    int n_short, n_long;
    const WinRows z = window_rows(rowptr, rescan_a, M, t, R, &n_short, &n_long);
    int u = 0, sp = z.q_unsplit;
    const int64_t r0 = (int64_t)t * W;
    for (int r = 0; r < z.nr; ++r) {
        int off;
        if ((z.split >> r) & 1u) { off = sp; sp += z.rlen[r]; } else { off = u; u += z.rlen[r]; }
        rowbase[r0 + r] = resptr[t] + off - rescan_a[rowptr[r0 + r]];
    }
}

// Per nonzero (CSR order): residual nonzeros to their places.  SDDMM: CSR order.
__global__ __launch_bounds__(256) void k_residual_fill(const int32_t *col, const uint8_t *val, int vsize, int n, Rule R, const int32_t *row_of,
                                                      const int32_t *resf_a, const int32_t *rescan_a, const int32_t *rowbase,
                                                      int32_t *a_perm, int32_t *a_row, int32_t *a_col, uint8_t *a_val,
                                                      const int32_t *resf_d, const int32_t *rescan_d,
                                                      int32_t *d_perm, int32_t *d_row, int32_t *d_col, uint8_t *d_val) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n) return;
    const bool ra = R.build_a && resf_a[p], rd = R.build_d && resf_d[p];
    if (!ra && !rd) return;
    const int i = row_of[p], c = col[p];
    if (ra) {
        const int d = rowbase[i] + rescan_a[p];
        a_perm[d] = p; a_row[d] = i; a_col[d] = c;
        if (vsize == 2) reinterpret_cast<uint16_t *>(a_val)[d] = reinterpret_cast<const uint16_t *>(val)[p];
        else reinterpret_cast<uint32_t *>(a_val)[d] = reinterpret_cast<const uint32_t *>(val)[p];
    }
    if (rd) {
        const int d = rescan_d[p];
        d_perm[d] = p; d_row[d] = i; d_col[d] = c;
        if (vsize == 2) reinterpret_cast<uint16_t *>(d_val)[d] = reinterpret_cast<const uint16_t *>(val)[p];
        else reinterpret_cast<uint32_t *>(d_val)[d] = reinterpret_cast<const uint32_t *>(val)[p];
    }
}

// Per SpMM task: first column of a row segment's entries (the host orders the segments by it), -1 for other tasks.
// Per flat SDDMM residual segment (cs entries of the residual list): its first column if the segment lies in one row, else -1.
__global__ __launch_bounds__(256) void k_segment_cols(const int32_t *res_row, const int32_t *res_col, int nres, int cs, int nseg, int32_t *seg_col) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nseg) return;
    const int64_t q = (int64_t)i * cs, q1 = q + cs < nres ? q + cs : nres;
    seg_col[i] = res_row[q] == res_row[q1 - 1] ? res_col[q] : -1;
}

__global__ __launch_bounds__(256) void k_task_cols(const libra_task_t *tasks, int nt, const int32_t *res_col, int32_t *task_col) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nt) return;
    task_col[i] = tasks[i].kind == LIBRA_TASK_CHUNK ? res_col[tasks[i].res_begin] : -1;
}

// ------------------------------------------------------------------------------------------
// host driver
// ------------------------------------------------------------------------------------------
struct Fail { int code; };
inline void hip_ok(hipError_t e) { if (e != hipSuccess) throw Fail{LIBRA_ERR_HIP}; }
inline unsigned blocks_for(int64_t n, int per) { return (unsigned)std::max<int64_t>(1, (n + per - 1) / per); }

void scan(const Layout &L, const int32_t *in, int32_t *out, size_t n, hipStream_t s) {
    size_t sz = L.tmp_bytes;
    hip_ok(rocprim::exclusive_scan(L.tmp, sz, in, out, (int32_t)0, n, rocprim::plus<int32_t>(), s));
}

template <class T>
void fetch(std::vector<T> &dst, const void *src, size_t n, hipStream_t s) {
    dst.resize(n);
    if (n) hip_ok(hipMemcpyAsync(dst.data(), src, n * sizeof(T), hipMemcpyDeviceToHost, s));
}

void fill_bytes(void *p, int value, size_t bytes, hipStream_t s) {
    if (bytes) hip_ok(hipMemsetAsync(p, value, bytes, s));
}

int32_t peek(const int32_t *p, hipStream_t s) {
    int32_t v = 0;
    hip_ok(hipMemcpyAsync(&v, p, sizeof v, hipMemcpyDeviceToHost, s));
    hip_ok(hipStreamSynchronize(s));
    return v;
}

}  // namespace

extern "C" int libra_plan_device_workspace(int64_t M, int64_t nnz, const libra_plan_opts_t *opts, size_t *bytes) {
    if (!bytes) return LIBRA_ERR_NULL;
    if (M < 1 || nnz < 0) return LIBRA_ERR_SHAPE;
    if (M >= (1ll << 31) - 64 || nnz >= (1ll << 31) - 64) return LIBRA_ERR_TOO_LARGE;
    Resolved o{};
    if (int rc = resolve_options(opts, LIBRA_F32, o)) return rc;       // the widest value type bounds the size
    if (o.W != W || o.KB != KB) return LIBRA_ERR_UNSUPPORTED;
    *bytes = make_layout(make_sizes(M, std::max<int64_t>(nnz, 1), o), 4, nullptr).total;
    return LIBRA_OK;
}

extern "C" int libra_plan_device_buffer_bound(int64_t M, int64_t nnz, int val_dtype, const libra_plan_opts_t *opts, size_t *bytes) {
    if (!bytes) return LIBRA_ERR_NULL;
    if (M < 1 || nnz < 0) return LIBRA_ERR_SHAPE;
    if (M >= (1ll << 31) - 64 || nnz >= (1ll << 31) - 64) return LIBRA_ERR_TOO_LARGE;
    if (val_dtype != LIBRA_F16 && val_dtype != LIBRA_BF16 && val_dtype != LIBRA_F32) return LIBRA_ERR_DTYPE;
    Resolved o{};
    if (int rc = resolve_options(opts, val_dtype, o)) return rc;
    if (o.W != W || o.KB != KB) return LIBRA_ERR_UNSUPPORTED;
    try {
        // a plan with the largest arrays this matrix size can produce (only the sizes matter)
        const Sizes z = make_sizes(M, std::max<int64_t>(nnz, 1), o);
        libra_plan_t fake;
        fake.M = M; fake.nnz = nnz; fake.vdt = val_dtype; fake.vsize = val_dtype == LIBRA_F32 ? 4 : 2;
        fake.o = o;
        for (SubPlan *sp : {&fake.spmm, &fake.sddmm}) {
            sp->n.blocks = z.nbmax; sp->n.col_slots = z.nbmax * KB; sp->n.bitmap_words = z.nbmax * 4;
            sp->n.dense = nnz; sp->n.res = nnz;
        }
        fake.spmm.n.zero_rows = M;
        fake.spmm.n.tasks = 2 * z.tasks_a_max + 64;                                // the die-aware order may add empty tasks
        fake.sddmm.n.tasks = 2 * (z.tasks_d_max + nnz / o.sddmm_Cs + 1) + 64;
        *bytes = plan_buffer_bytes(&fake) + 2 * align256((size_t)M * 4 + 16);      // + the two row lists of the edge softmax
    } catch (...) {
        return LIBRA_ERR_NOMEM;
    }
    return LIBRA_OK;
}

extern "C" int libra_plan_device(int64_t M, int64_t Kc, int64_t nnz, const int32_t *d_rowptr, const int32_t *d_col, const void *d_val,
                                 int val_dtype, const libra_plan_opts_t *opts, void *workspace, size_t workspace_bytes,
                                 void *plan_buf, size_t plan_bytes, int keep_host_copy, void *stream, libra_plan_t **out) {
    if (!out) return LIBRA_ERR_NULL;
    *out = nullptr;
    if (!d_rowptr) return LIBRA_ERR_NULL;
    if (M < 1 || Kc < 1 || nnz < 0) return LIBRA_ERR_SHAPE;
    if (M >= (1ll << 31) - 64 || Kc >= (1ll << 31) || nnz >= (1ll << 31) - 64) return LIBRA_ERR_TOO_LARGE;
    if (val_dtype != LIBRA_F16 && val_dtype != LIBRA_BF16 && val_dtype != LIBRA_F32) return LIBRA_ERR_DTYPE;
    Resolved o{};
    if (int rc = resolve_options(opts, val_dtype, o)) return rc;
    if (o.W != W || o.KB != KB) return LIBRA_ERR_UNSUPPORTED;
    if (nnz > 0 && (!d_col || !d_val || !workspace)) return LIBRA_ERR_NULL;
    if (!plan_buf) keep_host_copy = 1;          // the plan has to live somewhere
    hipStream_t s = (hipStream_t)stream;
    const auto t0 = std::chrono::steady_clock::now();
    // LIBRA_TRACE=1 in the environment prints where the call's time goes (stderr)
    const bool trace = std::getenv("LIBRA_TRACE") != nullptr;
    auto mark = [&](const char *what) {
        if (trace) std::fprintf(stderr, "[libra_plan_device] %-28s %8.3f ms\n", what,
                                1e3 * std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count());
    };

    libra_plan_t *P = new (std::nothrow) libra_plan_t();
    if (!P) return LIBRA_ERR_NOMEM;
    try {
        P->M = M; P->Kc = Kc; P->nnz = nnz; P->vdt = val_dtype; P->vsize = val_dtype == LIBRA_F32 ? 4 : 2;
        P->o = o;
        fetch(P->rowptr, d_rowptr, (size_t)M + 1, s);
        hip_ok(hipStreamSynchronize(s));
        if (P->rowptr[0] != 0 || P->rowptr[M] != nnz) throw Fail{LIBRA_ERR_ROWPTR};
        for (int64_t i = 0; i < M; ++i)
            if (P->rowptr[i + 1] < P->rowptr[i]) throw Fail{LIBRA_ERR_ROWPTR};
        if (nnz == 0) {
            // nothing to sort or scan: the plan of a matrix without nonzeros (one empty task per window) needs no device work
            const std::vector<int32_t> rp = P->rowptr;
            delete P;
            int rc = libra_plan(M, Kc, rp.data(), nullptr, nullptr, val_dtype, opts, out);
            if (rc == LIBRA_OK && plan_buf && (rc = libra_plan_upload(*out, plan_buf, plan_bytes, stream)) != LIBRA_OK) {
                libra_plan_destroy(*out);
                *out = nullptr;
            }
            return rc;
        }
        mark("rowptr on the host, checked");
        const Sizes z = make_sizes(M, nnz, o);
        const Layout L = make_layout(z, P->vsize, workspace);
        if (((uintptr_t)workspace & 255) || workspace_bytes < L.total) throw Fail{LIBRA_ERR_BUFFER};
        const int n = (int)nnz, nw = (int)z.nw;
        const int vsize = P->vsize;
        const uint8_t *val = reinterpret_cast<const uint8_t *>(d_val);
        int colbits = 1;
        while ((1ll << colbits) < Kc) ++colbits;
        Rule R{o.mode, o.fill && o.mode == LIBRA_MODE_HYBRID ? 1 : 0, o.tau_sddmm, o.Ts, o.Cs, o.short_len, o.build_spmm ? 1 : 0, o.build_sddmm ? 1 : 0, o.sddmm_Ts};
        const int tau_a = o.mode == LIBRA_MODE_DENSE_ONLY ? 1 : o.mode == LIBRA_MODE_SCALAR_ONLY ? W + 1 : o.tau_spmm;

        // ---- 1. census: sort the nonzeros of every window by (column, row) ----
        fill_bytes(L.ctr, 0, C_COUNT * sizeof(u64), s);
        hipLaunchKernelGGL(k_win_ptr, dim3(blocks_for(nw + 1, 256)), dim3(256), 0, s, d_rowptr, M, nw, L.win_ptr);
        hipLaunchKernelGGL(k_keys, dim3(blocks_for(n, 256)), dim3(256), 0, s, d_rowptr, d_col, M, Kc, n, L.key_in, L.row_of, L.ctr);
        {
            size_t sz = L.tmp_bytes;
            hip_ok(rocprim::segmented_radix_sort_pairs(L.tmp, sz, L.key_in, L.key_out, rocprim::counting_iterator<int32_t>(0), L.spos,
                                                       (unsigned)n, (unsigned)nw, L.win_ptr, L.win_ptr + 1, 0, (unsigned)(colbits + 4), s));
        }
        // ---- 2. vectors ----
        hipLaunchKernelGGL(k_census, dim3(blocks_for(n, 256)), dim3(256), 0, s, L.key_out, L.win_ptr, nw, n, L.hflag, L.einfo, L.ewin);
        fill_bytes(L.hflag + n, 0, sizeof(int32_t), s);
        scan(L, L.hflag, L.vid, (size_t)n + 1, s);
        hipLaunchKernelGGL(k_vectors, dim3(blocks_for(n, 256)), dim3(256), 0, s, L.key_out, L.hflag, L.vid, L.einfo, L.ewin, n, tau_a, colbits,
                           L.vfirst, L.vinfo, L.vcol, L.vwin, L.tflag, L.key2_in, L.ctr);
        hipLaunchKernelGGL(k_win_vptr, dim3(blocks_for(nw + 1, 256)), dim3(256), 0, s, L.win_ptr, L.vid, nw, n, L.ctr, L.win_vptr);
        u64 ctr[C_COUNT];
        hip_ok(hipMemcpyAsync(ctr, L.ctr, sizeof ctr, hipMemcpyDeviceToHost, s));
        hip_ok(hipStreamSynchronize(s));
        if (hipGetLastError() != hipSuccess) throw Fail{LIBRA_ERR_HIP};
        if (ctr[C_ERR] & 1) throw Fail{LIBRA_ERR_COLUMN};
        if (ctr[C_ERR] & 2) throw Fail{LIBRA_ERR_UNSORTED};
        const int nv = (int)ctr[C_NV];
        if (nv < 1 || nv > n) throw Fail{LIBRA_ERR_HIP};
        mark("census (sort 1, vectors)");
        // order of a window's vectors: NNZ descending, column ascending
        {
            size_t sz = L.tmp_bytes;
            hip_ok(rocprim::segmented_radix_sort_pairs(L.tmp, sz, L.key2_in, L.key2_out, rocprim::counting_iterator<int32_t>(0), L.sv,
                                                       (unsigned)nv, (unsigned)nw, L.win_vptr, L.win_vptr + 1, 0, (unsigned)(colbits + 4), s));
        }
        hipLaunchKernelGGL(k_sorted, dim3(blocks_for(nv, 256)), dim3(256), 0, s, L.sv, L.vinfo, L.vwin, L.win_vptr, nv, L.scnt, L.srank);
        fill_bytes(L.scnt + nv, 0, sizeof(int32_t), s);
        fill_bytes(L.tflag + nv, 0, sizeof(int32_t), s);
        scan(L, L.scnt, L.cum, (size_t)nv + 1, s);
        scan(L, L.tflag, L.taud, (size_t)nv + 1, s);
        // ---- 3. per window: dense vectors and blocks ----
        hipLaunchKernelGGL(k_window_counts, dim3(blocks_for(nw, 256)), dim3(256), 0, s, L.win_vptr, L.taud, L.cum, nw, R,
                           L.ntau, L.a.ndv, L.a.nb, L.d.ndv, L.d.nb, L.ctr);
        if (o.build_sddmm && o.mode == LIBRA_MODE_HYBRID && o.sddmm_min_dense_pct > 0) {
            // the whole-matrix utilisation rule: too small a dense share sends the whole SDDMM sub-plan to the scalar path
            u64 dense_d = 0;
            hip_ok(hipMemcpyAsync(&dense_d, L.ctr + C_DNNZ_D, sizeof dense_d, hipMemcpyDeviceToHost, s));
            hip_ok(hipStreamSynchronize(s));
            if (share_rule_fires(o, (int64_t)dense_d, nnz)) {
                fill_bytes(L.d.nb, 0, (size_t)nw * sizeof(int32_t), s);
                fill_bytes(L.d.ndv, 0, (size_t)nw * sizeof(int32_t), s);
                fill_bytes(L.ctr + C_DV_D, 0, 2 * sizeof(u64), s);              // C_DV_D and C_PAD_D are neighbours
            }
        }
        fill_bytes(L.a.nb + nw, 0, sizeof(int32_t), s);
        fill_bytes(L.d.nb + nw, 0, sizeof(int32_t), s);
        scan(L, L.a.nb, L.a.blkptr, (size_t)nw + 1, s);
        scan(L, L.d.nb, L.d.blkptr, (size_t)nw + 1, s);
        const int nbA = peek(L.a.blkptr + nw, s), nbD = peek(L.d.blkptr + nw, s);
        if (nbA < 0 || nbD < 0 || nbA > z.nbmax || nbD > z.nbmax) throw Fail{LIBRA_ERR_HIP};
        mark("sort 2, window counts");
        // ---- 4. slots, blocks, packed values ----
        fill_bytes(L.a.slotvec, 0xff, (size_t)nbA * KB * sizeof(int32_t), s);
        fill_bytes(L.d.slotvec, 0xff, (size_t)nbD * KB * sizeof(int32_t), s);
        fill_bytes(L.a.dflag, 0, (size_t)nv, s);
        fill_bytes(L.d.dflag, 0, (size_t)nv, s);
        hipLaunchKernelGGL(k_slots, dim3(blocks_for(nv, 256)), dim3(256), 0, s, L.vwin, L.win_vptr, L.srank, L.taud, L.ntau, L.a.ndv, L.a.blkptr,
                           L.d.ndv, L.d.blkptr, nv, R, L.a.slotvec, L.a.dflag, L.d.slotvec, L.d.dflag);
        const int nbs[2] = {nbA, nbD};
        const SubOut *subs[2] = {&L.a, &L.d};
        for (int k = 0; k < 2; ++k) {
            const SubOut &S = *subs[k];
            const int nb = nbs[k];
            if (nb > 0)
                hipLaunchKernelGGL(k_blocks, dim3(blocks_for((int64_t)nb * 16, 256)), dim3(256), 0, s, S.slotvec, L.vcol, L.vinfo, nb,
                                   S.blk_cols, S.bitmap, S.blknnz, S.blkmask, S.blkncols);
            fill_bytes(S.blknnz + nb, 0, sizeof(int32_t), s);
            scan(L, S.blknnz, S.blk_valptr, (size_t)nb + 1, s);
            if (nb > 0)
                hipLaunchKernelGGL(k_block_values, dim3(blocks_for((int64_t)nb * 16, 256)), dim3(256), 0, s, S.slotvec, L.vfirst, L.vinfo, S.bitmap,
                                   S.blk_valptr, L.spos, val, vsize, nb, S.dense_perm, S.dense_val);
        }
        // ---- 5. residual nonzeros and tasks ----
        hipLaunchKernelGGL(k_entry_flags, dim3(blocks_for(n, 256)), dim3(256), 0, s, L.hflag, L.vid, L.spos, L.a.dflag, L.d.dflag, n, R, L.a.resf, L.d.resf);
        fill_bytes(L.a.resf + n, 0, sizeof(int32_t), s);
        fill_bytes(L.d.resf + n, 0, sizeof(int32_t), s);
        scan(L, L.a.resf, L.a.rescan, (size_t)n + 1, s);
        scan(L, L.d.resf, L.d.rescan, (size_t)n + 1, s);
        hipLaunchKernelGGL((k_window_tasks<false>), dim3(blocks_for(nw, 128)), dim3(128), 0, s, d_rowptr, L.a.rescan, M, nw, R,
                           L.a.blkptr, L.a.blkmask, L.a.blkncols, L.d.blkptr, L.d.blkncols,
                           L.a.ntasks, L.nzero, L.nres, L.d.ntasks, L.ctr, L.a.tbase, L.zbase, L.resptr, L.d.tbase,
                           L.a.tasks, L.zero_rows, L.d.tasks);
        for (int32_t *p : {L.a.ntasks, L.nzero, L.nres, L.d.ntasks}) fill_bytes(p + nw, 0, sizeof(int32_t), s);
        scan(L, L.a.ntasks, L.a.tbase, (size_t)nw + 1, s);
        scan(L, L.nzero, L.zbase, (size_t)nw + 1, s);
        scan(L, L.nres, L.resptr, (size_t)nw + 1, s);
        scan(L, L.d.ntasks, L.d.tbase, (size_t)nw + 1, s);
        const int ntA = peek(L.a.tbase + nw, s), ntD = peek(L.d.tbase + nw, s), nz = peek(L.zbase + nw, s);
        const int nresA = peek(L.a.rescan + n, s), nresD = peek(L.d.rescan + n, s);
        const int dnnzA = peek(L.a.blk_valptr + nbA, s), dnnzD = peek(L.d.blk_valptr + nbD, s);
        if (ntA < 0 || ntA > z.tasks_a_max || ntD < 0 || ntD > z.tasks_d_max || nz < 0 || nz > M || nresA < 0 || nresA > n || nresD < 0 ||
            nresD > n || dnnzA < 0 || dnnzA > n || dnnzD < 0 || dnnzD > n)
            throw Fail{LIBRA_ERR_HIP};
        hipLaunchKernelGGL((k_window_tasks<true>), dim3(blocks_for(nw, 128)), dim3(128), 0, s, d_rowptr, L.a.rescan, M, nw, R,
                           L.a.blkptr, L.a.blkmask, L.a.blkncols, L.d.blkptr, L.d.blkncols,
                           L.a.ntasks, L.nzero, L.nres, L.d.ntasks, L.ctr, L.a.tbase, L.zbase, L.resptr, L.d.tbase,
                           L.a.tasks, L.zero_rows, L.d.tasks);
        const int64_t ngroups = (nw + LIBRA_LOCALITY_WINDOWS - 1) / LIBRA_LOCALITY_WINDOWS, nsample = share_samples(ngroups);
        hipLaunchKernelGGL(k_share, dim3((unsigned)nsample, 16), dim3(256), 0, s, L.win_vptr, L.vcol, nw, ngroups, nsample, L.ctr);
        if (o.build_spmm)
            hipLaunchKernelGGL(k_row_bases, dim3(blocks_for(nw, 128)), dim3(128), 0, s, d_rowptr, L.a.rescan, L.resptr, M, nw, R, L.rowbase);
        hipLaunchKernelGGL(k_residual_fill, dim3(blocks_for(n, 256)), dim3(256), 0, s, d_col, val, vsize, n, R, L.row_of,
                           L.a.resf, L.a.rescan, L.rowbase, L.a.res_perm, L.a.res_row, L.a.res_col, L.a.res_val,
                           L.d.resf, L.d.rescan, L.d.res_perm, L.d.res_row, L.d.res_col, L.d.res_val);
        if (o.build_spmm && ntA > 0)
            hipLaunchKernelGGL(k_task_cols, dim3(blocks_for(ntA, 256)), dim3(256), 0, s, L.a.tasks, ntA, L.a.res_col, L.task_col);
        const int nsegD = o.build_sddmm ? (nresD + o.sddmm_Cs - 1) / o.sddmm_Cs : 0;
        if (nsegD > 0)
            hipLaunchKernelGGL(k_segment_cols, dim3(blocks_for(nsegD, 256)), dim3(256), 0, s, L.d.res_row, L.d.res_col, nresD, o.sddmm_Cs, nsegD, L.seg_col);
        hip_ok(hipMemcpyAsync(ctr, L.ctr, sizeof ctr, hipMemcpyDeviceToHost, s));
        hip_ok(hipStreamSynchronize(s));
        if (hipGetLastError() != hipSuccess) throw Fail{LIBRA_ERR_HIP};
        P->stats.device_seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
        mark("blocks, residual, tasks");

        // ---- sizes; the task tables always come to the host (their order is made there); the big arrays only on request ----
        SubPlan &sa = P->spmm, &sd = P->sddmm;
        const int nts[2] = {ntA, ntD}, nres2[2] = {nresA, nresD}, dn[2] = {dnnzA, dnnzD};
        SubPlan *hs[2] = {&sa, &sd};
        P->host_arrays = keep_host_copy != 0;
        for (int k = 0; k < 2; ++k) {
            if (!(k == 0 ? o.build_spmm : o.build_sddmm)) continue;
            const SubOut &S = *subs[k];
            SubPlan &H = *hs[k];
            H.n.blocks = nbs[k]; H.n.col_slots = (int64_t)nbs[k] * KB; H.n.bitmap_words = (int64_t)nbs[k] * 4;
            H.n.dense = dn[k]; H.n.res = nres2[k]; H.n.zero_rows = k == 0 ? nz : 0;
            fetch(H.tasks, S.tasks, (size_t)nts[k], s);
            if (k == 0) fetch(H.task_col, L.task_col, (size_t)nts[k], s);
            if (k == 1) fetch(H.seg_col, L.seg_col, (size_t)nsegD, s);
            fetch(H.blk_valptr, S.blk_valptr, (size_t)nbs[k] + 1, s);
            if (!keep_host_copy) continue;
            fetch(H.win_blkptr, S.blkptr, (size_t)nw + 1, s);
            fetch(H.blk_cols, S.blk_cols, (size_t)nbs[k] * KB, s);
            fetch(H.blk_bitmap, S.bitmap, (size_t)nbs[k] * 4, s);
            fetch(H.dense_perm, S.dense_perm, (size_t)dn[k], s);
            fetch(H.dense_val, S.dense_val, (size_t)dn[k] * vsize, s);
            fetch(H.res_perm, S.res_perm, (size_t)nres2[k], s);
            fetch(H.res_row, S.res_row, (size_t)nres2[k], s);
            fetch(H.res_col, S.res_col, (size_t)nres2[k], s);
            fetch(H.res_val, S.res_val, (size_t)nres2[k] * vsize, s);
        }
        if (o.build_spmm && keep_host_copy) {
            fetch(sa.win_resptr, L.resptr, (size_t)nw + 1, s);
            fetch(sa.zero_rows, L.zero_rows, (size_t)nz, s);
        }
        hip_ok(hipStreamSynchronize(s));
        sa.dense_vectors = (int64_t)ctr[C_DV_A]; sa.pad_slots = (int64_t)ctr[C_PAD_A];
        sd.dense_vectors = (int64_t)ctr[C_DV_D]; sd.pad_slots = (int64_t)ctr[C_PAD_D];
        sa.short_rows = (int64_t)ctr[C_SHORT]; sa.long_rows = (int64_t)ctr[C_LONG]; sa.split_rows = (int64_t)ctr[C_SPLIT];
        P->stats.n_vectors = nv;
        P->stats.n_vectors_nnz1 = (int64_t)ctr[C_NNZ1];
        mark("copies to the host");
        const int64_t share[2] = {(int64_t)ctr[C_TOGETHER], (int64_t)ctr[C_APART]};
        finish_plan(P, nullptr, share);
        mark("task order, statistics");
        if (plan_buf) {
            // the plan's device copy straight from the workspace: no round trip through host memory
            auto src = [&](const SubOut &S, const int32_t *zero_rows) {
                return DeviceSource{S.blk_cols, S.blk_valptr, S.dense_perm, S.res_perm, S.res_row, S.res_col, zero_rows,
                                    reinterpret_cast<const uint64_t *>(S.bitmap), S.dense_val, S.res_val};
            };
            if (int rc = adopt_device_arrays(P, src(L.a, L.zero_rows), src(L.d, nullptr), plan_buf, plan_bytes, stream)) throw Fail{rc};
        }
        mark("plan buffer written");
        P->stats.plan_seconds = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    } catch (const Fail &f) {
        (void)hipStreamSynchronize(s);       // queued passes may still use the workspace the caller is about to free
        delete P;
        return f.code;
    } catch (...) {
        (void)hipStreamSynchronize(s);
        delete P;
        return LIBRA_ERR_NOMEM;
    }
    *out = P;
    return LIBRA_OK;
}

// ------------------------------------------------------------------------------------------
// Transposition of a CSR pattern on the device (the backward pass of SpMM multiplies by the transposed matrix).
// ------------------------------------------------------------------------------------------
namespace {
// one wave per 16 rows: key = (column, CSR position); a sort by key lists the nonzeros column by column, rows ascending
__global__ __launch_bounds__(64) void k_transpose_keys(const int32_t *rowptr, const int32_t *col, int64_t M, u64 *key, int32_t *row_of) {
    const int64_t w = blockIdx.x;
    const int lane = threadIdx.x;
    for (int r = 0; r < W; ++r) {
        const int64_t i = w * W + r;
        if (i >= M) break;
        const int s = rowptr[i], e = rowptr[i + 1];
        for (int p = s + lane; p < e; p += 64) {
            key[p] = ((u64)(uint32_t)col[p] << 32) | (u64)(uint32_t)p;
            row_of[p] = (int32_t)i;
        }
    }
}
__global__ __launch_bounds__(256) void k_transpose_fill(const u64 *skey, const int32_t *row_of, int n, int32_t *col_t, int32_t *perm_t) {
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= n) return;
    const int p = (int)(skey[q] & 0xffffffffull);
    perm_t[q] = p;
    col_t[q] = row_of[p];
}
// rowptr_t[c] = first sorted position whose column is >= c
__global__ __launch_bounds__(256) void k_transpose_rowptr(const u64 *skey, int n, int64_t Kc, int32_t *rowptr_t) {
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c > Kc) return;
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if ((int64_t)(skey[mid] >> 32) < c) lo = mid + 1; else hi = mid;
    }
    rowptr_t[c] = lo;
}

struct TLayout { u64 *key_in, *key_out; int32_t *row_of; void *tmp; size_t tmp_bytes, total; };
TLayout transpose_layout(int64_t nnz, void *base) {
    TLayout L{};
    Arena A{(char *)base};
    const size_t n = (size_t)std::max<int64_t>(nnz, 1);
    L.key_in = A.take<u64>(n);
    L.key_out = A.take<u64>(n);
    L.row_of = A.take<int32_t>(n);
    size_t sz = 0;
    (void)rocprim::radix_sort_keys(nullptr, sz, (u64 *)nullptr, (u64 *)nullptr, n, 0, 64);
    L.tmp_bytes = sz + 4096;
    L.tmp = A.take<uint8_t>(L.tmp_bytes);
    L.total = align256(A.off) + 256;
    return L;
}
}  // namespace

extern "C" int libra_csr_transpose_workspace(int64_t nnz, size_t *bytes) {
    if (!bytes) return LIBRA_ERR_NULL;
    if (nnz < 0) return LIBRA_ERR_SHAPE;
    if (nnz >= (1ll << 31) - 64) return LIBRA_ERR_TOO_LARGE;
    *bytes = transpose_layout(nnz, nullptr).total;
    return LIBRA_OK;
}

namespace {
// The passes of the transposition on a workspace that is known to be large enough and aligned.  Only launches kernels
// and the sort on `s`; nothing is allocated and the stream is not synchronised.
int transpose_passes(int64_t M, int64_t Kc, int n, const int32_t *d_rowptr, const int32_t *d_col, int32_t *d_rowptr_t,
                     int32_t *d_col_t, int32_t *d_perm_t, const TLayout &L, hipStream_t s) {
    int colbits = 1;
    while ((1ll << colbits) < Kc) ++colbits;
    const int64_t nw = (M + W - 1) / W;
    hipLaunchKernelGGL(k_transpose_keys, dim3((unsigned)nw), dim3(64), 0, s, d_rowptr, d_col, M, L.key_in, L.row_of);
    size_t sz = L.tmp_bytes;
    if (rocprim::radix_sort_keys(L.tmp, sz, L.key_in, L.key_out, (size_t)n, 0, (unsigned)(32 + colbits), s) != hipSuccess) return LIBRA_ERR_HIP;
    hipLaunchKernelGGL(k_transpose_fill, dim3(blocks_for(n, 256)), dim3(256), 0, s, L.key_out, L.row_of, n, d_col_t, d_perm_t);
    hipLaunchKernelGGL(k_transpose_rowptr, dim3(blocks_for(Kc + 1, 256)), dim3(256), 0, s, L.key_out, n, Kc, d_rowptr_t);
    return hipGetLastError() == hipSuccess ? LIBRA_OK : LIBRA_ERR_HIP;
}

int transpose_args(int64_t M, int64_t Kc, int64_t nnz, const int32_t *d_rowptr, const int32_t *d_col, int32_t *d_rowptr_t,
                   int32_t *d_col_t, int32_t *d_perm_t) {
    if (!d_rowptr || !d_rowptr_t) return LIBRA_ERR_NULL;
    if (M < 1 || Kc < 1 || nnz < 0) return LIBRA_ERR_SHAPE;
    if (M >= (1ll << 31) - 64 || Kc >= (1ll << 31) - 64 || nnz >= (1ll << 31) - 64) return LIBRA_ERR_TOO_LARGE;
    if (nnz > 0 && (!d_col || !d_col_t || !d_perm_t)) return LIBRA_ERR_NULL;
    return LIBRA_OK;
}

// rowptr of a transposed matrix without nonzeros: Kc + 1 zeros, written by a kernel (a memset node in a captured graph
// is not reliable on replays)
__global__ __launch_bounds__(256) void k_zero_i32(int32_t *p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}
}  // namespace

extern "C" int libra_csr_transpose_device(int64_t M, int64_t Kc, int64_t nnz, const int32_t *d_rowptr, const int32_t *d_col,
                                          int32_t *d_rowptr_t, int32_t *d_col_t, int32_t *d_perm_t,
                                          void *workspace, size_t workspace_bytes, void *stream) {
    if (int rc = transpose_args(M, Kc, nnz, d_rowptr, d_col, d_rowptr_t, d_col_t, d_perm_t)) return rc;
    hipStream_t s = (hipStream_t)stream;
    if (nnz == 0) {
        hipLaunchKernelGGL(k_zero_i32, dim3(blocks_for(Kc + 1, 256)), dim3(256), 0, s, d_rowptr_t, Kc + 1);
        return hipGetLastError() == hipSuccess ? LIBRA_OK : LIBRA_ERR_HIP;
    }
    if (!workspace) return LIBRA_ERR_NULL;
    const TLayout L = transpose_layout(nnz, workspace);
    if (((uintptr_t)workspace & 255) || workspace_bytes < L.total) return LIBRA_ERR_BUFFER;
    if (int rc = transpose_passes(M, Kc, (int)nnz, d_rowptr, d_col, d_rowptr_t, d_col_t, d_perm_t, L, s)) return rc;
    if (hipStreamSynchronize(s) != hipSuccess) return LIBRA_ERR_HIP;     // the workspace may go now
    return LIBRA_OK;
}

// ------------------------------------------------------------------------------------------
// The same transposition for callers that cannot allocate: its workspace is a fixed array in device memory that every
// GPU the library runs on holds from the moment the code object is loaded until the process ends.
// ------------------------------------------------------------------------------------------
namespace {
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)LIBRA_TRANSPOSE_STATIC_MAX_NNZ * 40;      // keys in, keys out, rows, sort storage
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

// In host code the array's name stands for the symbol, not for device memory: its address on the current device comes from
// hipGetSymbolAddress, once per device (every GPU has its own copy at its own address).
constexpr int MAX_DEVICES = 64;
std::mutex scratch_mutex;
void *scratch_ptr[MAX_DEVICES];

int static_scratch(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return LIBRA_ERR_HIP;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LIBRA_ERR_HIP;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return LIBRA_OK;
}
}  // namespace

extern "C" int libra_csr_transpose_device_static(int64_t M, int64_t Kc, int64_t nnz, const int32_t *d_rowptr, const int32_t *d_col,
                                                 int32_t *d_rowptr_t, int32_t *d_col_t, int32_t *d_perm_t, void *stream) {
    if (int rc = transpose_args(M, Kc, nnz, d_rowptr, d_col, d_rowptr_t, d_col_t, d_perm_t)) return rc;
    if (nnz > LIBRA_TRANSPOSE_STATIC_MAX_NNZ) return LIBRA_ERR_TOO_LARGE;
    hipStream_t s = (hipStream_t)stream;
    if (nnz == 0) {
        hipLaunchKernelGGL(k_zero_i32, dim3(blocks_for(Kc + 1, 256)), dim3(256), 0, s, d_rowptr_t, Kc + 1);
        return hipGetLastError() == hipSuccess ? LIBRA_OK : LIBRA_ERR_HIP;
    }
    void *ws = nullptr;
    if (int rc = static_scratch(&ws)) return rc;
    const TLayout L = transpose_layout(nnz, ws);
    if (L.total > STATIC_SCRATCH_BYTES) return LIBRA_ERR_TOO_LARGE;      // the sort asked for more storage than the array was sized for
    // every array of the layout is written by a pass before a later pass reads it: nothing of the previous call's
    // contents is read, so nothing has to be cleared
    return transpose_passes(M, Kc, (int)nnz, d_rowptr, d_col, d_rowptr_t, d_col_t, d_perm_t, L, s);
}
