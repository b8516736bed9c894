// gfx950 kernels and the compute half of the C ABI.
//
// One wavefront (64 lanes) owns one task of the plan's task table.
//
//   SpMM window task   dense blocks -> v_mfma_f32_16x16x16_f16 (A tile decoded from the
//                      block bitmap in registers, gathered B rows transposed through LDS),
//                      accumulators parked in an LDS C tile; then every row of the window
//                      is finished on the VALU: tile row + residual nonzeros, one coalesced
//                      store (or fp32 atomics for rows that have other writers).
//   SpMM chunk task    a segment of a decomposed long row, VALU, atomics.
//   SDDMM window task  X window x gathered Y rows on v_mfma_f32_16x16x32_f16 (both operands
//                      are contiguous along K, so they load straight into MFMA layout),
//                      sampled through the bitmap, write offsets by popcount.
//   SDDMM chunk task   per-nonzero dot products on the VALU with a cross-lane reduction.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <vector>

#include "plan_internal.h"

using namespace libra;

typedef _Float16 half_t;
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));

namespace {

constexpr int WAVE = 64;
constexpr int W = 16;    // window height the kernels are written for
constexpr int KB = 16;   // block width the kernels are written for

struct SpmmArgs {
    const libra_task_t *tasks;
    const int32_t *blk_cols;
    const uint64_t *blk_bitmap;
    const int32_t *blk_valptr;
    const void *dense_val;
    const int32_t *res_rowptr;
    const int32_t *res_col;
    const void *res_val;
    const void *B;
    float *C;
    int64_t ldb, ldc;
    int64_t M;
};

// 8 consecutive elements of a dense-operand row, widened to fp32.
template <class T> struct Row8;
template <> struct Row8<half_t> {
    static constexpr int PER_LANE = 8;
    __device__ static void load(const void *base, int64_t elem_off, float (&f)[8]) {
        half8_t h = *reinterpret_cast<const half8_t *>(reinterpret_cast<const half_t *>(base) + elem_off);
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = (float)h[e];
    }
    __device__ static float val(const void *base, int64_t i) { return (float)reinterpret_cast<const half_t *>(base)[i]; }
};
template <> struct Row8<float> {
    static constexpr int PER_LANE = 4;
    __device__ static void load(const void *base, int64_t elem_off, float (&f)[8]) {
        float4_t v = *reinterpret_cast<const float4_t *>(reinterpret_cast<const float *>(base) + elem_off);
#pragma unroll
        for (int e = 0; e < 4; ++e) f[e] = v[e];
    }
    __device__ static float val(const void *base, int64_t i) { return reinterpret_cast<const float *>(base)[i]; }
};

// ---------------------------------------------------------------------------------------
// SpMM.  N = feature columns handled by this launch, T = storage type of values and B.
// ---------------------------------------------------------------------------------------
template <class T, int N, bool DENSE>
__global__ __launch_bounds__(WAVE) void spmm_task_kernel(SpmmArgs a) {
    using R = Row8<T>;
    constexpr int PL = R::PER_LANE;          // elements of a row per lane
    constexpr int LPR = N / PL;              // lanes per row
    constexpr int RPW = WAVE / LPR;          // rows per wave pass
    static_assert(LPR >= 1 && LPR <= WAVE && WAVE % LPR == 0, "unsupported N");
    constexpr int LDC = N + 4;               // fp32 C tile row stride (floats)
    constexpr int LDB = N + 4;               // fp16 B stage row stride (halves): rows 4 apart land 8 banks apart
    __shared__ __attribute__((aligned(16))) float lds_c[(DENSE ? W : (RPW < 1 ? 1 : RPW)) * LDC];
    __shared__ __attribute__((aligned(16))) half_t lds_b[DENSE ? KB * LDB : 8];

    const libra_task_t t = a.tasks[blockIdx.x];
    const int lane = threadIdx.x;
    const int sub = lane % LPR;              // which PL-wide piece of the row
    const int grp = lane / LPR;              // which row of the pass

    if (t.kind == LIBRA_TASK_CHUNK) {
        // ---- a segment of a decomposed long row: groups stride over it, reduce in LDS, atomics ----
        float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int p = t.begin + grp; p < t.end; p += RPW) {
            const int64_t c = a.res_col[p];
            const float v = R::val(a.res_val, p);
            float b[8];
            R::load(a.B, c * a.ldb + sub * PL, b);
#pragma unroll
            for (int e = 0; e < PL; ++e) acc[e] = fmaf(v, b[e], acc[e]);
        }
#pragma unroll
        for (int e = 0; e < PL; ++e) lds_c[grp * LDC + sub * PL + e] = acc[e];
        __syncthreads();
        float *crow = a.C + (int64_t)t.id * a.ldc;
        for (int f = lane; f < N; f += WAVE) {
            float s = 0.f;
#pragma unroll
            for (int q = 0; q < RPW; ++q) s += lds_c[q * LDC + f];
            atomicAdd(crow + f, s);
        }
        return;
    }

    const int w = t.id;
    bool have_tile = false;
    if constexpr (DENSE) {
        if (t.end > t.begin) {
            have_tile = true;
            constexpr int NT = N / 16;
            const int g = lane >> 4, j = lane & 15;
            float4_t acc[NT];
#pragma unroll
            for (int n = 0; n < NT; ++n) acc[n] = float4_t{0.f, 0.f, 0.f, 0.f};
            for (int b = t.begin; b < t.end; ++b) {
                // gather the block's B rows into LDS (padding slots become zero rows)
#pragma unroll
                for (int k0 = 0; k0 < KB; k0 += RPW) {
                    const int k = k0 + grp;
                    if (RPW <= KB || k < KB) {
                        const int c = a.blk_cols[(int64_t)b * KB + k];
                        uint4 raw = make_uint4(0u, 0u, 0u, 0u);
                        if (c >= 0)
                            raw = *reinterpret_cast<const uint4 *>(reinterpret_cast<const half_t *>(a.B) + (int64_t)c * a.ldb + sub * 8);
                        uint2 *dst = reinterpret_cast<uint2 *>(&lds_b[k * LDB + sub * 8]);
                        dst[0] = make_uint2(raw.x, raw.y);
                        dst[1] = make_uint2(raw.z, raw.w);
                    }
                }
                // decode this lane's 4 A elements (row j, slots 4g..4g+3) from the bitmap
                const uint64_t *bm = a.blk_bitmap + (int64_t)b * 4;
                const int q = j >> 2;
                const uint64_t word = bm[q];
                int prefix = 0;
                if (q > 0) prefix += __popcll(bm[0]);
                if (q > 1) prefix += __popcll(bm[1]);
                if (q > 2) prefix += __popcll(bm[2]);
                const int bitpos = (j & 3) * 16 + 4 * g;
                prefix += __popcll(word & ((1ull << bitpos) - 1ull));
                const unsigned nib = (unsigned)(word >> bitpos) & 0xFu;
                const half_t *vals = reinterpret_cast<const half_t *>(a.dense_val) + a.blk_valptr[b] + prefix;
                half4_t af;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    af[e] = (nib >> e & 1u) ? vals[__popc(nib & ((1u << e) - 1u))] : (half_t)0;
                __syncthreads();
#pragma unroll
                for (int n = 0; n < NT; ++n) {
                    half4_t bf;
#pragma unroll
                    for (int e = 0; e < 4; ++e) bf[e] = lds_b[(4 * g + e) * LDB + 16 * n + j];
                    acc[n] = __builtin_amdgcn_mfma_f32_16x16x16f16(af, bf, acc[n], 0, 0, 0);
                }
                __syncthreads();
            }
            // park the accumulators: lane (g, j) holds rows 4g..4g+3, feature 16n + j
#pragma unroll
            for (int n = 0; n < NT; ++n)
#pragma unroll
                for (int e = 0; e < 4; ++e) lds_c[(4 * g + e) * LDC + 16 * n + j] = acc[n][e];
            __syncthreads();
        }
    }

    // ---- finish every row of the window on the VALU ----
    const uint32_t active = t.store_mask | t.atomic_mask;
    for (int r0 = 0; r0 < W; r0 += RPW) {
        const int r = r0 + grp;
        if (r >= W || !(active >> r & 1u)) continue;
        const int64_t row = (int64_t)w * W + r;
        float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (have_tile) {
#pragma unroll
            for (int e = 0; e < PL; ++e) acc[e] = lds_c[r * LDC + sub * PL + e];
        }
        if (t.scalar_mask >> r & 1u) {
            int p = a.res_rowptr[row];
            const int pe = a.res_rowptr[row + 1];
            for (; p + 4 <= pe; p += 4) {
                int64_t c[4];
                float v[4], b[4][8];
#pragma unroll
                for (int u = 0; u < 4; ++u) { c[u] = a.res_col[p + u]; v[u] = R::val(a.res_val, p + u); }
#pragma unroll
                for (int u = 0; u < 4; ++u) R::load(a.B, c[u] * a.ldb + sub * PL, b[u]);
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int e = 0; e < PL; ++e) acc[e] = fmaf(v[u], b[u][e], acc[e]);
            }
            for (; p < pe; ++p) {
                const int64_t c = a.res_col[p];
                const float v = R::val(a.res_val, p);
                float b[8];
                R::load(a.B, c * a.ldb + sub * PL, b);
#pragma unroll
                for (int e = 0; e < PL; ++e) acc[e] = fmaf(v, b[e], acc[e]);
            }
        }
        float *dst = a.C + row * a.ldc + sub * PL;
        if (t.store_mask >> r & 1u) {
            *reinterpret_cast<float4_t *>(dst) = float4_t{acc[0], acc[1], acc[2], acc[3]};
            if (PL == 8) *reinterpret_cast<float4_t *>(dst + 4) = float4_t{acc[4], acc[5], acc[6], acc[7]};
        } else {
#pragma unroll
            for (int e = 0; e < PL; ++e) atomicAdd(dst + e, acc[e]);
        }
    }
}

// Clear the rows that several tasks accumulate into.
__global__ __launch_bounds__(256) void zero_rows_kernel(const int32_t *rows, int64_t nrows, float *C, int64_t ldc, int n4) {
    const int64_t total = nrows * n4;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = i / n4;
        const int c4 = (int)(i - r * n4);
        *reinterpret_cast<float4_t *>(C + (int64_t)rows[r] * ldc + c4 * 4) = float4_t{0.f, 0.f, 0.f, 0.f};
    }
}

// ---------------------------------------------------------------------------------------
// SDDMM
// ---------------------------------------------------------------------------------------
struct SddmmArgs {
    const libra_task_t *tasks;
    const int32_t *blk_cols;
    const uint64_t *blk_bitmap;
    const int32_t *blk_valptr;
    const void *dense_val;
    const int32_t *dense_perm;
    const int32_t *res_row;
    const int32_t *res_col;
    const void *res_val;
    const int32_t *res_perm;
    const void *X;
    const void *Y;
    float *out;
    int64_t M;
};

template <int K>
__global__ __launch_bounds__(WAVE) void sddmm_window_kernel(SddmmArgs a) {
    constexpr int KS = K / 32;               // MFMA k-steps
    const libra_task_t t = a.tasks[blockIdx.x];
    const int lane = threadIdx.x;
    const int g = lane >> 4, j = lane & 15;
    const half_t *X = reinterpret_cast<const half_t *>(a.X);
    const half_t *Y = reinterpret_cast<const half_t *>(a.Y);
    // A operand: row j of the window, k = 32*s + 8g .. +7 (rows past M repeat the last row; never sampled)
    int64_t xr = (int64_t)t.id * W + j;
    if (xr >= a.M) xr = a.M - 1;
    half8_t xa[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) xa[s] = *reinterpret_cast<const half8_t *>(X + xr * K + 32 * s + 8 * g);
    for (int b = t.begin; b < t.end; ++b) {
        int c = a.blk_cols[(int64_t)b * KB + j];
        if (c < 0) c = 0;                    // padding slot: no bit is set in its column
        float4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            half8_t yb = *reinterpret_cast<const half8_t *>(Y + (int64_t)c * K + 32 * s + 8 * g);
            d = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[s], yb, d, 0, 0, 0);
        }
        // lane (g, j) holds D[4g+e][j]; rows 4g..4g+3 are word g of the bitmap, bit e*16 + j
        const uint64_t *bm = a.blk_bitmap + (int64_t)b * 4;
        const uint64_t word = bm[g];
        int prefix = a.blk_valptr[b];
        if (g > 0) prefix += __popcll(bm[0]);
        if (g > 1) prefix += __popcll(bm[1]);
        if (g > 2) prefix += __popcll(bm[2]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int bit = e * 16 + j;
            if (word >> bit & 1ull) {
                const int slot = prefix + __popcll(word & ((1ull << bit) - 1ull));
                a.out[a.dense_perm[slot]] = (float)reinterpret_cast<const half_t *>(a.dense_val)[slot] * d[e];
            }
        }
    }
}

template <class T, int K>
__global__ __launch_bounds__(WAVE) void sddmm_chunk_kernel(SddmmArgs a) {
    using R = Row8<T>;
    constexpr int PL = R::PER_LANE;
    constexpr int LPN = K / PL;              // lanes per nonzero
    constexpr int NPW = WAVE / LPN;          // nonzeros per wave pass
    static_assert(LPN >= 1 && LPN <= WAVE, "unsupported K");
    const libra_task_t t = a.tasks[blockIdx.x];
    const int lane = threadIdx.x;
    const int sub = lane % LPN, grp = lane / LPN;
    for (int q0 = t.begin; q0 < t.end; q0 += NPW) {
        const int q = q0 + grp;
        float s = 0.f;
        if (q < t.end) {
            float x[8], y[8];
            R::load(a.X, (int64_t)a.res_row[q] * K + sub * PL, x);
            R::load(a.Y, (int64_t)a.res_col[q] * K + sub * PL, y);
#pragma unroll
            for (int e = 0; e < PL; ++e) s = fmaf(x[e], y[e], s);
        }
#pragma unroll
        for (int m = 1; m < LPN; m <<= 1) s += __shfl_xor(s, m, WAVE);
        if (q < t.end && sub == 0) a.out[a.res_perm[q]] = R::val(a.res_val, q) * s;
    }
}

// ---------------------------------------------------------------------------------------
// Edge softmax (one wave per row, rows dealt round-robin) and value scatter
// ---------------------------------------------------------------------------------------
__device__ inline float wave_max(float v) {
#pragma unroll
    for (int m = 1; m < WAVE; m <<= 1) v = fmaxf(v, __shfl_xor(v, m, WAVE));
    return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int m = 1; m < WAVE; m <<= 1) v += __shfl_xor(v, m, WAVE);
    return v;
}

template <class TO>
__global__ __launch_bounds__(256) void edge_softmax_kernel(const int32_t *rowptr, int64_t M, const float *score, float scale, TO *out) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t i = wave; i < M; i += nwaves) {
        const int s = rowptr[i], e = rowptr[i + 1];
        if (s == e) continue;
        float mx = -INFINITY;
        for (int p = s + lane; p < e; p += WAVE) mx = fmaxf(mx, scale * score[p]);
        mx = wave_max(mx);
        float den = 0.f;
        for (int p = s + lane; p < e; p += WAVE) den += __expf(scale * score[p] - mx);
        den = wave_sum(den);
        const float inv = 1.f / den;
        for (int p = s + lane; p < e; p += WAVE) out[p] = (TO)(__expf(scale * score[p] - mx) * inv);
    }
}

template <class T>
__global__ __launch_bounds__(256) void gather_values_kernel(const T *src, const int32_t *perm, int64_t n, T *dst) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        dst[i] = src[perm[i]];
}

inline int hip_rc(hipError_t e) { return e == hipSuccess ? LIBRA_OK : LIBRA_ERR_HIP; }

template <class T, int N, bool DENSE>
int launch_spmm(const SpmmArgs &a, int64_t ntasks, hipStream_t s) {
    if (ntasks == 0) return LIBRA_OK;
    hipLaunchKernelGGL((spmm_task_kernel<T, N, DENSE>), dim3((unsigned)ntasks), dim3(WAVE), 0, s, a);
    return hip_rc(hipGetLastError());
}

int spmm_piece(const libra_plan_t *P, const void *B, int n, int64_t ldb, float *C, int64_t ldc, hipStream_t s) {
    const SubPlan &sp = P->spmm;
    SpmmArgs a{sp.dev.tasks, sp.dev.blk_cols, sp.dev.blk_bitmap, sp.dev.blk_valptr, sp.dev.dense_val,
               sp.dev.res_rowptr, sp.dev.res_col, sp.dev.res_val, B, C, ldb, ldc, P->M};
    if (!sp.zero_rows.empty()) {
        const int64_t total = (int64_t)sp.zero_rows.size() * (n / 4);
        const unsigned blocks = (unsigned)std::min<int64_t>((total + 255) / 256, 65536);
        hipLaunchKernelGGL(zero_rows_kernel, dim3(blocks), dim3(256), 0, s, sp.dev.zero_rows, (int64_t)sp.zero_rows.size(), C, ldc, n / 4);
        if (hipGetLastError() != hipSuccess) return LIBRA_ERR_HIP;
    }
    const int64_t nt = (int64_t)sp.tasks.size();
    if (P->vdt == LIBRA_F16) {
        switch (n) {
        case 32: return launch_spmm<half_t, 32, true>(a, nt, s);
        case 64: return launch_spmm<half_t, 64, true>(a, nt, s);
        case 128: return launch_spmm<half_t, 128, true>(a, nt, s);
        case 256: return launch_spmm<half_t, 256, true>(a, nt, s);
        }
    } else {
        switch (n) {
        case 16: return launch_spmm<float, 16, false>(a, nt, s);
        case 32: return launch_spmm<float, 32, false>(a, nt, s);
        case 64: return launch_spmm<float, 64, false>(a, nt, s);
        case 128: return launch_spmm<float, 128, false>(a, nt, s);
        case 256: return launch_spmm<float, 256, false>(a, nt, s);
        }
    }
    return LIBRA_ERR_UNSUPPORTED;
}

}  // namespace

// =========================================================================================
// C ABI: upload and compute
// =========================================================================================
namespace {
struct Slot { const void *src; size_t bytes; const void **dst; };

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

template <class V> Slot slot(const V &v, const void **dst) { return {v.data(), v.size() * sizeof(v[0]), dst}; }

void collect(libra_plan_t *P, std::vector<Slot> &s) {
    s.push_back(slot(P->rowptr, (const void **)&P->d_rowptr));
    for (SubPlan *sp : {&P->spmm, &P->sddmm}) {
        SubPlanDev &d = sp->dev;
        s.push_back(slot(sp->tasks, (const void **)&d.tasks));
        s.push_back(slot(sp->win_blkptr, (const void **)&d.win_blkptr));
        s.push_back(slot(sp->blk_cols, (const void **)&d.blk_cols));
        s.push_back(slot(sp->blk_bitmap, (const void **)&d.blk_bitmap));
        s.push_back(slot(sp->blk_valptr, (const void **)&d.blk_valptr));
        s.push_back(slot(sp->dense_val, (const void **)&d.dense_val));
        s.push_back(slot(sp->dense_perm, (const void **)&d.dense_perm));
        s.push_back(slot(sp->res_rowptr, (const void **)&d.res_rowptr));
        s.push_back(slot(sp->res_row, (const void **)&d.res_row));
        s.push_back(slot(sp->res_col, (const void **)&d.res_col));
        s.push_back(slot(sp->res_val, (const void **)&d.res_val));
        s.push_back(slot(sp->res_perm, (const void **)&d.res_perm));
        s.push_back(slot(sp->zero_rows, (const void **)&d.zero_rows));
    }
}
}  // namespace

extern "C" int libra_plan_device_bytes(const libra_plan_t *plan, size_t *bytes) {
    if (!plan || !bytes) return LIBRA_ERR_NULL;
    std::vector<Slot> s;
    collect(const_cast<libra_plan_t *>(plan), s);
    size_t total = 256;
    for (auto &x : s) total += align256(x.bytes + 16);     // 16 spare bytes: vector loads may read past a tail
    *bytes = total;
    return LIBRA_OK;
}

extern "C" int libra_plan_upload(libra_plan_t *plan, void *dev_buf, size_t bytes, void *stream) {
    if (!plan || !dev_buf) return LIBRA_ERR_NULL;
    size_t need = 0;
    libra_plan_device_bytes(plan, &need);
    if (bytes < need || ((uintptr_t)dev_buf & 255)) return LIBRA_ERR_BUFFER;
    hipStream_t s = (hipStream_t)stream;
    std::vector<Slot> slots;
    collect(plan, slots);
    size_t off = 0;
    for (auto &x : slots) {
        char *dst = (char *)dev_buf + off;
        *x.dst = dst;
        if (x.bytes && hipMemcpyAsync(dst, x.src, x.bytes, hipMemcpyHostToDevice, s) != hipSuccess) return LIBRA_ERR_HIP;
        off += align256(x.bytes + 16);
    }
    if (hipStreamSynchronize(s) != hipSuccess) return LIBRA_ERR_HIP;
    plan->dev_base = dev_buf;
    plan->dev_bytes = bytes;
    return LIBRA_OK;
}

extern "C" int libra_spmm(const libra_plan_t *P, const void *B, int32_t N, int64_t ldb, float *C, int64_t ldc, void *stream) {
    if (!P || !B || !C) return LIBRA_ERR_NULL;
    if (!P->o.build_spmm) return LIBRA_ERR_NOT_BUILT;
    if (!P->dev_base) return LIBRA_ERR_NOT_UPLOADED;
    if (P->o.W != W || P->o.KB != KB) return LIBRA_ERR_UNSUPPORTED;
    const int unit = P->vdt == LIBRA_F16 ? 32 : 16;
    if (N < unit || N > 512) return LIBRA_ERR_SHAPE;
    if (N % unit) return LIBRA_ERR_UNSUPPORTED;
    if (ldb < N || ldc < N) return LIBRA_ERR_SHAPE;
    if (ldb % (P->vdt == LIBRA_F16 ? 8 : 4) || ldc % 4) return LIBRA_ERR_UNSUPPORTED;
    if (((uintptr_t)B & 15) || ((uintptr_t)C & 15)) return LIBRA_ERR_BUFFER;
    hipStream_t s = (hipStream_t)stream;
    const int esz = P->vsize;
    // the feature dimension is cut into pieces the kernels are instantiated for
    for (int n0 = 0; n0 < N;) {
        int n = 256;
        while (n > N - n0) n >>= 1;
        int rc = spmm_piece(P, (const char *)B + (size_t)n0 * esz, n, ldb, C + n0, ldc, s);
        if (rc != LIBRA_OK) return rc;
        n0 += n;
    }
    return LIBRA_OK;
}

extern "C" int libra_sddmm(const libra_plan_t *P, const void *X, const void *Y, int32_t K, float *out, void *stream) {
    if (!P || !X || !Y) return LIBRA_ERR_NULL;
    if (!out && P->nnz > 0) return LIBRA_ERR_NULL;           // a matrix without nonzeros has no output
    if (!P->o.build_sddmm) return LIBRA_ERR_NOT_BUILT;
    if (!P->dev_base) return LIBRA_ERR_NOT_UPLOADED;
    if (P->o.W != W || P->o.KB != KB) return LIBRA_ERR_UNSUPPORTED;
    if (K <= 0) return LIBRA_ERR_SHAPE;
    if (K != 32 && K != 64 && K != 128) return LIBRA_ERR_UNSUPPORTED;
    if (((uintptr_t)X & 15) || ((uintptr_t)Y & 15) || ((uintptr_t)out & 3)) return LIBRA_ERR_BUFFER;
    hipStream_t s = (hipStream_t)stream;
    const SubPlan &sp = P->sddmm;
    SddmmArgs a{sp.dev.tasks, sp.dev.blk_cols, sp.dev.blk_bitmap, sp.dev.blk_valptr, sp.dev.dense_val, sp.dev.dense_perm,
                sp.dev.res_row, sp.dev.res_col, sp.dev.res_val, sp.dev.res_perm, X, Y, out, P->M};
    // window tasks come first in the table, residual segments after them
    const int64_t nw = sp.n_window_tasks, nc = sp.n_chunk_tasks;
    if (nw > 0) {
        if (P->vdt != LIBRA_F16) return LIBRA_ERR_UNSUPPORTED;
        switch (K) {
        case 32: hipLaunchKernelGGL((sddmm_window_kernel<32>), dim3((unsigned)nw), dim3(WAVE), 0, s, a); break;
        case 64: hipLaunchKernelGGL((sddmm_window_kernel<64>), dim3((unsigned)nw), dim3(WAVE), 0, s, a); break;
        case 128: hipLaunchKernelGGL((sddmm_window_kernel<128>), dim3((unsigned)nw), dim3(WAVE), 0, s, a); break;
        }
        if (hipGetLastError() != hipSuccess) return LIBRA_ERR_HIP;
    }
    if (nc > 0) {
        a.tasks = sp.dev.tasks + nw;
        if (P->vdt == LIBRA_F16) {
            switch (K) {
            case 32: hipLaunchKernelGGL((sddmm_chunk_kernel<half_t, 32>), dim3((unsigned)nc), dim3(WAVE), 0, s, a); break;
            case 64: hipLaunchKernelGGL((sddmm_chunk_kernel<half_t, 64>), dim3((unsigned)nc), dim3(WAVE), 0, s, a); break;
            case 128: hipLaunchKernelGGL((sddmm_chunk_kernel<half_t, 128>), dim3((unsigned)nc), dim3(WAVE), 0, s, a); break;
            }
        } else {
            switch (K) {
            case 32: hipLaunchKernelGGL((sddmm_chunk_kernel<float, 32>), dim3((unsigned)nc), dim3(WAVE), 0, s, a); break;
            case 64: hipLaunchKernelGGL((sddmm_chunk_kernel<float, 64>), dim3((unsigned)nc), dim3(WAVE), 0, s, a); break;
            case 128: hipLaunchKernelGGL((sddmm_chunk_kernel<float, 128>), dim3((unsigned)nc), dim3(WAVE), 0, s, a); break;
            }
        }
        if (hipGetLastError() != hipSuccess) return LIBRA_ERR_HIP;
    }
    return LIBRA_OK;
}

extern "C" int libra_edge_softmax(const libra_plan_t *P, const float *scores, float scale, void *vals_out, int out_dtype, void *stream) {
    if (!P) return LIBRA_ERR_NULL;
    if ((!scores || !vals_out) && P->nnz > 0) return LIBRA_ERR_NULL;
    if (out_dtype != LIBRA_F16 && out_dtype != LIBRA_F32) return LIBRA_ERR_DTYPE;
    if (!P->dev_base) return LIBRA_ERR_NOT_UPLOADED;
    hipStream_t s = (hipStream_t)stream;
    const unsigned blocks = (unsigned)std::min<int64_t>((P->M + 3) / 4, 1 << 16);
    if (out_dtype == LIBRA_F16)
        hipLaunchKernelGGL((edge_softmax_kernel<half_t>), dim3(blocks), dim3(256), 0, s, P->d_rowptr, P->M, scores, scale, (half_t *)vals_out);
    else
        hipLaunchKernelGGL((edge_softmax_kernel<float>), dim3(blocks), dim3(256), 0, s, P->d_rowptr, P->M, scores, scale, (float *)vals_out);
    return hip_rc(hipGetLastError());
}

extern "C" int libra_plan_set_values(libra_plan_t *P, const void *vals, int dtype, void *stream) {
    if (!P) return LIBRA_ERR_NULL;
    if (!vals && P->nnz > 0) return LIBRA_ERR_NULL;
    if (dtype != P->vdt) return LIBRA_ERR_DTYPE;
    if (!P->dev_base) return LIBRA_ERR_NOT_UPLOADED;
    hipStream_t s = (hipStream_t)stream;
    for (SubPlan *sp : {&P->spmm, &P->sddmm}) {
        struct { const int32_t *perm; void *dst; int64_t n; } seg[2] = {
            {sp->dev.dense_perm, sp->dev.dense_val, (int64_t)sp->dense_perm.size()},
            {sp->dev.res_perm, sp->dev.res_val, (int64_t)sp->res_perm.size()}};
        for (auto &g : seg) {
            if (g.n == 0) continue;
            const unsigned blocks = (unsigned)std::min<int64_t>((g.n + 255) / 256, 1 << 16);
            if (dtype == LIBRA_F16)
                hipLaunchKernelGGL((gather_values_kernel<half_t>), dim3(blocks), dim3(256), 0, s, (const half_t *)vals, g.perm, g.n, (half_t *)g.dst);
            else
                hipLaunchKernelGGL((gather_values_kernel<float>), dim3(blocks), dim3(256), 0, s, (const float *)vals, g.perm, g.n, (float *)g.dst);
            if (hipGetLastError() != hipSuccess) return LIBRA_ERR_HIP;
        }
    }
    return LIBRA_OK;
}
