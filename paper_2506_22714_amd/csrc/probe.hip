// Register-only probe of matrix-core / vector-ALU concurrency (the experiment of Section 3.1 of the paper, which
// motivates running both units at once): the same workgroups run (a) MFMA chains on half of their waves, (b) FMA chains
// on the other half, (c) both.  If the two units run side by side, (c) takes about max(a, b); if they exclude each
// other, about a + b.  Nothing touches memory inside the loops.
#include <hip/hip_runtime.h>

#include "libra.h"

namespace {

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));

// 8 waves per workgroup = 2 per SIMD: waves 0..3 are the matrix-core waves, waves 4..7 the vector-ALU waves; each SIMD
// gets one of each.  mode bit 0: matrix-core waves work; bit 1: vector-ALU waves work.
__global__ __launch_bounds__(512) void coissue_kernel(int mode, int iters, float *sink) {
    const int wave = threadIdx.x >> 6;
    float result = 0.f;
    if (wave < 4) {
        if (mode & 1) {
            const half4_t a = {(_Float16)1.0f, (_Float16)0.5f, (_Float16)0.25f, (_Float16)(threadIdx.x & 3)};
            const half4_t b = {(_Float16)0.5f, (_Float16)1.0f, (_Float16)2.0f, (_Float16)(blockIdx.x & 1)};
            float4_t acc[4] = {{0, 0, 0, 0}, {1, 1, 1, 1}, {2, 2, 2, 2}, {3, 3, 3, 3}};
            for (int i = 0; i < iters; ++i) {
#pragma unroll
                for (int k = 0; k < 4; ++k) acc[k] = __builtin_amdgcn_mfma_f32_16x16x16f16(a, b, acc[k], 0, 0, 0);
            }
            result = acc[0][0] + acc[1][1] + acc[2][2] + acc[3][3];
        }
    } else if (mode & 2) {
        float x[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) x[k] = (float)(threadIdx.x + k);
        const float m = 1.0001f, c = 0.5f;
        for (int i = 0; i < iters; ++i) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int k = 0; k < 8; ++k) x[k] = fmaf(x[k], m, c);
        }
        result = x[0] + x[1] + x[2] + x[3] + x[4] + x[5] + x[6] + x[7];
    }
    if (result == 12345.678f) sink[0] = result;         // keeps the loops alive; practically never true
}

}  // namespace

extern "C" int libra_probe_coissue(int iters, float *sink_dev, float times_us[3], void *stream) {
    if (!sink_dev || !times_us) return LIBRA_ERR_NULL;
    if (iters < 1 || iters > (1 << 24)) return LIBRA_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess) return LIBRA_ERR_HIP;
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return LIBRA_ERR_HIP;
    }
    int rc = LIBRA_OK;
    for (int mode = 1; mode <= 3 && rc == LIBRA_OK; ++mode) {
        float best = 1e30f;
        for (int rep = 0; rep < 4; ++rep) {          // the first repetition warms up
            bool ok = hipEventRecord(e0, s) == hipSuccess;
            hipLaunchKernelGGL(coissue_kernel, dim3(1024), dim3(512), 0, s, mode, iters, sink_dev);
            ok = ok && hipGetLastError() == hipSuccess && hipEventRecord(e1, s) == hipSuccess && hipEventSynchronize(e1) == hipSuccess;
            float ms = 0.f;
            ok = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
            if (!ok) { rc = LIBRA_ERR_HIP; break; }
            if (rep > 0 && ms < best) best = ms;
        }
        times_us[mode - 1] = best * 1e3f;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}

// ---------------------------------------------------------------------------------------------------------------
// Bare gather: the row fetches of an SpMM / SDDMM call and nothing else.  Lane groups of ROW_BYTES / 16 lanes fetch row
// idx[i] of a table (16 bytes per lane, U rows in flight per group), fold what arrives into one register and never write.
// Its time is the floor of any kernel that has to bring these rows, in this order, from the caches and HBM into a compute
// unit - the measured ceiling the task kernels are compared with.
// ---------------------------------------------------------------------------------------------------------------
namespace {
constexpr int GATHER_PER_WAVE = 256;     // consecutive indices per wave, as long as a row segment of the plan's tasks

template <int ROW_BYTES, int U>
__global__ __launch_bounds__(64) void gather_kernel(const uint4 *table, const int32_t *idx, int64_t n, float *sink) {
    constexpr int LPR = ROW_BYTES / 16, GROUPS = 64 / LPR, PER_GROUP = GATHER_PER_WAVE / GROUPS;
    static_assert(PER_GROUP % U == 0, "whole batches");
    const int lane = threadIdx.x, sub = lane % LPR, grp = lane / LPR;
    const int64_t base = (int64_t)blockIdx.x * GATHER_PER_WAVE + grp * PER_GROUP;
    uint32_t acc = 0;
    for (int p = 0; p < PER_GROUP; p += U) {
        int32_t c[U];
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) c[u] = idx[min(base + p + u, n - 1)];          // the tail repeats the last index
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = table[(int64_t)c[u] * LPR + sub];
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x12345679u) sink[0] = 1.f;              // keeps the loads alive; practically never true
}

// The same fetches with the most popular rows resident in LDS (the data-reuse argument of Section 4.2.1 taken to the
// compute unit's own memory): persistent workgroups of 1024 threads, one per compute unit, copy rows hub_rows[0 .. H) of
// the table into LDS once; an index c >= 0 is fetched from the table as before, an index c < 0 reads slot ~c of the LDS
// copy.  Table rows go through buffer loads whose range is the table, so an index outside it reads zeros.
template <int ROW_BYTES, int U>
__global__ __launch_bounds__(1024) void gather_hub_kernel(const void *table, uint32_t table_bytes, const int32_t *idx, int64_t n,
                                                          const int32_t *hub_rows, int H, float *sink) {
    constexpr int LPR = ROW_BYTES / 16, GROUPS = 64 / LPR, PER_GROUP = GATHER_PER_WAVE / GROUPS;
    static_assert(PER_GROUP % U == 0, "whole batches");
    extern __shared__ uint4 hub[];
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(table), 0, (int)table_bytes, 0x00020000);
    const int tid = threadIdx.x;
    for (int i = tid; i < H * LPR; i += (int)blockDim.x) {
        const uint32_t hr = (uint32_t)hub_rows[i / LPR];
        const uint32_t off = hr < table_bytes / ROW_BYTES ? hr * (uint32_t)ROW_BYTES + (uint32_t)(i % LPR) * 16u : 0xfffffff0u;
        hub[i] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, 0));
    }
    __syncthreads();
    const int lane = tid & 63, sub = lane % LPR, grp = lane / LPR, wave = tid >> 6, waves = (int)blockDim.x >> 6;
    const int64_t nchunks = (n + GATHER_PER_WAVE - 1) / GATHER_PER_WAVE;
    uint32_t acc = 0;
    for (int64_t ch = (int64_t)blockIdx.x * waves + wave; ch < nchunks; ch += (int64_t)gridDim.x * waves) {
        const int64_t base = ch * GATHER_PER_WAVE + grp * PER_GROUP;
#pragma unroll 1
        for (int p = 0; p < PER_GROUP; p += U) {
            int32_t c[U];
            uint4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) c[u] = idx[min(base + p + u, n - 1)];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                // a hub entry gets an offset past the table: the load returns zeros and moves nothing
                const uint32_t off = (uint32_t)c[u] < table_bytes / ROW_BYTES ? (uint32_t)c[u] * (uint32_t)ROW_BYTES + (uint32_t)sub * 16u : 0xfffffff0u;
                v[u] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, 0));
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (c[u] < 0 && H > 0) {
                    const uint4 h = hub[min(~c[u], H - 1) * LPR + sub];
                    v[u].x |= h.x; v[u].y |= h.y; v[u].z |= h.z; v[u].w |= h.w;
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
        }
    }
    if (acc == 0x12345679u) sink[0] = 1.f;
}

template <int ROW_BYTES>
int launch_gather_hub(const void *table, uint32_t table_bytes, const int32_t *idx, int64_t n, const int32_t *hub_rows, int H,
                      float *sink, int cus, hipStream_t s) {
    const size_t lds = (size_t)H * ROW_BYTES;
    auto kernel = gather_hub_kernel<ROW_BYTES, 8>;
    if (lds > 48 * 1024 && hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
        return LIBRA_ERR_HIP;
    hipLaunchKernelGGL(kernel, dim3((unsigned)cus), dim3(1024), lds, s, table, table_bytes, idx, n, hub_rows, H, sink);
    return hipGetLastError() == hipSuccess ? LIBRA_OK : LIBRA_ERR_HIP;
}
}  // namespace

extern "C" int libra_probe_gather(const void *table_dev, int64_t table_rows, int32_t row_bytes, const int32_t *idx_dev, int64_t n,
                                  float *sink_dev, void *stream) {
    if (!table_dev || !idx_dev || !sink_dev) return LIBRA_ERR_NULL;
    if (table_rows < 1 || n < 1 || n > (1ll << 40)) return LIBRA_ERR_SHAPE;
    if (((uintptr_t)table_dev & 15) || ((uintptr_t)idx_dev & 3)) return LIBRA_ERR_BUFFER;
    hipStream_t s = (hipStream_t)stream;
    const int64_t waves = (n + GATHER_PER_WAVE - 1) / GATHER_PER_WAVE;
    if (waves >= (1ll << 31)) return LIBRA_ERR_TOO_LARGE;
    const uint4 *t = reinterpret_cast<const uint4 *>(table_dev);
    const dim3 grid((unsigned)waves), block(64);
    switch (row_bytes) {
    case 64: hipLaunchKernelGGL((gather_kernel<64, 8>), grid, block, 0, s, t, idx_dev, n, sink_dev); break;
    case 128: hipLaunchKernelGGL((gather_kernel<128, 8>), grid, block, 0, s, t, idx_dev, n, sink_dev); break;
    case 256: hipLaunchKernelGGL((gather_kernel<256, 8>), grid, block, 0, s, t, idx_dev, n, sink_dev); break;
    default: return LIBRA_ERR_UNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? LIBRA_OK : LIBRA_ERR_HIP;
}

extern "C" int libra_probe_gather_hub(const void *table_dev, int64_t table_rows, int32_t row_bytes, const int32_t *idx_dev, int64_t n,
                                      const int32_t *hub_rows_dev, int32_t n_hub, float *sink_dev, void *stream) {
    if (!table_dev || !idx_dev || !sink_dev || (n_hub > 0 && !hub_rows_dev)) return LIBRA_ERR_NULL;
    if (table_rows < 1 || n < 1 || n > (1ll << 40) || n_hub < 0) return LIBRA_ERR_SHAPE;
    if (row_bytes != 64 && row_bytes != 128 && row_bytes != 256) return LIBRA_ERR_UNSUPPORTED;
    if (((uintptr_t)table_dev & 15) || ((uintptr_t)idx_dev & 3)) return LIBRA_ERR_BUFFER;
    if (table_rows * row_bytes >= (1ll << 32) - 16 || (int64_t)n_hub * row_bytes > LIBRA_PROBE_HUB_MAX_BYTES) return LIBRA_ERR_TOO_LARGE;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return LIBRA_ERR_HIP;
    hipStream_t s = (hipStream_t)stream;
    const uint32_t bytes = (uint32_t)(table_rows * row_bytes);
    switch (row_bytes) {
    case 64: return launch_gather_hub<64>(table_dev, bytes, idx_dev, n, hub_rows_dev, n_hub, sink_dev, cus, s);
    case 128: return launch_gather_hub<128>(table_dev, bytes, idx_dev, n, hub_rows_dev, n_hub, sink_dev, cus, s);
    default: return launch_gather_hub<256>(table_dev, bytes, idx_dev, n, hub_rows_dev, n_hub, sink_dev, cus, s);
    }
}
