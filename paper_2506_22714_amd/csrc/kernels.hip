// gfx950 kernels and the compute half of the C ABI.
//
// One wavefront (64 lanes) owns one task of the plan's task table.
//
//   SpMM task    dense blocks -> v_mfma_f32_16x16x16_f16: the A tile is decoded from the block
//                bitmap in registers (Section 4.4 of the paper), the gathered B rows are staged
//                in LDS and read back in MFMA operand layout with ds_read_b64_tr_b16.  The
//                accumulators are parked in an fp32 LDS tile of the window.  The residual
//                nonzeros of the task are then cut into equal contiguous runs, one per lane
//                group; a group keeps a row's partial sum in registers and adds it into the LDS
//                tile when the row changes.  Finally the tile is written once: plain coalesced
//                stores for rows this task owns, fp32 atomics for rows with other writers.
//                A segment of a decomposed long row is the same task with no blocks and one
//                atomic output row.
//   SDDMM window task  X window x gathered Y rows on v_mfma_f32_16x16x32_f16 (both operands are
//                contiguous along K, so they load straight into MFMA layout), sampled through
//                the bitmap, write offsets by popcount.
//   SDDMM segment task per-nonzero dot products on the VALU with a cross-lane reduction.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <type_traits>
#include <vector>

#include "plan_internal.h"

using namespace libra;

typedef _Float16 half_t;
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef short short8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf8_t __attribute__((ext_vector_type(8)));
struct bf16_t { uint16_t bits; };     // bfloat16 storage: the upper half of a binary32

namespace {

constexpr int WAVE = 64;
constexpr int W = 16;    // window height the kernels are written for
constexpr int KB = 16;   // block width the kernels are written for

// SDDMM window tasks take their dense blocks in groups of SD_GROUP; the 16-bit output records of a group are stored in
// ascending CSR position with the LDS stage slot of their product (see sddmm_window_task).
constexpr int SD_GROUP = 4;
__host__ __device__ inline int sd_stage_slot(int block_in_group, int row, int slot) {
    return block_in_group * 256 + (row % 4) * 64 + (row / 4) * 16 + slot;
}
inline bool sorted_records(const libra_plan_t *P) { return P->vdt != LIBRA_F32 && P->o.W == W && P->o.KB == KB; }

struct SpmmArgs {
    const DevTask *tasks;
    const int32_t *blk_cols;
    const uint64_t *blk_bitmap;
    const int32_t *blk_valptr;
    const void *dense_val;
    const void *res_ent;
    const void *B;
    float *C;
    int64_t ldb, ldc;
    int32_t tasks_per_die;  // the table holds die k's tasks (dispatch positions k, k + 8, ...) contiguously from k * tasks_per_die on
    int32_t pieces;         // the launch covers `pieces` adjacent column pieces of N features each: every task runs once per piece
    int32_t phase;          // 0: a task does all its work; 1: dense blocks only; 2: residual nonzeros only, added to what phase 1 wrote
};

// Per storage type: how a lane reads its piece of a dense-operand row and a residual entry.
template <class T> struct Elem;
template <> struct Elem<half_t> {
    static constexpr int PER_LANE = 8;                   // 16 bytes
    typedef uint4 raw_t;
    typedef uint16_t val_t;                              // a residual entry's value as stored
    static constexpr int VALS_PER_WORD = 2;
    __device__ static raw_t load(const void *base, int64_t elem_off) {
        return *reinterpret_cast<const uint4 *>(reinterpret_cast<const half_t *>(base) + elem_off);
    }
    __device__ static void fma(float v, const raw_t &r, float (&acc)[8]) {
        half8_t h;
        __builtin_memcpy(&h, &r, 16);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf(v, (float)h[e], acc[e]);
    }
    __device__ static float dot(const raw_t &x, const raw_t &y, float s) {
        half8_t a, b;
        __builtin_memcpy(&a, &x, 16);
        __builtin_memcpy(&b, &y, 16);
#pragma unroll
        for (int e = 0; e < 8; ++e) s = fmaf((float)a[e], (float)b[e], s);
        return s;
    }
    __device__ static float pair_lo(uint32_t w) {
        const uint16_t lo = (uint16_t)(w & 0xffffu);
        half_t h;
        __builtin_memcpy(&h, &lo, 2);
        return (float)h;
    }
    __device__ static float pair_hi(uint32_t w) {
        const uint16_t hi = (uint16_t)(w >> 16);
        half_t h;
        __builtin_memcpy(&h, &hi, 2);
        return (float)h;
    }
    __device__ static void mask(raw_t &r, uint32_t keep) { r.x &= keep; r.y &= keep; r.z &= keep; r.w &= keep; }
    // the lane's 16 bytes of row `col`: one 32x32->64 multiply-add for the address
    __device__ static raw_t load_row(const void *base, int32_t col, uint32_t ld_bytes, int sub) {
        const char *p = reinterpret_cast<const char *>(base) + ((uint64_t)(uint32_t)col * ld_bytes + (uint32_t)sub * 16u);
        return *reinterpret_cast<const uint4 *>(p);
    }
    __device__ static float word_val(uint32_t bits) {
        const uint16_t lo = (uint16_t)bits;
        half_t h;
        __builtin_memcpy(&h, &lo, 2);
        return (float)h;
    }
};
template <> struct Elem<bf16_t> : Elem<half_t> {
    // same 16-byte pieces and 2-byte entry values as binary16; only the widening differs (a shift)
    __device__ static float widen(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
    __device__ static void fma(float v, const raw_t &r, float (&acc)[8]) {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc[2 * e] = fmaf(v, __uint_as_float(w[e] << 16), acc[2 * e]);
            acc[2 * e + 1] = fmaf(v, __uint_as_float(w[e] & 0xffff0000u), acc[2 * e + 1]);
        }
    }
    __device__ static float dot(const raw_t &x, const raw_t &y, float s) {
        const uint32_t a[4] = {x.x, x.y, x.z, x.w}, b[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            s = fmaf(__uint_as_float(a[e] << 16), __uint_as_float(b[e] << 16), s);
            s = fmaf(__uint_as_float(a[e] & 0xffff0000u), __uint_as_float(b[e] & 0xffff0000u), s);
        }
        return s;
    }
    __device__ static float pair_lo(uint32_t w) { return __uint_as_float(w << 16); }
    __device__ static float pair_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
    __device__ static float word_val(uint32_t bits) { return widen(bits & 0xffffu); }
};
template <> struct Elem<float> {
    static constexpr int PER_LANE = 4;                   // 16 bytes
    typedef float4_t raw_t;
    typedef float val_t;
    static constexpr int VALS_PER_WORD = 1;
    __device__ static raw_t load(const void *base, int64_t elem_off) {
        return *reinterpret_cast<const float4_t *>(reinterpret_cast<const float *>(base) + elem_off);
    }
    __device__ static void fma(float v, const raw_t &r, float (&acc)[8]) {
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] = fmaf(v, r[e], acc[e]);
    }
    __device__ static float dot(const raw_t &x, const raw_t &y, float s) {
#pragma unroll
        for (int e = 0; e < 4; ++e) s = fmaf(x[e], y[e], s);
        return s;
    }
    __device__ static float pair_lo(uint32_t w) { return __uint_as_float(w); }
    __device__ static float pair_hi(uint32_t w) { return __uint_as_float(w); }
    __device__ static void mask(raw_t &r, uint32_t keep) {
#pragma unroll
        for (int e = 0; e < 4; ++e) r[e] = __uint_as_float(__float_as_uint(r[e]) & keep);
    }
    __device__ static raw_t load_row(const void *base, int32_t col, uint32_t ld_bytes, int sub) {
        const char *p = reinterpret_cast<const char *>(base) + ((uint64_t)(uint32_t)col * ld_bytes + (uint32_t)sub * 16u);
        return *reinterpret_cast<const float4_t *>(p);
    }
    __device__ static float word_val(uint32_t bits) { return __uint_as_float(bits); }
};

// NW 32-bit words from an LDS address aligned to their size (16 bytes from four words up): 16-byte reads issued back to
// back; every word then goes through an opaque move, so that it is read once and whole however its fields are used.
template <int NW>
__device__ inline void lds_words(const void *lds, uint32_t (&w)[NW]) {
    static_assert(NW == 2 || NW % 4 == 0, "8 bytes, or whole 16-byte reads");
    if constexpr (NW == 2) {
        const uint2 v = *reinterpret_cast<const uint2 *>(lds);
        w[0] = v.x; w[1] = v.y;
    } else {
#pragma unroll
        for (int k = 0; k < NW / 4; ++k) {
            const uint4 v = reinterpret_cast<const uint4 *>(lds)[k];
            w[4 * k] = v.x; w[4 * k + 1] = v.y; w[4 * k + 2] = v.z; w[4 * k + 3] = v.w;
        }
    }
#pragma unroll
    for (int k = 0; k < NW; ++k) asm volatile("" : "+v"(w[k]));
}
// entry i of the blocked layout: its word and its value
template <class V>
__device__ inline void load_blocked_entry(const void *base, int64_t i, uint32_t &word, V &val) {
    const char *blk = reinterpret_cast<const char *>(base) + (i / RES_BLOCK) * (RES_BLOCK * (4 + (int)sizeof(V)));
    const int slot = (int)(i % RES_BLOCK);
    word = reinterpret_cast<const uint32_t *>(blk)[slot];
    val = reinterpret_cast<const V *>(blk + RES_BLOCK * 4)[slot];
}

__device__ inline void global_add(float *p, float v) {
    __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One 16x16 tile step on the matrix cores for either 16-bit storage type; operands are passed as raw bits.
template <class T>
__device__ inline float4_t mfma_k16(short4_t a, short4_t b, float4_t c) {
    if constexpr (std::is_same<T, half_t>::value) {
        half4_t ha, hb;
        __builtin_memcpy(&ha, &a, 8);
        __builtin_memcpy(&hb, &b, 8);
        return __builtin_amdgcn_mfma_f32_16x16x16f16(ha, hb, c, 0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b, c, 0, 0, 0);
    }
}
template <class T>
__device__ inline float4_t mfma_k32(const uint4 &a, const uint4 &b, float4_t c) {
    if constexpr (std::is_same<T, half_t>::value) {
        half8_t ha, hb;
        __builtin_memcpy(&ha, &a, 16);
        __builtin_memcpy(&hb, &b, 16);
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(ha, hb, c, 0, 0, 0);
    } else {
        bf8_t ba, bb;
        __builtin_memcpy(&ba, &a, 16);
        __builtin_memcpy(&bb, &b, 16);
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(ba, bb, c, 0, 0, 0);
    }
}
// fp32 -> storage type of the softmax output (round to nearest even)
template <class TO> __device__ inline TO to_storage(float x) { return (TO)x; }
template <> __device__ inline bf16_t to_storage<bf16_t>(float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return bf16_t{(uint16_t)((u >> 16) | 0x40u)};      // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return bf16_t{(uint16_t)(u >> 16)};
}

// Workgroup b of a launch runs on die b mod 8, so the records of the tasks that one die runs are stored next to each
// other: a 128-byte line of the table then serves four consecutive workgroups of one die instead of four dies.
static_assert(LIBRA_XCDS == 8, "task_slot divides by the number of dies with a shift");
__device__ inline int64_t task_slot(unsigned b, int per_die) { return (int64_t)(b & (LIBRA_XCDS - 1)) * per_die + (b >> 3); }

// ---------------------------------------------------------------------------------------
// SpMM.  N = feature columns handled by this launch, T = storage type of values and B.
//
// A task is latency-bound unless few dependent memory round trips carry many row fetches, so
// the kernel is organised around round trips: (1) the task record; (2) all the metadata of the
// task at once - residual entries, block column ids, block bitmaps - staged in LDS; (3..) the
// B-row fetches in large batches whose addresses come from LDS, never from another global load.
// ---------------------------------------------------------------------------------------

// Orders the LDS accesses of one wavefront (the hardware runs a wave's LDS instructions in order;
// this only stops the compiler from moving them across the point).
__device__ inline void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

#ifndef SPMM_U
#define SPMM_U 8
#endif
// Register budget: a 128-column task is held to four waves per SIMD by its 10 KB of LDS anyway; narrower ones gain
// from six (community N=64: 176 -> 139 us, power-law N=64: 49 -> 45 us), which four fetches in flight per group allow.
template <class T, int N>
__global__ __launch_bounds__(WAVE) __attribute__((amdgpu_waves_per_eu(N >= 128 ? 4 : 6))) void spmm_task_kernel(SpmmArgs a) {
    using E = Elem<T>;
    typedef typename E::val_t val_t;
    constexpr bool F32 = std::is_same<T, float>::value;        // fp32 storage: v_mfma_f32_16x16x4_f32, operands straight from the stage
    constexpr bool DENSE = true;
    constexpr int PL = E::PER_LANE;          // elements of a row per lane
    constexpr int LPR = N / PL;              // lanes per row
    constexpr int RPW = WAVE / LPR;          // lane groups per wave
    static_assert(LPR >= 1 && LPR <= WAVE && WAVE % LPR == 0, "unsupported N");
    constexpr int LDC = N + 4;               // fp32 tile row stride (floats)
    constexpr int BPI = 1;                   // dense blocks staged in LDS at a time (the stage then fits inside the tile's bytes)
    constexpr int LDBS = N + 16;             // stage row stride in elements: 4 consecutive 16-bit rows / 2 consecutive fp32 rows cover all 32 banks
    constexpr int TILE_BYTES = W * LDC * 4;
    constexpr int STAGE_BYTES = DENSE ? BPI * KB * LDBS * (int)sizeof(T) : 0;
    constexpr int SMEM = TILE_BYTES > STAGE_BYTES ? TILE_BYTES : STAGE_BYTES;
    constexpr int ECAP = 128;                // residual entries staged per round
    constexpr int BCAP = 8;                  // dense blocks whose metadata is staged per round
    constexpr int U = N >= 128 ? SPMM_U : SPMM_U / 2;   // B-row fetches in flight per lane group (narrow rows: fewer, for more waves)
    // the B stage (dense phase) and the C tile (afterwards) share the same LDS bytes
    __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM];
    __shared__ __attribute__((aligned(16))) uint32_t ent_lds[ECAP];          // the staged entries' words (column | row in window) ...
    __shared__ __attribute__((aligned(16))) val_t val_lds[ECAP];             // ... and values
    __shared__ __attribute__((aligned(16))) int32_t cols_lds[DENSE ? BCAP * KB : 4];
    __shared__ __attribute__((aligned(16))) uint64_t bm_lds[DENSE ? WAVE : 2];   // BCAP * 4 words used
    float *tile = reinterpret_cast<float *>(smem);

    // workgroup b: die b mod 8, then the pieces of one task next to each other (they read the same plan data through
    // the same L2), then the die's next task
    const unsigned round = blockIdx.x >> 3, piece = round % (unsigned)a.pieces;
    const DevTask t = a.tasks[(int64_t)(blockIdx.x & (LIBRA_XCDS - 1)) * a.tasks_per_die + round / (unsigned)a.pieces];
    const char *Bp = reinterpret_cast<const char *>(a.B) + (size_t)piece * N * sizeof(T);
    float *Cp = a.C + (size_t)piece * N;
    const int lane = threadIdx.x;
    const int sub = lane % LPR;              // which PL-wide piece of a row
    const int grp = lane / LPR;              // which lane group
    const uint32_t atomic_mask = t.masks & 0xffffu, store_mask = t.masks >> 16;
    const uint32_t out_mask = atomic_mask | store_mask;
    // The two-kernel mode (the paper's sequential schedule of Section 4.4.1: matrix-unit part, then scalar part) runs
    // the table twice.  Phase 1 takes the tasks that have blocks and writes all their rows; phase 2 takes the tasks that
    // have residual nonzeros or own rows that phase 1 did not write, and adds to rows that phase 1 wrote.
    const int nblk_all = t.blk_end - t.blk_begin;
    if (a.phase == 1 && nblk_all == 0) return;
    const int nblk = a.phase == 2 ? 0 : nblk_all;
    const int L = a.phase == 1 ? 0 : t.res_end - t.res_begin;
    if (a.phase == 2 && nblk_all > 0 && L == 0) return;
    const bool add_to_c = a.phase == 2 && nblk_all > 0;
    const uint32_t ldb_bytes = (uint32_t)a.ldb * (uint32_t)sizeof(T);

    // ---- round trip 2: all metadata of the task (first round of each kind) ----
    // Loads are issued unconditionally from clamped (always valid) addresses and unused results are
    // masked afterwards: a load inside a branch makes the compiler wait for all earlier loads first.
    // First round of each kind of metadata, all loads in flight together, then the LDS writes.
    {
        const int nE = min(L, ECAP), nb = min(nblk, BCAP);
        uint32_t tmp[ECAP / WAVE];
        val_t tmp_val[ECAP / WAVE];
#pragma unroll
        for (int k = 0; k < ECAP / WAVE; ++k)
            load_blocked_entry(a.res_ent, (int64_t)t.res_begin + max(min(k * WAVE + lane, nE - 1), 0), tmp[k], tmp_val[k]);
        if constexpr (DENSE) {
            const int32_t *csrc = a.blk_cols + (int64_t)t.blk_begin * KB;
            int32_t c[BCAP * KB / WAVE];
#pragma unroll
            for (int k = 0; k < BCAP * KB / WAVE; ++k) c[k] = csrc[max(min(k * WAVE + lane, nb * KB - 1), 0)];
            const uint64_t w = a.blk_bitmap[(int64_t)t.blk_begin * 4 + max(min(lane, nb * 4 - 1), 0)];
#pragma unroll
            for (int k = 0; k < BCAP * KB / WAVE; ++k) cols_lds[k * WAVE + lane] = c[k];
            bm_lds[lane] = w;        // all 64 lanes write (the upper ones a copy of the last word): under a `lane < 32` branch
                                     // the compiler moves the load there too and issues it only after the loads before it returned
        }
#pragma unroll
        for (int k = 0; k < ECAP / WAVE; ++k) {
            ent_lds[k * WAVE + lane] = tmp[k];
            val_lds[k * WAVE + lane] = tmp_val[k];
        }
    }
    // later rounds of a task with more than BCAP blocks are fetched in place
    auto fetch_blocks = [&](int b0, int nb) {
        if constexpr (DENSE) {
            const int32_t *csrc = a.blk_cols + (int64_t)(t.blk_begin + b0) * KB;
            int32_t c[BCAP * KB / WAVE];
#pragma unroll
            for (int k = 0; k < BCAP * KB / WAVE; ++k) c[k] = csrc[min(k * WAVE + lane, nb * KB - 1)];
            const uint64_t w = a.blk_bitmap[(int64_t)(t.blk_begin + b0) * 4 + min(lane, nb * 4 - 1)];
#pragma unroll
            for (int k = 0; k < BCAP * KB / WAVE; ++k) cols_lds[k * WAVE + lane] = c[k];
            bm_lds[lane] = w;        // all 64 lanes write (the upper ones a copy of the last word): under a `lane < 32` branch
                                     // the compiler moves the load there too and issues it only after the loads before it returned
        }
    };
    wave_sync();

    bool tile_ready = false;
    if constexpr (DENSE) {
        if (nblk > 0) {
            tile_ready = true;
            constexpr int NT = N / 16;
            constexpr int PASSES = BPI * KB / RPW;               // wave loads per staged group of BPI blocks
            constexpr int H = (N <= 128 && !F32) ? 2 : 1;        // staged groups per round trip (more costs registers, i.e. waves)
            constexpr int FPI = BPI * H;                         // blocks fetched per round trip
            static_assert(BPI * KB % RPW == 0 && PASSES >= 1, "stage shape");
            typedef typename std::conditional<F32, float, uint16_t>::type stage_t;
            stage_t *stage = reinterpret_cast<stage_t *>(smem);
            const int g = lane >> 4, j = lane & 15;
            float4_t acc[NT];
#pragma unroll
            for (int n = 0; n < NT; ++n) acc[n] = float4_t{0.f, 0.f, 0.f, 0.f};
            int vbase = t.val_begin;                             // first packed value of the current block
            for (int b0 = 0; b0 < nblk; b0 += BCAP) {
                const int nbr = min(BCAP, nblk - b0);
                if (b0 > 0) {
                    wave_sync();
                    fetch_blocks(b0, nbr);
                    wave_sync();
                }
                for (int bb = 0; bb < nbr; bb += FPI) {
                    const int nb = min(FPI, nbr - bb);
                    // one round trip: the B rows of up to FPI blocks (padding slots become zero rows) ...
                    typename E::raw_t raw[H][PASSES];
                    int cc[H][PASSES];
                    // all column ids first (LDS reads back to back), then all fetches
#pragma unroll
                    for (int h = 0; h < H; ++h)
#pragma unroll
                        for (int ps = 0; ps < PASSES; ++ps)
                            cc[h][ps] = cols_lds[bb * KB + min(h * BPI * KB + ps * RPW + grp, nb * KB - 1)];
#pragma unroll
                    for (int h = 0; h < H; ++h)
#pragma unroll
                        for (int ps = 0; ps < PASSES; ++ps) {
                            const int k = h * BPI * KB + ps * RPW + grp;
                            const int c = cc[h][ps];
                            // a padding slot fetches row 0 and is cleared by a mask the compiler cannot see through
                            // (so that it keeps the fetch outside any branch)
                            uint32_t keep = (k < nb * KB && c >= 0) ? 0xffffffffu : 0u;
                            asm volatile("" : "+v"(keep));
                            raw[h][ps] = E::load_row(Bp, keep ? c : 0, ldb_bytes, sub);
                            E::mask(raw[h][ps], keep);
                        }
                    // ... and this lane's 4 A elements (row j, slots 4g..4g+3) of each block, decoded from its bitmap
                    typedef typename std::conditional<F32, float, short>::type aval_t;
                    typedef typename std::conditional<F32, float4_t, short4_t>::type afrag_t;
                    // All value loads of the FPI blocks are issued before any of them is used: unconditional loads (an unset
                    // slot reads a neighbouring value, at most 3 values past the array's end, inside its 16 spare bytes; a
                    // block past the last one repeats the last one), and the selects afterwards.  With two blocks per round
                    // trip an opaque move sits between the two: without it the compiler moves a load under its select's
                    // condition and waits block by block (community N=128 261 -> 255 us with it, GAT graph N=64 624 -> 581 us
                    // against the same code without it); with one block per round trip (fp32) it only forces the wait early
                    // (community 388 -> 436 us) and is left out.
                    afrag_t af[FPI];
                    typedef typename std::conditional<F32, float, int>::type areg_t;
                    areg_t av[FPI][4];
                    unsigned nib[FPI];
                    {
                        int vb = vbase;
#pragma unroll
                        for (int x = 0; x < FPI; ++x) {
                            const uint64_t *bm = &bm_lds[(bb + min(x, nb - 1)) * 4];
                            const uint64_t w0 = bm[0], w1 = bm[1], w2 = bm[2], w3 = bm[3];
                            const int q = j >> 2;
                            const uint64_t word = q == 0 ? w0 : q == 1 ? w1 : q == 2 ? w2 : w3;
                            const int c0 = __popcll(w0), c1 = __popcll(w1), c2 = __popcll(w2), c3 = __popcll(w3);
                            int prefix = (q > 0 ? c0 : 0) + (q > 1 ? c1 : 0) + (q > 2 ? c2 : 0);
                            const int bitpos = (j & 3) * 16 + 4 * g;
                            prefix += __popcll(word & ((1ull << bitpos) - 1ull));
                            nib[x] = x < nb ? (unsigned)(word >> bitpos) & 0xFu : 0u;
                            const aval_t *vals = reinterpret_cast<const aval_t *>(a.dense_val) + vb + prefix;
#pragma unroll
                            for (int e = 0; e < 4; ++e) av[x][e] = (areg_t)vals[__popc(nib[x] & ((1u << e) - 1u))];
                            if (x + 1 < nb) vb += c0 + c1 + c2 + c3;       // the next block's values follow; a repeated block re-reads its own
                            if (x < nb) vbase += c0 + c1 + c2 + c3;
                        }
                    }
#pragma unroll
                    for (int x = 0; x < FPI; ++x)
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if constexpr (FPI > 1) asm volatile("" : "+v"(av[x][e]));
#pragma unroll
                    for (int x = 0; x < FPI; ++x)
#pragma unroll
                        for (int e = 0; e < 4; ++e) af[x][e] = (nib[x] >> e & 1u) ? (aval_t)av[x][e] : (aval_t)0;
                    // the fetched rows go through the LDS stage BPI blocks at a time
#pragma unroll
                    for (int h = 0; h < H; ++h) {
                        if (h * BPI < nb) {
                            wave_sync();         // the previous operand reads are done
#pragma unroll
                            for (int ps = 0; ps < PASSES; ++ps) {
                                const int k = ps * RPW + grp;
                                *reinterpret_cast<typename E::raw_t *>(&stage[k * LDBS + sub * PL]) = raw[h][ps];
                            }
                            wave_sync();
#pragma unroll
                            for (int x = 0; x < BPI; ++x) {
                                if (h * BPI + x < nb) {
                                    if constexpr (F32) {
                                        // k-step e of the 16x16x4 product takes column slot 4g + e from lane group g (the same
                                        // slots as this lane's 4 A elements): B[4g+e][16n+j] is a plain 4-byte read
                                        const float *src = &stage[(x * KB + 4 * g) * LDBS + j];
#pragma unroll
                                        for (int n = 0; n < NT; ++n)
#pragma unroll
                                            for (int e = 0; e < 4; ++e)
                                                acc[n] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[h * BPI + x][e], src[e * LDBS + 16 * n], acc[n], 0, 0, 0);
                                    } else {
                                        // lane i of a 16-lane block points at row i/4, halves 4(i%4)..+3 of the 32-byte row piece;
                                        // the transposing read hands lane j the four rows' element j: B[4g+e][16n+j], e = 0..3
                                        const uint16_t *src = &stage[(x * KB + 4 * g + (j >> 2)) * LDBS + 4 * (j & 3)];
#pragma unroll
                                        for (int n = 0; n < NT; ++n) {
                                            const short4_t r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                                                (short4_t __attribute__((address_space(3))) *)(src + 16 * n));
                                            acc[n] = mfma_k16<T>(af[h * BPI + x], r, acc[n]);
                                        }
                                    }
                                }
                            }
                        }
                    }
                }
            }
            wave_sync();
            // park the accumulators: lane (g, j) holds rows 4g..4g+3, feature 16n + j
#pragma unroll
            for (int n = 0; n < NT; ++n)
#pragma unroll
                for (int e = 0; e < 4; ++e) tile[(4 * g + e) * LDC + 16 * n + j] = acc[n][e];
        }
    }
    constexpr int LPF = N / 4;                                   // lanes per tile row at 4 floats each
    constexpr int RPP = WAVE / LPF >= 1 ? WAVE / LPF : 1;        // tile rows per wave pass
    static_assert(LPF <= WAVE, "N too wide for one wave pass");
    const int rr = lane / LPF, cl = lane % LPF;
    if (!tile_ready) {
        // clear the output rows of the tile
#pragma unroll
        for (int r0 = 0; r0 < W; r0 += RPP) {
            const int r = r0 + rr;
            if (out_mask >> r & 1u) *reinterpret_cast<float4_t *>(&tile[r * LDC + cl * 4]) = float4_t{0.f, 0.f, 0.f, 0.f};
        }
    }
    wave_sync();

    // ---- residual nonzeros, ECAP per round: equal contiguous runs per lane group, row sums flushed into the tile ----
    for (int e0 = 0; e0 < L; e0 += ECAP) {
        const int nE = min(ECAP, L - e0);
        // the next round's entries go in flight now and wait in registers until this round is done
        const int nE_next = min(ECAP, L - e0 - ECAP);
        uint32_t next_ent[ECAP / WAVE];
        val_t next_val[ECAP / WAVE];
        if (nE_next > 0) {
#pragma unroll
            for (int k = 0; k < ECAP / WAVE; ++k)
                load_blocked_entry(a.res_ent, (int64_t)t.res_begin + e0 + ECAP + min(k * WAVE + lane, nE_next - 1), next_ent[k], next_val[k]);
        }
        // runs are whole batches of U entries (the longest run, which sets the time of the round, needs no more batches
        // for it), so a batch is U consecutive entries from an aligned base address and never leaves the staged array
        static_assert(ECAP % U == 0, "a batch must not straddle the end of the staged entries");
        const int per = ((nE + RPW - 1) / RPW + U - 1) / U * U;
        const int q0 = min(grp * per, nE);
        const int q1 = min(nE, q0 + per);
        // A row is added into the tile by the group that holds its first entry (plain read-add-write:
        // one owner per row).  A group whose run starts inside a row keeps that row's partial sum in
        // registers instead and adds it after the others, in group order, so the order of additions is fixed.
        bool first_is_shared = q0 > 0 && q0 < q1 && ((ent_lds[q0 - 1] ^ ent_lds[q0]) >> RES_ROW_SHIFT) == 0;
        int kept_row = -1;
        float kept[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        int cur = -1;
        float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        auto add_to_tile = [&](int r, const float (&v)[8]) {
#pragma unroll
            for (int e = 0; e < PL; e += 4) {
                float4_t *p = reinterpret_cast<float4_t *>(&tile[r * LDC + sub * PL + e]);
                float4_t x = *p;
                x[0] += v[e]; x[1] += v[e + 1]; x[2] += v[e + 2]; x[3] += v[e + 3];
                *p = x;
            }
        };
        auto flush = [&]() {
            if (first_is_shared) {
                first_is_shared = false;
                kept_row = cur;
#pragma unroll
                for (int e = 0; e < PL; ++e) kept[e] = acc[e];
            } else {
                add_to_tile(cur, acc);
            }
        };
        for (int q = q0; q < q1; q += U) {
            // all entry reads, then all row fetches, back to back
            typename E::raw_t raw[U];
            const bool full = q + U <= q1;
            // U consecutive entries from one aligned base address; slots past the run hold valid entries whose fetch is
            // harmless and whose product is never formed
            constexpr int VPW = E::VALS_PER_WORD;
            int ecol[U], erow[U];
            float eval[U];
            {
                uint32_t cr[U], vw[U / VPW];
                lds_words<U>(ent_lds + q, cr);
                lds_words<U / VPW>(val_lds + q, vw);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    ecol[u] = (int)(cr[u] & RES_COL_MASK);
                    erow[u] = (int)(cr[u] >> RES_ROW_SHIFT);
                    eval[u] = (u % VPW) ? E::pair_hi(vw[u / VPW]) : E::pair_lo(vw[u / VPW]);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) raw[u] = E::load_row(Bp, ecol[u], ldb_bytes, sub);
            bool one_row = full;
#pragma unroll
            for (int u = 1; u < U; ++u) one_row = one_row && erow[u] == erow[0];
            if (one_row) {
                // common case (long rows, segments of decomposed rows): the whole batch belongs to one row
                const int r = erow[0];
                if (r != cur) {
                    if (cur >= 0) flush();
#pragma unroll
                    for (int e = 0; e < PL; ++e) acc[e] = 0.f;
                    cur = r;
                }
#pragma unroll
                for (int u = 0; u < U; ++u) E::fma(eval[u], raw[u], acc);
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (q + u < q1) {
                        const int r = erow[u];
                        if (r != cur) {
                            if (cur >= 0) flush();
#pragma unroll
                            for (int e = 0; e < PL; ++e) acc[e] = 0.f;
                            cur = r;
                        }
                        E::fma(eval[u], raw[u], acc);
                    }
                }
            }
        }
        if (cur >= 0) flush();
        for (int gq = 1; gq < RPW; ++gq) {
            wave_sync();
            if (grp == gq && kept_row >= 0) add_to_tile(kept_row, kept);
        }
        if (nE_next > 0) {
            wave_sync();
#pragma unroll
            for (int k = 0; k < ECAP / WAVE; ++k) {
                ent_lds[k * WAVE + lane] = next_ent[k];
                val_lds[k * WAVE + lane] = next_val[k];
            }
            wave_sync();
        }
    }
    wave_sync();

    // ---- write the tile once: a wave pass covers RPP rows, LPF lanes per row ----
    {
        float *cbase = Cp + (int64_t)t.id * W * a.ldc;
#pragma unroll
        for (int r0 = 0; r0 < W; r0 += RPP) {
            const int r = r0 + rr;
            if (!(out_mask >> r & 1u)) continue;
            float *dst = cbase + (int64_t)r * a.ldc;
            if (store_mask >> r & 1u) {
                // streaming store: C is written once and not read again by this call
                float4_t x = *reinterpret_cast<const float4_t *>(&tile[r * LDC + cl * 4]);
                if (add_to_c) {           // stream order: phase 1 has written the row
                    const float4_t y = *reinterpret_cast<const float4_t *>(dst + cl * 4);
                    x[0] += y[0]; x[1] += y[1]; x[2] += y[2]; x[3] += y[3];
                }
                __builtin_nontemporal_store(x, reinterpret_cast<float4_t *>(dst + cl * 4));
            } else {
                // each atomic instruction covers LPF consecutive floats of the row
#pragma unroll
                for (int e = 0; e < 4; ++e) global_add(dst + e * LPF + cl, tile[r * LDC + e * LPF + cl]);
            }
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
    const DevTask *tasks;
    const int32_t *blk_cols;
    const uint64_t *blk_bitmap;
    const int32_t *blk_valptr;
    const uint2 *dense_pv;      // per packed dense nonzero: CSR position, value bits
    int32_t n_dense;
    const SdEnt *res_ent;
    const void *X;
    const void *Y;
    float *out;
    int64_t M;
    int32_t tasks_per_die;      // as in SpmmArgs
    int32_t pattern_only;       // nonzero: out_p = <X_i, Y_j>, A's values are not applied
};

// Sum over the LPN consecutive lanes of a group; every lane of the group gets the total.
// Steps inside a 16-lane row are DPP moves (no LDS traffic); wider groups finish with wave shuffles.
template <int LPN>
__device__ inline float group_sum(float s) {
    auto dpp = [](float v, auto ctrl) {
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), decltype(ctrl)::value, 0xf, 0xf, true));
    };
    if constexpr (LPN >= 2) s += dpp(s, std::integral_constant<int, 0xB1>{});      // quad_perm [1,0,3,2]
    if constexpr (LPN >= 4) s += dpp(s, std::integral_constant<int, 0x4E>{});      // quad_perm [2,3,0,1]
    if constexpr (LPN >= 8) s += dpp(s, std::integral_constant<int, 0x141>{});     // row_half_mirror
    if constexpr (LPN >= 16) s += dpp(s, std::integral_constant<int, 0x140>{});    // row_mirror
#pragma unroll
    for (int m = 16; m < LPN; m <<= 1) s += __shfl_xor(s, m, WAVE);
    return s;
}

// Dense blocks of one window: D = Xwin * Y[cols]^T on the MFMA (both operands are contiguous along K: 16-byte global
// loads straight into the operand registers).  The blocks of a task are taken in groups of SD_GROUP; a group's 16 x 16
// products go to an LDS stage as they come out of the matrix cores (slot sd_stage_slot(block, row, column slot): lane l
// writes its e-th accumulator of block x to x * 256 + e * 64 + l, no bank conflicts, no bitmap needed), and the group's
// output records - {CSR position, value | stage slot << 16}, stored at plan time in ascending CSR position inside every
// group - are then read by consecutive lanes: coalesced record loads, and stores that fall into the row-contiguous runs
// of the output instead of one 4-byte store per matrix-core lane (the write-back of Section 4.4.2, with the popcount
// offsets resolved when the plan is built).
template <class T, int K>
__device__ inline void sddmm_window_task(const SddmmArgs &a, const DevTask &t, float *stage) {
    constexpr int KS = K / 32;               // MFMA k-steps
    constexpr int BB = K <= 64 ? 4 : 2;      // blocks whose Y rows are in registers together
    constexpr int RU = 4;                    // record loads in flight per lane
    static_assert(SD_GROUP % BB == 0, "a group is whole register batches");
    const int lane = threadIdx.x % WAVE;
    const int g = lane >> 4, j = lane & 15;
    const uint16_t *X = reinterpret_cast<const uint16_t *>(a.X);
    const uint16_t *Y = reinterpret_cast<const uint16_t *>(a.Y);
    // A operand: row j of the window, k = 32*s + 8g .. +7 (rows past M repeat the last row; no record points at them)
    const int64_t xr = min((int64_t)t.id * W + j, a.M - 1);
    uint4 xa[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) xa[s] = *reinterpret_cast<const uint4 *>(X + xr * K + 32 * s + 8 * g);
    for (int b0 = t.blk_begin; b0 < t.blk_end; b0 += SD_GROUP) {
        const int nb = min(SD_GROUP, t.blk_end - b0);
        int col[SD_GROUP];
#pragma unroll
        for (int x = 0; x < SD_GROUP; ++x) col[x] = a.blk_cols[(int64_t)(b0 + min(x, nb - 1)) * KB + j];
        const int v0 = a.blk_valptr[b0], v1 = a.blk_valptr[b0 + nb];
        // the first records of the group travel with the Y rows
        uint2 rec[RU];
#pragma unroll
        for (int u = 0; u < RU; ++u) rec[u] = a.dense_pv[min(v0 + u * WAVE + lane, a.n_dense - 1)];
#pragma unroll
        for (int h = 0; h < SD_GROUP; h += BB) {
            if (h < nb) {
                uint4 yb[BB][KS];
#pragma unroll
                for (int x = 0; x < BB; ++x) {
                    const int c = max(col[h + x], 0);            // padding slot (or a block past the group): no record points at it
#pragma unroll
                    for (int s = 0; s < KS; ++s) yb[x][s] = *reinterpret_cast<const uint4 *>(Y + (int64_t)c * K + 32 * s + 8 * g);
                }
#pragma unroll
                for (int x = 0; x < BB; ++x) {
                    float4_t d = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s = 0; s < KS; ++s) d = mfma_k32<T>(xa[s], yb[x][s], d);
#pragma unroll
                    for (int e = 0; e < 4; ++e) stage[(h + x) * 256 + e * WAVE + lane] = d[e];
                }
            }
        }
        wave_sync();
        for (int q = v0; q < v1; q += RU * WAVE) {
            if (q > v0) {
#pragma unroll
                for (int u = 0; u < RU; ++u) rec[u] = a.dense_pv[min(q + u * WAVE + lane, a.n_dense - 1)];
            }
#pragma unroll
            for (int u = 0; u < RU; ++u)
                if (q + u * WAVE + lane < v1)
                    a.out[(int32_t)rec[u].x] = (a.pattern_only ? 1.f : Elem<T>::word_val(rec[u].y)) * stage[rec[u].y >> 16];
        }
        wave_sync();                         // the next group overwrites the stage
    }
}

// Residual nonzeros: LPN lanes per nonzero, NPW nonzeros per wave pass, U passes in one batch of loads.
// The same for fp32 storage: v_mfma_f32_16x16x4_f32.  A lane (g, j) fetches X[row j][16t + 4g .. +3] and Y[col j][16t + 4g .. +3] as
// 16-byte loads; k-step 4t + e of the product takes element e of both, i.e. lane group g contributes k = 16t + 4g + e to
// that step - any assignment of the k's to steps and lane groups gives the same sum as long as both operands use it.
// (fp32 records are 8 bytes of position and value with no room for a stage slot: they stay in bit order and this task keeps
// the per-lane popcount offsets and 4-byte stores.)
template <int K>
__device__ inline void sddmm_window_task_f32(const SddmmArgs &a, const DevTask &t) {
    constexpr int KT = K / 16;               // 16-byte pieces per lane and operand row
    constexpr int BB = K <= 32 ? 4 : K <= 64 ? 2 : 1;      // blocks per batch (register budget)
    const int lane = threadIdx.x % WAVE;
    const int g = lane >> 4, j = lane & 15;
    const float *X = reinterpret_cast<const float *>(a.X);
    const float *Y = reinterpret_cast<const float *>(a.Y);
    const int64_t xr = min((int64_t)t.id * W + j, a.M - 1);
    float4_t xa[KT];
#pragma unroll
    for (int s = 0; s < KT; ++s) xa[s] = *reinterpret_cast<const float4_t *>(X + xr * K + 16 * s + 4 * g);
    for (int b0 = t.blk_begin; b0 < t.blk_end; b0 += BB) {
        int col[BB], vptr[BB];
        uint64_t word[BB];
#pragma unroll
        for (int x = 0; x < BB; ++x) {
            const int b = min(b0 + x, t.blk_end - 1);
            col[x] = a.blk_cols[(int64_t)b * KB + j];
            word[x] = a.blk_bitmap[(int64_t)b * 4 + g];          // rows 4g..4g+3 of the block, bit e*16 + j
            vptr[x] = a.blk_valptr[b];
        }
        float4_t yb[BB][KT];
#pragma unroll
        for (int x = 0; x < BB; ++x) {
            const int c = max(col[x], 0);                        // padding slot: no bit is set in its column
#pragma unroll
            for (int s = 0; s < KT; ++s) yb[x][s] = *reinterpret_cast<const float4_t *>(Y + (int64_t)c * K + 16 * s + 4 * g);
        }
        int slot[BB][4];
#pragma unroll
        for (int x = 0; x < BB; ++x) {
            const int cnt = __popcll(word[x]);
            const int c0 = __builtin_amdgcn_readlane(cnt, 0), c1 = __builtin_amdgcn_readlane(cnt, 16), c2 = __builtin_amdgcn_readlane(cnt, 32);
            const int prefix = vptr[x] + (g > 0 ? c0 : 0) + (g > 1 ? c1 : 0) + (g > 2 ? c2 : 0);
#pragma unroll
            for (int e = 0; e < 4; ++e) slot[x][e] = prefix + __popcll(word[x] & ((1ull << (e * 16 + j)) - 1ull));
        }
        uint2 pv[BB][4];
#pragma unroll
        for (int x = 0; x < BB; ++x)
#pragma unroll
            for (int e = 0; e < 4; ++e) pv[x][e] = a.dense_pv[min(slot[x][e], a.n_dense - 1)];
        float4_t d[BB];
#pragma unroll
        for (int x = 0; x < BB; ++x) {
            d[x] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KT; ++s)
#pragma unroll
                for (int e = 0; e < 4; ++e) d[x] = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[s][e], yb[x][s][e], d[x], 0, 0, 0);
        }
#pragma unroll
        for (int x = 0; x < BB; ++x)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (b0 + x < t.blk_end && (word[x] >> (e * 16 + j) & 1ull))
                    a.out[(int32_t)pv[x][e].x] = (a.pattern_only ? 1.f : __uint_as_float(pv[x][e].y)) * d[x][e];
    }
}

template <class T, int K>
__device__ inline void sddmm_segment_task(const SddmmArgs &a, const DevTask &t) {
    using E = Elem<T>;
    constexpr int PL = E::PER_LANE;
    constexpr int LPN = K / PL;              // lanes per nonzero
    constexpr int NPW = WAVE / LPN;          // nonzeros per wave pass
    constexpr int U = LPN <= 8 ? 8 : 4;      // passes in flight
    static_assert(LPN >= 4 && LPN % 4 == 0 && LPN <= WAVE, "unsupported K (whole quads per nonzero)");
    const int lane = threadIdx.x % WAVE;
    const int sub = lane % LPN, grp = lane / LPN;
    for (int q0 = t.res_begin; q0 < t.res_end; q0 += NPW * U) {
        // An entry is 4 words (row, col, position, value bits).  Each lane of a quad fetches one of them (a quad then
        // costs the texture path 16 bytes instead of 64) and the quad shares them with DPP moves.
        uint32_t word[U];
        uint4 ent[U];
        typename E::raw_t x[U], y[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            word[u] = reinterpret_cast<const uint32_t *>(a.res_ent)[(int64_t)min(q0 + u * NPW + grp, t.res_end - 1) * 4 + (sub & 3)];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int w = (int)word[u];
            ent[u].x = (uint32_t)__builtin_amdgcn_update_dpp(0, w, 0x00, 0xf, 0xf, true);      // quad_perm [0,0,0,0]
            ent[u].y = (uint32_t)__builtin_amdgcn_update_dpp(0, w, 0x55, 0xf, 0xf, true);      // quad_perm [1,1,1,1]
            ent[u].z = (uint32_t)__builtin_amdgcn_update_dpp(0, w, 0xAA, 0xf, 0xf, true);      // quad_perm [2,2,2,2]
            ent[u].w = (uint32_t)__builtin_amdgcn_update_dpp(0, w, 0xFF, 0xf, 0xf, true);      // quad_perm [3,3,3,3]
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            x[u] = E::load(a.X, (int64_t)(int32_t)ent[u].x * K + sub * PL);
            y[u] = E::load(a.Y, (int64_t)(int32_t)ent[u].y * K + sub * PL);
        }
        float s[U];
#pragma unroll
        for (int u = 0; u < U; ++u) s[u] = group_sum<LPN>(E::dot(x[u], y[u], 0.f));
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (sub == 0 && q0 + u * NPW + grp < t.res_end) a.out[(int32_t)ent[u].z] = (a.pattern_only ? 1.f : E::word_val(ent[u].w)) * s[u];
    }
}

// One launch for both kinds of SDDMM task: the window tasks, heaviest first, then the residual segments.  A workgroup is
// WPB waves, each with a task of its own; nothing is shared between them but the compute unit.  Workgroup b runs on die
// b mod 8 and takes WPB consecutive tasks of that die's part of the table.  WPB = 4 is used when the table is in the
// die-aware order: its consecutive tasks are then neighbouring windows (or runs of consecutive segments) that read the
// same rows of Y, and four of them on one compute unit find each other's rows in its L1 (community matrix, K = 64:
// matrix-unit-only 249 -> 208 us, hybrid 265 -> 247 us, same box).  Elsewhere one wave per workgroup is better (power-law
// graph 31.0 vs 32.3 us: a workgroup's slots are only free again when its slowest wave has finished).
template <class T, int K, int WPB>
__global__ __launch_bounds__(WAVE * WPB) void sddmm_task_kernel(SddmmArgs a) {
    __shared__ float stage_all[std::is_same<T, float>::value ? 1 : WPB * SD_GROUP * 256];
    const unsigned wave = threadIdx.x / WAVE;
    const unsigned seq = (blockIdx.x >> 3) * WPB + wave;                // position in the die's part of the table
    if (seq >= (unsigned)a.tasks_per_die) return;
    const DevTask t = a.tasks[(int64_t)(blockIdx.x & (LIBRA_XCDS - 1)) * a.tasks_per_die + seq];
    if (t.kind == LIBRA_TASK_WINDOW) {
        if constexpr (std::is_same<T, float>::value) sddmm_window_task_f32<K>(a, t);
        else sddmm_window_task<T, K>(a, t, stage_all + wave * (SD_GROUP * 256));
        return;
    }
    sddmm_segment_task<T, K>(a, t);
}

// ---------------------------------------------------------------------------------------
// Edge softmax (one wave per row, rows dealt round-robin) and value scatter
// ---------------------------------------------------------------------------------------
// Maximum over a group of LPN (2, 4, 8 or 16) neighbouring lanes of a DPP row; every lane gets the result.
template <int LPN>
__device__ inline float group_max(float s) {
    static_assert(LPN == 2 || LPN == 4 || LPN == 8 || LPN == 16, "inside one DPP row");
    auto dpp = [](float v, auto ctrl) {
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), decltype(ctrl)::value, 0xf, 0xf, true));
    };
    if constexpr (LPN >= 2) s = fmaxf(s, dpp(s, std::integral_constant<int, 0xB1>{}));      // quad_perm [1,0,3,2]
    if constexpr (LPN >= 4) s = fmaxf(s, dpp(s, std::integral_constant<int, 0x4E>{}));      // quad_perm [2,3,0,1]
    if constexpr (LPN >= 8) s = fmaxf(s, dpp(s, std::integral_constant<int, 0x141>{}));     // row_half_mirror
    if constexpr (LPN >= 16) s = fmaxf(s, dpp(s, std::integral_constant<int, 0x140>{}));    // row_mirror
    return s;
}
constexpr int SHORT_LANES = 8;                  // lanes per row of up to 64 nonzeros
constexpr int SHORT_LOADS = 64 / SHORT_LANES;   // scores per lane


// Rows of up to 64 nonzeros (the bulk of a graph): SHORT_LANES lanes per row, read once and kept in registers.
template <class TO>
__device__ inline void edge_softmax_short_rows(unsigned block, unsigned nblocks, const int32_t *rowptr, int64_t M, const float *score, float scale, TO *out) {
    constexpr int SL = SHORT_LANES, KPL = SHORT_LOADS;
    const int l = threadIdx.x % SL;
    const int64_t group = ((int64_t)block * blockDim.x + threadIdx.x) / SL;
    const int64_t ngroups = ((int64_t)nblocks * blockDim.x) / SL;
    for (int64_t i = group; i < M; i += ngroups) {
        const int s = rowptr[i], n = rowptr[i + 1] - s;
        if (n == 0 || n > 64) continue;         // longer rows are listed at plan time and run below
        {
            float v[KPL];
#pragma unroll
            for (int k = 0; k < KPL; ++k) v[k] = score[s + min(l + SL * k, n - 1)];
            float mx = -INFINITY;
#pragma unroll
            for (int k = 0; k < KPL; ++k) {
                v[k] = l + SL * k < n ? scale * v[k] : -INFINITY;
                mx = fmaxf(mx, v[k]);
            }
            mx = group_max<SL>(mx);
            float den = 0.f;
#pragma unroll
            for (int k = 0; k < KPL; ++k) { v[k] = __expf(v[k] - mx); den += v[k]; }      // exp(-inf) = 0 for the padding
            const float inv = 1.f / group_sum<SL>(den);
#pragma unroll
            for (int k = 0; k < KPL; ++k)
                if (l + SL * k < n) out[s + l + SL * k] = to_storage<TO>(v[k] * inv);
        }
    }
}

// Rows listed at plan time: 65 .. LIBRA_SOFTMAX_LONG_ROW nonzeros, THREADS = MEDIUM_LANES lanes per row (whole groups
// of lanes inside a wave), and longer ones, one 256-thread workgroup per row.  A thread takes UNR scores per round, all loads in flight
// together; the row's maximum and denominator come from one pass (running maximum, sum rescaled when it grows); the second
// pass writes, from the registers if the whole row fitted one round and from a second read (cache) otherwise.
template <int THREADS>
__device__ inline float list_sum(float x, float *red) {
#pragma unroll
    for (int m = 1; m < (THREADS < WAVE ? THREADS : WAVE); m <<= 1) x += __shfl_xor(x, m, WAVE);
    if constexpr (THREADS > WAVE) {
        __syncthreads();                // earlier readers of `red` are done
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
        __syncthreads();
        x = 0.f;
#pragma unroll
        for (int w = 0; w < THREADS / WAVE; ++w) x += red[w];
    }
    return x;
}
template <int THREADS>
__device__ inline float list_max(float x, float *red) {
#pragma unroll
    for (int m = 1; m < (THREADS < WAVE ? THREADS : WAVE); m <<= 1) x = fmaxf(x, __shfl_xor(x, m, WAVE));
    if constexpr (THREADS > WAVE) {
        __syncthreads();
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
        __syncthreads();
        x = red[0];
#pragma unroll
        for (int w = 1; w < THREADS / WAVE; ++w) x = fmaxf(x, red[w]);
    }
    return x;
}

template <class TO, int THREADS, int UNR>
__device__ inline void edge_softmax_listed_row(unsigned block, const int32_t *rowptr, const int32_t *rows, int nrows, const float *score, float scale, TO *out) {
    __shared__ float red[4];
    static_assert(THREADS == 256 || (THREADS <= WAVE && WAVE % THREADS == 0), "a workgroup per row, or whole groups of lanes inside a wave");
    const int tid = (int)threadIdx.x % THREADS;
    const int w = (int)((block * 256u + threadIdx.x) / THREADS);
    if (w >= nrows) return;             // whole lane groups or whole workgroups leave together
    const int64_t i = rows[w];
    const int s = rowptr[i], n = rowptr[i + 1] - s;
    const float *sc = score + s;
    float v[UNR];
    auto fetch = [&](int q0) {          // clamped addresses, padding becomes -inf afterwards
#pragma unroll
        for (int u = 0; u < UNR; ++u) v[u] = sc[min(q0 + u * THREADS + tid, n - 1)];
#pragma unroll
        for (int u = 0; u < UNR; ++u) v[u] = q0 + u * THREADS + tid < n ? scale * v[u] : -INFINITY;
    };
    float m = -INFINITY, d = 0.f;
    for (int q0 = 0; q0 < n; q0 += THREADS * UNR) {
        fetch(q0);
        float bm = v[0];
#pragma unroll
        for (int u = 1; u < UNR; ++u) bm = fmaxf(bm, v[u]);
        const float nm = fmaxf(m, bm);
        if (nm > -INFINITY) {           // this thread has seen a score
            float acc = 0.f;
#pragma unroll
            for (int u = 0; u < UNR; ++u) acc += __expf(v[u] - nm);
            d = d * __expf(m - nm) + acc;       // m = -inf: d is 0 and exp(-inf) = 0
            m = nm;
        }
    }
    const float mx = list_max<THREADS>(m, red);
    const float den = list_sum<THREADS>(m > -INFINITY ? d * __expf(m - mx) : 0.f, red);
    const float inv = 1.f / den;
    const bool in_registers = n <= THREADS * UNR;
    for (int q0 = 0; q0 < n; q0 += THREADS * UNR) {
        if (!in_registers) fetch(q0);
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int q = q0 + u * THREADS + tid;
            if (q < n) out[s + q] = to_storage<TO>(__expf(v[u] - mx) * inv);
        }
    }
}

// The three row classes in one launch of 256-thread workgroups: first one workgroup per long row (the plan lists them
// longest first: the longest row sets the time of its class, so it starts first and the rest of the launch runs beside
// it), then 256 / MEDIUM_LANES medium rows per workgroup, then the workgroups that walk the rows of 64 nonzeros or fewer.
// GAT graph (2^20 rows, 60.7 M nonzeros): 196 us as three launches, 159 us as one, 150 us with 32 instead of 64 lanes per
// medium row (more rows in flight per wave; 16 lanes: 149 us).
constexpr int MEDIUM_LANES = 32;        // lanes per medium row
struct SoftmaxRows {
    const int32_t *rowptr, *long_rows, *medium_rows;
    int64_t M;
    int32_t nlong, nmedium;
    uint32_t medium_blocks, short_blocks;
};
__host__ inline SoftmaxRows softmax_rows(const libra_plan_t *P) {
    SoftmaxRows r{P->d_rowptr, P->d_long_rows, P->d_medium_rows, P->M, (int32_t)P->long_rows.size(), (int32_t)P->medium_rows.size(), 0u, 0u};
    r.medium_blocks = ((uint32_t)r.nmedium + 256u / MEDIUM_LANES - 1u) / (256u / MEDIUM_LANES);
    r.short_blocks = (uint32_t)std::min<int64_t>((P->M * SHORT_LANES + 255) / 256, 1 << 18);
    return r;
}
template <class TO>
__global__ __launch_bounds__(256) void edge_softmax_kernel(SoftmaxRows r, const float *score, float scale, TO *out) {
    const unsigned b = blockIdx.x;
    if (b < (unsigned)r.nlong) edge_softmax_listed_row<TO, 256, 16>(b, r.rowptr, r.long_rows, r.nlong, score, scale, out);
    else if (b < (unsigned)r.nlong + r.medium_blocks) edge_softmax_listed_row<TO, MEDIUM_LANES, 8>(b - (unsigned)r.nlong, r.rowptr, r.medium_rows, r.nmedium, score, scale, out);
    else edge_softmax_short_rows<TO>(b - (unsigned)r.nlong - r.medium_blocks, r.short_blocks, r.rowptr, r.M, score, scale, out);
}

// Backward of the edge softmax: dscore_p = scale * alpha_p * (dalpha_p - sum_row alpha_q dalpha_q).  Same three row
// classes as the forward kernels.
template <class TA> __device__ inline float from_storage(TA x) { return (float)x; }
template <> __device__ inline float from_storage<bf16_t>(bf16_t x) { return __uint_as_float((uint32_t)x.bits << 16); }

template <class TA>
__device__ inline void edge_softmax_bwd_short_rows(unsigned block, unsigned nblocks, const int32_t *rowptr, int64_t M, const TA *alpha, const float *dalpha, float scale, float *dscore) {
    constexpr int SL = SHORT_LANES, KPL = SHORT_LOADS;
    const int l = threadIdx.x % SL;
    const int64_t group = ((int64_t)block * blockDim.x + threadIdx.x) / SL;
    const int64_t ngroups = ((int64_t)nblocks * blockDim.x) / SL;
    for (int64_t i = group; i < M; i += ngroups) {
        const int s = rowptr[i], n = rowptr[i + 1] - s;
        if (n == 0 || n > 64) continue;
        // clamped addresses, all loads in flight together; the padding contributes zero
        TA ar[KPL];
        float a[KPL], g[KPL], dot = 0.f;
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            const int q = s + min(l + SL * k, n - 1);
            ar[k] = alpha[q];
            g[k] = dalpha[q];
        }
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            a[k] = l + SL * k < n ? from_storage<TA>(ar[k]) : 0.f;
            dot += a[k] * g[k];
        }
        dot = group_sum<SL>(dot);
#pragma unroll
        for (int k = 0; k < KPL; ++k)
            if (l + SL * k < n) dscore[s + l + SL * k] = scale * a[k] * (g[k] - dot);
    }
}

// MEDIUM_LANES lanes per listed row (65 .. LIBRA_SOFTMAX_LONG_ROW nonzeros), or one 256-thread workgroup per listed long row;
// UNR pairs per thread and round, as in the forward kernel
template <class TA, int THREADS, int UNR>
__device__ inline void edge_softmax_bwd_listed_row(unsigned block, const int32_t *rowptr, const int32_t *rows, int nrows, const TA *alpha, const float *dalpha, float scale, float *dscore) {
    __shared__ float red[4];
    static_assert(THREADS == 256 || (THREADS <= WAVE && WAVE % THREADS == 0), "a workgroup per row, or whole groups of lanes inside a wave");
    const int tid = (int)threadIdx.x % THREADS;
    const int w = (int)((block * 256u + threadIdx.x) / THREADS);
    if (w >= nrows) return;             // whole lane groups or whole workgroups leave together
    const int64_t i = rows[w];
    const int s = rowptr[i], n = rowptr[i + 1] - s;
    float a[UNR], g[UNR];
    auto fetch = [&](int q0) {          // clamped addresses; padding contributes zero
        TA ar[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int q = min(q0 + u * THREADS + tid, n - 1);
            ar[u] = alpha[s + q];
            g[u] = dalpha[s + q];
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) a[u] = q0 + u * THREADS + tid < n ? from_storage<TA>(ar[u]) : 0.f;
    };
    float dot = 0.f;
    for (int q0 = 0; q0 < n; q0 += THREADS * UNR) {
        fetch(q0);
#pragma unroll
        for (int u = 0; u < UNR; ++u) dot += a[u] * g[u];
    }
    dot = list_sum<THREADS>(dot, red);
    const bool in_registers = n <= THREADS * UNR;
    for (int q0 = 0; q0 < n; q0 += THREADS * UNR) {
        if (!in_registers) fetch(q0);
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int q = q0 + u * THREADS + tid;
            if (q < n) dscore[s + q] = scale * a[u] * (g[u] - dot);
        }
    }
}

template <class TA>
__global__ __launch_bounds__(256) void edge_softmax_bwd_kernel(SoftmaxRows r, const TA *alpha, const float *dalpha, float scale, float *dscore) {
    const unsigned b = blockIdx.x;
    if (b < (unsigned)r.nlong) edge_softmax_bwd_listed_row<TA, 256, 8>(b, r.rowptr, r.long_rows, r.nlong, alpha, dalpha, scale, dscore);
    else if (b < (unsigned)r.nlong + r.medium_blocks) edge_softmax_bwd_listed_row<TA, MEDIUM_LANES, 8>(b - (unsigned)r.nlong, r.rowptr, r.medium_rows, r.nmedium, alpha, dalpha, scale, dscore);
    else edge_softmax_bwd_short_rows<TA>(b - (unsigned)r.nlong - r.medium_blocks, r.short_blocks, r.rowptr, r.M, alpha, dalpha, scale, dscore);
}

// dst[i * stride + offset] (as T) = src[perm[i]]: new values into a packed array or into entry records
template <class T>
__global__ __launch_bounds__(256) void scatter_values_kernel(const T *src, const int32_t *perm, int64_t n, void *dst, int stride, int offset) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        *reinterpret_cast<T *>(reinterpret_cast<char *>(dst) + i * stride + offset) = src[perm[i]];
}

// new values into the 16-bit SDDMM output records, which carry their own CSR position (and keep their stage slot)
__global__ __launch_bounds__(256) void refresh_record_values_kernel(const uint16_t *src, int64_t n, SdPv *rec) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        rec[i].val = (rec[i].val & 0xffff0000u) | src[rec[i].perm];
}

// the same into the value runs of the blocked entry layout
// 16-bit values, eight consecutive destinations per thread: the permutation arrives as two 16-byte loads and the values
// leave as one 16-byte store (a group of eight never straddles a block of the blocked layout: 64 values per block).
// BLOCKED: the value runs of the blocked SpMM entries; otherwise a plain array of 16-bit values.
template <bool BLOCKED>
__global__ __launch_bounds__(256) void scatter_values16_x8_kernel(const uint16_t *src, const int32_t *perm, int64_t n, unsigned char *dst) {
    static_assert(RES_BLOCK % 8 == 0, "a group of eight values stays inside one block");
    const int64_t groups = n / 8;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, nthreads = (int64_t)gridDim.x * blockDim.x;
    auto where = [&](int64_t i) {
        return BLOCKED ? dst + (i / RES_BLOCK) * (RES_BLOCK * 6) + RES_BLOCK * 4 + (i % RES_BLOCK) * 2 : dst + i * 2;
    };
    for (int64_t g = tid; g < groups; g += nthreads) {
        const int4 p0 = reinterpret_cast<const int4 *>(perm)[2 * g], p1 = reinterpret_cast<const int4 *>(perm)[2 * g + 1];
        const uint32_t v0 = src[p0.x], v1 = src[p0.y], v2 = src[p0.z], v3 = src[p0.w];
        const uint32_t v4 = src[p1.x], v5 = src[p1.y], v6 = src[p1.z], v7 = src[p1.w];
        *reinterpret_cast<uint4 *>(where(g * 8)) = uint4{v0 | v1 << 16, v2 | v3 << 16, v4 | v5 << 16, v6 | v7 << 16};
    }
    for (int64_t i = groups * 8 + tid; i < n; i += nthreads) *reinterpret_cast<uint16_t *>(where(i)) = src[perm[i]];
}
template <class T>
__global__ __launch_bounds__(256) void scatter_blocked_values_kernel(const T *src, const int32_t *perm, int64_t n, unsigned char *dst) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        reinterpret_cast<T *>(dst + (i / RES_BLOCK) * (RES_BLOCK * (4 + (int)sizeof(T))) + RES_BLOCK * 4)[i % RES_BLOCK] = src[perm[i]];
}

inline int hip_rc(hipError_t e) { return e == hipSuccess ? LIBRA_OK : LIBRA_ERR_HIP; }

template <class T, int N>
int launch_spmm(const SpmmArgs &a, int64_t ntasks, hipStream_t s) {
    if (ntasks == 0) return LIBRA_OK;
    hipLaunchKernelGGL((spmm_task_kernel<T, N>), dim3((unsigned)(ntasks * a.pieces)), dim3(WAVE), 0, s, a);
    return hip_rc(hipGetLastError());
}

int spmm_launch(const libra_plan_t *P, const SpmmArgs &a, int n, int64_t nt, hipStream_t s);

// `pieces` adjacent pieces of n columns each, one launch
int spmm_piece(const libra_plan_t *P, const void *B, int n, int pieces, int64_t ldb, float *C, int64_t ldc, hipStream_t s) {
    const SubPlan &sp = P->spmm;
    const int64_t per_die = ((int64_t)sp.tasks.size() + LIBRA_XCDS - 1) / LIBRA_XCDS;
    SpmmArgs a{sp.dev.tasks, sp.dev.blk_cols, sp.dev.blk_bitmap, sp.dev.blk_valptr, sp.dev.dense_val,
               sp.dev.res_ent, B, C, ldb, ldc, (int32_t)per_die, pieces, 0};
    if (sp.n.zero_rows) {
        const int n4 = n * pieces / 4;
        const int64_t total = sp.n.zero_rows * n4;
        const unsigned blocks = (unsigned)std::min<int64_t>((total + 255) / 256, 65536);
        hipLaunchKernelGGL(zero_rows_kernel, dim3(blocks), dim3(256), 0, s, sp.dev.zero_rows, sp.n.zero_rows, C, ldc, n4);
        if (hipGetLastError() != hipSuccess) return LIBRA_ERR_HIP;
    }
    const int64_t nt = per_die * LIBRA_XCDS;         // every slot of the table (the last few may hold empty tasks)
    if (P->o.two_kernels && a.phase == 0) {
        // ablation / debugging schedule: the matrix-unit part and the scalar part as two launches on the stream
        for (int phase = 1; phase <= 2; ++phase) {
            SpmmArgs b = a;
            b.phase = phase;
            if (int rc = spmm_launch(P, b, n, nt, s)) return rc;
        }
        return LIBRA_OK;
    }
    return spmm_launch(P, a, n, nt, s);
}

int spmm_launch(const libra_plan_t *P, const SpmmArgs &a, int n, int64_t nt, hipStream_t s) {
    if (P->vdt == LIBRA_F16) {
        switch (n) {
        case 32: return launch_spmm<half_t, 32>(a, nt, s);
        case 64: return launch_spmm<half_t, 64>(a, nt, s);
        case 128: return launch_spmm<half_t, 128>(a, nt, s);
        }
    } else if (P->vdt == LIBRA_BF16) {
        switch (n) {
        case 32: return launch_spmm<bf16_t, 32>(a, nt, s);
        case 64: return launch_spmm<bf16_t, 64>(a, nt, s);
        case 128: return launch_spmm<bf16_t, 128>(a, nt, s);
        }
    } else {
        switch (n) {
        case 16: return launch_spmm<float, 16>(a, nt, s);
        case 32: return launch_spmm<float, 32>(a, nt, s);
        case 64: return launch_spmm<float, 64>(a, nt, s);
        case 128: return launch_spmm<float, 128>(a, nt, s);
        }
    }
    return LIBRA_ERR_UNSUPPORTED;
}

}  // namespace

// =========================================================================================
// C ABI: upload and compute
// =========================================================================================
namespace {
size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Lays arrays out back to back (256-byte aligned, 16 spare bytes each) and copies them from host memory, from
// device memory, or only reserves their place (arrays that a kernel packs afterwards).
struct Uploader {
    char *base = nullptr;     // nullptr: size pass only
    size_t off = 0;
    hipStream_t s = nullptr;
    bool ok = true;
    template <class P>
    void put(const void *host_src, const void *dev_src, size_t bytes, P *&dst) {
        if (base) {
            dst = reinterpret_cast<P *>(base + off);
            if (bytes && host_src && hipMemcpyAsync(base + off, host_src, bytes, hipMemcpyHostToDevice, s) != hipSuccess) ok = false;
            if (bytes && !host_src && dev_src && hipMemcpyAsync(base + off, dev_src, bytes, hipMemcpyDeviceToDevice, s) != hipSuccess) ok = false;
        }
        off += align256(bytes + 16);
    }
    template <class V, class P>
    void putv(const V &v, P *&dst) { put(v.data(), nullptr, v.size() * sizeof(v[0]), dst); }
};

// Slots of the device task table: the table's length rounded up to whole rounds of the dies.
size_t task_slots(int64_t ntasks) { return (size_t)((ntasks + LIBRA_XCDS - 1) / LIBRA_XCDS) * LIBRA_XCDS; }

// Device task records, die by die (see task_slot); the slots past the last task hold empty tasks.
std::vector<DevTask> pack_tasks(const libra_plan_t *P, const SubPlan &sp, bool spmm) {
    const size_t per_die = task_slots((int64_t)sp.tasks.size()) / LIBRA_XCDS;
    const DevTask empty{0, 0, 0, 0, 0, 0u, (uint32_t)(spmm ? LIBRA_TASK_WINDOW : LIBRA_TASK_CHUNK), 0};
    std::vector<DevTask> out(per_die * LIBRA_XCDS, empty);
    for (size_t i = 0; i < sp.tasks.size(); ++i) {
        const libra_task_t &t = sp.tasks[i];
        DevTask d{t.id, t.blk_begin, t.blk_end, t.res_begin, t.res_end, (t.atomic_mask & 0xffffu) | (t.store_mask << 16),
                  (uint32_t)t.kind, t.kind == LIBRA_TASK_WINDOW ? sp.blk_valptr[t.blk_begin] : 0};
        if (spmm && t.kind == LIBRA_TASK_CHUNK) {
            // a segment of a decomposed row = a task of the row's window with one atomic output row
            d.id = t.id / P->o.W;
            d.blk_begin = d.blk_end = 0;
            d.masks = 1u << (t.id % P->o.W);
        }
        out[(i % LIBRA_XCDS) * per_die + i / LIBRA_XCDS] = d;
    }
    return out;
}

// Host staging of everything the kernels read in packed form; alive until the copies have finished.
struct Staging {
    std::vector<DevTask> tasks_a, tasks_d;
    std::vector<unsigned char> res_blocks;  // SpMM residual entries: blocked words and values
    std::vector<SdEnt> sdent;
    std::vector<SdPv> sdpv;
};

// Record layouts written on the device when the arrays come from the device planner.
template <class V>
__global__ __launch_bounds__(256) void pack_blocked_entries_kernel(const int32_t *col, const V *val, const int32_t *row, int64_t n, unsigned char *out) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        unsigned char *blk = out + (i / RES_BLOCK) * (RES_BLOCK * (4 + (int)sizeof(V)));
        const int slot = (int)(i % RES_BLOCK);
        reinterpret_cast<uint32_t *>(blk)[slot] = (uint32_t)col[i] | (uint32_t)(row[i] % W) << RES_ROW_SHIFT;
        reinterpret_cast<V *>(blk + RES_BLOCK * 4)[slot] = val[i];
    }
}
template <class V>
__global__ __launch_bounds__(256) void pack_sddmm_entries_kernel(const int32_t *row, const int32_t *col, const int32_t *perm, const V *val, int64_t n, SdEnt *out) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        out[i] = SdEnt{row[i], col[i], perm[i], (uint32_t)val[i]};
}
template <class V>
__global__ __launch_bounds__(256) void pack_sddmm_values_kernel(const int32_t *perm, const V *val, int64_t n, SdPv *out) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        out[i] = SdPv{perm[i], (uint32_t)val[i]};
}

// 16-bit SDDMM output records written on the device: one wave per window task.  Per group of SD_GROUP blocks the CSR
// positions of the group's packed values go to LDS; a lane then takes 4 bits of each block's bitmap, and for each set bit
// finds the packed value (popcount of the bits below), its rank among the group's positions (a count over the LDS array),
// and writes the record to that rank.
__global__ __launch_bounds__(WAVE) void pack_sddmm_sorted_records_kernel(const DevTask *tasks, const uint64_t *blk_bitmap, const int32_t *blk_valptr,
                                                                         const int32_t *dense_perm, const uint16_t *dense_val, SdPv *out) {
    __shared__ int32_t pos[SD_GROUP * 256];
    const DevTask t = tasks[blockIdx.x];                 // any order: every window task once
    if (t.kind != LIBRA_TASK_WINDOW) return;
    const int lane = threadIdx.x;
    for (int b0 = t.blk_begin; b0 < t.blk_end; b0 += SD_GROUP) {
        const int nb = min(SD_GROUP, t.blk_end - b0);
        const int v0 = blk_valptr[b0], n = blk_valptr[b0 + nb] - v0;
        for (int i = lane; i < n; i += WAVE) pos[i] = dense_perm[v0 + i];
        __syncthreads();
        for (int x = 0; x < nb; ++x) {
            const int b = b0 + x;
            const uint64_t word = blk_bitmap[(int64_t)b * 4 + lane / 16];       // bits 64 (lane / 16) .. + 63 of the block
            const int sh = (lane % 16) * 4;
            int before = 0;                                                     // set bits of the block below this lane's four
            for (int w = 0; w < lane / 16; ++w) before += __popcll(blk_bitmap[(int64_t)b * 4 + w]);
            before += __popcll(word & ((1ull << sh) - 1ull));
            int q = blk_valptr[b] + before;
            for (int e = 0; e < 4; ++e) {
                if (!(word >> (sh + e) & 1ull)) continue;
                const int bit = lane * 4 + e;
                const int32_t p = dense_perm[q];
                int rank = 0;
                for (int i = 0; i < n; ++i) rank += pos[i] < p;
                out[v0 + rank] = SdPv{p, (uint32_t)dense_val[q] | (uint32_t)sd_stage_slot(x, bit / KB, bit % KB) << 16};
                ++q;
            }
        }
        __syncthreads();
    }
}

// st == nullptr: size pass.  da/dd == nullptr: the arrays come from the plan's host vectors; otherwise from
// device memory, and the packed record arrays are only reserved here (adopt_device_arrays fills them).
void layout(libra_plan_t *P, Uploader &u, Staging *st, const DeviceSource *da, const DeviceSource *dd) {
    u.put(st ? (const void *)P->rowptr.data() : nullptr, nullptr, (size_t)(P->M + 1) * 4, P->d_rowptr);
    u.putv(P->long_rows, P->d_long_rows);
    u.putv(P->medium_rows, P->d_medium_rows);
    SubPlan &sa = P->spmm, &sd = P->sddmm;
    const size_t vs = (size_t)P->vsize;
    const bool from_host = st && !da;
    auto H = [&](const void *p) { return from_host ? p : nullptr; };
    // ---- SpMM ----
    if (st) st->tasks_a = pack_tasks(P, sa, true);
    u.put(st ? (const void *)st->tasks_a.data() : nullptr, nullptr, task_slots(sa.n.tasks) * sizeof(DevTask), sa.dev.tasks);
    u.put(H(sa.blk_cols.data()), da ? da->blk_cols : nullptr, (size_t)sa.n.col_slots * 4, sa.dev.blk_cols);
    u.put(H(sa.blk_bitmap.data()), da ? da->blk_bitmap : nullptr, (size_t)sa.n.bitmap_words * 8, sa.dev.blk_bitmap);
    u.put(H(sa.blk_valptr.data()), da ? da->blk_valptr : nullptr, P->o.build_spmm ? (size_t)(sa.n.blocks + 1) * 4 : 0, sa.dev.blk_valptr);
    u.put(H(sa.dense_val.data()), da ? da->dense_val : nullptr, (size_t)sa.n.dense * vs, sa.dev.dense_val);
    u.put(H(sa.dense_perm.data()), da ? da->dense_perm : nullptr, (size_t)sa.n.dense * 4, sa.dev.dense_perm);
    const size_t nres = (size_t)sa.n.res;
    const size_t res_bytes = res_blocked_bytes(nres + 1, vs);      // + 1: a task without entries still reads the slot at its (clamped) first index
    if (from_host) {
        const int Wp = P->o.W;
        st->res_blocks.assign(res_bytes, 0);
        for (size_t i = 0; i < nres; ++i) {
            unsigned char *blk = st->res_blocks.data() + i / RES_BLOCK * res_block_bytes(vs);
            const uint32_t word = (uint32_t)sa.res_col[i] | (uint32_t)(sa.res_row[i] % Wp) << RES_ROW_SHIFT;
            std::memcpy(blk + i % RES_BLOCK * 4, &word, 4);
            std::memcpy(blk + RES_BLOCK * 4 + i % RES_BLOCK * vs, sa.res_val.data() + i * vs, vs);
        }
    }
    u.put(from_host ? (const void *)st->res_blocks.data() : nullptr, nullptr, res_bytes, sa.dev.res_ent);
    u.put(H(sa.res_perm.data()), da ? da->res_perm : nullptr, nres * 4, sa.dev.res_perm);
    u.put(H(sa.zero_rows.data()), da ? da->zero_rows : nullptr, (size_t)sa.n.zero_rows * 4, sa.dev.zero_rows);
    // ---- SDDMM ----
    if (st) st->tasks_d = pack_tasks(P, sd, false);
    u.put(st ? (const void *)st->tasks_d.data() : nullptr, nullptr, task_slots(sd.n.tasks) * sizeof(DevTask), sd.dev.tasks);
    u.put(H(sd.blk_cols.data()), dd ? dd->blk_cols : nullptr, (size_t)sd.n.col_slots * 4, sd.dev.blk_cols);
    u.put(H(sd.blk_bitmap.data()), dd ? dd->blk_bitmap : nullptr, (size_t)sd.n.bitmap_words * 8, sd.dev.blk_bitmap);
    u.put(H(sd.blk_valptr.data()), dd ? dd->blk_valptr : nullptr, P->o.build_sddmm ? (size_t)(sd.n.blocks + 1) * 4 : 0, sd.dev.blk_valptr);
    const size_t ndd = (size_t)sd.n.dense;
    if (from_host) {
        st->sdpv.resize(ndd);
        for (size_t i = 0; i < ndd; ++i) {
            uint32_t bits = 0;
            std::memcpy(&bits, sd.dense_val.data() + i * vs, vs);
            st->sdpv[i] = {sd.dense_perm[i], bits};
        }
        if (sorted_records(P)) {
            // 16-bit records: inside every group of SD_GROUP blocks of a window task, ascending CSR position, each with the
            // stage slot of its product
            std::vector<SdPv> grp;
            for (const libra_task_t &t : sd.tasks) {
                if (t.kind != LIBRA_TASK_WINDOW) continue;
                for (int32_t b0 = t.blk_begin; b0 < t.blk_end; b0 += SD_GROUP) {
                    const int32_t b1 = std::min(t.blk_end, b0 + SD_GROUP);
                    grp.clear();
                    for (int32_t b = b0; b < b1; ++b) {
                        int32_t q = sd.blk_valptr[b];
                        for (int bit = 0; bit < W * KB; ++bit)
                            if (sd.blk_bitmap[(size_t)b * 4 + bit / 64] >> (bit % 64) & 1u) {
                                SdPv r = st->sdpv[q++];
                                r.val |= (uint32_t)sd_stage_slot(b - b0, bit / KB, bit % KB) << 16;
                                grp.push_back(r);
                            }
                    }
                    std::sort(grp.begin(), grp.end(), [](const SdPv &x, const SdPv &y) { return x.perm < y.perm; });
                    std::copy(grp.begin(), grp.end(), st->sdpv.begin() + sd.blk_valptr[b0]);
                }
            }
        }
    }
    u.put(from_host ? (const void *)st->sdpv.data() : nullptr, nullptr, ndd * sizeof(SdPv), sd.dev.dense_pv);
    u.put(H(sd.dense_perm.data()), dd ? dd->dense_perm : nullptr, ndd * 4, sd.dev.dense_perm);
    const size_t nrd = (size_t)sd.n.res;
    if (from_host) {
        st->sdent.resize(nrd);
        for (size_t i = 0; i < nrd; ++i) {
            uint32_t bits = 0;
            std::memcpy(&bits, sd.res_val.data() + i * vs, vs);
            st->sdent[i] = {sd.res_row[i], sd.res_col[i], sd.res_perm[i], bits};
        }
    }
    u.put(from_host ? (const void *)st->sdent.data() : nullptr, nullptr, nrd * sizeof(SdEnt), sd.dev.res_ent);
    u.put(H(sd.res_perm.data()), dd ? dd->res_perm : nullptr, nrd * 4, sd.dev.res_perm);
}
}  // namespace

size_t libra::plan_buffer_bytes(const libra_plan_t *plan) {
    Uploader u;
    layout(const_cast<libra_plan_t *>(plan), u, nullptr, nullptr, nullptr);
    return u.off + 256;
}

int libra::adopt_device_arrays(libra_plan_t *P, const DeviceSource &da, const DeviceSource &dd, void *dev_buf, size_t bytes, void *stream) {
    if (!dev_buf) return LIBRA_ERR_NULL;
    if (bytes < plan_buffer_bytes(P) || ((uintptr_t)dev_buf & 255)) return LIBRA_ERR_BUFFER;
    if (P->Kc > (int64_t)RES_COL_MASK + 1) return LIBRA_ERR_UNSUPPORTED;    // a residual entry keeps its column in RES_ROW_SHIFT bits
    hipStream_t s = (hipStream_t)stream;
    try {
        Staging st;
        Uploader u;
        u.base = (char *)dev_buf;
        u.s = s;
        layout(P, u, &st, &da, &dd);
        auto grid = [](int64_t n) { return dim3((unsigned)std::min<int64_t>((n + 255) / 256, 1 << 16)); };
        const SubPlan &sa = P->spmm, &sd = P->sddmm;
        if (sa.n.res) {
            if (P->vdt == LIBRA_F32)
                hipLaunchKernelGGL((pack_blocked_entries_kernel<float>), grid(sa.n.res), dim3(256), 0, s, da.res_col,
                                   (const float *)da.res_val, da.res_row, sa.n.res, (unsigned char *)sa.dev.res_ent);
            else
                hipLaunchKernelGGL((pack_blocked_entries_kernel<uint16_t>), grid(sa.n.res), dim3(256), 0, s, da.res_col,
                                   (const uint16_t *)da.res_val, da.res_row, sa.n.res, (unsigned char *)sa.dev.res_ent);
        }
        if (sd.n.res) {
            if (P->vdt == LIBRA_F32)
                hipLaunchKernelGGL((pack_sddmm_entries_kernel<uint32_t>), grid(sd.n.res), dim3(256), 0, s, dd.res_row, dd.res_col, dd.res_perm,
                                   (const uint32_t *)dd.res_val, sd.n.res, (SdEnt *)sd.dev.res_ent);
            else
                hipLaunchKernelGGL((pack_sddmm_entries_kernel<uint16_t>), grid(sd.n.res), dim3(256), 0, s, dd.res_row, dd.res_col, dd.res_perm,
                                   (const uint16_t *)dd.res_val, sd.n.res, (SdEnt *)sd.dev.res_ent);
        }
        if (sd.n.dense) {
            if (P->vdt == LIBRA_F32)
                hipLaunchKernelGGL((pack_sddmm_values_kernel<uint32_t>), grid(sd.n.dense), dim3(256), 0, s, dd.dense_perm,
                                   (const uint32_t *)dd.dense_val, sd.n.dense, (SdPv *)sd.dev.dense_pv);
            else if (sorted_records(P))       // reads the task table that layout() has just queued for copying on this stream
                hipLaunchKernelGGL(pack_sddmm_sorted_records_kernel, dim3((unsigned)task_slots(sd.n.tasks)), dim3(WAVE), 0, s, sd.dev.tasks,
                                   dd.blk_bitmap, dd.blk_valptr, dd.dense_perm, (const uint16_t *)dd.dense_val, (SdPv *)sd.dev.dense_pv);
            else
                hipLaunchKernelGGL((pack_sddmm_values_kernel<uint16_t>), grid(sd.n.dense), dim3(256), 0, s, dd.dense_perm,
                                   (const uint16_t *)dd.dense_val, sd.n.dense, (SdPv *)sd.dev.dense_pv);
        }
        if (hipGetLastError() != hipSuccess || hipStreamSynchronize(s) != hipSuccess || !u.ok) return LIBRA_ERR_HIP;
    } catch (...) {
        return LIBRA_ERR_NOMEM;
    }
    P->dev_base = dev_buf;
    P->dev_bytes = bytes;
    return LIBRA_OK;
}

extern "C" int libra_plan_device_bytes(const libra_plan_t *plan, size_t *bytes) {
    if (!plan || !bytes) return LIBRA_ERR_NULL;
    *bytes = plan_buffer_bytes(plan);
    return LIBRA_OK;
}

extern "C" int libra_plan_upload(libra_plan_t *plan, void *dev_buf, size_t bytes, void *stream) {
    if (!plan || !dev_buf) return LIBRA_ERR_NULL;
    if (!plan->host_arrays) return LIBRA_ERR_NOT_BUILT;      // built on the device without a host copy: nothing to upload
    size_t need = 0;
    libra_plan_device_bytes(plan, &need);
    if (bytes < need || ((uintptr_t)dev_buf & 255)) return LIBRA_ERR_BUFFER;
    if (plan->Kc > (int64_t)RES_COL_MASK + 1) return LIBRA_ERR_UNSUPPORTED;      // a residual entry keeps its column in RES_ROW_SHIFT bits
    try {
        Staging st;
        Uploader u;
        u.base = (char *)dev_buf;
        u.s = (hipStream_t)stream;
        layout(plan, u, &st, nullptr, nullptr);
        if (hipStreamSynchronize(u.s) != hipSuccess || !u.ok) return LIBRA_ERR_HIP;
    } catch (...) {
        return LIBRA_ERR_NOMEM;
    }
    plan->dev_base = dev_buf;
    plan->dev_bytes = bytes;
    return LIBRA_OK;
}

extern "C" int libra_spmm(const libra_plan_t *P, const void *B, int32_t N, int64_t ldb, float *C, int64_t ldc, void *stream) {
    if (!P || !B || !C) return LIBRA_ERR_NULL;
    if (!P->o.build_spmm) return LIBRA_ERR_NOT_BUILT;
    if (!P->dev_base) return LIBRA_ERR_NOT_UPLOADED;
    if (P->o.W != W || P->o.KB != KB) return LIBRA_ERR_UNSUPPORTED;
    const int unit = P->vdt != LIBRA_F32 ? 32 : 16;
    if (N < unit || N > 512) return LIBRA_ERR_SHAPE;
    if (N % unit) return LIBRA_ERR_UNSUPPORTED;
    // a kernel forms a row's byte offset as a 32 x 32 -> 64 bit product: the row stride in bytes has to fit in 32 bits
    if (ldb < N || ldc < N || ldb * (int64_t)P->vsize >= (1ll << 32)) return LIBRA_ERR_SHAPE;
    if (ldb % (P->vdt != LIBRA_F32 ? 8 : 4) || ldc % 4) return LIBRA_ERR_UNSUPPORTED;
    if (((uintptr_t)B & 15) || ((uintptr_t)C & 15)) return LIBRA_ERR_BUFFER;
    hipStream_t s = (hipStream_t)stream;
    const int esz = P->vsize;
    // the feature dimension is cut into pieces the kernels are instantiated for; at most 128 columns, the widest
    // piece whose tile leaves four waves per SIMD (a 256-column piece ran at two and took 2.5x the time of a 128-column one)
    for (int n0 = 0; n0 < N;) {
        int n = 128;
        while (n > N - n0) n >>= 1;
        // The 128-column pieces of a wide operand go into one launch when the plan keeps neighbouring windows on one die
        // (matrices whose windows share columns: the pieces of a task then share the plan's data and the launch has one
        // tail; community N=256: 535 -> 508 us).  Elsewhere they run one after the other: together they would compete for
        // the L2 with twice the rows of B (power-law N=512: 267 us apart, 354 us together).
        const int pieces = (n == 128 && P->o.xcd_order == 1) ? (N - n0) / 128 : 1;
        int rc = spmm_piece(P, (const char *)B + (size_t)n0 * esz, n, pieces, ldb, C + n0, ldc, s);
        if (rc != LIBRA_OK) return rc;
        n0 += n * pieces;
    }
    return LIBRA_OK;
}

namespace {
int sddmm_call(const libra_plan_t *P, const void *X, const void *Y, int32_t K, float *out, void *stream, int pattern_only);
}
extern "C" int libra_sddmm(const libra_plan_t *P, const void *X, const void *Y, int32_t K, float *out, void *stream) {
    return sddmm_call(P, X, Y, K, out, stream, 0);
}
extern "C" int libra_sddmm_pattern(const libra_plan_t *P, const void *X, const void *Y, int32_t K, float *out, void *stream) {
    return sddmm_call(P, X, Y, K, out, stream, 1);
}
namespace {
int sddmm_call(const libra_plan_t *P, const void *X, const void *Y, int32_t K, float *out, void *stream, int pattern_only) {
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
    SddmmArgs a{sp.dev.tasks, sp.dev.blk_cols, sp.dev.blk_bitmap, sp.dev.blk_valptr,
                reinterpret_cast<const uint2 *>(sp.dev.dense_pv), (int32_t)sp.n.dense,
                reinterpret_cast<const SdEnt *>(sp.dev.res_ent), X, Y, out, P->M, 0, pattern_only};
    if (sp.tasks.empty()) return LIBRA_OK;
    a.tasks_per_die = (int32_t)(((int64_t)sp.tasks.size() + LIBRA_XCDS - 1) / LIBRA_XCDS);
    auto launch = [&](auto wpb) {
        constexpr int WPB = decltype(wpb)::value;
        const dim3 grid((unsigned)((a.tasks_per_die + WPB - 1) / WPB * LIBRA_XCDS)), block(WAVE * WPB);
        if (P->vdt == LIBRA_F16) {
            switch (K) {
            case 32: hipLaunchKernelGGL((sddmm_task_kernel<half_t, 32, WPB>), grid, block, 0, s, a); break;
            case 64: hipLaunchKernelGGL((sddmm_task_kernel<half_t, 64, WPB>), grid, block, 0, s, a); break;
            case 128: hipLaunchKernelGGL((sddmm_task_kernel<half_t, 128, WPB>), grid, block, 0, s, a); break;
            }
        } else if (P->vdt == LIBRA_BF16) {
            switch (K) {
            case 32: hipLaunchKernelGGL((sddmm_task_kernel<bf16_t, 32, WPB>), grid, block, 0, s, a); break;
            case 64: hipLaunchKernelGGL((sddmm_task_kernel<bf16_t, 64, WPB>), grid, block, 0, s, a); break;
            case 128: hipLaunchKernelGGL((sddmm_task_kernel<bf16_t, 128, WPB>), grid, block, 0, s, a); break;
            }
        } else {
            switch (K) {
            case 32: hipLaunchKernelGGL((sddmm_task_kernel<float, 32, WPB>), grid, block, 0, s, a); break;
            case 64: hipLaunchKernelGGL((sddmm_task_kernel<float, 64, WPB>), grid, block, 0, s, a); break;
            case 128: hipLaunchKernelGGL((sddmm_task_kernel<float, 128, WPB>), grid, block, 0, s, a); break;
            }
        }
    };
    if (P->o.xcd_order == 1) launch(std::integral_constant<int, 4>{});
    else launch(std::integral_constant<int, 1>{});
    if (hipGetLastError() != hipSuccess) return LIBRA_ERR_HIP;
    return LIBRA_OK;
}
}  // namespace

extern "C" int libra_edge_softmax(const libra_plan_t *P, const float *scores, float scale, void *vals_out, int out_dtype, void *stream) {
    if (!P) return LIBRA_ERR_NULL;
    if ((!scores || !vals_out) && P->nnz > 0) return LIBRA_ERR_NULL;
    if (out_dtype != LIBRA_F16 && out_dtype != LIBRA_BF16 && out_dtype != LIBRA_F32) return LIBRA_ERR_DTYPE;
    if (!P->dev_base) return LIBRA_ERR_NOT_UPLOADED;
    hipStream_t s = (hipStream_t)stream;
    if (P->nnz == 0) return LIBRA_OK;
    const SoftmaxRows r = softmax_rows(P);
    const unsigned blocks = (unsigned)r.nlong + r.medium_blocks + r.short_blocks;
    auto run = [&](auto tag) {
        typedef decltype(tag) TO;
        hipLaunchKernelGGL((edge_softmax_kernel<TO>), dim3(blocks), dim3(256), 0, s, r, scores, scale, reinterpret_cast<TO *>(vals_out));
    };
    if (out_dtype == LIBRA_F16) run(half_t{});
    else if (out_dtype == LIBRA_BF16) run(bf16_t{});
    else run(float{});
    return hip_rc(hipGetLastError());
}

extern "C" int libra_edge_softmax_backward(const libra_plan_t *P, const void *alpha, int alpha_dtype, const float *dalpha, float scale,
                                           float *dscores, void *stream) {
    if (!P) return LIBRA_ERR_NULL;
    if ((!alpha || !dalpha || !dscores) && P->nnz > 0) return LIBRA_ERR_NULL;
    if (alpha_dtype != LIBRA_F16 && alpha_dtype != LIBRA_BF16 && alpha_dtype != LIBRA_F32) return LIBRA_ERR_DTYPE;
    if (!P->dev_base) return LIBRA_ERR_NOT_UPLOADED;
    hipStream_t s = (hipStream_t)stream;
    if (P->nnz == 0) return LIBRA_OK;
    const SoftmaxRows r = softmax_rows(P);
    const unsigned blocks = (unsigned)r.nlong + r.medium_blocks + r.short_blocks;
    auto run = [&](auto tag) {
        typedef decltype(tag) TA;
        hipLaunchKernelGGL((edge_softmax_bwd_kernel<TA>), dim3(blocks), dim3(256), 0, s, r, reinterpret_cast<const TA *>(alpha), dalpha, scale, dscores);
    };
    if (alpha_dtype == LIBRA_F16) run(half_t{});
    else if (alpha_dtype == LIBRA_BF16) run(bf16_t{});
    else run(float{});
    return hip_rc(hipGetLastError());
}

extern "C" int libra_plan_set_values(libra_plan_t *P, const void *vals, int dtype, void *stream) {
    return libra_plan_set_values_for(P, vals, dtype, LIBRA_OP_SPMM | LIBRA_OP_SDDMM, stream);
}

extern "C" int libra_plan_set_values_for(libra_plan_t *P, const void *vals, int dtype, int ops, void *stream) {
    if (!P) return LIBRA_ERR_NULL;
    if (!(ops & (LIBRA_OP_SPMM | LIBRA_OP_SDDMM)) || (ops & ~(LIBRA_OP_SPMM | LIBRA_OP_SDDMM))) return LIBRA_ERR_OPTION;
    if (!vals && P->nnz > 0) return LIBRA_ERR_NULL;
    if (dtype != P->vdt) return LIBRA_ERR_DTYPE;
    if (!P->dev_base) return LIBRA_ERR_NOT_UPLOADED;
    hipStream_t s = (hipStream_t)stream;
    const bool f16 = dtype != LIBRA_F32;       // 16-bit values are moved as raw bits
    const int vs = P->vsize;
    struct Seg { const int32_t *perm; void *dst; int64_t n; int stride, offset; };
    const SubPlan &sa = P->spmm, &sd = P->sddmm;
    const Seg segs[4] = {
        {sa.dev.dense_perm, sa.dev.dense_val, sa.n.dense, vs, 0},
        {sa.dev.res_perm, sa.dev.res_ent, sa.n.res, 0, 0},                  // stride 0: the blocked entry layout
        {sd.dev.dense_perm, sd.dev.dense_pv, sd.n.dense, (int)sizeof(SdPv), 4},
        {sd.dev.res_perm, sd.dev.res_ent, sd.n.res, (int)sizeof(SdEnt), 12}};
    for (int k = 0; k < 4; ++k) {
        const Seg &g = segs[k];
        if (g.n == 0 || !(ops & (k < 2 ? LIBRA_OP_SPMM : LIBRA_OP_SDDMM))) continue;
        const unsigned blocks = (unsigned)std::min<int64_t>((g.n + 255) / 256, 1 << 16);
        const unsigned blocks8 = (unsigned)std::min<int64_t>((g.n / 8 + 255) / 256 + 1, 1 << 16);
        if (k == 2 && sorted_records(P))
            hipLaunchKernelGGL(refresh_record_values_kernel, dim3(blocks), dim3(256), 0, s, (const uint16_t *)vals, g.n, (SdPv *)g.dst);
        else if (g.stride == 0 && f16)
            hipLaunchKernelGGL((scatter_values16_x8_kernel<true>), dim3(blocks8), dim3(256), 0, s, (const uint16_t *)vals, g.perm, g.n, (unsigned char *)g.dst);
        else if (g.stride == 2 && g.offset == 0 && f16)
            hipLaunchKernelGGL((scatter_values16_x8_kernel<false>), dim3(blocks8), dim3(256), 0, s, (const uint16_t *)vals, g.perm, g.n, (unsigned char *)g.dst);
        else if (g.stride == 0)
            hipLaunchKernelGGL((scatter_blocked_values_kernel<float>), dim3(blocks), dim3(256), 0, s, (const float *)vals, g.perm, g.n, (unsigned char *)g.dst);
        else if (f16)
            hipLaunchKernelGGL((scatter_values_kernel<uint16_t>), dim3(blocks), dim3(256), 0, s, (const uint16_t *)vals, g.perm, g.n, g.dst, g.stride, g.offset);
        else
            hipLaunchKernelGGL((scatter_values_kernel<float>), dim3(blocks), dim3(256), 0, s, (const float *)vals, g.perm, g.n, g.dst, g.stride, g.offset);
        if (hipGetLastError() != hipSuccess) return LIBRA_ERR_HIP;
    }
    return LIBRA_OK;
}
