/*
 * CPU oracle for the sparse hot path.  TEST INFRASTRUCTURE ONLY: the product
 * library never links, loads or calls anything in this directory.
 *
 * What it computes is the plain definition of the two operators the paper
 * accelerates (Section 2.2, "Programming Sparse Operators on TCUs"; cost
 * model of Section 4.2, Eq. 2 and Eq. 4):
 *
 *   SpMM   C[i,n]  = sum_{p in row i} val[p] * B[col[p], n]
 *   SDDMM  out[p]  = val[p] * sum_k X[i,k] * Y[col[p],k]      (p in row i)
 *
 * and the row-wise edge softmax that sits between them in an attention GNN
 * layer (Section 5.5, AGNN = SDDMM -> softmax -> SpMM).
 *
 * Inputs are widened exactly from their storage type (IEEE binary16, bfloat16
 * or binary32) to double; all accumulation is in double, in CSR order, with no
 * blocking or reordering.  OpenMP splits ROWS over threads for timing only;
 * the order of additions inside a row never changes.
 *
 * Each routine can also emit S = the same sum over absolute values, which the
 * tests use as the natural scale of an output that cancels to ~0.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1, ORACLE_F32 = 2 };

/* IEEE 754 binary16 -> double, written from the format definition:
 * 1 sign, 5 exponent (bias 15), 10 fraction bits. */
double oracle_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);                 /* subnormal: f * 2^-10 * 2^-14 */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(f | 0x400), e - 25);    /* (1 + f/1024) * 2^(e-15) */
    return sign ? -v : v;
}

/* bfloat16 is the upper half of a binary32. */
double oracle_bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static inline double load_elem(const void *p, int dt, size_t i)
{
    switch (dt) {
    case ORACLE_F16:  return oracle_half_to_double(((const uint16_t *)p)[i]);
    case ORACLE_BF16: return oracle_bf16_to_double(((const uint16_t *)p)[i]);
    default:          return (double)((const float *)p)[i];
    }
}

void oracle_widen(const void *in, int dt, int64_t n, double *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = load_elem(in, dt, (size_t)i);
}

static int pick_threads(int nthreads)
{
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
    return nthreads;
#else
    (void)nthreads;
    return 1;
#endif
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * SpMM on a list of rows (rows == NULL: all rows 0..M-1, nrows ignored).
 * C and S are dense [nrows_out x N] double, row r of the output belongs to
 * rows[r] (or to row r).  S may be NULL.
 */
int oracle_spmm(int64_t M, const int32_t *rowptr, const int32_t *col,
                const void *val, int vdt,
                const void *B, int bdt, int64_t N, int64_t ldb,
                const int64_t *rows, int64_t nrows,
                double *C, double *S, int nthreads)
{
    if (!rowptr || !C || N <= 0 || ldb < N) return -1;
    int64_t R = rows ? nrows : M;
    int nt = pick_threads(nthreads);
    (void)nt;
#pragma omp parallel for schedule(dynamic, 64) num_threads(nt)
    for (int64_t r = 0; r < R; ++r) {
        int64_t i = rows ? rows[r] : r;
        double *c = C + (size_t)r * (size_t)N;
        double *s = S ? S + (size_t)r * (size_t)N : NULL;
        for (int64_t n = 0; n < N; ++n) c[n] = 0.0;
        if (s) for (int64_t n = 0; n < N; ++n) s[n] = 0.0;
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            double a = load_elem(val, vdt, (size_t)p);
            size_t base = (size_t)col[p] * (size_t)ldb;
            for (int64_t n = 0; n < N; ++n) {
                double b = load_elem(B, bdt, base + (size_t)n);
                c[n] += a * b;
                if (s) s[n] += fabs(a) * fabs(b);
            }
        }
    }
    return 0;
}

/*
 * SDDMM.  If idx == NULL all nnz entries are produced in CSR order.
 * Otherwise only entries idx[0..nidx) are produced; idx_row[q] is the row that
 * holds CSR position idx[q].
 */
int oracle_sddmm(int64_t M, const int32_t *rowptr, const int32_t *col,
                 const void *val, int vdt,
                 const void *X, const void *Y, int xdt, int64_t K,
                 const int64_t *idx, const int64_t *idx_row, int64_t nidx,
                 double *out, double *S, int nthreads)
{
    if (!rowptr || !out || K <= 0) return -1;
    int nt = pick_threads(nthreads);
    (void)nt;
    if (!idx) {
#pragma omp parallel for schedule(dynamic, 64) num_threads(nt)
        for (int64_t i = 0; i < M; ++i) {
            for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
                double acc = 0.0, sacc = 0.0;
                size_t xb = (size_t)i * (size_t)K, yb = (size_t)col[p] * (size_t)K;
                for (int64_t k = 0; k < K; ++k) {
                    double x = load_elem(X, xdt, xb + (size_t)k);
                    double y = load_elem(Y, xdt, yb + (size_t)k);
                    acc += x * y;
                    sacc += fabs(x) * fabs(y);
                }
                double a = load_elem(val, vdt, (size_t)p);
                out[p] = a * acc;
                if (S) S[p] = fabs(a) * sacc;
            }
        }
    } else {
#pragma omp parallel for schedule(static) num_threads(nt)
        for (int64_t q = 0; q < nidx; ++q) {
            int64_t p = idx[q], i = idx_row[q];
            double acc = 0.0, sacc = 0.0;
            size_t xb = (size_t)i * (size_t)K, yb = (size_t)col[p] * (size_t)K;
            for (int64_t k = 0; k < K; ++k) {
                double x = load_elem(X, xdt, xb + (size_t)k);
                double y = load_elem(Y, xdt, yb + (size_t)k);
                acc += x * y;
                sacc += fabs(x) * fabs(y);
            }
            double a = load_elem(val, vdt, (size_t)p);
            out[q] = a * acc;
            if (S) S[q] = fabs(a) * sacc;
        }
    }
    return 0;
}

/*
 * Row-wise edge softmax over CSR-ordered scores:
 *   alpha[p] = exp(scale*score[p] - mx_i) / sum_{q in row i} exp(scale*score[q] - mx_i),
 *   mx_i = max over row i of scale*score.
 */
int oracle_edge_softmax(int64_t M, const int32_t *rowptr, const double *score,
                        double scale, double *alpha, int nthreads)
{
    if (!rowptr || !score || !alpha) return -1;
    int nt = pick_threads(nthreads);
    (void)nt;
#pragma omp parallel for schedule(dynamic, 256) num_threads(nt)
    for (int64_t i = 0; i < M; ++i) {
        int64_t s = rowptr[i], e = rowptr[i + 1];
        if (s == e) continue;
        double mx = -INFINITY;
        for (int64_t p = s; p < e; ++p) {
            double v = scale * score[p];
            if (v > mx) mx = v;
        }
        double den = 0.0;
        for (int64_t p = s; p < e; ++p) den += exp(scale * score[p] - mx);
        for (int64_t p = s; p < e; ++p) alpha[p] = exp(scale * score[p] - mx) / den;
    }
    return 0;
}
