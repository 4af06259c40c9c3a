/*
 * CPU oracle for the out-of-place tensor transposition
 *
 *     B[Pi(i_1..i_N)]  <-  alpha * A[i_1..i_N]  +  beta * B[Pi(i_1..i_N)]        (paper Eq. 1)
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a plain, slow, obviously
 * correct nested-loop transposer that shares nothing with the HIP library: no
 * headers, no helpers, no tables.  Only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may call it.
 *
 * Conventions (paper Section 1, storage paragraph after Eq. 1):
 *   - column-major ("Fortran") storage: the leftmost index has stride 1.
 *   - 0-based here.  sizes[k] is the extent of A's k-th index.
 *   - perm[j] is the index of A that becomes the j-th index of B, i.e. the
 *     capital-Pi list of Eq. 1: Pi(i1,i2,i3) = (i2,i3,i1) is perm = {1,2,0}.
 *     The parallel-code listing of Section 3.5 (permutation (i3,i2,i1)) fixes this
 *     reading: its B address has i3 at stride 1.
 *
 * Walk: B is visited in the order of its linear offsets (the loop order of the paper's
 * reference routine, Section 4.2), an odometer over B's multi-index keeps the matching
 * offset into A.  No index fusion, no
 * tiling, no reordering.
 *
 * Arithmetic, per element, in the precision of the data type, round to nearest
 * even, no contraction other than the fused multiply-adds written out below
 * (compile with -ffp-contract=off):
 *   real,    alpha == 1 and beta == 0 :  r = a                     (bits moved unchanged)
 *   real,    beta == 0                :  r = alpha * a             (B is never read)
 *   real,    beta != 0                :  t = beta * b;  r = fma(alpha, a, t)
 *   complex product  z = s * x        :  z.re = fma(s.re, x.re, -(s.im * x.im))
 *                                        z.im = fma(s.re, x.im,   s.im * x.re )
 *   complex, alpha == (1,0), beta == 0:  r = a
 *   complex, beta == 0                :  r = alpha * a
 *   complex, beta != 0                :  p = alpha * a;  q = beta * b;  r = p + q (componentwise)
 * Mixed precision (A and B of different precision; the paper names the feature and no
 * more): alpha and beta are double precision, every element of A (and of B when beta != 0)
 * is widened to double -- exact -- the formulas above are evaluated in double, and the
 * result is rounded once, to nearest even, to B's precision when B is single.
 * The paper leaves the evaluation order open; this is the reading both sides of the
 * parity tests follow.
 *
 * Parity pins (tests/test_oracle_pins.py): closed-form address map of the Section 3.5
 * listing, 2-D case == textbook matrix transpose, identity == axpby, round trip with
 * the inverse permutation, composition, merged-index invariant of Section 3 stage (1),
 * brute-force element map on tiny tensors, numpy.transpose on Fortran-ordered arrays,
 * exact rational arithmetic for the alpha/beta formulas; for sub-tensors (lda / ldb):
 * numpy slicing of the enclosing arrays, untouched elements outside the sub-tensor, the
 * strided brute-force element map, and ld = size reproducing the dense result.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

enum { ORACLE_F32 = 0, ORACLE_F64 = 1, ORACLE_C64 = 2, ORACLE_C128 = 3,
       /* A and B of different precision (Table 1, --dataType sd / ds / cz / zc): first letter A, second B */
       ORACLE_F32_F64 = 4, ORACLE_F64_F32 = 5, ORACLE_C64_C128 = 6, ORACLE_C128_C64 = 7 };
enum { ORACLE_MAX_DIM = 16 };

/* Odometer over B's multi-index (j_0 fastest).  offA and offB follow along. */
typedef struct {
    int     n;
    int64_t sizeB[ORACLE_MAX_DIM];    /* sizeB[j]  = sizes[perm[j]]                    */
    int64_t stepA[ORACLE_MAX_DIM];    /* stepA[j]  = stride in A of the index perm[j]  */
    int64_t stepB[ORACLE_MAX_DIM];    /* stepB[j]  = stride in B of B's j-th index     */
    int64_t idx[ORACLE_MAX_DIM];
    int64_t offA, offB;
} walker_t;

/*
 * Strides.  A tensor may be a part of a larger one (Table 1, --lda / --ldb; Section 3):
 * lda[k] >= sizes[k] is the extent of the enclosing tensor along A's k-th index, so
 * strideA[0] = 1 and strideA[k] = strideA[k-1] * lda[k-1]; ldb[j] >= sizes[perm[j]] does the
 * same for B's j-th index.  NULL means the tensor is dense (ld = size).  `count` is the
 * position, in B's index space, of the element the walk starts from.
 */
static void walker_init(walker_t* w, int n, const int64_t* sizes, const int* perm,
                        const int64_t* lda, const int64_t* ldb, int64_t count)
{
    int64_t strideA[ORACLE_MAX_DIM], strideB[ORACLE_MAX_DIM];
    strideA[0] = 1;
    for (int k = 1; k < n; ++k) strideA[k] = strideA[k - 1] * (lda ? lda[k - 1] : sizes[k - 1]);
    strideB[0] = 1;
    for (int j = 1; j < n; ++j) strideB[j] = strideB[j - 1] * (ldb ? ldb[j - 1] : sizes[perm[j - 1]]);
    w->n = n;
    w->offA = 0;
    w->offB = 0;
    for (int j = 0; j < n; ++j) {
        w->sizeB[j] = sizes[perm[j]];
        w->stepA[j] = strideA[perm[j]];
        w->stepB[j] = strideB[j];
        w->idx[j]   = count % w->sizeB[j];
        count      /= w->sizeB[j];
        w->offA    += w->idx[j] * w->stepA[j];
        w->offB    += w->idx[j] * w->stepB[j];
    }
}

static inline void walker_next(walker_t* w)
{
    for (int j = 0; j < w->n; ++j) {
        w->idx[j] += 1;
        w->offA   += w->stepA[j];
        w->offB   += w->stepB[j];
        if (w->idx[j] < w->sizeB[j]) return;
        w->offA   -= w->sizeB[j] * w->stepA[j];
        w->offB   -= w->sizeB[j] * w->stepB[j];
        w->idx[j]  = 0;
    }
}

static void run_f32(walker_t w, int64_t lo, int64_t hi, float alpha, float beta,
                    const float* A, float* B)
{
    const int copy = (alpha == 1.0f && beta == 0.0f), overwrite = (beta == 0.0f);
    for (int64_t count = lo; count < hi; ++count, walker_next(&w)) {
        const int64_t offB = w.offB;
        const float a = A[w.offA];
        if (copy)            B[offB] = a;
        else if (overwrite)  B[offB] = alpha * a;
        else { const float t = beta * B[offB]; B[offB] = fmaf(alpha, a, t); }
    }
}

static void run_f64(walker_t w, int64_t lo, int64_t hi, double alpha, double beta,
                    const double* A, double* B)
{
    const int copy = (alpha == 1.0 && beta == 0.0), overwrite = (beta == 0.0);
    for (int64_t count = lo; count < hi; ++count, walker_next(&w)) {
        const int64_t offB = w.offB;
        const double a = A[w.offA];
        if (copy)            B[offB] = a;
        else if (overwrite)  B[offB] = alpha * a;
        else { const double t = beta * B[offB]; B[offB] = fma(alpha, a, t); }
    }
}

static void run_c64(walker_t w, int64_t lo, int64_t hi, const float* alpha, const float* beta,
                    const float* A, float* B)
{
    const float ar = alpha[0], ai = alpha[1], br = beta[0], bi = beta[1];
    const int overwrite = (br == 0.0f && bi == 0.0f);
    const int copy = overwrite && (ar == 1.0f && ai == 0.0f);
    for (int64_t count = lo; count < hi; ++count, walker_next(&w)) {
        const int64_t offB = w.offB;
        const float xr = A[2 * w.offA], xi = A[2 * w.offA + 1];
        if (copy) { B[2 * offB] = xr; B[2 * offB + 1] = xi; continue; }
        const float pr = fmaf(ar, xr, -(ai * xi));
        const float pi = fmaf(ar, xi,   ai * xr);
        if (overwrite) { B[2 * offB] = pr; B[2 * offB + 1] = pi; continue; }
        const float yr = B[2 * offB], yi = B[2 * offB + 1];
        const float qr = fmaf(br, yr, -(bi * yi));
        const float qi = fmaf(br, yi,   bi * yr);
        B[2 * offB]     = pr + qr;
        B[2 * offB + 1] = pi + qi;
    }
}

static void run_c128(walker_t w, int64_t lo, int64_t hi, const double* alpha, const double* beta,
                     const double* A, double* B)
{
    const double ar = alpha[0], ai = alpha[1], br = beta[0], bi = beta[1];
    const int overwrite = (br == 0.0 && bi == 0.0);
    const int copy = overwrite && (ar == 1.0 && ai == 0.0);
    for (int64_t count = lo; count < hi; ++count, walker_next(&w)) {
        const int64_t offB = w.offB;
        const double xr = A[2 * w.offA], xi = A[2 * w.offA + 1];
        if (copy) { B[2 * offB] = xr; B[2 * offB + 1] = xi; continue; }
        const double pr = fma(ar, xr, -(ai * xi));
        const double pi = fma(ar, xi,   ai * xr);
        if (overwrite) { B[2 * offB] = pr; B[2 * offB + 1] = pi; continue; }
        const double yr = B[2 * offB], yi = B[2 * offB + 1];
        const double qr = fma(br, yr, -(bi * yi));
        const double qi = fma(br, yi,   bi * yr);
        B[2 * offB]     = pr + qr;
        B[2 * offB + 1] = pi + qi;
    }
}

/* Mixed precision, real: TA / TB are float or double, arithmetic in double. */
#define ORACLE_RUN_REAL_MIXED(NAME, TA, TB)                                                        \
static void NAME(walker_t w, int64_t lo, int64_t hi, double alpha, double beta,                   \
                 const TA* A, TB* B)                                                               \
{                                                                                                  \
    const int copy = (alpha == 1.0 && beta == 0.0), overwrite = (beta == 0.0);                     \
    for (int64_t count = lo; count < hi; ++count, walker_next(&w)) {                               \
        const int64_t offB = w.offB;                                                               \
        const double a = (double)A[w.offA];                                                        \
        double r;                                                                                  \
        if (copy)            r = a;                                                                \
        else if (overwrite)  r = alpha * a;                                                        \
        else { const double t = beta * (double)B[offB]; r = fma(alpha, a, t); }                    \
        B[offB] = (TB)r;                                                                           \
    }                                                                                              \
}
ORACLE_RUN_REAL_MIXED(run_sd, float, double)
ORACLE_RUN_REAL_MIXED(run_ds, double, float)

/* Mixed precision, complex. */
#define ORACLE_RUN_COMPLEX_MIXED(NAME, TA, TB)                                                     \
static void NAME(walker_t w, int64_t lo, int64_t hi, const double* alpha, const double* beta,     \
                 const TA* A, TB* B)                                                               \
{                                                                                                  \
    const double ar = alpha[0], ai = alpha[1], br = beta[0], bi = beta[1];                         \
    const int overwrite = (br == 0.0 && bi == 0.0);                                                \
    const int copy = overwrite && (ar == 1.0 && ai == 0.0);                                        \
    for (int64_t count = lo; count < hi; ++count, walker_next(&w)) {                               \
        const int64_t offB = w.offB;                                                               \
        const double xr = (double)A[2 * w.offA], xi = (double)A[2 * w.offA + 1];                   \
        if (copy) { B[2 * offB] = (TB)xr; B[2 * offB + 1] = (TB)xi; continue; }                    \
        const double pr = fma(ar, xr, -(ai * xi));                                                 \
        const double pi = fma(ar, xi,   ai * xr);                                                  \
        if (overwrite) { B[2 * offB] = (TB)pr; B[2 * offB + 1] = (TB)pi; continue; }               \
        const double yr = (double)B[2 * offB], yi = (double)B[2 * offB + 1];                       \
        const double qr = fma(br, yr, -(bi * yi));                                                 \
        const double qi = fma(br, yi,   bi * yr);                                                  \
        B[2 * offB]     = (TB)(pr + qr);                                                           \
        B[2 * offB + 1] = (TB)(pi + qi);                                                           \
    }                                                                                              \
}
ORACLE_RUN_COMPLEX_MIXED(run_cz, float, double)
ORACLE_RUN_COMPLEX_MIXED(run_zc, double, float)

/*
 * Returns 0 on success, a negative number for an argument the definition does not
 * cover (ndim out of range, extent < 1, perm not a permutation, unknown dtype, a leading
 * dimension smaller than its extent).
 * alpha / beta point to one scalar of the data type (two reals for complex types;
 * double precision for the mixed types).
 * lda / ldb: see walker_init; NULL = dense.  Elements of B outside the sub-tensor are
 * neither read nor written.
 * nthreads > 1 splits the elements, in B's index order, into equal contiguous slabs
 * (OpenMP); every element is still computed by the same statements.
 */
int ttc_oracle_transpose_ld(int dtype, int ndim, const int64_t* sizes, const int* perm,
                            const int64_t* lda, const int64_t* ldb,
                            const void* alpha, const void* beta,
                            const void* A, void* B, int nthreads)
{
    if (ndim < 1 || ndim > ORACLE_MAX_DIM) return -1;
    if (dtype < ORACLE_F32 || dtype > ORACLE_C128_C64) return -2;
    int seen[ORACLE_MAX_DIM] = {0};
    int64_t total = 1;
    for (int k = 0; k < ndim; ++k) {
        if (sizes[k] < 1) return -3;
        if (perm[k] < 0 || perm[k] >= ndim || seen[perm[k]]) return -4;
        seen[perm[k]] = 1;
        total *= sizes[k];
    }
    for (int k = 0; k < ndim; ++k) {
        if (lda && lda[k] < sizes[k]) return -5;
        if (ldb && ldb[k] < sizes[perm[k]]) return -5;
    }
    if (nthreads < 1) nthreads = 1;
    if ((int64_t)nthreads > total) nthreads = (int)total;

#pragma omp parallel for num_threads(nthreads) schedule(static)
    for (int t = 0; t < nthreads; ++t) {
        const int64_t lo = total * t / nthreads, hi = total * (t + 1) / nthreads;
        walker_t w;
        walker_init(&w, ndim, sizes, perm, lda, ldb, lo);
        switch (dtype) {
        case ORACLE_F32:  run_f32 (w, lo, hi, *(const float*)alpha,  *(const float*)beta,  A, B); break;
        case ORACLE_F64:  run_f64 (w, lo, hi, *(const double*)alpha, *(const double*)beta, A, B); break;
        case ORACLE_C64:  run_c64 (w, lo, hi, alpha, beta, A, B); break;
        case ORACLE_C128: run_c128(w, lo, hi, alpha, beta, A, B); break;
        case ORACLE_F32_F64:  run_sd(w, lo, hi, *(const double*)alpha, *(const double*)beta, A, B); break;
        case ORACLE_F64_F32:  run_ds(w, lo, hi, *(const double*)alpha, *(const double*)beta, A, B); break;
        case ORACLE_C64_C128: run_cz(w, lo, hi, alpha, beta, A, B); break;
        case ORACLE_C128_C64: run_zc(w, lo, hi, alpha, beta, A, B); break;
        }
    }
    return 0;
}

/* Dense tensors: the operation of Eq. 1 as stated. */
int ttc_oracle_transpose(int dtype, int ndim, const int64_t* sizes, const int* perm,
                         const void* alpha, const void* beta,
                         const void* A, void* B, int nthreads)
{
    return ttc_oracle_transpose_ld(dtype, ndim, sizes, perm, NULL, NULL, alpha, beta, A, B, nthreads);
}
