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
 * Walk: B is visited linearly (the loop order of the paper's reference routine,
 * Section 4.2: "output tensor accessed in a perfectly linear fashion"), an odometer
 * over B's multi-index keeps the matching offset into A.  No index fusion, no
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
 * The paper leaves the evaluation order open; this is the reading both sides of the
 * parity tests follow.
 *
 * Parity pins (tests/test_oracle_pins.py): closed-form address map of the Section 3.5
 * listing, 2-D case == textbook matrix transpose, identity == axpby, round trip with
 * the inverse permutation, composition, merged-index invariant of Section 3 stage (1),
 * brute-force element map on tiny tensors, numpy.transpose on Fortran-ordered arrays,
 * exact rational arithmetic for the alpha/beta formulas.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

enum { ORACLE_F32 = 0, ORACLE_F64 = 1, ORACLE_C64 = 2, ORACLE_C128 = 3 };
enum { ORACLE_MAX_DIM = 16 };

/* Odometer over B's multi-index (j_0 fastest).  offA follows along. */
typedef struct {
    int     n;
    int64_t sizeB[ORACLE_MAX_DIM];    /* sizeB[j]  = sizes[perm[j]]                    */
    int64_t stepA[ORACLE_MAX_DIM];    /* stepA[j]  = stride in A of the index perm[j]  */
    int64_t idx[ORACLE_MAX_DIM];
    int64_t offA;
} walker_t;

static void walker_init(walker_t* w, int n, const int64_t* sizes, const int* perm, int64_t offB)
{
    int64_t strideA[ORACLE_MAX_DIM];
    strideA[0] = 1;
    for (int k = 1; k < n; ++k) strideA[k] = strideA[k - 1] * sizes[k - 1];
    w->n = n;
    w->offA = 0;
    for (int j = 0; j < n; ++j) {
        w->sizeB[j] = sizes[perm[j]];
        w->stepA[j] = strideA[perm[j]];
        w->idx[j]   = offB % w->sizeB[j];     /* position of B offset offB in B's index space */
        offB       /= w->sizeB[j];
        w->offA    += w->idx[j] * w->stepA[j];
    }
}

static inline void walker_next(walker_t* w)
{
    for (int j = 0; j < w->n; ++j) {
        w->idx[j] += 1;
        w->offA   += w->stepA[j];
        if (w->idx[j] < w->sizeB[j]) return;
        w->offA   -= w->sizeB[j] * w->stepA[j];
        w->idx[j]  = 0;
    }
}

static void run_f32(walker_t w, int64_t lo, int64_t hi, float alpha, float beta,
                    const float* A, float* B)
{
    const int copy = (alpha == 1.0f && beta == 0.0f), overwrite = (beta == 0.0f);
    for (int64_t offB = lo; offB < hi; ++offB, walker_next(&w)) {
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
    for (int64_t offB = lo; offB < hi; ++offB, walker_next(&w)) {
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
    for (int64_t offB = lo; offB < hi; ++offB, walker_next(&w)) {
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
    for (int64_t offB = lo; offB < hi; ++offB, walker_next(&w)) {
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

/*
 * Returns 0 on success, a negative number for an argument the definition does not
 * cover (ndim out of range, extent < 1, perm not a permutation, unknown dtype).
 * alpha / beta point to one scalar of the data type (two reals for complex types).
 * nthreads > 1 splits B's linear range into equal contiguous slabs (OpenMP); every
 * element is still computed by the same statements.
 */
int ttc_oracle_transpose(int dtype, int ndim, const int64_t* sizes, const int* perm,
                         const void* alpha, const void* beta,
                         const void* A, void* B, int nthreads)
{
    if (ndim < 1 || ndim > ORACLE_MAX_DIM) return -1;
    if (dtype < ORACLE_F32 || dtype > ORACLE_C128) return -2;
    int seen[ORACLE_MAX_DIM] = {0};
    int64_t total = 1;
    for (int k = 0; k < ndim; ++k) {
        if (sizes[k] < 1) return -3;
        if (perm[k] < 0 || perm[k] >= ndim || seen[perm[k]]) return -4;
        seen[perm[k]] = 1;
        total *= sizes[k];
    }
    if (nthreads < 1) nthreads = 1;
    if ((int64_t)nthreads > total) nthreads = (int)total;

#pragma omp parallel for num_threads(nthreads) schedule(static)
    for (int t = 0; t < nthreads; ++t) {
        const int64_t lo = total * t / nthreads, hi = total * (t + 1) / nthreads;
        walker_t w;
        walker_init(&w, ndim, sizes, perm, lo);
        switch (dtype) {
        case ORACLE_F32:  run_f32 (w, lo, hi, *(const float*)alpha,  *(const float*)beta,  A, B); break;
        case ORACLE_F64:  run_f64 (w, lo, hi, *(const double*)alpha, *(const double*)beta, A, B); break;
        case ORACLE_C64:  run_c64 (w, lo, hi, alpha, beta, A, B); break;
        case ORACLE_C128: run_c128(w, lo, hi, alpha, beta, A, B); break;
        }
    }
    return 0;
}
