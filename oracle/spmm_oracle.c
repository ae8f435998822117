/*
 * CPU oracle for the hybrid SpMM path -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, slow, obviously-correct definitions in fp64.  Nothing here is shared
 * with (or derived from) the HIP implementation, and the product never calls it.
 *
 *   oracle_spmm      Z[i,j] = sum_{k in row i} val[k] * X[colInd[k], j]
 *                    -- the scalar-core SpMM definition (Alg. 1; aggregation
 *                    Z = A X, Eq. 1).  Duplicate (i, col) entries are summed.
 *   oracle_gemm      T[i,c] = sum_r X[i,r] * W[r,c]   (update X W, Eq. 2)
 *
 * Inputs are the stored bits the GPU sees (fp32, bf16, fp16 or fp64), each
 * widened exactly to fp64 before use; all sums are accumulated in fp64 in
 * index order.  OpenMP only splits the outermost row loop.
 */
#include <stdint.h>
#include <string.h>
#include <stddef.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { DT_F32 = 0, DT_BF16 = 1, DT_F16 = 2, DT_F64 = 3 };

static double widen_bf16(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double widen_f16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0)
        v = ldexp((double)frac, -24);               /* subnormal: frac * 2^-10 * 2^-14 */
    else if (expo == 31)
        v = frac ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)frac / 1024.0, expo - 15);
    return sign ? -v : v;
}

static double load_elem(const void *base, int dtype, int64_t idx)
{
    switch (dtype) {
    case DT_F32:  return (double)((const float *)base)[idx];
    case DT_BF16: return widen_bf16(((const uint16_t *)base)[idx]);
    case DT_F16:  return widen_f16(((const uint16_t *)base)[idx]);
    default:      return ((const double *)base)[idx];
    }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Z = A X for rows listed in `rows` (n_sel of them; rows == NULL means rows
 * 0..n_sel-1).  Output row r of Z (leading dimension ldz) holds the result for
 * matrix row rows[r].  use_abs != 0 computes sum |val| * |X| instead (the
 * magnitude bound used to scale error tolerances). */
void oracle_spmm(int64_t n_sel, const int64_t *rows,
                 const int32_t *rowptr, const int32_t *colind, const float *vals,
                 const void *X, int x_dtype, int64_t ldx, int32_t d,
                 double *Z, int64_t ldz, int use_abs)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t r = 0; r < n_sel; ++r) {
        int64_t i = rows ? rows[r] : r;
        for (int32_t j = 0; j < d; ++j) {
            double res = 0.0;
            for (int64_t k = rowptr[i]; k < rowptr[i + 1]; ++k) {
                double a = (double)vals[k];
                double x = load_elem(X, x_dtype, (int64_t)colind[k] * ldx + j);
                if (use_abs) { a = fabs(a); x = fabs(x); }
                res += a * x;
            }
            Z[r * ldz + j] = res;
        }
    }
}

/* T = X W for rows listed in `rows` (NULL = 0..n_sel-1); X is n x k (ldx), W is
 * k x n_out (ldw), T is n_sel x n_out (ldt).  use_abs: |X| |W|. */
void oracle_gemm(int64_t n_sel, const int64_t *rows,
                 const void *X, int x_dtype, int64_t ldx, int32_t k_dim,
                 const void *W, int w_dtype, int64_t ldw, int32_t n_out,
                 double *T, int64_t ldt, int use_abs)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t r = 0; r < n_sel; ++r) {
        int64_t i = rows ? rows[r] : r;
        for (int32_t c = 0; c < n_out; ++c) {
            double acc = 0.0;
            for (int32_t q = 0; q < k_dim; ++q) {
                double x = load_elem(X, x_dtype, i * ldx + q);
                double w = load_elem(W, w_dtype, (int64_t)q * ldw + c);
                if (use_abs) { x = fabs(x); w = fabs(w); }
                acc += x * w;
            }
            T[r * ldt + c] = acc;
        }
    }
}
