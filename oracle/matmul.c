/* Oracle arithmetic -- TEST INFRASTRUCTURE ONLY, never linked into the library.
 *
 * C = A B by its definition (Section 2.1: A is m x k, B is k x n, C is m x n,
 * C[i][j] = sum over l of A[i][l] * B[l][j]), as an i-k-j triple loop in fp64.
 * Inputs may be fp64, fp32 or bf16 bit patterns; fp32 and bf16 are widened
 * exactly (every such value is representable in fp64), so for bf16 workloads
 * the oracle multiplies the very same rounded values the GPU path reads.
 * No blocking, no reordering: rows of C are independent, so the only
 * parallelism is an OpenMP loop over i, and the sum over l runs in ascending l.
 *
 * The replica sum (reduce_replicas, Table 1; Section 4.2, last paragraph) is
 * C_0 + C_1 + ... in ascending replica index, in fp32, because the partial
 * results it adds are the fp32 tiles that the path holds.
 */
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F64 = 0, ORACLE_F32 = 1, ORACLE_BF16 = 2 };

static inline double widen(const void *base, int64_t idx, int dtype)
{
    if (dtype == ORACLE_F64) return ((const double *)base)[idx];
    if (dtype == ORACLE_F32) return (double)((const float *)base)[idx];
    /* bf16: the upper 16 bits of an IEEE fp32 */
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* C[m x n] (fp64, leading dimension ldc) = A[m x k] (lda) * B[k x n] (ldb).
 * Row-major.  Returns 0, or -1 for a bad dtype / negative size. */
int oracle_matmul(int dtype,
                  const void *A, int64_t lda,
                  const void *B, int64_t ldb,
                  double *C, int64_t ldc,
                  int64_t m, int64_t k, int64_t n)
{
    if (dtype < ORACLE_F64 || dtype > ORACLE_BF16 || m < 0 || k < 0 || n < 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        double *c = C + i * ldc;
        for (int64_t j = 0; j < n; ++j) c[j] = 0.0;
        for (int64_t l = 0; l < k; ++l) {
            const double a = widen(A, i * lda + l, dtype);
            for (int64_t j = 0; j < n; ++j) c[j] += a * widen(B, l * ldb + j, dtype);
        }
    }
    return 0;
}

/* out[rows x cols] (fp32, ldo) = ((parts[0] + parts[1]) + parts[2]) + ...
 * Each part is rows x cols fp32 with its own leading dimension.  `out` may be
 * one of the parts (the origin replica's tile). */
int oracle_reduce_replicas(const float *const *parts, const int64_t *ld, int32_t nparts,
                           float *out, int64_t ldo, int64_t rows, int64_t cols)
{
    if (nparts < 1 || rows < 0 || cols < 0) return -1;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j) {
            float s = parts[0][i * ld[0] + j];
            for (int32_t r = 1; r < nparts; ++r) s = s + parts[r][i * ld[r] + j];
            out[i * ldo + j] = s;
        }
    return 0;
}

/* Threads the OpenMP loop over i will use (1 when built without OpenMP). */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
