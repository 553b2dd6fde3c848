/*
 * TEST INFRASTRUCTURE -- CPU oracle for the symmetric rank-k update and the
 * Cholesky factorisation.  It is the yardstick the GPU library is compared
 * with; it is never part of the product path and shares no code with it.
 *
 * What is computed is the plain definition of the two kernels, i.e. the
 * triple loops of the paper's Algorithm 1 (SYRK) and Algorithm 2 (Cholesky),
 * Section 3.  The paper's communication-avoiding schedules (TBS, LBC,
 * Section 5) execute exactly the same set of scalar operations in another
 * order (Section 5, first paragraph), so the definition is the oracle.
 *
 * Readings of the paper taken here:
 *  - Algorithm 1 is written as C += A*A^T.  The Cholesky trailing update of
 *    Algorithm 5 needs C -= A*A^T, so the update is generalised to
 *        C[i][j] <- beta*C[i][j] + alpha * sum_k A[i][k]*A[j][k],  j <= i,
 *    which gives Algorithm 1 for alpha = beta = 1.
 *  - The loop bounds of Algorithm 1 (j = 1..i) include the diagonal; the sets
 *    S and C of Section 3 drop i = j only for the lower-bound proofs.
 *  - beta == 0 means "C is write-only": the old value is not read, so a NaN
 *    stored there does not propagate (BLAS convention; the paper is silent).
 *  - Only entries with j <= i are ever read or written.
 *  - Algorithm 2 takes sqrt of the pivot without a test.  Here a pivot that
 *    is not > 0 (or is NaN) stops the factorisation and its 1-based index is
 *    returned (LAPACK convention); 0 means success.
 *
 * Storage: row-major, leading dimensions lda / ldc counted in elements.
 *
 * Parallelism: OpenMP over the outermost loop whose iterations are
 * independent (rows i of C in SYRK; rows i of the trailing matrix inside one
 * elimination step k of Cholesky).  No blocking, no BLAS, no reordering of
 * the k-sum.
 */
#include <math.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Algorithm 1 in working precision (double accumulation, k ascending). */
void oracle_syrk_lower_f64(int64_t N, int64_t M, double alpha,
                           const double *A, int64_t lda,
                           double beta, double *C, int64_t ldc)
{
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < N; ++i) {
        for (int64_t j = 0; j <= i; ++j) {
            double s = 0.0;
            for (int64_t k = 0; k < M; ++k)
                s += A[i * lda + k] * A[j * lda + k];
            if (beta == 0.0)
                C[i * ldc + j] = alpha * s;
            else
                C[i * ldc + j] = beta * C[i * ldc + j] + alpha * s;
        }
    }
}

/* Algorithm 1 with the k-sum carried in long double (x87 80-bit, 64-bit
 * significand): each product of two doubles is formed in long double, the
 * sum is rounded to double once at the end.  This is the parity yardstick:
 * its own rounding error (about M * 2^-64 relative to sum |a||a|) is far
 * below the tolerance the GPU result is held to. */
void oracle_syrk_lower_f64_ext(int64_t N, int64_t M, double alpha,
                               const double *A, int64_t lda,
                               double beta, double *C, int64_t ldc)
{
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < N; ++i) {
        for (int64_t j = 0; j <= i; ++j) {
            long double s = 0.0L;
            for (int64_t k = 0; k < M; ++k)
                s += (long double)A[i * lda + k] * (long double)A[j * lda + k];
            long double r = (long double)alpha * s;
            if (beta != 0.0)
                r += (long double)beta * (long double)C[i * ldc + j];
            C[i * ldc + j] = (double)r;
        }
    }
}

/* A sample of Algorithm 1: entry t of out is the updated value of
 * C[ii[t]][jj[t]] (ii[t] >= jj[t]), computed as in the _ext routine, C itself
 * is left untouched.  Lets a test check single entries of a matrix that is
 * too large to recompute in full. */
void oracle_syrk_lower_f64_ext_sample(int64_t M, double alpha,
                                      const double *A, int64_t lda,
                                      double beta, const double *C, int64_t ldc,
                                      int64_t nsample, const int64_t *ii,
                                      const int64_t *jj, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < nsample; ++t) {
        const int64_t i = ii[t], j = jj[t];
        long double s = 0.0L;
        for (int64_t k = 0; k < M; ++k)
            s += (long double)A[i * lda + k] * (long double)A[j * lda + k];
        long double r = (long double)alpha * s;
        if (beta != 0.0)
            r += (long double)beta * (long double)C[i * ldc + j];
        out[t] = (double)r;
    }
}

/* Algorithm 2: right-looking Cholesky, in place, lower triangle only.
 * Returns 0, or the 1-based index of the first pivot that is not > 0. */
int64_t oracle_potrf_lower_f64(int64_t N, double *A, int64_t lda)
{
    for (int64_t k = 0; k < N; ++k) {
        const double p = A[k * lda + k];
        if (!(p > 0.0))
            return k + 1;
        const double d = sqrt(p);
        A[k * lda + k] = d;
#pragma omp parallel for schedule(static) if (N - k > 256)
        for (int64_t i = k + 1; i < N; ++i) {
            const double lik = A[i * lda + k] / d;
            A[i * lda + k] = lik;
        }
        /* the update of row i needs the scaled column entries A[j][k] of all
         * rows j <= i, hence the scaling loop is completed first */
#pragma omp parallel for schedule(dynamic, 16) if (N - k > 256)
        for (int64_t i = k + 1; i < N; ++i) {
            const double lik = A[i * lda + k];
            for (int64_t j = k + 1; j <= i; ++j)
                A[i * lda + j] -= lik * A[j * lda + k];
        }
    }
    return 0;
}

/* Residual pieces for a factor L (lower triangle of a row-major array):
 * returns sum over i>=j of ( (L*L^T)[i][j] - S[i][j] )^2 counted twice for
 * i>j (the Frobenius norm of the symmetric difference), with the inner sum
 * in long double.  *norm2 receives the same count of S[i][j]^2. */
double oracle_llt_residual_sq(int64_t N, const double *L, int64_t ldl,
                              const double *S, int64_t lds, double *norm2)
{
    long double acc = 0.0L, nrm = 0.0L;
#pragma omp parallel for schedule(dynamic, 4) reduction(+ : acc, nrm)
    for (int64_t i = 0; i < N; ++i) {
        for (int64_t j = 0; j <= i; ++j) {
            long double s = 0.0L;
            for (int64_t k = 0; k <= j; ++k)
                s += (long double)L[i * ldl + k] * (long double)L[j * ldl + k];
            const long double d = s - (long double)S[i * lds + j];
            const long double w = (i == j) ? 1.0L : 2.0L;
            acc += w * d * d;
            nrm += w * (long double)S[i * lds + j] * (long double)S[i * lds + j];
        }
    }
    *norm2 = (double)nrm;
    return (double)acc;
}

/* ---------------------------------------------------------------------------
 * Two more kernels that use an input twice (the paper's conclusion names the
 * extension to "other kernels which use the same input several times" as
 * future work; it defines neither, so these are the textbook definitions,
 * written as the same kind of triple loop as Algorithm 1).
 *
 * SYR2K, lower triangle:
 *   C[i][j] <- beta*C[i][j] + alpha * sum_k (A[i][k]*B[j][k] + B[i][k]*A[j][k]),  j <= i.
 * Gram matrix, lower triangle (A is N x M, C is M x M):
 *   C[i][j] <- beta*C[i][j] + alpha * sum_k A[k][i]*A[k][j],  j <= i.
 * `ext` != 0 carries the sums in long double (the parity yardstick), 0 is the
 * plain double loop.  beta == 0: C is write-only.  Entries above the diagonal
 * are neither read nor written.
 * ------------------------------------------------------------------------- */
void oracle_syr2k_lower_f64(int64_t N, int64_t M, double alpha,
                            const double *A, int64_t lda,
                            const double *B, int64_t ldb,
                            double beta, double *C, int64_t ldc, int ext)
{
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < N; ++i) {
        for (int64_t j = 0; j <= i; ++j) {
            if (ext) {
                long double s = 0.0L;
                for (int64_t k = 0; k < M; ++k) {
                    s += (long double)A[i * lda + k] * (long double)B[j * ldb + k];
                    s += (long double)B[i * ldb + k] * (long double)A[j * lda + k];
                }
                long double r = (long double)alpha * s;
                if (beta != 0.0)
                    r += (long double)beta * (long double)C[i * ldc + j];
                C[i * ldc + j] = (double)r;
            } else {
                double s = 0.0;
                for (int64_t k = 0; k < M; ++k) {
                    s += A[i * lda + k] * B[j * ldb + k];
                    s += B[i * ldb + k] * A[j * lda + k];
                }
                if (beta == 0.0)
                    C[i * ldc + j] = alpha * s;
                else
                    C[i * ldc + j] = beta * C[i * ldc + j] + alpha * s;
            }
        }
    }
}

void oracle_gram_lower_f64(int64_t N, int64_t M, double alpha,
                           const double *A, int64_t lda,
                           double beta, double *C, int64_t ldc, int ext)
{
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j <= i; ++j) {
            if (ext) {
                long double s = 0.0L;
                for (int64_t k = 0; k < N; ++k)
                    s += (long double)A[k * lda + i] * (long double)A[k * lda + j];
                long double r = (long double)alpha * s;
                if (beta != 0.0)
                    r += (long double)beta * (long double)C[i * ldc + j];
                C[i * ldc + j] = (double)r;
            } else {
                double s = 0.0;
                for (int64_t k = 0; k < N; ++k)
                    s += A[k * lda + i] * A[k * lda + j];
                if (beta == 0.0)
                    C[i * ldc + j] = alpha * s;
                else
                    C[i * ldc + j] = beta * C[i * ldc + j] + alpha * s;
            }
        }
    }
}
