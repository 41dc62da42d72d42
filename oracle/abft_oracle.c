/*
 * CPU oracle for the checksum-protected GEMM  --  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct loops.  Only tests, the smoke check and the
 * benchmark's CPU-baseline leg may call this; the product (the HIP library)
 * never does and shares no code with it.
 *
 * What is computed follows the paper's checksum description (Sec. III-B.1,
 * paragraph "Checksums"): for Y = X * W^T the input is summed over its rows,
 * the weight is reduced over its output dimension, and the dot product of the
 * two length-K vectors must equal the sum of all outputs.  The classic
 * row/column form the paper cites as its origin (Sec. I, Sec. II-B, Huang and
 * Abraham) keeps the two vector products un-summed:
 *      column checksum  cc = (e^T A) B      (length N, guards columns)
 *      row checksum     rc = A (B e)        (length M, guards rows)
 * and compares them with e^T C and C e.  The paper's scalar is the sum of
 * either vector.
 *
 * All matrices are addressed logically: element (r, c) of X lives at
 * X[r * rs + c * cs], so one routine serves both storage orders of B.
 * Every dot product runs with k ascending, one accumulator per output, in
 * int64 (integer path) or fp64 (floating-point path).  No blocking, no
 * intrinsics; OpenMP splits rows of the output only.
 */
#include <stdint.h>
#include <stddef.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* C[i][j] = sum_k A(i,k) * B(k,j), int8 inputs, int64 accumulate. C is M x N row-major. */
void oracle_gemm_i8(const int8_t *A, long a_rs, long a_cs,
                    const int8_t *B, long b_rs, long b_cs,
                    long M, long N, long K, int64_t *C)
{
#pragma omp parallel for schedule(static)
    for (long i = 0; i < M; ++i) {
        for (long j = 0; j < N; ++j) {
            int64_t s = 0;
            for (long k = 0; k < K; ++k)
                s += (int64_t)A[i * a_rs + k * a_cs] * (int64_t)B[k * b_rs + j * b_cs];
            C[i * N + j] = s;
        }
    }
}

/* Same product for already-decoded fp64 inputs, fp64 accumulate. */
void oracle_gemm_f64(const double *A, long a_rs, long a_cs,
                     const double *B, long b_rs, long b_cs,
                     long M, long N, long K, double *C)
{
#pragma omp parallel for schedule(static)
    for (long i = 0; i < M; ++i) {
        for (long j = 0; j < N; ++j) {
            double s = 0.0;
            for (long k = 0; k < K; ++k)
                s += A[i * a_rs + k * a_cs] * B[k * b_rs + j * b_cs];
            C[i * N + j] = s;
        }
    }
}

/* Input-side checksum vectors (both of length K):
 *   a[k] = sum_i A(i,k)   -- the input batch summed over its rows
 *   b[k] = sum_j B(k,j)   -- the weight reduced over its output dimension */
void oracle_encode_i64(const int64_t *A, long a_rs, long a_cs,
                       const int64_t *B, long b_rs, long b_cs,
                       long M, long N, long K, int64_t *a, int64_t *b)
{
    for (long k = 0; k < K; ++k) {
        int64_t s = 0;
        for (long i = 0; i < M; ++i) s += A[i * a_rs + k * a_cs];
        a[k] = s;
        int64_t t = 0;
        for (long j = 0; j < N; ++j) t += B[k * b_rs + j * b_cs];
        b[k] = t;
    }
}

void oracle_encode_f64(const double *A, long a_rs, long a_cs,
                       const double *B, long b_rs, long b_cs,
                       long M, long N, long K, double *a, double *b)
{
    for (long k = 0; k < K; ++k) {
        double s = 0.0;
        for (long i = 0; i < M; ++i) s += A[i * a_rs + k * a_cs];
        a[k] = s;
        double t = 0.0;
        for (long j = 0; j < N; ++j) t += B[k * b_rs + j * b_cs];
        b[k] = t;
    }
}

/* Predicted checksums from the inputs alone:
 *   cc[j] = sum_k a[k] B(k,j),  rc[i] = sum_k A(i,k) b[k],  s = sum_k a[k] b[k].
 * Integers: exact in int64 (callers keep |values| small enough; see the Python
 * wrapper's range assertion). */
void oracle_predict_i64(const int64_t *A, long a_rs, long a_cs,
                        const int64_t *B, long b_rs, long b_cs,
                        const int64_t *a, const int64_t *b,
                        long M, long N, long K,
                        int64_t *cc, int64_t *rc, int64_t *s)
{
    for (long j = 0; j < N; ++j) {
        int64_t t = 0;
        for (long k = 0; k < K; ++k) t += a[k] * B[k * b_rs + j * b_cs];
        cc[j] = t;
    }
    for (long i = 0; i < M; ++i) {
        int64_t t = 0;
        for (long k = 0; k < K; ++k) t += A[i * a_rs + k * a_cs] * b[k];
        rc[i] = t;
    }
    int64_t t = 0;
    for (long k = 0; k < K; ++k) t += a[k] * b[k];
    *s = t;
}

void oracle_predict_f64(const double *A, long a_rs, long a_cs,
                        const double *B, long b_rs, long b_cs,
                        const double *a, const double *b,
                        long M, long N, long K,
                        double *cc, double *rc, double *s)
{
    for (long j = 0; j < N; ++j) {
        double t = 0.0;
        for (long k = 0; k < K; ++k) t += a[k] * B[k * b_rs + j * b_cs];
        cc[j] = t;
    }
    for (long i = 0; i < M; ++i) {
        double t = 0.0;
        for (long k = 0; k < K; ++k) t += A[i * a_rs + k * a_cs] * b[k];
        rc[i] = t;
    }
    double t = 0.0;
    for (long k = 0; k < K; ++k) t += a[k] * b[k];
    *s = t;
}

/* Observed checksums of an M x N row-major matrix X (the output as stored):
 *   cc[j] = sum_i X[i][j],  rc[i] = sum_j X[i][j],  s = sum of everything. */
void oracle_observe_i64(const int64_t *X, long M, long N,
                        int64_t *cc, int64_t *rc, int64_t *s)
{
    for (long j = 0; j < N; ++j) {
        int64_t t = 0;
        for (long i = 0; i < M; ++i) t += X[i * N + j];
        cc[j] = t;
    }
    int64_t tot = 0;
    for (long i = 0; i < M; ++i) {
        int64_t t = 0;
        for (long j = 0; j < N; ++j) t += X[i * N + j];
        rc[i] = t;
        tot += t;
    }
    *s = tot;
}

void oracle_observe_f64(const double *X, long M, long N,
                        double *cc, double *rc, double *s)
{
    for (long j = 0; j < N; ++j) {
        double t = 0.0;
        for (long i = 0; i < M; ++i) t += X[i * N + j];
        cc[j] = t;
    }
    double tot = 0.0;
    for (long i = 0; i < M; ++i) {
        double t = 0.0;
        for (long j = 0; j < N; ++j) t += X[i * N + j];
        rc[i] = t;
        tot += t;
    }
    *s = tot;
}
