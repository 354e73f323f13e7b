/*
 * CPU oracle for the error-corrected SGEMM: TEST INFRASTRUCTURE ONLY.
 *
 * Nothing in the product path may call into this file.  It holds the two plain
 * definitions every result is judged against:
 *
 *   - the FP64 reference product of the FP32 inputs (the C_FP64 of Eq. eval-matmul,
 *     "toFP64(A) . toFP64(B)" computed in FP64), and
 *   - a naive FP32 matrix product as an FP32 SIMT unit would form it: one running
 *     FP32 sum per output element, k ascending, every multiply and every add rounded
 *     to nearest on its own (the file is built with -ffp-contract=off, so the
 *     compiler cannot fuse them).
 *
 * Both take the operands already laid out as plain row-major arrays,
 *   opA : M x K,  opA[i*K + k]      opB : K x N,  opB[k*N + j]
 *   Cin, Cout : M x N, [i*N + j]
 * (the Python wrapper does the transposition / leading-dimension bookkeeping, which
 * moves data but does no arithmetic).  The loop nest is i, k, j: for a fixed (i, j)
 * the running sum still sees k = 0, 1, 2, ... in order, exactly like the textbook
 * i, j, k nest; the only reason for the order is that the j loop walks memory
 * contiguously.  There is no blocking, unrolling by hand, or reassociation.
 *
 * The scaling step follows BLAS: Cout = alpha * sum + beta * Cin, and Cin is not
 * read at all when beta == 0.
 */
#include <stdint.h>
#include <stddef.h>
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

void oracle_gemm_fp32_naive(int64_t M, int64_t N, int64_t K, float alpha,
                            const float *opA, const float *opB, float beta,
                            const float *Cin, float *Cout)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < M; ++i) {
        float *acc = Cout + i * N;
        for (int64_t j = 0; j < N; ++j)
            acc[j] = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            const float a = opA[i * K + k];
            const float *b = opB + k * N;
            for (int64_t j = 0; j < N; ++j) {
                const float prod = a * b[j];
                acc[j] = acc[j] + prod;
            }
        }
        if (beta == 0.0f) {
            for (int64_t j = 0; j < N; ++j)
                acc[j] = alpha * acc[j];
        } else {
            const float *cin = Cin + i * N;
            for (int64_t j = 0; j < N; ++j) {
                const float scaled_sum = alpha * acc[j];
                const float scaled_cin = beta * cin[j];
                acc[j] = scaled_sum + scaled_cin;
            }
        }
    }
}

void oracle_gemm_fp64_ref(int64_t M, int64_t N, int64_t K, double alpha,
                          const float *opA, const float *opB, double beta,
                          const float *Cin, double *Cout)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < M; ++i) {
        double *acc = Cout + i * N;
        for (int64_t j = 0; j < N; ++j)
            acc[j] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double a = (double)opA[i * K + k];
            const float *b = opB + k * N;
            for (int64_t j = 0; j < N; ++j) {
                const double prod = a * (double)b[j];
                acc[j] = acc[j] + prod;
            }
        }
        if (beta == 0.0) {
            for (int64_t j = 0; j < N; ++j)
                acc[j] = alpha * acc[j];
        } else {
            const float *cin = Cin + i * N;
            for (int64_t j = 0; j < N; ++j) {
                const double scaled_sum = alpha * acc[j];
                const double scaled_cin = beta * (double)cin[j];
                acc[j] = scaled_sum + scaled_cin;
            }
        }
    }
}
