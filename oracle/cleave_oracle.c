/*
 * CPU oracle for Cleave's sub-GEMM hot path -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain reference that the tests and the benchmark's
 * cpu-baseline leg compare the GPU library against.  Nothing in the product
 * path may link, load or call it, and it shares no code with the HIP sources.
 *
 * What it computes (Cleave, Sec. 4.1 "Search space of GEMM"): a GEMM with
 * inputs A (m x n) and B (n x q) produces O (m x q); a device that receives
 * alpha rows of A and beta columns of B returns the alpha x beta sub-block
 * A' o B' of O, and the union of those sub-blocks is O.  Because the paper
 * preserves the numerical semantics of every GEMM (Sec. 3.2 "Seamless
 * training"), the reference result is simply the undecomposed product, in
 * fp64, over the stored input values.
 *
 * Everything here works on fp64 row-major operands that already are the
 * logical op(A) (M x K) and op(B) (K x N): the Python wrapper widens the
 * stored bf16/fp32 values (exactly) and applies any transpose as a data
 * layout step before calling in.
 *
 * Loop order is i-k-j with a scalar accumulation per output element in
 * ascending k; no blocking, no intrinsics, no BLAS.  OpenMP spreads the rows
 * of the output over the host cores.
 */
#include <stddef.h>
#include <stdint.h>
#include <omp.h>

/* Number of threads the parallel loops below will use. */
int oracle_num_threads(void) { return omp_get_max_threads(); }

/*
 * C[i, j] = sum_{k = k_begin}^{k_end - 1} A[i, k] * B[k, j]
 * for i in [0, M), j in [0, N).
 *
 * A: M rows, leading dimension lda (>= k_end), row-major.
 * B: at least k_end rows, leading dimension ldb (>= N), row-major.
 * C: M x N, leading dimension ldc, overwritten.
 *
 * With k_begin = 0 and k_end = K this is the undecomposed GEMM; with a
 * sub-range it is the partial product one K-split task contributes.  The
 * count of floating-point operations is 2*M*N*(k_end-k_begin), the
 * convention of the paper's computation-cost term (Sec. 4.1, Eq.
 * computation-cost).
 */
void oracle_gemm_f64(int64_t M, int64_t N, int64_t k_begin, int64_t k_end,
                     const double *A, int64_t lda,
                     const double *B, int64_t ldb,
                     double *C, int64_t ldc)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        double *c = C + i * ldc;
        for (int64_t j = 0; j < N; ++j)
            c[j] = 0.0;
        for (int64_t k = k_begin; k < k_end; ++k) {
            const double a = A[i * lda + k];
            const double *b = B + k * ldb;
            for (int64_t j = 0; j < N; ++j)
                c[j] += a * b[j];
        }
    }
}

/*
 * Parameter-server aggregation of K-split partial blocks (Sec. 3.2: the PS
 * aggregates the computed outputs).  `parts` holds `S` blocks of `count`
 * fp32 values each, block s at parts + s*stride.  The sum is a left fold in
 * fp32, ascending s: ((P0 + P1) + P2) + ...  Plain IEEE single adds, so the
 * result is reproducible bit for bit from the same partials.
 */
void oracle_fold_f32(int64_t S, int64_t count, int64_t stride,
                     const float *parts, float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < count; ++e) {
        volatile float acc = parts[e];
        for (int64_t s = 1; s < S; ++s) {
            volatile float t = acc + parts[s * stride + e];
            acc = t;
        }
        out[e] = acc;
    }
}

/* Same fold in fp64, for the oracle's own invariants. */
void oracle_fold_f64(int64_t S, int64_t count, int64_t stride,
                     const double *parts, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < count; ++e) {
        double acc = parts[e];
        for (int64_t s = 1; s < S; ++s)
            acc = acc + parts[s * stride + e];
        out[e] = acc;
    }
}
