/* Plain float32 matrix product with every output element accumulated over k strictly in order, one
 * fused multiply-add per term: c = fma(a_ik, b_kj, c).  This is the summation order of a single
 * accumulator that walks K from 0 to K-1 (what a matrix-core tile does), unlike a blocked BLAS sgemm,
 * which sums partial blocks.  Host test helper for the fp32 rounding floor of the Newton-DB
 * iteration (paper Section 3.3); it is neither part of the library nor of the oracle.
 *   C[n][n] = A[n][n] B[n][n], row-major.  upper != 0: only the elements on or above the diagonal
 *   are computed and the rest mirrored (the residual product in symmetric mode). */
#include <math.h>
#include <string.h>

void seq_sgemm(int n, const float* A, const float* B, float* C, int upper) {
#pragma omp parallel for schedule(dynamic, 8)
    for (int i = 0; i < n; ++i) {
        float* c = C + (size_t)i * n;
        memset(c, 0, sizeof(float) * (size_t)n);
        const int j0 = upper ? i : 0;
        for (int k = 0; k < n; ++k) {
            const float a = A[(size_t)i * n + k];
            const float* b = B + (size_t)k * n;
            for (int j = j0; j < n; ++j) c[j] = fmaf(a, b[j], c[j]);
        }
    }
    if (upper) {
#pragma omp parallel for schedule(dynamic, 8)
        for (int i = 1; i < n; ++i)
            for (int j = 0; j < i; ++j) C[(size_t)i * n + j] = C[(size_t)j * n + i];
    }
}
