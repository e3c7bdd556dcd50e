/* Plain ascending-k fp32 contraction (TEST INFRASTRUCTURE ONLY; part of the CPU oracle's pins).
 *
 * Section 3.1 of the paper fixes the arithmetic of a mixed-precision contraction: half-precision operands, sums
 * accumulated in single precision.  This file states that literally, with no blocking, tiling or reordering:
 * for every output element, one fp32 accumulator that takes the products in ascending k.  The oracle's layer code
 * contracts with NumPy's matmul (a BLAS routine that blocks and orders the sum as it likes); tests/ pin that
 * library step against this definition (the two may differ only by fp32 summation order).
 *
 *   y[m][n] = sum_{k ascending} x[m][k] * w[n][k]          x: M x K, w: N x K, y: M x N, all row-major fp32
 *
 * Each product of two fp16-representable values is exact in fp32, so mul-then-add and a fused multiply-add give the
 * same bits; the compiler is told not to contract anyway (-ffp-contract=off) and not to reassociate (no -ffast-math).
 * Rows of y are independent, so the row loop may run on several threads without changing any element's order. */
#include <stddef.h>

void oracle_contract_nt_f32(const float* x, const float* w, float* y, long M, long N, long K) {
#pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m) {
        for (long n = 0; n < N; ++n) {
            float acc = 0.0f;
            for (long k = 0; k < K; ++k) acc += x[m * K + k] * w[n * K + k];
            y[m * N + n] = acc;
        }
    }
}
