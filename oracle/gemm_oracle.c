/*
 * CPU oracle for the local matrix multiplies of a tensor-parallel FC layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct
 * definition that the GPU library is checked against.  It shares no code with
 * the GPU path and the product never calls it.
 *
 * What is computed (paper Sec. IV-A, the paragraph that introduces the three
 * matrix multiplies of an FC layer, and Algorithm 1 lines 3, 11 and 13):
 *   forward          O      = I    x W
 *   backward (data)  dL/dI  = dL/dO x W^T
 *   backward (weight)dL/dW  = I^T  x dL/dO
 * Every one of them is a plain product  C[M,N] = sum_k a(i,k) * b(k,j)  whose
 * operands are bf16 values held in row-major buffers.  The way a(i,k) and
 * b(k,j) are found in the buffers is the "mode" of Sec. IV-C:
 *   NN: A is [M,K], B is [K,N]   a(i,k)=A[i*K+k]  b(k,j)=B[k*N+j]
 *   NT: A is [M,K], B is [N,K]   a(i,k)=A[i*K+k]  b(k,j)=B[j*K+k]
 *   TN: A is [K,M], B is [K,N]   a(i,k)=A[k*M+i]  b(k,j)=B[k*N+j]
 *
 * Arithmetic: each bf16 value is decoded exactly to fp64, products and sums
 * are fp64, k runs upward from 0, the result is left in fp64 (no rounding to
 * bf16 here).  A bf16 x bf16 product has at most 16 significant bits, so every
 * product is exact in fp64; only the K-term sum rounds (relative error at most
 * about K * 2^-53 of sum |a||b|).
 *
 * Parity pins: tests/test_oracle_pins.py (brute force in exact integer
 * arithmetic, identity, transpose identity, linearity, closed forms, finite
 * differences of the forward, numpy fp64 matmul).
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>

enum { ORACLE_NN = 0, ORACLE_NT = 1, ORACLE_TN = 2 };

/* bf16 -> fp64, exact: a bf16 is the upper half of an IEEE binary32. */
static inline double bf16_to_f64(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static inline double elem_a(const uint16_t *A, int layout, int64_t M, int64_t K,
                            int64_t i, int64_t k)
{
    return bf16_to_f64(layout == ORACLE_TN ? A[k * M + i] : A[i * K + k]);
}

static inline double elem_b(const uint16_t *B, int layout, int64_t N, int64_t K,
                            int64_t k, int64_t j)
{
    return bf16_to_f64(layout == ORACLE_NT ? B[j * K + k] : B[k * N + j]);
}

/*
 * Full product.  C is [M,N] row-major fp64, written by this call.
 * Rows of C are independent, so they are shared out over OpenMP threads; within
 * a row every C[i][j] is the sum over k = 0..K-1 in that order.
 * Returns 0, or -1 on a bad argument.
 */
int oracle_gemm_bf16_f64(int64_t M, int64_t N, int64_t K, int layout,
                         const uint16_t *A, const uint16_t *B, double *C,
                         int nthreads)
{
    if (M < 0 || N < 0 || K < 0 || layout < 0 || layout > 2) return -1;
    if (M == 0 || N == 0) return 0;
    if (!C || (K > 0 && (!A || !B))) return -1;
    if (nthreads < 1) nthreads = 1;

#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int64_t i = 0; i < M; ++i) {
        double *c = C + i * N;
        if (layout == ORACLE_NT) {
            /* both operands run along k in memory: one dot product per (i,j) */
            for (int64_t j = 0; j < N; ++j) {
                double s = 0.0;
                for (int64_t k = 0; k < K; ++k)
                    s += elem_a(A, layout, M, K, i, k) * elem_b(B, layout, N, K, k, j);
                c[j] = s;
            }
        } else {
            /* B rows run along j in memory: add a(i,k) * B[k,:] for k = 0,1,.. */
            for (int64_t j = 0; j < N; ++j) c[j] = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                const double a = elem_a(A, layout, M, K, i, k);
                for (int64_t j = 0; j < N; ++j)
                    c[j] += a * elem_b(B, layout, N, K, k, j);
            }
        }
    }
    return 0;
}

/*
 * The same definition evaluated only at the nsamp positions (ii[s], jj[s]):
 * out[s] = sum_k a(ii[s],k) * b(k,jj[s]).  For problem sizes whose full
 * product would take the CPU many minutes.
 */
int oracle_gemm_bf16_f64_at(int64_t M, int64_t N, int64_t K, int layout,
                            const uint16_t *A, const uint16_t *B,
                            int64_t nsamp, const int64_t *ii, const int64_t *jj,
                            double *out, int nthreads)
{
    if (M < 0 || N < 0 || K < 0 || layout < 0 || layout > 2 || nsamp < 0) return -1;
    if (nsamp == 0) return 0;
    if (!ii || !jj || !out || (K > 0 && (!A || !B))) return -1;
    for (int64_t s = 0; s < nsamp; ++s)
        if (ii[s] < 0 || ii[s] >= M || jj[s] < 0 || jj[s] >= N) return -1;
    if (nthreads < 1) nthreads = 1;

#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int64_t s = 0; s < nsamp; ++s) {
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k)
            acc += elem_a(A, layout, M, K, ii[s], k) * elem_b(B, layout, N, K, k, jj[s]);
        out[s] = acc;
    }
    return 0;
}
