/*
 * stl_oracle.c -- plain fp64 CPU oracle of the Strassen-Tile (STL) operator.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct reference
 * that the GPU library is checked against.  Only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may call it; the product path never does.
 * It shares no code, header, table or helper with the HIP kernels.
 *
 * Notation (paper, Section "Strassen-Tile Operator", Definition 3.1 / Eq. (2)),
 * with the letters used throughout this repository:
 *   X  : m x k activations,  W : k x n weights,  C = X <> W : m x n
 *   t  : tile size,  r : tensor rank,  M=m/t, K=k/t, N=n/t tile counts
 *   E_X, E_W, D : r x t^2 row-major (Definition 3.1); the decoder is applied as D^T
 *   vec(T)[a*t+b] = T[a][b]   (row-major vectorisation of a t x t tile)
 *   What[p][L][J] = (E_W vec W_{L,J})_p            (encoded weight planes, Remark
 *                                                   "Fake Encoding" and the plane
 *                                                   definition before Claim 3.4)
 *
 * Everything is double precision; nothing is blocked, fused or reordered beyond
 * what the definition states.  OpenMP, when enabled, only distributes
 * independent output tiles (forward) or independent output entries (backward)
 * over threads; each entry is still summed in the written order.
 *
 * Parity pins (see tests): exact bases r=t^3 and Strassen (r=7 at t=2, r=49 at
 * t=4) reproduce X*W; contraction with the bilinear-map tensor sum_p E_X(x)E_W(x)D;
 * bilinearity; additivity over rank subsets; finite differences and Euler
 * identities for every gradient.  No function here is "parity unpinned".
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* element (a,b) of tile (I,L) of a row-major matrix with `ld` columns */
#define TILE_AT(A, ld, t, I, L, a, b) ((A)[((size_t)(I) * (t) + (a)) * (size_t)(ld) + (size_t)(L) * (t) + (b)])

int stl_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void stl_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/*
 * W-encoding (definition of the planes W^(p) before Claim 3.4; Remark on keeping
 * only encoded tiles): What[p][L][J] = sum_q E_W[p][q] * vec(W_{L,J})[q].
 * W is k x n row-major; What is r x K x N, plane-major, each plane row-major.
 */
void stl_oracle_encode_weight(int64_t k, int64_t n, int t, int r,
                              const double *W, const double *E_W, double *What)
{
    const int64_t K = k / t, N = n / t;
    const int tt = t * t;
    for (int p = 0; p < r; ++p)
        for (int64_t L = 0; L < K; ++L)
            for (int64_t J = 0; J < N; ++J) {
                double s = 0.0;
                for (int a = 0; a < t; ++a)
                    for (int b = 0; b < t; ++b)
                        s += E_W[(size_t)p * tt + a * t + b] * TILE_AT(W, n, t, L, J, a, b);
                What[((size_t)p * K + L) * N + J] = s;
            }
}

/*
 * X-encoding into planes (step (i) of the three-step algorithm):
 * Xhat[p][I][L] = sum_q E_X[p][q] * vec(X_{I,L})[q].   Xhat is r x M x K.
 */
void stl_oracle_encode_x(int64_t m, int64_t k, int t, int r,
                         const double *X, const double *E_X, double *Xhat)
{
    const int64_t M = m / t, K = k / t;
    const int tt = t * t;
    for (int p = 0; p < r; ++p)
        for (int64_t I = 0; I < M; ++I)
            for (int64_t L = 0; L < K; ++L) {
                double s = 0.0;
                for (int a = 0; a < t; ++a)
                    for (int b = 0; b < t; ++b)
                        s += E_X[(size_t)p * tt + a * t + b] * TILE_AT(X, k, t, I, L, a, b);
                Xhat[((size_t)p * M + I) * K + L] = s;
            }
}

/*
 * Forward, Eq. (2) taken literally, restricted to output tiles
 * I in [I0,I1), J in [J0,J1) (the full operator is I0=J0=0, I1=M, J1=N):
 *
 *   vec(C_{I,J}) = D^T ( sum_L (E_X vec X_{I,L}) (.) What[:,L,J] )
 *
 * The encoded sum (the "encoding of C_{I,J}") is optionally returned in
 * Yhat_blk[p][I-I0][J-J0] (may be NULL).  C_blk is (I1-I0)*t x (J1-J0)*t
 * row-major.  The decode is applied once per output tile, after the L sum.
 */
void stl_oracle_forward_block(int64_t m, int64_t k, int64_t n, int t, int r,
                              const double *X, const double *What,
                              const double *E_X, const double *D,
                              int64_t I0, int64_t I1, int64_t J0, int64_t J1,
                              double *C_blk, double *Yhat_blk)
{
    const int64_t K = k / t, N = n / t;
    const int tt = t * t;
    const int64_t nI = I1 - I0, nJ = J1 - J0;
    const int64_t ldc = nJ * t;
    (void)m;
#pragma omp parallel
    {
        double *acc = (double *)malloc(sizeof(double) * (size_t)r);
        double *xh = (double *)malloc(sizeof(double) * (size_t)r);
#pragma omp for collapse(2) schedule(static)
        for (int64_t I = I0; I < I1; ++I)
            for (int64_t J = J0; J < J1; ++J) {
                for (int p = 0; p < r; ++p) acc[p] = 0.0;
                for (int64_t L = 0; L < K; ++L) {
                    /* E_X * vec(X_{I,L}) */
                    for (int p = 0; p < r; ++p) {
                        double s = 0.0;
                        for (int a = 0; a < t; ++a)
                            for (int b = 0; b < t; ++b)
                                s += E_X[(size_t)p * tt + a * t + b] * TILE_AT(X, k, t, I, L, a, b);
                        xh[p] = s;
                    }
                    /* Hadamard product with the encoded weight tile, summed over L */
                    for (int p = 0; p < r; ++p)
                        acc[p] += xh[p] * What[((size_t)p * K + L) * N + J];
                }
                if (Yhat_blk)
                    for (int p = 0; p < r; ++p)
                        Yhat_blk[((size_t)p * nI + (I - I0)) * nJ + (J - J0)] = acc[p];
                /* decode: vec(C_{I,J})[q] = sum_p D[p][q] * acc[p] */
                for (int a = 0; a < t; ++a)
                    for (int b = 0; b < t; ++b) {
                        double s = 0.0;
                        for (int p = 0; p < r; ++p) s += D[(size_t)p * tt + a * t + b] * acc[p];
                        C_blk[((size_t)(I - I0) * t + a) * ldc + (size_t)(J - J0) * t + b] = s;
                    }
            }
        free(acc);
        free(xh);
    }
}

void stl_oracle_forward(int64_t m, int64_t k, int64_t n, int t, int r,
                        const double *X, const double *What,
                        const double *E_X, const double *D,
                        double *C, double *Yhat)
{
    stl_oracle_forward_block(m, k, n, t, r, X, What, E_X, D, 0, m / t, 0, n / t, C, Yhat);
}

/*
 * Backward.  The paper only states that gradients w.r.t. the encoders, the
 * decoder and the weights exist (Section "Strassen-Tile Operator", first
 * paragraph); the formulas below are the chain rule through the three linear
 * steps encode -> per-plane product -> decode, for the scalar loss <dC, C>:
 *
 *   dc[I][J][q]   := tile view of dC
 *   dD[p][q]      = sum_{I,J} Yhat[p][I][J] * dc[I][J][q]
 *   dYhat[p][I][J]= sum_q D[p][q] * dc[I][J][q]
 *   dXhat[p][I][L]= sum_J dYhat[p][I][J] * What[p][L][J]
 *   dWhat[p][L][J]= sum_I Xhat[p][I][L] * dYhat[p][I][J]
 *   dx[I][L][q]   = sum_p E_X[p][q] * dXhat[p][I][L]          -> dX
 *   dE_X[p][q]    = sum_{I,L} dXhat[p][I][L] * x[I][L][q]
 *
 * Outputs: dX m x k, dWhat r x K x N, dE_X r x t^2, dD r x t^2 (all overwritten).
 * Any output pointer may be NULL to skip it.
 */
void stl_oracle_backward(int64_t m, int64_t k, int64_t n, int t, int r,
                         const double *X, const double *What,
                         const double *E_X, const double *D, const double *dC,
                         double *dX, double *dWhat, double *dE_X, double *dD)
{
    const int64_t M = m / t, K = k / t, N = n / t;
    const int tt = t * t;
    double *Xhat = (double *)malloc(sizeof(double) * (size_t)r * M * K);
    double *Yhat = (double *)malloc(sizeof(double) * (size_t)r * M * N);
    double *dYhat = (double *)malloc(sizeof(double) * (size_t)r * M * N);
    double *dXhat = (double *)malloc(sizeof(double) * (size_t)r * M * K);

    stl_oracle_encode_x(m, k, t, r, X, E_X, Xhat);

    /* Yhat[p] = Xhat[p] * What[p]  (Claim 3.4) */
#pragma omp parallel for collapse(2) schedule(static)
    for (int p = 0; p < r; ++p)
        for (int64_t I = 0; I < M; ++I)
            for (int64_t J = 0; J < N; ++J) {
                double s = 0.0;
                for (int64_t L = 0; L < K; ++L)
                    s += Xhat[((size_t)p * M + I) * K + L] * What[((size_t)p * K + L) * N + J];
                Yhat[((size_t)p * M + I) * N + J] = s;
            }

    /* dYhat: D applied (not transposed) to the tile view of dC */
#pragma omp parallel for collapse(2) schedule(static)
    for (int p = 0; p < r; ++p)
        for (int64_t I = 0; I < M; ++I)
            for (int64_t J = 0; J < N; ++J) {
                double s = 0.0;
                for (int a = 0; a < t; ++a)
                    for (int b = 0; b < t; ++b)
                        s += D[(size_t)p * tt + a * t + b] * TILE_AT(dC, n, t, I, J, a, b);
                dYhat[((size_t)p * M + I) * N + J] = s;
            }

    if (dD) {
#pragma omp parallel for schedule(static)
        for (int pq = 0; pq < r * tt; ++pq) {
            const int p = pq / tt, q = pq % tt, a = q / t, b = q % t;
            double s = 0.0;
            for (int64_t I = 0; I < M; ++I)
                for (int64_t J = 0; J < N; ++J)
                    s += Yhat[((size_t)p * M + I) * N + J] * TILE_AT(dC, n, t, I, J, a, b);
            dD[pq] = s;
        }
    }

    /* dXhat[p] = dYhat[p] * What[p]^T */
#pragma omp parallel for collapse(2) schedule(static)
    for (int p = 0; p < r; ++p)
        for (int64_t I = 0; I < M; ++I)
            for (int64_t L = 0; L < K; ++L) {
                double s = 0.0;
                for (int64_t J = 0; J < N; ++J)
                    s += dYhat[((size_t)p * M + I) * N + J] * What[((size_t)p * K + L) * N + J];
                dXhat[((size_t)p * M + I) * K + L] = s;
            }

    if (dWhat) {
        /* dWhat[p] = Xhat[p]^T * dYhat[p] */
#pragma omp parallel for collapse(2) schedule(static)
        for (int p = 0; p < r; ++p)
            for (int64_t L = 0; L < K; ++L)
                for (int64_t J = 0; J < N; ++J) {
                    double s = 0.0;
                    for (int64_t I = 0; I < M; ++I)
                        s += Xhat[((size_t)p * M + I) * K + L] * dYhat[((size_t)p * M + I) * N + J];
                    dWhat[((size_t)p * K + L) * N + J] = s;
                }
    }

    if (dX) {
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t I = 0; I < M; ++I)
            for (int64_t L = 0; L < K; ++L)
                for (int a = 0; a < t; ++a)
                    for (int b = 0; b < t; ++b) {
                        double s = 0.0;
                        for (int p = 0; p < r; ++p)
                            s += E_X[(size_t)p * tt + a * t + b] * dXhat[((size_t)p * M + I) * K + L];
                        TILE_AT(dX, k, t, I, L, a, b) = s;
                    }
    }

    if (dE_X) {
#pragma omp parallel for schedule(static)
        for (int pq = 0; pq < r * tt; ++pq) {
            const int p = pq / tt, q = pq % tt, a = q / t, b = q % t;
            double s = 0.0;
            for (int64_t I = 0; I < M; ++I)
                for (int64_t L = 0; L < K; ++L)
                    s += dXhat[((size_t)p * M + I) * K + L] * TILE_AT(X, k, t, I, L, a, b);
            dE_X[pq] = s;
        }
    }

    free(Xhat);
    free(Yhat);
    free(dYhat);
    free(dXhat);
}
