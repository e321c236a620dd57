// Tile-level linear maps of the STL operator: encode (step (i) of Algorithm 1), decode
// (step (iii)) and the two basis-gradient reductions.  All of these stream a matrix once
// through HBM; arithmetic is fp32.
#include "stl_kernels.h"
#include "stl_device.h"

namespace stl {

// ---------------------------------------------------------------------------------------
// encode:  P[p][I][L] = sum_q E[p][q] * A[4I + q/4][4L + q%4]        (planes of encoded tiles)
// One thread per tile; lanes run along L so that every row segment and every plane row is
// read / written contiguously by a wavefront.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void encode_kernel(const T *__restrict__ A, const T *__restrict__ E,
                                                     T *__restrict__ P, int R, int Cc, int r)
{
    __shared__ float sE[64 * 16];
    const int tid = threadIdx.y * blockDim.x + threadIdx.x;
    for (int i = tid; i < r * 16; i += 256) sE[i] = Elem<T>::ld(E + i);
    __syncthreads();

    const int L = blockIdx.x * blockDim.x + threadIdx.x;
    const int I = blockIdx.y * blockDim.y + threadIdx.y;
    if (L >= Cc || I >= R) return;

    const size_t ld = (size_t)Cc * 4;
    float x[16];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) x[a * 4 + b] = Elem<T>::ld(A + ((size_t)I * 4 + a) * ld + (size_t)L * 4 + b);

    const size_t plane = (size_t)R * Cc;
    T *out = P + (size_t)I * Cc + L;
    for (int p = 0; p < r; ++p) {
        float s = 0.f;
#pragma unroll
        for (int q = 0; q < 16; ++q) s = fmaf(sE[p * 16 + q], x[q], s);
        Elem<T>::st(out + (size_t)p * plane, s);
    }
}

// ---------------------------------------------------------------------------------------
// decode:  Cmat[4I + q/4][4J + q%4] = sum_p Dm[p][q] * P[p][I][J]     (+ optional GELU)
// ---------------------------------------------------------------------------------------
template <typename T, bool GELU>
__global__ __launch_bounds__(256) void decode_kernel(const T *__restrict__ P, const T *__restrict__ Dm,
                                                     T *__restrict__ Cmat, int R, int Cc, int r)
{
    __shared__ float sD[64 * 16];
    const int tid = threadIdx.y * blockDim.x + threadIdx.x;
    for (int i = tid; i < r * 16; i += 256) sD[i] = Elem<T>::ld(Dm + i);
    __syncthreads();

    const int J = blockIdx.x * blockDim.x + threadIdx.x;
    const int I = blockIdx.y * blockDim.y + threadIdx.y;
    if (J >= Cc || I >= R) return;

    const size_t plane = (size_t)R * Cc;
    const T *in = P + (size_t)I * Cc + J;
    float c[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) c[q] = 0.f;
    for (int p = 0; p < r; ++p) {
        const float y = Elem<T>::ld(in + (size_t)p * plane);
#pragma unroll
        for (int q = 0; q < 16; ++q) c[q] = fmaf(sD[p * 16 + q], y, c[q]);
    }
    const size_t ld = (size_t)Cc * 4;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            float v = c[a * 4 + b];
            if (GELU) v = gelu_erf(v);
            Elem<T>::st(Cmat + ((size_t)I * 4 + a) * ld + (size_t)J * 4 + b, v);
        }
}

// ---------------------------------------------------------------------------------------
// basis gradients:  G[p][q] (+)= sum_{I,J} P[p][I][J] * V[4I + q/4][4J + q%4]
// (dD with P=Yhat, V=dC;  dE_X with P=dXhat, V=X).  Two deterministic stages: every block
// sums a fixed range of tiles in a fixed order into part[block][p][q]; the second stage
// adds the partials in block order.  No atomics, so results are bitwise reproducible.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void outer_partial_kernel(const T *__restrict__ P, const T *__restrict__ V,
                                                            float *__restrict__ part, int R, int Cc, int r,
                                                            int tiles_per_block)
{
    // 256 threads: q = tid & 15, tile lane = tid >> 4 (16 tiles in flight); loop over planes.
    __shared__ float red[16][16];
    const int q = threadIdx.x & 15, tl = threadIdx.x >> 4;
    const size_t T_total = (size_t)R * Cc;
    const size_t t0 = (size_t)blockIdx.x * tiles_per_block;
    size_t t1 = t0 + tiles_per_block;
    if (t1 > T_total) t1 = T_total;
    const size_t ld = (size_t)Cc * 4;
    for (int p = 0; p < r; ++p) {
        float s = 0.f;
        for (size_t tile = t0 + tl; tile < t1; tile += 16) {
            const size_t I = tile / Cc, J = tile % Cc;
            const float v = Elem<T>::ld(V + (I * 4 + (q >> 2)) * ld + J * 4 + (q & 3));
            const float y = Elem<T>::ld(P + (size_t)p * T_total + tile);
            s = fmaf(y, v, s);
        }
        red[tl][q] = s;
        __syncthreads();
        if (tl == 0) {
            float tot = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) tot += red[i][q];
            part[((size_t)blockIdx.x * r + p) * 16 + q] = tot;
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(256) void outer_final_kernel(const float *__restrict__ part, float *__restrict__ G,
                                                          int nblocks, int n_out, int accumulate)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_out) return;
    float s = 0.f;
    for (int b = 0; b < nblocks; ++b) s += part[(size_t)b * n_out + i];
    G[i] = accumulate ? G[i] + s : s;
}

// ---------------------------------------------------------------------------------------
// host launchers
// ---------------------------------------------------------------------------------------
template <typename T>
static hipError_t launch_encode_t(const void *A, const void *E, void *P, int R, int Cc, int r, hipStream_t s)
{
    dim3 block(64, 4), grid((Cc + 63) / 64, (R + 3) / 4);
    hipLaunchKernelGGL(encode_kernel<T>, grid, block, 0, s, (const T *)A, (const T *)E, (T *)P, R, Cc, r);
    return hipGetLastError();
}

hipError_t launch_encode(int dtype, const void *A, const void *E, void *P, int R, int Cc, int r, hipStream_t s)
{
    return dtype == 0 ? launch_encode_t<float>(A, E, P, R, Cc, r, s) : launch_encode_t<bf16_t>(A, E, P, R, Cc, r, s);
}

template <typename T>
static hipError_t launch_decode_t(const void *P, const void *Dm, void *Cmat, int R, int Cc, int r, bool gelu,
                                  hipStream_t s)
{
    dim3 block(64, 4), grid((Cc + 63) / 64, (R + 3) / 4);
    if (gelu)
        hipLaunchKernelGGL((decode_kernel<T, true>), grid, block, 0, s, (const T *)P, (const T *)Dm, (T *)Cmat, R, Cc, r);
    else
        hipLaunchKernelGGL((decode_kernel<T, false>), grid, block, 0, s, (const T *)P, (const T *)Dm, (T *)Cmat, R, Cc, r);
    return hipGetLastError();
}

hipError_t launch_decode(int dtype, const void *P, const void *Dm, void *Cmat, int R, int Cc, int r, bool gelu,
                         hipStream_t s)
{
    return dtype == 0 ? launch_decode_t<float>(P, Dm, Cmat, R, Cc, r, gelu, s)
                      : launch_decode_t<bf16_t>(P, Dm, Cmat, R, Cc, r, gelu, s);
}

int outer_reduce_blocks(int64_t tiles)
{
    int64_t nb = (tiles + OUTER_TILES_PER_BLOCK - 1) / OUTER_TILES_PER_BLOCK;
    return (int)nb;
}

hipError_t launch_outer_reduce(int dtype, const void *P, const void *V, float *G, float *part, int R, int Cc, int r,
                               int accumulate, hipStream_t s)
{
    const int nb = outer_reduce_blocks((int64_t)R * Cc);
    if (dtype == 0)
        hipLaunchKernelGGL(outer_partial_kernel<float>, dim3(nb), dim3(256), 0, s, (const float *)P, (const float *)V,
                           part, R, Cc, r, OUTER_TILES_PER_BLOCK);
    else
        hipLaunchKernelGGL(outer_partial_kernel<bf16_t>, dim3(nb), dim3(256), 0, s, (const bf16_t *)P,
                           (const bf16_t *)V, part, R, Cc, r, OUTER_TILES_PER_BLOCK);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int n_out = r * 16;
    hipLaunchKernelGGL(outer_final_kernel, dim3((n_out + 255) / 256), dim3(256), 0, s, part, G, nb, n_out, accumulate);
    return hipGetLastError();
}

}  // namespace stl
