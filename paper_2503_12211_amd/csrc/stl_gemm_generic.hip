// Any-shape batched plane product on the vector ALUs (fp32 multiply-add).  This is the path
// for fp32 storage and for bf16 shapes the MFMA kernel does not take (ragged contiguous
// dimensions).  LDS-tiled 64x64x16, 256 threads, 4x4 outputs per thread.
#include "stl_kernels.h"
#include "stl_device.h"


namespace stl {

template <typename T, typename TO, bool ACC>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const T *__restrict__ A, const T *__restrict__ B,
                                                           TO *__restrict__ Out, int Mi, int Nj, int Kl, int a_km,
                                                           int b_km, int a_pg, int b_pg, int o_pg, int batch, int nb)
{
    __shared__ float sA[16][64 + 4];
    __shared__ float sB[16][64 + 4];
  for (int z = blockIdx.z; z < batch * nb; z += gridDim.z) {      // (stacked problem, plane) pairs
    const int p = z % batch, pb = z / batch;
    const int a_r0 = pb * (a_km ? Kl : Mi), b_r0 = pb * (b_km ? Kl : Nj), o_r0 = pb * Mi;
    // element (row, col) of plane p of an operand stored [row][col] with `ld` columns, rows in groups of pg
    auto at = [&](int row, int col, int pg, int ld) { return plane_row_base(row, pg, batch, ld) + (size_t)p * pg * ld + col; };
    const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.f;

    for (int l0 = 0; l0 < Kl; l0 += 16) {
        for (int e = threadIdx.x; e < 64 * 16; e += 256) {
            // pick the index that is contiguous in memory as the fast one
            int ii, ll;
            if (!a_km) { ll = e & 15; ii = e >> 4; } else { ii = e & 63; ll = e >> 6; }
            const int gi = i0 + ii, gl = l0 + ll;
            sA[ll][ii] = (gi < Mi && gl < Kl) ? Elem<T>::ld(A + (a_km ? at(a_r0 + gl, gi, a_pg, Mi) : at(a_r0 + gi, gl, a_pg, Kl))) : 0.f;
            int jj, l2;
            if (!b_km) { l2 = e & 15; jj = e >> 4; } else { jj = e & 63; l2 = e >> 6; }
            const int gj = j0 + jj, gl2 = l0 + l2;
            sB[l2][jj] = (gj < Nj && gl2 < Kl) ? Elem<T>::ld(B + (b_km ? at(b_r0 + gl2, gj, b_pg, Nj) : at(b_r0 + gj, gl2, b_pg, Kl))) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int l = 0; l < 16; ++l) {
            float a[4], b[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { a[u] = sA[l][ty * 4 + u]; b[u] = sB[l][tx * 4 + u]; }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[u][v] = fmaf(a[u], b[v], acc[u][v]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int gi = i0 + ty * 4 + u, gj = j0 + tx * 4 + v;
            if (gi < Mi && gj < Nj) {
                TO *o = Out + at(o_r0 + gi, gj, o_pg, Nj);
                if (ACC) Elem<TO>::st(o, Elem<TO>::ld(o) + acc[u][v]);
                else Elem<TO>::st(o, acc[u][v]);
            }
        }
    __syncthreads();
  }
}

template <typename T, typename TO, bool ACC>
static hipError_t launch_t(const GemmDesc &g, const void *A, const void *B, void *Out, hipStream_t s)
{
    const long zs = (long)g.batch * g.nb;
    dim3 grid((g.Nj + 63) / 64, (g.Mi + 63) / 64, (unsigned)(zs > 65535 ? 65535 : zs));
    hipLaunchKernelGGL((gemm_generic_kernel<T, TO, ACC>), grid, dim3(256), 0, s, (const T *)A, (const T *)B, (TO *)Out,
                       g.Mi, g.Nj, g.Kl, (int)g.a_kmajor, (int)g.b_kmajor, g.a_rows_per_group(), g.b_rows_per_group(),
                       g.o_rows_per_group(), g.batch, g.nb);
    return hipGetLastError();
}

hipError_t launch_plane_gemm_generic(int dtype, const GemmDesc &g, const void *A, const void *B, void *Out,
                                     hipStream_t s)
{
    if ((g.Mi + 63) / 64 > 65535) return hipErrorInvalidValue;
    if (dtype == 0) {
        return g.accumulate ? launch_t<float, float, true>(g, A, B, Out, s) : launch_t<float, float, false>(g, A, B, Out, s);
    }
    if (g.out_f32)
        return g.accumulate ? launch_t<bf16_t, float, true>(g, A, B, Out, s)
                            : launch_t<bf16_t, float, false>(g, A, B, Out, s);
    return launch_t<bf16_t, bf16_t, false>(g, A, B, Out, s);
}

hipError_t launch_plane_gemm(int dtype, const GemmDesc &g, const void *A, const void *B, void *Out, hipStream_t s)
{
    if (dtype == 1 && plane_gemm_pipe_eligible(g)) return launch_plane_gemm_pipe(g, A, B, Out, s);
    if (dtype == 1 && plane_gemm_mfma_eligible(g)) return launch_plane_gemm_mfma(g, A, B, Out, s);
    return launch_plane_gemm_generic(dtype, g, A, B, Out, s);
}

}  // namespace stl
