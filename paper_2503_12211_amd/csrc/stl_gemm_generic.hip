// Any-shape batched plane product on the matrix cores in fp32 (v_mfma_f32_32x32x2_f32: fp32 operands, fp32
// accumulation).  This is the path for fp32 storage and for bf16 shapes the bf16 MFMA kernels do not take (ragged
// contiguous dimensions; their values are widened to fp32 on the way into LDS, which is exact).  LDS-tiled
// 128 x 128 x 16, 256 threads = four wavefronts of 64 x 64; edges are zero-filled on load and masked on store.
#include "stl_kernels.h"
#include "stl_device.h"


namespace stl {

// MFMA accumulator layout of v_mfma_f32_32x32x2_f32: lane (j = lane % 32, h = lane / 32) supplies A[row j][k = h] and
// B[k = h][column j]; accumulator e of the lane is C[row 8 (e / 4) + 4 h + e % 4][column j].
template <typename T, typename TO, bool ACC>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const T *__restrict__ A, const T *__restrict__ B,
                                                           TO *__restrict__ Out, int Mi, int Nj, int Kl, int a_km,
                                                           int b_km, int a_pg, int b_pg, int o_pg, int batch, int nb)
{
    constexpr int BT = 128, KC = 16, PAD = 4;          // 128 x 128 block, 16 contraction elements per step
    __shared__ float sA[KC][BT + PAD];                 // [l][i]: a fragment read takes 32 consecutive i of one l
    __shared__ float sB[KC][BT + PAD];                 // [l][j]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wi = (wave >> 1) * 64, wj = (wave & 1) * 64;      // four wavefronts, 64 x 64 each (2 x 2 MFMA tiles)
    const int fj = lane & 31, fh = lane >> 5;
  for (int by = blockIdx.y; by * BT < Mi; by += gridDim.y)        // block rows beyond the grid's second extent
  for (int z = blockIdx.z; z < batch * nb; z += gridDim.z) {      // (stacked problem, plane) pairs
    const int p = z % batch, pb = z / batch;
    const int a_r0 = pb * (a_km ? Kl : Mi), b_r0 = pb * (b_km ? Kl : Nj), o_r0 = pb * Mi;
    // element (row, col) of plane p of an operand stored [row][col] with `ld` columns, rows in groups of pg
    auto at = [&](int row, int col, int pg, int ld) { return plane_row_base(row, pg, batch, ld) + (size_t)p * pg * ld + col; };
    const int i0 = by * BT, j0 = blockIdx.x * BT;
    f32x16_t acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

    for (int l0 = 0; l0 < Kl; l0 += KC) {
        for (int e = threadIdx.x; e < BT * KC; e += 256) {
            // pick the index that is contiguous in memory as the fast one
            int ii, ll;
            if (!a_km) { ll = e & (KC - 1); ii = e / KC; } else { ii = e & (BT - 1); ll = e / BT; }
            const int gi = i0 + ii, gl = l0 + ll;
            sA[ll][ii] = (gi < Mi && gl < Kl) ? Elem<T>::ld(A + (a_km ? at(a_r0 + gl, gi, a_pg, Mi) : at(a_r0 + gi, gl, a_pg, Kl))) : 0.f;
            int jj, l2;
            if (!b_km) { l2 = e & (KC - 1); jj = e / KC; } else { jj = e & (BT - 1); l2 = e / BT; }
            const int gj = j0 + jj, gl2 = l0 + l2;
            sB[l2][jj] = (gj < Nj && gl2 < Kl) ? Elem<T>::ld(B + (b_km ? at(b_r0 + gl2, gj, b_pg, Nj) : at(b_r0 + gj, gl2, b_pg, Kl))) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int l = 0; l < KC; l += 2) {
            float fa[2], fb[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                fa[u] = sA[l + fh][wi + 32 * u + fj];
                fb[u] = sB[l + fh][wj + 32 * u + fj];
            }
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int v = 0; v < 2; ++v) acc[u][v] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[u], fb[v], acc[u][v], 0, 0, 0);
        }
        __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int v = 0; v < 2; ++v)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int gi = i0 + wi + 32 * u + 8 * (e >> 2) + 4 * fh + (e & 3), gj = j0 + wj + 32 * v + fj;
                if (gi < Mi && gj < Nj) {
                    TO *o = Out + at(o_r0 + gi, gj, o_pg, Nj);
                    if (ACC) Elem<TO>::st(o, Elem<TO>::ld(o) + acc[u][v][e]);
                    else Elem<TO>::st(o, acc[u][v][e]);
                }
            }
  }
}

template <typename T, typename TO, bool ACC>
static hipError_t launch_t(const GemmDesc &g, const void *A, const void *B, void *Out, hipStream_t s)
{
    const long zs = (long)g.batch * g.nb;
    const int rows = (g.Mi + 127) / 128;
    dim3 grid((g.Nj + 127) / 128, (unsigned)(rows > 65535 ? 65535 : rows), (unsigned)(zs > 65535 ? 65535 : zs));   // the kernel strides over both
    hipLaunchKernelGGL((gemm_generic_kernel<T, TO, ACC>), grid, dim3(256), 0, s, (const T *)A, (const T *)B, (TO *)Out,
                       g.Mi, g.Nj, g.Kl, (int)g.a_kmajor, (int)g.b_kmajor, g.a_rows_per_group(), g.b_rows_per_group(),
                       g.o_rows_per_group(), g.batch, g.nb);
    return hipGetLastError();
}

hipError_t launch_plane_gemm_generic(int dtype, const GemmDesc &g, const void *A, const void *B, void *Out,
                                     hipStream_t s)
{
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
    if (dtype == 1 && plane_gemm_wide_eligible(g)) return launch_plane_gemm_wide(g, A, B, Out, s);
    if (dtype == 1 && plane_gemm_pipe_eligible(g)) return launch_plane_gemm_pipe(g, A, B, Out, s);
    if (dtype == 1 && plane_gemm_mfma_eligible(g)) return launch_plane_gemm_mfma(g, A, B, Out, s);
    return launch_plane_gemm_generic(dtype, g, A, B, Out, s);
}

}  // namespace stl
