// Forward variants that keep the r encoded output planes on chip (Definition 3.1 / Eq. (2) evaluated per
// output block: encode -> per-plane MFMA accumulation over L -> one decode per output tile):
//
//   EPILOGUE: Xhat comes from HBM (written by the encode kernel); the plane products and the decode run here.
//   FUSED:    X itself is read; the encode of every X sub-block runs here on MFMA, so no plane tensor ever
//             touches HBM (optionally Yhat is written for the backward pass).
//
// One workgroup (4 wavefronts) owns a block of 32 x 32 output tiles (128 x 128 entries of C) and ALL r <= 32
// planes of it: wavefront w accumulates planes w, w+4, ... (one 32x32x16 MFMA tile per plane, K = 16 tile
// columns L per step).  Operand sub-blocks arrive by LDS-DMA, double buffered.  After the L loop the r x 1024
// fp32 accumulators are exchanged through LDS and every thread decodes 4 tiles with D in fp32.
//
// Decode needs all planes of a tile in one workgroup, and r accumulator planes leave room for only ~1K output
// tiles per workgroup, so each operand element fetched from L2 feeds few MACs (16 flop per byte against 128 for a
// one-plane 256 x 256 block): this kernel is bound by the L2 -> LDS path, not by MFMA, and at every shape where the
// plane products take a measurable time the three-launch path is faster (6 x at the benchmark shape, where this
// kernel moves 26 GB through L2 at 20 TB/s, the rate the L2 -> LDS path gives).  It wins only where the whole
// operator is bound by launch latency: one launch instead of three for problems of a few microseconds, which is
// where the automatic variant choice uses it.
#include "stl_kernels.h"
#include "stl_device.h"

namespace stl {
namespace fused {

typedef short v4i16_t __attribute__((ext_vector_type(4)));
#define STL_LDS_PTR(p) ((__attribute__((address_space(3))) char *)(p))

constexpr int BI = 32, BJ = 32, KC = 16;          // block: 32 x 32 tiles, 16 tile columns of X per step
constexpr int SX_BYTES = 4 * BI * KC * 4 * 2;     // X sub-block: 128 rows x 64 entries  = 16 KB
constexpr int SD_BYTES = 32 * 16 * 4;             // decoder in fp32
// per plane: Xhat stage 32 x 16 bf16 = 1 KB, What stage 16 x 32 bf16 = 1 KB, exchanged accumulators 32 x 32 fp32 = 4 KB
template <int RP, bool ENCODE>
constexpr int smem_bytes()
{
    const int loop = ENCODE ? 2 * SX_BYTES + RP * 1024 + 2 * RP * 1024 : 2 * RP * 1024 + 2 * RP * 1024;
    const int exch = RP * 4096;
    return (loop > exch ? loop : exch) + SD_BYTES;
}

__device__ __forceinline__ void dma16(const bf16_t *g, uint32_t lds_wave_base)
{
    // LDS-DMA, 16 bytes per lane, lane L lands at lds_wave_base + 16 L.  Inline assembly so that the loop below
    // orders these loads itself (vmcnt + barrier) instead of the compiler draining them before every LDS read.
    const uint32_t l = __builtin_amdgcn_readfirstlane(lds_wave_base);
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(l) : "memory", "m0");
}
__device__ __forceinline__ void wait_dma() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void barrier() { asm volatile("s_barrier" ::: "memory"); }

// ENCODE: true = FUSED (reads X), false = EPILOGUE (reads Xhat).  RP: planes padded to 8, 16 or 32 (sizes the LDS
// stages and the accumulators, so that small r leaves room for several workgroups per CU).
template <int RP, bool ENCODE, bool GELU>
__global__ __launch_bounds__(256) void stl_block_kernel(const bf16_t *__restrict__ Xin,   // X (m x k) or Xhat (r x M x K)
                                                        const bf16_t *__restrict__ What, const bf16_t *__restrict__ E,
                                                        const bf16_t *__restrict__ Dm, bf16_t *__restrict__ C,
                                                        bf16_t *__restrict__ Ysave, int M, int K, int N, int r,
                                                        int blocks_j, int pg)
{
    extern __shared__ __align__(16) char smem[];
    // layout: [A-side staging x2][What stage x2]; the exchange buffer reuses everything after the L loop
    constexpr int PW = RP / 4;                        // planes per wavefront
    constexpr int SXH_BYTES = RP * 1024, SW_BYTES = RP * 1024;
    constexpr int A_STAGE = ENCODE ? SX_BYTES : SXH_BYTES;
    char *sA = smem;                                  // 2 stages of X (FUSED) or Xhat (EPILOGUE)
    char *sXh = smem + 2 * A_STAGE;                   // FUSED only: encoded stage, single buffer
    char *sW = sXh + (ENCODE ? SXH_BYTES : 0);        // 2 stages
    float *sD = reinterpret_cast<float *>(smem + smem_bytes<RP, ENCODE>() - SD_BYTES);
    const uint32_t lds0 = (uint32_t)(uintptr_t)STL_LDS_PTR(smem);
    const uint32_t ldsA = lds0, ldsW = lds0 + (uint32_t)(sW - smem);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int I0 = (blockIdx.x / blocks_j) * BI, J0 = (blockIdx.x % blocks_j) * BJ;
    const size_t k_elems = (size_t)K * 4, n_elems = (size_t)N * 4;

    for (int i = tid; i < r * 16; i += 256) sD[i] = bf16_to_f32(Dm[i]);

    // ---- DMA sources ------------------------------------------------------------------------------------
    // What: one instruction per plane (16 L rows x 64 bytes); lane -> (L = lane/4, 16-byte chunk = lane%4)
    const bf16_t *srcW[PW];
    {
        int jc = J0 + 8 * (lane & 3);
        jc = jc < N ? jc : N - 8;                     // columns past the edge feed only discarded outputs
#pragma unroll
        for (int t = 0; t < PW; ++t) {
            const int p = wave * PW + t;
            srcW[t] = What + ((size_t)(p < r ? p : 0) * K + (lane >> 2)) * N + jc;
        }
    }
    // A side
    const bf16_t *srcA[ENCODE ? 4 : PW];
    if (ENCODE) {
        // X sub-block: 128 rows x 128 bytes; instruction q covers rows 8q..8q+7; lane -> (row, 16-byte slot);
        // the slot holds logical chunk slot ^ ((row/4) & 7) so that the encode's 8-byte reads spread over banks
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int row = 8 * (wave * 4 + t) + (lane >> 3);
            const int c16 = (lane & 7) ^ ((row >> 2) & 7);
            long gr = (long)I0 * 4 + row;
            gr = gr < (long)M * 4 ? gr : (long)M * 4 - 1;
            srcA[t] = Xin + (size_t)gr * k_elems + 8 * c16;
        }
    } else {
        // Xhat: one instruction per plane (32 I rows x 32 bytes); lane -> (I = lane/2, half = lane%2)
        int gi = I0 + (lane >> 1);
        gi = gi < M ? gi : M - 1;
#pragma unroll
        for (int t = 0; t < PW; ++t) {
            const int p = wave * PW + t;
            srcA[t] = Xin + plane_row_base(gi, pg, r, K) + (size_t)(p < r ? p : 0) * pg * K + 8 * (lane & 1);
        }
    }
    auto issue = [&](int stage) {
        if (ENCODE) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                dma16(srcA[t], ldsA + stage * SX_BYTES + (wave * 4 + t) * 1024);
                srcA[t] += KC * 4;                    // 16 tile columns = 64 entries further
            }
        } else {
#pragma unroll
            for (int t = 0; t < PW; ++t) {
                dma16(srcA[t], ldsA + stage * SXH_BYTES + (wave * PW + t) * 1024);
                srcA[t] += KC;
            }
        }
#pragma unroll
        for (int t = 0; t < PW; ++t) {
            dma16(srcW[t], ldsW + stage * SW_BYTES + (wave * PW + t) * 1024);
            srcW[t] += (size_t)KC * N;
        }
    };

    // ---- encode operands (FUSED): E fragment, lane (plane = lane%32, h): E[plane][8h .. 8h+7] ------------------
    bf16x8_t fe;
    {
        u32x4_t ev = {0u, 0u, 0u, 0u};
        if (ENCODE && (lane & 31) < r) ev = *reinterpret_cast<const u32x4_t *>(E + (lane & 31) * 16 + 8 * (lane >> 5));
        fe = __builtin_bit_cast(bf16x8_t, ev);
    }

    // ---- fragment offsets --------------------------------------------------------------------------------
    const int frow = lane & 31, fh = lane >> 5;
    const int offA = frow * 32 + fh * 16;             // Xhat stage of one plane: [I][16 L], 32-byte rows
    int offB[2];                                      // What stage of one plane: [16 L][32 J], 64-byte rows
    {
        const int i = lane & 15, blk = (lane >> 4) & 1;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) offB[kk] = (8 * fh + 4 * kk + (i >> 2)) * 64 + (16 * blk + 4 * (i & 3)) * 2;
    }

    f32x16_t acc[PW];
#pragma unroll
    for (int t = 0; t < PW; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;

    const int nch = K / KC;
    issue(0);
    for (int c = 0; c < nch; ++c) {
        wait_dma();
        barrier();                                    // stage c landed for all; stage c+1's buffers are free
        if (c + 1 < nch) issue((c + 1) & 1);
        const char *stA = sA + (c & 1) * A_STAGE;
        const char *stW = sW + (c & 1) * SW_BYTES;
        const char *stXh = ENCODE ? sXh : stA;
        if (ENCODE) {
            // wavefront w encodes tile columns L = 4w .. 4w+3 of the 32 tile rows: 4 MFMAs, rows = planes,
            // columns = tile rows I; lane (I, h) supplies rows 2h, 2h+1 of tile (I, L)
            f32x16_t en[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int L = 4 * wave + u;
                u32x2_t x0, x1;
                {
                    const int row = 4 * frow + 2 * fh;
                    const int slot = (L >> 1) ^ (frow & 7);
                    x0 = *reinterpret_cast<const u32x2_t *>(stA + row * 128 + slot * 16 + (L & 1) * 8);
                    x1 = *reinterpret_cast<const u32x2_t *>(stA + (row + 1) * 128 + slot * 16 + (L & 1) * 8);
                }
                const u32x4_t bv = {x0[0], x0[1], x1[0], x1[1]};
                f32x16_t zero;
#pragma unroll
                for (int e = 0; e < 16; ++e) zero[e] = 0.f;
                en[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fe, __builtin_bit_cast(bf16x8_t, bv), zero, 0, 0, 0);
            }
            // accumulator e: plane 8*(e/4) + 4h + e%4, tile row I = lane%32; pack the 4 L values -> 8 bytes
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int p = 8 * (e >> 2) + 4 * fh + (e & 3);
                if (p < RP) {
                    const u32x2_t w = {pack_bf16x2(en[0][e], en[1][e]), pack_bf16x2(en[2][e], en[3][e])};
                    *reinterpret_cast<u32x2_t *>(sXh + p * 1024 + frow * 32 + wave * 8) = w;
                }
            }
            wait_lds();
            barrier();                                // encoded stage visible to all wavefronts
        }
#pragma unroll
        for (int t = 0; t < PW; ++t) {
            const int p = wave + 4 * t;
            if (p < r) {
                const bf16x8_t a = *reinterpret_cast<const bf16x8_t *>(stXh + p * 1024 + offA);
                const v4i16_t b0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) v4i16_t *)STL_LDS_PTR(stW + p * 1024 + offB[0]));
                const v4i16_t b1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) v4i16_t *)STL_LDS_PTR(stW + p * 1024 + offB[1]));
                struct { v4i16_t lo, hi; } both = {b0, b1};
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8_t, both), acc[t], 0, 0, 0);
            }
        }
    }

    // ---- exchange: accumulator e of plane p is Yhat[p][I = 8*(e/4) + 4h + e%4][J = lane%32] ---------------------
    barrier();
    float *sY = reinterpret_cast<float *>(smem);      // [p][I][J]
#pragma unroll
    for (int t = 0; t < PW; ++t) {
        const int p = wave + 4 * t;
        if (p < r) {
#pragma unroll
            for (int e = 0; e < 16; ++e) sY[(p * BI + 8 * (e >> 2) + 4 * fh + (e & 3)) * BJ + frow] = acc[t][e];
        }
    }
    __syncthreads();

    // ---- decode: 4 tiles per thread ---------------------------------------------------------------------------
#pragma unroll 1
    for (int it = 0; it < 4; ++it) {
        const int id = tid + 256 * it, I = id >> 5, J = id & 31;
        const int gi = I0 + I, gj = J0 + J;
        float cq[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) cq[q] = 0.f;
        for (int p = 0; p < r; ++p) {
            const float y = sY[(p * BI + I) * BJ + J];
            if (Ysave != nullptr && gi < M && gj < N) Ysave[plane_row_base(gi, pg, r, N) + (size_t)p * pg * N + gj] = f32_to_bf16(y);
#pragma unroll
            for (int q = 0; q < 16; ++q) cq[q] = fmaf(sD[p * 16 + q], y, cq[q]);
        }
        if (gi < M && gj < N) {
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                float c0 = cq[4 * a], c1 = cq[4 * a + 1], c2 = cq[4 * a + 2], c3 = cq[4 * a + 3];
                if (GELU) { c0 = gelu_erf(c0); c1 = gelu_erf(c1); c2 = gelu_erf(c2); c3 = gelu_erf(c3); }
                const u32x2_t w = {pack_bf16x2(c0, c1), pack_bf16x2(c2, c3)};
                *reinterpret_cast<u32x2_t *>(C + ((size_t)gi * 4 + a) * n_elems + (size_t)gj * 4) = w;
            }
        }
    }
}

}  // namespace fused

bool block_forward_eligible(int dtype, int M, int K, int N, int r)
{
    return dtype == 1 && r >= 1 && r <= 32 && (K % fused::KC) == 0 && (N % 8) == 0 && N >= 8 && M >= 1;
}

template <int RP, bool ENCODE, bool GELU>
static hipError_t launch_block_t(const void *Xin, const void *What, const void *E, const void *Dm, void *C, void *Ysave,
                                 int M, int K, int N, int r, int pg, hipStream_t s)
{
    auto kern = fused::stl_block_kernel<RP, ENCODE, GELU>;
    constexpr int smem = fused::smem_bytes<RP, ENCODE>();
    static_assert(smem <= 160 * 1024, "LDS budget");
    // once per instantiation (initialisation of a function-local static is thread-safe)
    static const hipError_t attr_err =
        hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (attr_err != hipSuccess) return attr_err;
    const int bi = (M + fused::BI - 1) / fused::BI, bj = (N + fused::BJ - 1) / fused::BJ;
    const long total = (long)bi * bj;
    if (total > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(256), smem, s, (const bf16_t *)Xin, (const bf16_t *)What,
                       (const bf16_t *)E, (const bf16_t *)Dm, (bf16_t *)C, (bf16_t *)Ysave, M, K, N, r, bj, pg);
    return hipGetLastError();
}

template <int RP>
static hipError_t launch_block_rp(bool encode_in_kernel, const void *Xin, const void *What, const void *E,
                                  const void *Dm, void *C, void *Ysave, int M, int K, int N, int r, bool gelu, int pg,
                                  hipStream_t s)
{
    if (encode_in_kernel)
        return gelu ? launch_block_t<RP, true, true>(Xin, What, E, Dm, C, Ysave, M, K, N, r, pg, s)
                    : launch_block_t<RP, true, false>(Xin, What, E, Dm, C, Ysave, M, K, N, r, pg, s);
    return gelu ? launch_block_t<RP, false, true>(Xin, What, E, Dm, C, Ysave, M, K, N, r, pg, s)
                : launch_block_t<RP, false, false>(Xin, What, E, Dm, C, Ysave, M, K, N, r, pg, s);
}

hipError_t launch_block_forward(bool encode_in_kernel, const void *Xin, const void *What, const void *E, const void *Dm,
                                void *C, void *Ysave, int M, int K, int N, int r, bool gelu, int pg, hipStream_t s)
{
    if (pg <= 0) pg = M;
    if (r <= 8) return launch_block_rp<8>(encode_in_kernel, Xin, What, E, Dm, C, Ysave, M, K, N, r, gelu, pg, s);
    if (r <= 16) return launch_block_rp<16>(encode_in_kernel, Xin, What, E, Dm, C, Ysave, M, K, N, r, gelu, pg, s);
    return launch_block_rp<32>(encode_in_kernel, Xin, What, E, Dm, C, Ysave, M, K, N, r, gelu, pg, s);
}

}  // namespace stl
