// Probe of the two resources the pipelined plane-product kernel lives on, in that kernel's own access pattern:
// the L2 -> LDS path (LDS-DMA loads, global_load_lds_dwordx4) and the matrix cores (32x32x16 bf16 MFMA).
// One workgroup of eight wavefronts per CU walks over the same (plane, 256 x 256 block) list as the library's
// kernel at the benchmark shape (r planes of M x K times K x N tiles) and per 32-element contraction stage either
//   * only issues the loads of the stage (nobody reads the data),          mode bit 0
//   * only issues the stage's sixteen MFMAs per wavefront on register operands, mode bit 1
//   * or both, interleaved as in the library's kernel.
// The first operand ([row][l]: 64 contiguous bytes per row and stage) can be fetched as the kernel does it today --
// half a 128-byte line per row and stage -- or as whole lines (64 contraction elements per row every second stage):
// same bytes, half the number of L2 requests for that operand.                mode bit 2 = whole lines
// Results are timings only; this file is measurement code, not part of the library.
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>
#include <type_traits>

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

__device__ __forceinline__ void dma16(const uint16_t *g, uint32_t lds_wave_base)
{
    const uint32_t l = __builtin_amdgcn_readfirstlane(lds_wave_base);
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(l) : "memory", "m0");
}

template <int MODE>
__global__ __launch_bounds__(512) void probe_kernel(const uint16_t *__restrict__ A, const uint16_t *__restrict__ B, int Mi,
                                                    int Nj, int Kl, int planes, float *__restrict__ sink)
{
    constexpr bool DMA = MODE & 1, MFMA = MODE & 2, WIDE = MODE & 4;
    extern __shared__ __align__(16) char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char *)smem);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tiles_m = Mi / 256, tiles_n = Nj / 256, per_plane = tiles_m * tiles_n, total = per_plane * planes;
    const int nks = Kl / 32;
    f32x16_t acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    bf16x8_t va[4], vb[2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) va[i][e] = (__bf16)(0.01f * (lane + i + e));
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) vb[i][e] = (__bf16)(0.02f * (lane - i - e));

    for (int v = blockIdx.x; v < total; v += gridDim.x) {
        int lid = v;
        if ((total & 7) == 0 && (gridDim.x & 7) == 0) lid = (v & 7) * (total >> 3) + (v >> 3);
        const int p = lid / per_plane, rem = lid - p * per_plane;
        const int i0 = (rem / tiles_n) * 256, j0 = (rem % tiles_n) * 256;
        const uint16_t *Ap = A + (size_t)p * Mi * Kl, *Bp = B + (size_t)p * Kl * Nj;
        for (int s = 0; s < nks; ++s) {
            const uint32_t slot = lds0 + (uint32_t)(s & 3) * 16384u;
            if (DMA) {
                if (!WIDE) {
                    // [row][l] operand, half lines: instruction q covers rows 16q .. 16q+15, four 16-byte chunks per row
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const int q = 2 * wave + j, row = 16 * q + (lane >> 2), c = lane & 3;
                        dma16(Ap + (size_t)(i0 + row) * Kl + s * 32 + 8 * c, slot + q * 1024);
                    }
                } else {
                    // whole lines: instruction q covers rows 8q .. 8q+7, eight chunks (64 contraction elements) per row;
                    // the upper half of the rows is fetched in the even stage of a pair, the lower half in the odd one
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const int q = 16 * (s & 1) + 2 * wave + j, row = 8 * q + (lane >> 3), c = lane & 7;
                        dma16(Ap + (size_t)(i0 + row) * Kl + (s & ~1) * 32 + 8 * c, lds0 + (uint32_t)((s >> 1) & 1) * 32768u + q * 1024);
                    }
                }
                // [l][row] operand: instruction q covers contraction rows 2q, 2q+1, 32 chunks (256 columns) per row
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int q = 2 * wave + j, k = 2 * q + (lane >> 5), nc = lane & 31;
                    dma16(Bp + (size_t)(s * 32 + k) * Nj + j0 + 8 * nc, lds0 + 65536u + (uint32_t)(s & 3) * 16384u + q * 1024);
                }
            }
            if (MFMA) {
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vb[i & 1], va[i >> 1], acc[i], 0, 0, 0);
            }
            // at most three stages of loads in flight per wavefront, as in the library's ring
            if (DMA) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) t += acc[i][e];
    if (t == 12345.678f) sink[threadIdx.x] = t;     // keeps the products alive; never true
}

// Second form of the probe: whole-line loads only, with the number of load instructions a wavefront may leave in flight
// at the end of a stage (DEPTH, four instructions per stage), the placement of the loads (SPREAD: one after every fourth
// MFMA instead of all four in front of the stage's MFMAs; 2, 3: the same with the wavefronts staggered) and a workgroup
// barrier per stage (BAR) as parameters.
template <int MODE, int DEPTH, int SPREAD, int BAR>
__global__ __launch_bounds__(512) void probe_depth_kernel(const uint16_t *__restrict__ A, const uint16_t *__restrict__ B, int Mi,
                                                          int Nj, int Kl, int planes, float *__restrict__ sink)
{
    constexpr bool DMA = MODE & 1, MFMA = MODE & 2, ZERO = MODE & 8;   // ZERO: all-zero MFMA operands (least switching)
    extern __shared__ __align__(16) char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char *)smem);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tiles_m = Mi / 256, tiles_n = Nj / 256, per_plane = tiles_m * tiles_n, total = per_plane * planes;
    const int nks = Kl / 32;
    // MFMA (of every four) after which this wavefront issues a load: the same for all (SPREAD 1), or staggered so that the
    // eight wavefronts of the workgroup never issue theirs together (2: by wavefront pair, 3: by wavefront index mod 4)
    // pair forms: wavefronts w and w + 4 (SPREAD 4) or 2i and 2i + 1 (SPREAD 5); the first of a pair issues all eight loads
    const int partner = __builtin_amdgcn_readfirstlane(SPREAD == 4 ? (wave ^ 4) : (wave ^ 1));
    const bool loader = SPREAD == 4 ? __builtin_amdgcn_readfirstlane(wave) < 4 : (__builtin_amdgcn_readfirstlane(wave) & 1) == 0;
    const int issue_after = SPREAD == 2 ? __builtin_amdgcn_readfirstlane((wave >> 1) & 3)
                          : SPREAD == 3 ? __builtin_amdgcn_readfirstlane(wave & 3) : 1;
    f32x16_t acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    bf16x8_t va[4], vb[2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) va[i][e] = ZERO ? (__bf16)0.f : (__bf16)(0.01f * (lane + i + e));
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) vb[i][e] = ZERO ? (__bf16)0.f : (__bf16)(0.02f * (lane - i - e));

    for (int v = blockIdx.x; v < total; v += gridDim.x) {
        int lid = v;
        if ((total & 7) == 0 && (gridDim.x & 7) == 0) lid = (v & 7) * (total >> 3) + (v >> 3);
        const int p = lid / per_plane, rem = lid - p * per_plane;
        const int i0 = (rem / tiles_n) * 256, j0 = (rem % tiles_n) * 256;
        const uint16_t *Ap = A + (size_t)p * Mi * Kl, *Bp = B + (size_t)p * Kl * Nj;
        for (int s = 0; s < nks; ++s) {
            // the four loads of wavefront index w (entries 4h .. 4h+3): this wavefront's own (h = 0) and, where one wavefront
            // of a pair issues for both (SPREAD 4, 5), its partner's (h = 1)
            const uint16_t *src[8];
            uint32_t dst[8];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int w = h == 0 ? wave : partner;
#pragma unroll
                for (int j = 0; j < 2; ++j) {   // whole lines of the [row][l] operand
                    const int q = 16 * (s & 1) + 2 * w + j, row = 8 * q + (lane >> 3), c = lane & 7;
                    src[4 * h + j] = Ap + (size_t)(i0 + row) * Kl + (s & ~1) * 32 + 8 * c;
                    dst[4 * h + j] = lds0 + (uint32_t)((s >> 1) & 1) * 32768u + q * 1024;
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int q = 2 * w + j, k = 2 * q + (lane >> 5), nc = lane & 31;
                    src[4 * h + 2 + j] = Bp + (size_t)(s * 32 + k) * Nj + j0 + 8 * nc;
                    dst[4 * h + 2 + j] = lds0 + 65536u + (uint32_t)(s & 3) * 16384u + q * 1024;
                }
            }
            if (DMA && !SPREAD) {
#pragma unroll
                for (int j = 0; j < 4; ++j) dma16(src[j], dst[j]);
            }
            if (MFMA) {
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vb[i & 1], va[i >> 1], acc[i], 0, 0, 0);
                        if (SPREAD >= 4) {              // one wavefront of each pair issues the loads of both
                            __builtin_amdgcn_sched_barrier(0);
                            if (DMA && (i & 1) == 1 && loader) {
                                dma16(src[ks * 4 + (i >> 1)], dst[ks * 4 + (i >> 1)]);
                                __builtin_amdgcn_sched_barrier(0);
                            }
                        } else if (SPREAD) {
                            __builtin_amdgcn_sched_barrier(0);
                            if (DMA && (i & 3) == issue_after) {
                                dma16(src[ks * 2 + (i >> 2)], dst[ks * 2 + (i >> 2)]);
                                __builtin_amdgcn_sched_barrier(0);
                            }
                        }
                    }
            } else if (DMA && SPREAD) {
#pragma unroll
                for (int j = 0; j < 4; ++j) dma16(src[j], dst[j]);
            }
            static_assert(!(SPREAD >= 4) || ((MODE & 3) == 3), "the pair forms exist for loads + MFMA only");
            if (DMA) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(DEPTH) : "memory");
            if (BAR) asm volatile("s_barrier" ::: "memory");
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) t += acc[i][e];
    if (t == 12345.678f) sink[threadIdx.x] = t;     // keeps the products alive; never true
}

// Third form: no LDS at all for the first operand.  Every wavefront owns 32 rows of the block and loads its own MFMA
// fragments of that operand straight from memory into registers (lane = (row, half of the 16-element step): 16 bytes),
// RING steps ahead, with ordinary loads the compiler tracks; the second operand stays in registers.  Measures what
// register-returning loads cost the matrix cores, against the LDS-DMA loads of the other forms.  The contraction length
// is fixed (1024 elements = 64 steps, unrolled) so that every ring index and every "is there a next step" is a constant.
template <int I, int N, class F>
__device__ __forceinline__ void probe_static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        probe_static_for<I + 1, N>(f);
    }
}

template <int RING>
__global__ __launch_bounds__(512) void probe_direct_kernel(const uint16_t *__restrict__ A, const uint16_t *__restrict__ B, int Mi,
                                                           int Nj, int Kl, int planes, float *__restrict__ sink)
{
    (void)B;
    constexpr int STEPS = 64;                               // Kl == 1024, checked by the caller
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tiles_m = Mi / 256, tiles_n = Nj / 256, per_plane = tiles_m * tiles_n, total = per_plane * planes;
    f32x16_t acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    bf16x8_t vb[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) vb[i][e] = (__bf16)(0.02f * (lane - i - e));

    for (int v = blockIdx.x; v < total; v += gridDim.x) {
        int lid = v;
        if ((total & 7) == 0 && (gridDim.x & 7) == 0) lid = (v & 7) * (total >> 3) + (v >> 3);
        const int p = lid / per_plane, rem = lid - p * per_plane;
        const int i0 = (rem / tiles_n) * 256;
        // this lane's row of the block and its half of every 16-element step: 16-byte pieces at rowp + 16 * step
        const uint16_t *rowp = A + (size_t)p * Mi * Kl + (size_t)(i0 + 32 * wave + (lane & 31)) * Kl + 8 * (lane >> 5);
        bf16x8_t ring[RING];
#pragma unroll
        for (int d = 0; d < RING; ++d) ring[d] = *reinterpret_cast<const bf16x8_t *>(rowp + 16 * d);
        __builtin_amdgcn_sched_barrier(0);
        probe_static_for<0, STEPS>([&](auto t_c) {
            constexpr int t = decltype(t_c)::value, d = t % RING;
            const bf16x8_t va = ring[d];
            if constexpr (t + RING < STEPS) ring[d] = *reinterpret_cast<const bf16x8_t *>(rowp + 16 * (t + RING));
            __builtin_amdgcn_sched_barrier(0);              // the load stays RING steps ahead of its use
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vb[i & 1], va, acc[i], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        });
    }
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) t += acc[i][e];
    if (t == 12345.678f) sink[threadIdx.x] = t;     // keeps the products alive; never true
}

template <class K>
static float time_kernel(K kern, const uint16_t *A, const uint16_t *B, int Mi, int Nj, int Kl, int planes, float *sink, int grid,
                         int iters)
{
    const int smem = 131072;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess) return -1.f;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -1.f;
    for (int i = 0; i < 3; ++i) hipLaunchKernelGGL(kern, dim3(grid), dim3(512), smem, 0, A, B, Mi, Nj, Kl, planes, sink);
    (void)hipEventRecord(e0, 0);
    for (int i = 0; i < iters; ++i) hipLaunchKernelGGL(kern, dim3(grid), dim3(512), smem, 0, A, B, Mi, Nj, Kl, planes, sink);
    (void)hipEventRecord(e1, 0);
    if (hipEventSynchronize(e1) != hipSuccess) return -1.f;
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return ms / iters;
}

template <int MODE>
static float run(const uint16_t *A, const uint16_t *B, int Mi, int Nj, int Kl, int planes, float *sink, int grid, int iters)
{
    auto kern = probe_kernel<MODE>;
    const int smem = 131072;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess) return -1.f;
    hipEvent_t e0, e1;
    hipEventCreate(&e0);
    hipEventCreate(&e1);
    for (int i = 0; i < 3; ++i) hipLaunchKernelGGL(kern, dim3(grid), dim3(512), smem, 0, A, B, Mi, Nj, Kl, planes, sink);
    hipEventRecord(e0, 0);
    for (int i = 0; i < iters; ++i) hipLaunchKernelGGL(kern, dim3(grid), dim3(512), smem, 0, A, B, Mi, Nj, Kl, planes, sink);
    hipEventRecord(e1, 0);
    if (hipEventSynchronize(e1) != hipSuccess) return -1.f;
    float ms = 0.f;
    hipEventElapsedTime(&ms, e0, e1);
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    return ms / iters;
}

// mode: bit 0 loads, bit 1 MFMAs, bit 2 whole-line loads of the first operand.  A: planes x Mi x Kl, B: planes x Kl x Nj
// (device pointers, bf16 bit patterns), sink: 512 floats.  Returns milliseconds per launch, negative on error.
extern "C" float stl_probe_run(int mode, const void *A, const void *B, int Mi, int Nj, int Kl, int planes, void *sink, int grid,
                               int iters)
{
    if (Mi % 256 || Nj % 256 || Kl % 64 || planes < 1 || grid < 1 || iters < 1) return -2.f;
    const uint16_t *a = (const uint16_t *)A, *b = (const uint16_t *)B;
    float *s = (float *)sink;
    switch (mode) {
        case 1: return run<1>(a, b, Mi, Nj, Kl, planes, s, grid, iters);
        case 2: return run<2>(a, b, Mi, Nj, Kl, planes, s, grid, iters);
        case 3: return run<3>(a, b, Mi, Nj, Kl, planes, s, grid, iters);
        case 5: return run<5>(a, b, Mi, Nj, Kl, planes, s, grid, iters);
        case 7: return run<7>(a, b, Mi, Nj, Kl, planes, s, grid, iters);
    }
    return -2.f;
}

// Depth form.  id = 100 * placement + depth: placement 0 = loads in front of the stage's MFMAs, 1 = spread between them,
// 2 = spread and a barrier per stage, 3 / 4 = staggered by wavefront pair without / with the barrier, 5 / 6 = staggered by
// wavefront index mod 4 (depth 8 only), 7 / 8 = wavefronts w < 4 issue the loads of w and w + 4 without / with the barrier,
// 9 / 11 = even wavefronts issue the loads of 2i and 2i + 1 (depth 16 only: eight loads per stage and loading wavefront);
// id 3000 / 3008 = MFMAs only / loads between the MFMAs with all-zero MFMA operands; id 4004 / 4008 = the direct form with
// 4 / 8 steps of register prefetch (Kl = 1024 only); depth (instructions in flight at the end of a stage) one of 4, 8, 16, 32, 48 for
// placement 0 and 4, 8, 16, 32 for the others; id 1000 + depth (8, 16, 32) = loads only; id 2000 / 2001 = MFMAs only
// without / with the barrier.  Same arguments and return value as stl_probe_run.
extern "C" float stl_probe_depth_run(int id, const void *A, const void *B, int Mi, int Nj, int Kl, int planes, void *sink, int grid,
                                     int iters)
{
    if (Mi % 256 || Nj % 256 || Kl % 64 || planes < 1 || grid < 1 || iters < 1) return -2.f;
    const uint16_t *a = (const uint16_t *)A, *b = (const uint16_t *)B;
    float *s = (float *)sink;
#define STL_PROBE_CASE(ID, M, D, S, Bb) \
    case ID: return time_kernel(probe_depth_kernel<M, D, S, Bb>, a, b, Mi, Nj, Kl, planes, s, grid, iters);
    switch (id) {
        STL_PROBE_CASE(2000, 2, 0, 0, 0)
        STL_PROBE_CASE(2001, 2, 0, 0, 1)
        STL_PROBE_CASE(1008, 1, 8, 0, 0)
        STL_PROBE_CASE(1016, 1, 16, 0, 0)
        STL_PROBE_CASE(1032, 1, 32, 0, 0)
        STL_PROBE_CASE(4, 3, 4, 0, 0)
        STL_PROBE_CASE(8, 3, 8, 0, 0)
        STL_PROBE_CASE(16, 3, 16, 0, 0)
        STL_PROBE_CASE(32, 3, 32, 0, 0)
        STL_PROBE_CASE(48, 3, 48, 0, 0)
        STL_PROBE_CASE(104, 3, 4, 1, 0)
        STL_PROBE_CASE(108, 3, 8, 1, 0)
        STL_PROBE_CASE(116, 3, 16, 1, 0)
        STL_PROBE_CASE(132, 3, 32, 1, 0)
        STL_PROBE_CASE(204, 3, 4, 1, 1)
        STL_PROBE_CASE(208, 3, 8, 1, 1)
        STL_PROBE_CASE(216, 3, 16, 1, 1)
        STL_PROBE_CASE(232, 3, 32, 1, 1)
        STL_PROBE_CASE(308, 3, 8, 2, 0)
        STL_PROBE_CASE(408, 3, 8, 2, 1)
        STL_PROBE_CASE(508, 3, 8, 3, 0)
        STL_PROBE_CASE(608, 3, 8, 3, 1)
        STL_PROBE_CASE(716, 3, 16, 4, 0)
        STL_PROBE_CASE(816, 3, 16, 4, 1)
        STL_PROBE_CASE(916, 3, 16, 5, 0)
        STL_PROBE_CASE(1116, 3, 16, 5, 1)
        STL_PROBE_CASE(3000, 10, 0, 0, 0)
        STL_PROBE_CASE(3008, 11, 8, 1, 0)
        case 4004: if (Kl != 1024) return -2.f; return time_kernel(probe_direct_kernel<4>, a, b, Mi, Nj, Kl, planes, s, grid, iters);
        case 4008: if (Kl != 1024) return -2.f; return time_kernel(probe_direct_kernel<8>, a, b, Mi, Nj, Kl, planes, s, grid, iters);
    }
#undef STL_PROBE_CASE
    return -2.f;
}
