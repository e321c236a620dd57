// Host stand-in for <hip/hip_runtime.h>, test infrastructure only (tests/test_cpu_address_check.py).
// The library's sources are compiled for the CPU against this header and every kernel launch is executed thread by
// thread, so that AddressSanitizer sees each global-memory access of the real index arithmetic: an access outside a
// buffer is reported here instead of faulting a GPU.  Matrix-core products, transposing LDS reads and barriers are
// stubs and LDS contents are meaningless: no address in these kernels depends on loaded data.  Launches with many
// blocks run a sample of them (first, last, a stride through the middle) unless CPU_ALL_BLOCKS is set.
#pragma once
#include <cmath>
#include <cstdint>
#include <cstddef>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#define __global__
#define __device__
#define __host__
#define __forceinline__ inline
#define __shared__ static
#define __launch_bounds__(...)
#define __align__(n) __attribute__((aligned(n)))
struct dim3 { unsigned x, y, z; dim3(unsigned a = 1, unsigned b = 1, unsigned c = 1) : x(a), y(b), z(c) {} };
inline dim3 threadIdx, blockIdx, blockDim, gridDim;
typedef int hipError_t;
typedef void *hipStream_t;
enum { hipSuccess = 0, hipErrorInvalidValue = 1 };
enum { hipFuncAttributeMaxDynamicSharedMemorySize = 0, hipDeviceAttributeMultiprocessorCount = 1 };
inline hipError_t hipGetLastError() { return 0; }
inline const char *hipGetErrorString(hipError_t) { return "cpu"; }
inline hipError_t hipFuncSetAttribute(const void *, int, int) { return 0; }
inline hipError_t hipGetDevice(int *d) { *d = 0; return 0; }
inline hipError_t hipDeviceGetAttribute(int *v, int, int) { *v = 256; return 0; }
#define HIP_SYMBOL(x) (&(x))
inline hipError_t hipGetSymbolAddress(void **p, const void *sym) { *p = const_cast<void *>(sym); return 0; }
inline const char *g_kernel_name = "";
inline size_t g_dyn_lds = 0;          // dynamic LDS bytes the current launch asked for
inline char *g_dyn_lds_buf = nullptr; // a heap block that ends where those bytes end: LDS accesses past them are reported
inline char *cpu_dyn_lds_ptr() { return g_dyn_lds_buf; }
// device limits of gfx950 that a launch must respect (LDS per workgroup, threads per workgroup, grid extents)
constexpr size_t kCpuMaxLds = 160 * 1024;
inline void cpu_check_launch(const char *name, dim3 grid, dim3 block, size_t smem)
{
    const unsigned long threads = (unsigned long)block.x * block.y * block.z;
    if (smem > kCpuMaxLds || threads > 1024 || grid.x > 0x7fffffffu || grid.y > 65535u || grid.z > 65535u) {
        fprintf(stderr, "runtime error: launch of %s outside device limits: grid (%u,%u,%u) block (%u,%u,%u) dynamic LDS %zu\n", name,
                grid.x, grid.y, grid.z, block.x, block.y, block.z, smem);
        abort();
    }
}
template <typename F>
inline void cpu_launch(const char *name, dim3 grid, dim3 block, size_t smem, F f)
{
    g_kernel_name = name;
    g_dyn_lds = smem;
    cpu_check_launch(name, grid, block, smem);
    if (getenv("CPU_VERBOSE")) { fprintf(stderr, "  launch %s grid (%u,%u,%u) block (%u,%u,%u)\n", name, grid.x, grid.y, grid.z, block.x, block.y, block.z); fflush(stderr); }
    if (grid.x == 0 || grid.y == 0 || grid.z == 0 || block.x * block.y * block.z == 0) { fprintf(stderr, "EMPTY LAUNCH %s\n", name); abort(); }
    gridDim = grid; blockDim = block;
    const size_t lds_tot = (smem + 255) / 256 * 256 + 256;
    char *lds_block = (char *)aligned_alloc(256, lds_tot);
    memset(lds_block, 0, lds_tot);
    g_dyn_lds_buf = lds_block + (lds_tot - smem) / 16 * 16;
    // visit a sample of blocks: all if few, else first, last and a stride through the middle
    const unsigned long nb = (unsigned long)grid.x * grid.y * grid.z;
    const char *all = getenv("CPU_ALL_BLOCKS");
    const unsigned long stride = (all || nb <= 64) ? 1 : (nb / 48 | 1);
    auto run_block = [&](unsigned long b) {
        blockIdx = dim3((unsigned)(b % grid.x), (unsigned)((b / grid.x) % grid.y), (unsigned)(b / ((unsigned long)grid.x * grid.y)));
        for (unsigned tz = 0; tz < block.z; ++tz)
            for (unsigned ty = 0; ty < block.y; ++ty)
                for (unsigned tx = 0; tx < block.x; ++tx) { threadIdx = dim3(tx, ty, tz); f(); }
    };
    for (unsigned long b = 0; b < nb; b += stride) run_block(b);
    if ((nb - 1) % stride) run_block(nb - 1);
    g_dyn_lds_buf = nullptr;
    free(lds_block);
}
#define hipLaunchKernelGGL(kern, grid, block, smem, stream, ...) cpu_launch(#kern, grid, block, (size_t)(smem), [&]() { kern(__VA_ARGS__); })
inline float __uint_as_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
#define __syncthreads() ((void)0)
#define __builtin_amdgcn_readfirstlane(x) (x)
#define __builtin_amdgcn_sched_barrier(x) ((void)0)
#define __builtin_amdgcn_rcpf(x) (1.0f / (x))
#define __builtin_amdgcn_exp2f(x) exp2f(x)
#define __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, x, y, z) (c)
#define __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, x, y, z) (c)
#define __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, x, y, z) (c)
typedef short cpu_v4i16 __attribute__((ext_vector_type(4)));
#define __builtin_amdgcn_ds_read_tr16_b64_v4i16(p) (cpu_v4i16{0, 0, 0, 0})
// a 16-byte global read (stands in for the LDS-DMA load): touch the bytes so that the sanitizer checks them
inline void cpu_touch16(const void *g);
// lds: byte offset of the wavefront's 1 KB destination inside the launch's dynamic LDS (the host form of a kernel
// counts LDS addresses from the start of its dynamic array); lane L's 16 bytes land at lds + 16 L
inline void cpu_touch16(const void *g, uint32_t lds)
{
    const size_t lane = (threadIdx.x + blockDim.x * (threadIdx.y + (size_t)blockDim.y * threadIdx.z)) & 63;
    if ((lds & 15) || (size_t)lds + 16 * lane + 16 > g_dyn_lds) {
        fprintf(stderr, "runtime error: LDS-DMA destination %u + 16*%zu outside the %zu bytes of dynamic LDS (%s)\n", lds, lane, g_dyn_lds, g_kernel_name);
        abort();
    }
    cpu_touch16(g);
}
inline void cpu_touch16(const void *g) { if ((uintptr_t)g & 15) { fprintf(stderr, "runtime error: LDS-DMA source %p is not 16-byte aligned (%s)\n", g, g_kernel_name); abort(); } volatile uint64_t a = ((const volatile uint64_t *)g)[0], b = ((const volatile uint64_t *)g)[1]; (void)a; (void)b; }
#define __builtin_amdgcn_sched_group_barrier(a, b, c) ((void)0)
// agent-scope atomics, fences and sleeps of the kernels that synchronise workgroups through counters: threads run one
// after the other here, so a counter that is waited for always reads as reached
#define __HIP_MEMORY_SCOPE_AGENT 0
#define __hip_atomic_load(p, order, scope) (0xffffffffu)
#define __hip_atomic_fetch_add(p, v, order, scope) (*(p) += (v), *(p) - (v))
#define __hip_atomic_fetch_or(p, v, order, scope) (*(p) |= (v))
#define __builtin_amdgcn_fence(order, scope) ((void)0)
#define __builtin_amdgcn_s_sleep(n) ((void)0)
