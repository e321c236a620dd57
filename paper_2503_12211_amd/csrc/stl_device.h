// Device-side helpers shared by the STL kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace stl {

typedef uint16_t bf16_t;  // raw bfloat16 bits in memory

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));

// fp32 -> bf16, round-to-nearest-even (NaN stays NaN): gfx950 has a packed hardware conversion
// (v_cvt_pk_bf16_f32), which the compiler selects for this vector conversion.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    const f32x2_t f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }

// 16-byte store that is written through the XCD's L2 to memory (cache-coherence bits sc0 sc1: system scope), for data that
// workgroups on another XCD read later in the same launch: when the store has completed (vmcnt) the data is where every
// L2 fetches from, with no write-back of the whole cache.  THROUGH = false is the ordinary store.
template <bool THROUGH>
__device__ __forceinline__ void store16(void *p, u32x4_t v)
{
    if constexpr (THROUGH) {
        asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(p), "v"(v) : "memory");
    } else {
        *reinterpret_cast<u32x4_t *>(p) = v;
    }
}

// storage-type traits: load as fp32, store from fp32
template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float ld(const float *p) { return *p; }
    static __device__ __forceinline__ void st(float *p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float ld(const bf16_t *p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void st(bf16_t *p, float v) { *p = f32_to_bf16(v); }
};

// Plane tensors [p][tile row][tile column] are stored in groups of `pg` tile rows: element (p, I, J) of an
// r x R x Cc tensor lives at ((I / pg) * r + p) * pg * Cc + (I % pg) * Cc + J.  pg = R is the plain plane-major
// layout (weights and their gradients); the activation-side tensors use groups of 64 tile rows, which keeps the r
// segments belonging to one tile row within r * 64 * Cc elements of each other instead of a whole plane apart
// (the kernels that walk over all planes of a tile row run a fifth faster on it) and still leaves 64 consecutive
// rows of a plane contiguous for the plane products.  Inside a group the distance between planes is pg * Cc.
__host__ __device__ __forceinline__ size_t plane_row_base(int I, int pg, int r, int Cc)
{
    const int g = I / pg;
    return ((size_t)g * r * pg + (size_t)(I - g * pg)) * Cc;
}

// erf-form GELU in fp32, h * Phi(h), branch-free.  Phi(h) = erfc(-h / sqrt 2) / 2 with the rational-exponential
// approximation of Abramowitz & Stegun 7.1.26,  erfc(x) ~ (a1 s + ... + a5 s^5) exp(-x^2),  s = 1 / (1 + p x),  x >= 0,
// whose absolute error is below 1.5e-7 (the library erff costs about three times the instructions and diverges on
// |x| < 1, which made the GELU the bottleneck of the HBM-bound decode kernels).  |gelu error| <= 7.5e-8 |h|.
__device__ __forceinline__ float gelu_erf(float h)
{
    const float x = fabsf(h) * 0.70710678118654752440f;
    const float s = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
    float poly = fmaf(s, 1.061405429f, -1.453152027f);
    poly = fmaf(poly, s, 1.421413741f);
    poly = fmaf(poly, s, -0.284496736f);
    poly = fmaf(poly, s, 0.254829592f);
    const float half_erfc = 0.5f * poly * s * __builtin_amdgcn_exp2f(-1.44269504088896340736f * x * x);
    return h * (h < 0.f ? half_erfc : 1.0f - half_erfc);
}

}  // namespace stl
