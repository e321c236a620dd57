// Inter-layer step of two stacked STL layers (Algorithm 2, its Steps 3 and 1 taken together):
//     Xhat2[s][I][J] = sum_q E2[s][q] * act( sum_p D1[p][q] * Yhat1[p][I][J] ),
// i.e. decode the first layer's encoded output tile, apply the activation, encode it for the next layer,
// without the hidden activation ever going to HBM: output tile (I, J) of layer 1 is input tile (I, L = J)
// of layer 2, so the whole step is local to a tile.  One pass: read r1 planes, write r2 planes.
//
// Both small contractions run on v_mfma_f32_16x16x32_bf16.  Decode: rows = the 16 tile entries, columns =
// 16 tiles, K = planes; a lane (tile, kq) is left with entries 4kq..4kq+3 of its tile.  Rounded to bf16 and
// padded with four zeros these four values ARE the lane's operand fragment of the second product
// (rows = tiles, K slot 8kq+e <-> entry 4kq+e for e < 4, zero weight on the other slots), so nothing moves
// between the two products.  The tiles of decode product u are picked as J0 + 8*(lane/4) + 4*(u%2) + 32*(u/2) + lane%4;
// then a lane of the second product (plane, kq) ends up with tiles J0 + 32h + 8kq .. +7 of its plane from
// products 2h, 2h+1: one 16-byte chunk each, which goes back through the LDS slab so that the planes are stored
// as they were loaded, in whole 128-byte lines.
#include "stl_kernels.h"
#include "stl_device.h"

namespace stl {

typedef short v4i16_t __attribute__((ext_vector_type(4)));

template <bool GELU, int KC>   // KC = number of 32-plane groups of the larger of the two ranks (1: <= 32, 2: <= 64)
__global__ __launch_bounds__(256) void recode_mfma_kernel(const bf16_t *__restrict__ P, const bf16_t *__restrict__ Dm,
                                                          const bf16_t *__restrict__ E2, bf16_t *__restrict__ Q, int R,
                                                          int Cc, int r1, int r2, int chunks, int pg)
{
    constexpr int ROWB = 128;                               // bytes per LDS row (64 tiles)
    __shared__ __align__(16) char slab_all[4][KC * 32 * ROWB];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    char *slab = slab_all[wave];
    const int j = lane & 15, kq = lane >> 4;
    const int ng2 = (r2 + 15) >> 4;

    // decode fragments: lane (entry q = j, kq) holds D1[32g + 8kq + e][q], e = 0..7
    bf16x8_t fa[KC];
#pragma unroll
    for (int g = 0; g < KC; ++g) {
        uint32_t w[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            const int p0 = 32 * g + 8 * kq + 2 * e2;
            const uint32_t lo = p0 < r1 ? Dm[p0 * 16 + j] : 0u, hi = p0 + 1 < r1 ? Dm[(p0 + 1) * 16 + j] : 0u;
            w[e2] = lo | (hi << 16);
        }
        fa[g] = __builtin_bit_cast(bf16x8_t, u32x4_t{w[0], w[1], w[2], w[3]});
    }
    // encode fragments: lane (plane 16g2 + j, kq) holds E2[plane][4kq + e] in K slots 8kq + e, e < 4; zeros above
    bf16x8_t eb[4];
#pragma unroll
    for (int g2 = 0; g2 < 4; ++g2) {
        const int pl = 16 * g2 + j;
        u32x2_t ev = {0u, 0u};
        if (pl < r2) ev = *reinterpret_cast<const u32x2_t *>(E2 + pl * 16 + 4 * kq);
        eb[g2] = __builtin_bit_cast(bf16x8_t, u32x4_t{ev[0], ev[1], 0u, 0u});
    }
    // 16-byte chunk swizzle of a slab row: one transposing read touches rows (planes) that differ in bits 0, 1
    // (lane/4 inside a 16-lane group) and bits 3, 4 (kq), and in each row the chunks 2*(lane%4) + u/2.  Bit 0 of
    // the row already alternates the bank half (128-byte rows); the other three bits shift the chunk index.
    auto swz = [](int row) { return ((row >> 1) & 1) | (((row >> 3) & 3) << 1); };

    const size_t plane = (size_t)pg * Cc;
    const long items = (long)R * chunks;
    // (tile row, chunk) of this wavefront's item, advanced without a division per round
    const long stride = (long)gridDim.x * 4;
    int In = (int)(((long)blockIdx.x * 4 + wave) / chunks), ckn = (int)(((long)blockIdx.x * 4 + wave) % chunks);
    const int dI = (int)(stride / chunks), dck = (int)(stride % chunks);

    // lane -> (plane within group of 8, 16-byte chunk = 8 tiles).  The plane segments of the NEXT item are fetched
    // into registers while the current item is computed and stored, so that a wavefront always has loads in flight.
    const int pr = lane >> 3, ch = lane & 7;
    u32x4_t pre[KC * 4];
    auto fetch = [&](int Ii, int cki) {
        const int Jl = cki * 64 + 8 * ch;
        const size_t rowb = Ii < R ? plane_row_base(Ii, pg, r1, Cc) : 0;
#pragma unroll
        for (int g8 = 0; g8 < KC * 4; ++g8) {
            const int pl = 8 * g8 + pr;
            u32x4_t v = {0u, 0u, 0u, 0u};
            if (Ii < R && pl < r1 && Jl < Cc) v = *reinterpret_cast<const u32x4_t *>(P + rowb + (size_t)pl * plane + Jl);
            pre[g8] = v;
        }
    };
    fetch(In, ckn);

    for (long item0 = (long)blockIdx.x * 4; item0 < items; item0 += stride) {
        const int I = In, J0 = ckn * 64;
        const bool live = I < R;
        // The slab is private to the wavefront and a wavefront's LDS operations execute in order: these writes
        // land after the previous round's fragment reads and before this round's, without a workgroup barrier
        // (which would also make the wavefront wait for the loads it has just put in flight).
#pragma unroll
        for (int g8 = 0; g8 < KC * 4; ++g8) {
            const int pl = 8 * g8 + pr;
            *reinterpret_cast<u32x4_t *>(slab + pl * ROWB + ((ch ^ swz(pl)) << 4)) = pre[g8];
        }
        In += dI;
        ckn += dck;
        if (ckn >= chunks) { ckn -= chunks; ++In; }
        if (item0 + stride < items) fetch(In, ckn);
        if (!live) continue;

        bf16x8_t hf[4];                                     // activation of this lane's tile in product u, entries 4kq..4kq+3
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int g = 0; g < KC; ++g) {
                v4i16_t t[2];
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    // source address of this lane inside its 16-lane group: plane 32g + 8kq + 4kk + j/4, tiles
                    // 8*(j%4) + 4*(u%2) + 32*(u/2) .. +3 (the group's lane 4c + e receives tile 8c + 4*(u%2) + 32*(u/2) + e)
                    const int row = 32 * g + 8 * kq + 4 * kk + (j >> 2);
                    const int col = 8 * (j & 3) + 4 * (u & 1) + 32 * (u >> 1);
                    const char *src = slab + row * ROWB + (((col >> 3) ^ swz(row)) << 4) + ((col & 7) << 1);
                    t[kk] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16_t *)(
                        (__attribute__((address_space(3))) char *)src));
                }
                struct { v4i16_t a, b; } both = {t[0], t[1]};
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[g], __builtin_bit_cast(bf16x8_t, both), acc, 0, 0, 0);
            }
            float c0 = acc[0], c1 = acc[1], c2 = acc[2], c3 = acc[3];
            if (GELU) { c0 = gelu_erf(c0); c1 = gelu_erf(c1); c2 = gelu_erf(c2); c3 = gelu_erf(c3); }
            hf[u] = __builtin_bit_cast(bf16x8_t, u32x4_t{pack_bf16x2(c0, c1), pack_bf16x2(c2, c3), 0u, 0u});
        }

        // second product: rows = tiles (row 4c + e of product u is tile J0 + 8c + 4*(u%2) + 32*(u/2) + e), columns =
        // planes; products 2h and 2h+1 leave this lane with the 8 consecutive tiles J0 + 32h + 8kq .. +7 = chunk 4h + kq
        // of its plane.  The results go back through the slab (all its fragments are in registers by now; LDS
        // operations of a wavefront execute in order) and leave as whole 128-byte lines, 8 planes per store
        // instruction: stores of 64 bytes per plane ran a fifth slower.
        auto swo = [](int row) { return ((row >> 1) & 1) << 2; };
#pragma unroll
        for (int g2 = 0; g2 < 2 * KC; ++g2) {
            if (g2 < ng2) {
                f32x4_t o[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
                    o[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hf[u], eb[g2], zero, 0, 0, 0);
                }
                const int pl = 16 * g2 + j;
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const f32x4_t a = o[2 * half], b = o[2 * half + 1];
                    const u32x4_t w = {pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(b[0], b[1]),
                                       pack_bf16x2(b[2], b[3])};
                    *reinterpret_cast<u32x4_t *>(slab + pl * ROWB + (((4 * half + kq) ^ swo(pl)) << 4)) = w;
                }
            }
        }
        const size_t rowb_out = plane_row_base(I, pg, r2, Cc);
#pragma unroll
        for (int g8 = 0; g8 < KC * 4; ++g8) {
            const int pl = 8 * g8 + pr;
            if (pl < r2 && J0 + 8 * ch < Cc) {
                const u32x4_t w = *reinterpret_cast<const u32x4_t *>(slab + pl * ROWB + ((ch ^ swo(pl)) << 4));
                *reinterpret_cast<u32x4_t *>(Q + rowb_out + (size_t)pl * plane + J0 + 8 * ch) = w;
            }
        }
    }
}

bool recode_eligible(int dtype, int Cc) { return dtype == 1 && (Cc % 8) == 0; }

hipError_t launch_recode(const void *P, const void *Dm, const void *E2, void *Q, int R, int Cc, int r1, int r2, bool gelu,
                         int pg, hipStream_t s)
{
    if (pg <= 0) pg = R;
    const int chunks = (Cc + 63) / 64;
    const long items = (long)R * chunks;
    long blocks = (items + 3) / 4;
    if (blocks > 8192) blocks = 8192;                       // grid-stride over (tile row, 64-tile chunk) items
    const dim3 grid((unsigned)blocks), block(256);
    const bf16_t *p = (const bf16_t *)P, *d = (const bf16_t *)Dm, *e = (const bf16_t *)E2;
    bf16_t *q = (bf16_t *)Q;
    if (r1 <= 32 && r2 <= 32) {
        if (gelu) hipLaunchKernelGGL((recode_mfma_kernel<true, 1>), grid, block, 0, s, p, d, e, q, R, Cc, r1, r2, chunks, pg);
        else hipLaunchKernelGGL((recode_mfma_kernel<false, 1>), grid, block, 0, s, p, d, e, q, R, Cc, r1, r2, chunks, pg);
    } else {
        if (gelu) hipLaunchKernelGGL((recode_mfma_kernel<true, 2>), grid, block, 0, s, p, d, e, q, R, Cc, r1, r2, chunks, pg);
        else hipLaunchKernelGGL((recode_mfma_kernel<false, 2>), grid, block, 0, s, p, d, e, q, R, Cc, r1, r2, chunks, pg);
    }
    return hipGetLastError();
}

}  // namespace stl
