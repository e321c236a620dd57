// Per-wavefront item loops of the bf16 tile maps on the matrix cores (encode: step (i) of Algorithm 1, decode: step (iii),
// each optionally with the basis-gradient sum of the backward pass).  Shared by the stand-alone kernels and by the
// kernel that runs them between plane-product blocks.
#pragma once
#include "stl_kernels.h"
#include "stl_device.h"

namespace stl {

typedef short v4i16_t __attribute__((ext_vector_type(4)));

// The item loop of one wavefront: items `first`, `first + stride`, ... below `end`, an item being (tile row index of the
// launch, 64-tile chunk) = item / chunks, item % chunks.  sT and slab are LDS areas private to the wavefront
// (sT: 64 x 32 bytes, used with OUTER only; slab: KC * 32 * 128 bytes); dacc accumulates the basis gradient (OUTER).
// `lane` is the caller's lane id (threadIdx.x % 64).  No workgroup barrier inside: wavefronts of a workgroup may run
// different numbers of items.
// THROUGH: the plane stores are written through to memory (see store16).  DEPTH: items whose operands are in flight
// at once (in registers) -- 1 where dozens of wavefronts per CU hide the latency, more where only eight run.
template <int KC, bool OUTER, bool THROUGH = false, int DEPTH = 1>
__device__ __forceinline__ void encode_items(const bf16_t *__restrict__ A, const bf16_t *__restrict__ E, bf16_t *__restrict__ P,
                                             const bf16_t *__restrict__ Qp, int R, int Cc, int r, int chunks, int pg, const RowMap &rm,
                                             long first, long stride, long end, char *sT, char *slab, f32x4_t (&dacc)[4], int lane)
{
    constexpr int ROWB = 128;                               // bytes per plane row of the slab (64 tiles)
    // 16-byte chunk swizzle of a plane row: a fragment read takes chunk 4sx + kq of 16 rows; odd/even rows already
    // alternate the bank half, bit 1 of the row moves the chunk to the other four positions
    auto swz = [](int row) { return ((row >> 1) & 1) << 2; };
    const int pr = lane >> 3, ch = lane & 7;                // loader role: plane within a group of 8, 8-tile chunk
    const int j = lane & 15, kq = lane >> 4;
    const int ng = (r + 15) >> 4;
    const size_t ld = (size_t)Cc * 4, plane = (size_t)pg * Cc;

    // encoder fragments: lane (plane 16g + j, kq) holds E[plane][4kq + e] in K slots 8kq + e, e < 4; zeros above
    bf16x8_t eb[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int pl = 16 * g + j;
        u32x2_t ev = {0u, 0u};
        if (pl < r) ev = *reinterpret_cast<const u32x2_t *>(E + pl * 16 + 4 * kq);
        eb[g] = __builtin_bit_cast(bf16x8_t, u32x4_t{ev[0], ev[1], 0u, 0u});
    }
    // tile (relative to J0) of this lane in product u, and its row in the LDS slab: rows t and t^4 are swapped where
    // bit 3 of t is set, so that the four 4-tile groups of one write (and the four 8-tile groups of one transposing
    // read) fall into both halves of the banks
    int trel[4], srow[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        trel[u] = 8 * (j >> 2) + 4 * (u & 1) + 32 * (u >> 1) + (j & 3);
        srow[u] = trel[u] ^ (((trel[u] >> 3) & 1) << 2);
    }

    u32x2_t xa[DEPTH][4];                   // this lane's tile rows, one per product
    u32x4_t qa[DEPTH][OUTER ? KC * 4 : 1];  // plane segments, loader role: plane 8*g8 + pr, tiles 8ch .. 8ch+7
    auto fetch = [&](int d, long item) {
        const int Ii = (int)(item / chunks), cki = (int)(item - (long)Ii * chunks);
        const int J0 = cki * 64;
        const int Ia = Ii < R ? rm.tile_row(Ii) : 0;        // Ii counts the tile rows of this launch, Ia is the tile row itself
        const size_t rowb = plane_row_base(Ia, pg, r, Cc);
        const bool row_ok = Ii < R && kq < rm.valid(Ia);    // a null row reads as zero
        const size_t r0 = rm.row0(Ia);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            u32x2_t v = {0u, 0u};
            if (row_ok && J0 + trel[u] < Cc) v = *reinterpret_cast<const u32x2_t *>(A + (r0 + kq) * ld + (size_t)(J0 + trel[u]) * 4);
            xa[d][u] = v;
        }
        if (OUTER) {
#pragma unroll
            for (int g8 = 0; g8 < KC * 4; ++g8) {
                const int pl = 8 * g8 + pr, tk = J0 + 8 * ch;
                u32x4_t v = {0u, 0u, 0u, 0u};
                if (Ii < R && pl < r && tk < Cc) v = *reinterpret_cast<const u32x4_t *>(Qp + rowb + (size_t)pl * plane + tk);
                qa[d][g8] = v;
            }
        }
    };
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
        if (first + d * stride < end) fetch(d, first + d * stride);

    for (long base = first; base < end; base += DEPTH * stride)
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
        const long item0 = base + d * stride;
        if (item0 >= end) break;
        const int Iidx = (int)(item0 / chunks), J0 = (int)(item0 - (long)Iidx * chunks) * 64;
        u32x2_t x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) x[u] = xa[d][u];
        // plane segments -> slab (private to the wavefront, whose LDS operations execute in order: no barrier)
        if (OUTER) {
#pragma unroll
            for (int g8 = 0; g8 < KC * 4; ++g8) {
                const int pl = 8 * g8 + pr;
                *reinterpret_cast<u32x4_t *>(slab + pl * ROWB + ((ch ^ swz(pl)) << 4)) = qa[d][g8];
            }
        }
        if (item0 + DEPTH * stride < end) fetch(d, item0 + DEPTH * stride);
        if (Iidx >= R) continue;
        const int I = rm.tile_row(Iidx);

        // tile rows -> second slab
        if (OUTER) {
#pragma unroll
            for (int u = 0; u < 4; ++u) *reinterpret_cast<u32x2_t *>(sT + srow[u] * 32 + 8 * kq) = x[u];
        }

        // basis gradient: K = 32 tiles per product; B fragment of lane (entry j, kq) = tiles 32sx + 8kq .. +7 of entry j
#pragma unroll
        for (int sx = 0; sx < (OUTER ? 2 : 0); ++sx) {
            v4i16_t t[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                // source address of this lane inside its 16-lane group: tile row (32sx + 8kq + 4h) + j/4, entries 4*(j%4)..
                const int t0 = 32 * sx + 8 * kq + 4 * h;
                const int row = (t0 ^ (((t0 >> 3) & 1) << 2)) + (j >> 2);
                t[h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16_t *)(
                    (__attribute__((address_space(3))) char *)(sT + row * 32 + 8 * (j & 3))));
            }
            struct { v4i16_t a, b; } both = {t[0], t[1]};
            const bf16x8_t fb = __builtin_bit_cast(bf16x8_t, both);
#pragma unroll
            for (int g = 0; g < 2 * KC; ++g)
                if (g < ng) {
                    const int pl = 16 * g + j;
                    const bf16x8_t fp = *reinterpret_cast<const bf16x8_t *>(slab + pl * ROWB + (((4 * sx + kq) ^ swz(pl)) << 4));
                    dacc[g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fp, fb, dacc[g], 0, 0, 0);
                }
        }

        // encode: rows = tiles, columns = planes.  The results go through the plane slab (its fragments have been read
        // above; LDS operations of a wavefront execute in order) so that they leave as whole 128-byte lines, 8 planes
        // per store instruction, like the loads.
#pragma unroll
        for (int g = 0; g < 2 * KC; ++g) {
            if (g < ng) {
                f32x4_t o[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
                    const bf16x8_t hf = __builtin_bit_cast(bf16x8_t, u32x4_t{x[u][0], x[u][1], 0u, 0u});
                    o[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hf, eb[g], zero, 0, 0, 0);
                }
                const int pl = 16 * g + j;                  // products 2h, 2h+1: tiles 32h + 8kq .. +7 = chunk 4h + kq
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const f32x4_t a = o[2 * half], b = o[2 * half + 1];
                    const u32x4_t w = {pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(b[0], b[1]),
                                       pack_bf16x2(b[2], b[3])};
                    *reinterpret_cast<u32x4_t *>(slab + pl * ROWB + (((4 * half + kq) ^ swz(pl)) << 4)) = w;
                }
            }
        }
        const size_t rowb_out = plane_row_base(I, pg, r, Cc);
#pragma unroll
        for (int g8 = 0; g8 < KC * 4; ++g8) {
            const int pl = 8 * g8 + pr;
            if (pl < r && J0 + 8 * ch < Cc) {
                const u32x4_t w = *reinterpret_cast<const u32x4_t *>(slab + pl * ROWB + ((ch ^ swz(pl)) << 4));
                store16<THROUGH>(P + rowb_out + (size_t)pl * plane + J0 + 8 * ch, w);
            }
        }
    }

}

// The item loop of one wavefront, items as in encode_items.  slab: KC * 32 * 128 bytes of LDS private to the
// wavefront; sT: 64 x 32 bytes (OUTER only); oacc accumulates the basis gradient (OUTER).  No workgroup barrier inside.
template <bool GELU, int KC, bool OUTER, int DEPTH = 1>   // DEPTH as in encode_items
__device__ __forceinline__ void decode_items(const bf16_t *__restrict__ P, const bf16_t *__restrict__ Dm, bf16_t *__restrict__ Cmat,
                                             int R, int Cc, int r, int chunks, const bf16_t *__restrict__ V, int pg, const RowMap &rm,
                                             long first, long stride, long end, char *sT, char *slab, f32x4_t (&oacc)[4], int lane)
{
    constexpr int ROWB = 128;                               // bytes per LDS row (64 tiles)
    const int ngroups = (r + 15) >> 4;
    const int j = lane & 15, kq = lane >> 4;
    // row of tile `lane` in sT: rows t and t^4 are swapped where bit 3 of t is set, so that the four 4-tile groups one
    // transposing read touches fall into both halves of the banks
    const int strow = lane ^ (((lane >> 3) & 1) << 2);

    // A fragments: lane (entry q = j, kq) holds D[32g + 8kq + e][q], e = 0..7
    bf16x8_t fa[KC];
#pragma unroll
    for (int g = 0; g < KC; ++g) {
        uint32_t w[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            const int p0 = 32 * g + 8 * kq + 2 * e2;
            const uint32_t lo = p0 < r ? Dm[p0 * 16 + j] : 0u, hi = p0 + 1 < r ? Dm[(p0 + 1) * 16 + j] : 0u;
            w[e2] = lo | (hi << 16);
        }
        fa[g] = __builtin_bit_cast(bf16x8_t, u32x4_t{w[0], w[1], w[2], w[3]});
    }
    // swizzle of the 16-byte chunk index inside a row, so that the 8 plane rows one transposing read touches
    // (planes 0-3 and 8-11, or 4-7 and 12-15, of a 16-tile column group) fall into different bank windows
    auto swz = [](int row) { return ((((row >> 1) & 1) | (((row >> 3) & 1) << 1)) << 1); };

    const size_t plane = (size_t)pg * Cc;
    const size_t ld = (size_t)Cc * 4;

    // Loader role of a lane: plane 8*g8 + pr, 16-byte chunk ch (8 tiles) -- whole 128-byte lines, 8 planes per
    // instruction; with OUTER also tile J0 + lane of V (4 rows x 8 bytes).  The NEXT item's operands are fetched into
    // registers while the current item is computed and stored.
    const int pr = lane >> 3, ch = lane & 7;
    u32x4_t pre[DEPTH][KC * 4];
    u32x2_t xpre[DEPTH][OUTER ? 4 : 1];
    auto fetch = [&](int d, long item) {
        const int Ii = (int)(item / chunks), cki = (int)(item - (long)Ii * chunks);
        const int Jl = cki * 64 + 8 * ch;
        const int Ia = Ii < R ? rm.tile_row(Ii) : 0;        // Ii counts the tile rows of this launch, Ia is the tile row itself
        const size_t rowb = plane_row_base(Ia, pg, r, Cc);
#pragma unroll
        for (int g8 = 0; g8 < KC * 4; ++g8) {
            const int pl = 8 * g8 + pr;
            u32x4_t v = {0u, 0u, 0u, 0u};       // planes >= r stay zero (they meet zero D entries, but must be finite)
            if (Ii < R && pl < r && Jl < Cc) v = *reinterpret_cast<const u32x4_t *>(P + rowb + (size_t)pl * plane + Jl);
            pre[d][g8] = v;
        }
        if (OUTER) {
            const int Jt = cki * 64 + lane, nv = rm.valid(Ia);
            const size_t r0 = rm.row0(Ia);
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                u32x2_t xv = {0u, 0u};
                if (Ii < R && Jt < Cc && a < nv) xv = *reinterpret_cast<const u32x2_t *>(V + (r0 + a) * ld + (size_t)Jt * 4);
                xpre[d][a] = xv;
            }
        }
    };
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
        if (first + d * stride < end) fetch(d, first + d * stride);

    for (long base = first; base < end; base += DEPTH * stride)
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
        const long item0 = base + d * stride;
        if (item0 >= end) break;
        const int In = (int)(item0 / chunks), J0 = (int)(item0 - (long)In * chunks) * 64;
        const bool live = In < R;
        const int I = live ? rm.tile_row(In) : 0;
        // slab and sV belong to this wavefront alone and its LDS operations execute in order: the writes below land
        // after the previous round's fragment reads without a workgroup barrier (which would also make the wavefront
        // wait for the loads it is about to put in flight)
#pragma unroll
        for (int g8 = 0; g8 < KC * 4; ++g8) {
            const int pl = 8 * g8 + pr;
            *reinterpret_cast<u32x4_t *>(slab + pl * ROWB + ((ch ^ swz(pl)) << 4)) = pre[d][g8];
        }
        if (OUTER) {
            // lane = tile J0 + lane: its 16 entries (4 rows x 8 bytes) as two 16-byte writes, tile-major; they come back
            // as "entry x 4 consecutive tiles" through the transposing read below
            *reinterpret_cast<u32x4_t *>(sT + strow * 32) = u32x4_t{xpre[d][0][0], xpre[d][0][1], xpre[d][1][0], xpre[d][1][1]};
            *reinterpret_cast<u32x4_t *>(sT + strow * 32 + 16) = u32x4_t{xpre[d][2][0], xpre[d][2][1], xpre[d][3][0], xpre[d][3][1]};
        }
        if (item0 + DEPTH * stride < end) fetch(d, item0 + DEPTH * stride);
        if (live && OUTER) {
            // K = 32 tiles per MFMA: A = planes x tiles from the slab (lane: plane 16g + j, tiles 32s + 8kq ..),
            // B = tiles x entries from sT (lane: entry j, same tiles)
#pragma unroll
            for (int sx = 0; sx < 2; ++sx) {
                v4i16_t tb[2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    // source address of this lane inside its 16-lane group: tile row (32sx + 8kq + 4h) + j/4, entries 4*(j%4)..
                    const int t0 = 32 * sx + 8 * kq + 4 * h;
                    const int row = (t0 ^ (((t0 >> 3) & 1) << 2)) + (j >> 2);
                    tb[h] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16_t *)(
                        (__attribute__((address_space(3))) char *)(sT + row * 32 + 8 * (j & 3))));
                }
                struct { v4i16_t a, b; } both_b = {tb[0], tb[1]};
                const bf16x8_t fb = __builtin_bit_cast(bf16x8_t, both_b);
#pragma unroll
                for (int g = 0; g < 2 * KC; ++g) {
                    if (g < ngroups) {
                        const int pl = 16 * g + j;
                        const bf16x8_t fp = *reinterpret_cast<const bf16x8_t *>(slab + pl * ROWB + (((4 * sx + kq) ^ swz(pl)) << 4));
                        oacc[g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fp, fb, oacc[g], 0, 0, 0);
                    }
                }
            }
        }
        if (live) {
            const int nv_out = rm.valid(I);
            const size_t r0_out = rm.row0(I);
#pragma unroll
            for (int u = 0; u < 4; ++u) {                   // 16 tiles per MFMA
                f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int g = 0; g < KC; ++g) {
                    v4i16_t t[2];
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk) {
                        // source row for this lane of the 16-lane group: plane 32g + 8kq + 4kk + j/4, tiles 16u + 4(j%4)
                        const int row = 32 * g + 8 * kq + 4 * kk + (j >> 2);
                        const int col = 16 * u + 4 * (j & 3);
                        const char *src = slab + row * ROWB + ((((col >> 3)) ^ swz(row)) << 4) + ((col & 7) << 1);
                        t[kk] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16_t *)(
                            (__attribute__((address_space(3))) char *)src));
                    }
                    struct { v4i16_t a, b; } both = {t[0], t[1]};
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[g], __builtin_bit_cast(bf16x8_t, both), acc, 0, 0, 0);
                }
                // lane holds row a = kq of tile J0 + 16u + j: entries acc[0..3]
                const int J = J0 + 16 * u + j;
                if (J < Cc && kq < nv_out) {
                    float c0 = acc[0], c1 = acc[1], c2 = acc[2], c3 = acc[3];
                    if (GELU) { c0 = gelu_erf(c0); c1 = gelu_erf(c1); c2 = gelu_erf(c2); c3 = gelu_erf(c3); }
                    const u32x2_t w = {pack_bf16x2(c0, c1), pack_bf16x2(c2, c3)};
                    *reinterpret_cast<u32x2_t *>(Cmat + (r0_out + kq) * ld + (size_t)J * 4) = w;
                }
            }
        }
    }
}

}  // namespace stl
