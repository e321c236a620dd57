// Encode of a matrix and a basis gradient against other planes in one pass over the matrix (bf16):
//     P[p][I][J]  = sum_q E[p][q] * a[I][J][q]                  (a = 4x4 tile view of A)
//     G[p][q]    += sum_{I,J} Qp[p][I][J] * a[I][J][q]
// In the backward pass A = dC, E = D, P = dYhat, Qp = Yhat, G = dD: dC is read from HBM once for both results.
//
// Both contractions run on v_mfma_f32_16x16x32_bf16.
//  * Encode: rows = tiles, columns = planes, K = tile entries.  A lane (tile, kq) loads row kq of its tile (8 bytes,
//    entries 4kq..4kq+3) straight from HBM; padded with four zeros this is its operand fragment (K slot 8kq+e <->
//    entry 4kq+e for e < 4, zero weight on the other slots).  The tile of lane j in product u is
//    J0 + 8*(j/4) + 4*(u%2) + 32*(u/2) + j%4, which leaves a lane of the result (plane, kq) with 8 consecutive tiles
//    per product pair: 16-byte stores, 64 contiguous bytes per plane and instruction.
//  * Basis gradient: rows = planes, columns = tile entries, K = 32 tiles.  The plane segments of the item (128 bytes per
//    plane) are loaded as whole cache lines, 8 planes per instruction, into a wavefront-private LDS slab [plane][tile]
//    and read back as fragments (8 consecutive tiles of a plane = 16 bytes; fetching those 64-byte half lines
//    straight from HBM, 16 planes per instruction, ran a quarter slower).  The tile rows already in registers are
//    written tile-major into a second private slab (one 8-byte write each) and come back as "entry x 4 consecutive
//    tiles" through the transposing ds_read_b64_tr_b16.
// The next item's operands are fetched while the current one is processed; every block writes one partial of G to
// `part`, added up in block order by a second kernel (no floating-point atomics: bitwise reproducible).
#include "stl_kernels.h"
#include "stl_device.h"

namespace stl {

typedef short v4i16_t __attribute__((ext_vector_type(4)));

// OUTER = false: the encode alone (Qp, part unused) -- the same whole-line stores through the slab, used for plain encodes
template <int KC, bool OUTER>   // KC = number of 32-plane groups (1: r <= 32, 2: r <= 64)
__global__ __launch_bounds__(256) void encode_outer16_kernel(const bf16_t *__restrict__ A, const bf16_t *__restrict__ E,
                                                             bf16_t *__restrict__ P, const bf16_t *__restrict__ Qp,
                                                             float *__restrict__ part, int R, int Cc, int r, int chunks, int pg,
                                                             RowMap rm)
{
    constexpr int ROWB = 128;                               // bytes per plane row of the slab (64 tiles)
    __shared__ __align__(16) char sT_all[OUTER ? 4 : 1][OUTER ? 64 * 32 : 16];   // per wavefront: [tile][16 entries] bf16
    __shared__ __align__(16) char slab_all[4][KC * 32 * ROWB];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    char *sT = sT_all[OUTER ? wave : 0], *slab = slab_all[wave];
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
    f32x4_t dacc[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) dacc[g] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // tile (relative to J0) of this lane in product u, and its row in the LDS slab: rows t and t^4 are swapped where
    // bit 3 of t is set, so that the four 4-tile groups of one write (and the four 8-tile groups of one transposing
    // read) fall into both halves of the banks
    int trel[4], srow[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        trel[u] = 8 * (j >> 2) + 4 * (u & 1) + 32 * (u >> 1) + (j & 3);
        srow[u] = trel[u] ^ (((trel[u] >> 3) & 1) << 2);
    }

    const long items = (long)R * chunks;
    const long stride = (long)gridDim.x * 4;
    int In = (int)(((long)blockIdx.x * 4 + wave) / chunks), ckn = (int)(((long)blockIdx.x * 4 + wave) % chunks);
    const int dI = (int)(stride / chunks), dck = (int)(stride % chunks);

    u32x2_t xa[4];          // this lane's tile rows, one per product
    u32x4_t qa[KC * 4];     // plane segments, loader role: plane 8*g8 + pr, tiles 8ch .. 8ch+7
    auto fetch = [&](int Ii, int cki) {
        const int J0 = cki * 64;
        const int Ia = Ii < R ? rm.tile_row(Ii) : 0;        // Ii counts the tile rows of this launch, Ia is the tile row itself
        const size_t rowb = plane_row_base(Ia, pg, r, Cc);
        const bool row_ok = Ii < R && kq < rm.valid(Ia);    // a null row reads as zero
        const size_t r0 = rm.row0(Ia);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            u32x2_t v = {0u, 0u};
            if (row_ok && J0 + trel[u] < Cc) v = *reinterpret_cast<const u32x2_t *>(A + (r0 + kq) * ld + (size_t)(J0 + trel[u]) * 4);
            xa[u] = v;
        }
        if (OUTER) {
#pragma unroll
            for (int g8 = 0; g8 < KC * 4; ++g8) {
                const int pl = 8 * g8 + pr, tk = J0 + 8 * ch;
                u32x4_t v = {0u, 0u, 0u, 0u};
                if (Ii < R && pl < r && tk < Cc) v = *reinterpret_cast<const u32x4_t *>(Qp + rowb + (size_t)pl * plane + tk);
                qa[g8] = v;
            }
        }
    };
    fetch(In, ckn);

    for (long item0 = (long)blockIdx.x * 4; item0 < items; item0 += stride) {
        const int Iidx = In, J0 = ckn * 64;
        u32x2_t x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) x[u] = xa[u];
        // plane segments -> slab (private to the wavefront, whose LDS operations execute in order: no barrier)
        if (OUTER) {
#pragma unroll
            for (int g8 = 0; g8 < KC * 4; ++g8) {
                const int pl = 8 * g8 + pr;
                *reinterpret_cast<u32x4_t *>(slab + pl * ROWB + ((ch ^ swz(pl)) << 4)) = qa[g8];
            }
        }
        In += dI;
        ckn += dck;
        if (ckn >= chunks) { ckn -= chunks; ++In; }
        if (item0 + stride < items) fetch(In, ckn);
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
                *reinterpret_cast<u32x4_t *>(P + rowb_out + (size_t)pl * plane + J0 + 8 * ch) = w;
            }
        }
    }

    if (!OUTER) return;
    // accumulator e of group g: plane 16g + 4kq + e, tile entry j; fixed-order sum over the four wavefronts
    __syncthreads();                                        // every wavefront is done with its slab
    float *red = reinterpret_cast<float *>(&slab_all[0][0]); // 4 x (32 KC x 16) floats = the slabs' size
#pragma unroll
    for (int g = 0; g < 2 * KC; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) red[wave * (KC * 512) + (16 * g + 4 * kq + e) * 16 + j] = dacc[g][e];
    __syncthreads();
    for (int i = threadIdx.x; i < r * 16; i += 256)
        part[(size_t)blockIdx.x * r * 16 + i] =
            ((red[i] + red[KC * 512 + i]) + red[2 * KC * 512 + i]) + red[3 * KC * 512 + i];
}

bool encode_outer_eligible(int dtype, int Cc) { return dtype == 1 && (Cc % 8) == 0; }

int encode_outer_blocks(int R, int Cc)
{
    const long items = (long)R * ((Cc + 63) / 64);
    const long blocks = (items + 3) / 4;
    return (int)(blocks > 1024 ? 1024 : blocks);
}

hipError_t launch_encode_outer(const void *A, const void *E, void *P, const void *Qp, float *G, float *part, int R, int Cc,
                               int r, int accumulate, int pg, hipStream_t s, RowMap rm, bool final_sum)
{
    if (pg <= 0) pg = R;
    R = rm.count(R);                                        // tile rows this launch walks over
    if (R <= 0) return hipErrorInvalidValue;
    const int chunks = (Cc + 63) / 64;
    const int nb = encode_outer_blocks(R, Cc);
    if (r <= 32)
        hipLaunchKernelGGL((encode_outer16_kernel<1, true>), dim3(nb), dim3(256), 0, s, (const bf16_t *)A, (const bf16_t *)E,
                           (bf16_t *)P, (const bf16_t *)Qp, part, R, Cc, r, chunks, pg, rm);
    else
        hipLaunchKernelGGL((encode_outer16_kernel<2, true>), dim3(nb), dim3(256), 0, s, (const bf16_t *)A, (const bf16_t *)E,
                           (bf16_t *)P, (const bf16_t *)Qp, part, R, Cc, r, chunks, pg, rm);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !final_sum) return e;
    return launch_outer_final(part, G, nb, r * 16, accumulate, s);
}

// the encode alone through the same kernel (bf16, Cc % 8 == 0): grid-stride over (tile row, 64-tile chunk) items
hipError_t launch_encode_lines(const void *A, const void *E, void *P, int R, int Cc, int r, int pg, hipStream_t s, RowMap rm)
{
    if (pg <= 0) pg = R;
    R = rm.count(R);
    if (R <= 0) return hipSuccess;
    const int chunks = (Cc + 63) / 64;
    const long items = (long)R * chunks;
    long blocks = (items + 3) / 4;
    if (blocks > 8192) blocks = 8192;
    if (r <= 32)
        hipLaunchKernelGGL((encode_outer16_kernel<1, false>), dim3((unsigned)blocks), dim3(256), 0, s, (const bf16_t *)A,
                           (const bf16_t *)E, (bf16_t *)P, (const bf16_t *)nullptr, (float *)nullptr, R, Cc, r, chunks, pg, rm);
    else
        hipLaunchKernelGGL((encode_outer16_kernel<2, false>), dim3((unsigned)blocks), dim3(256), 0, s, (const bf16_t *)A,
                           (const bf16_t *)E, (bf16_t *)P, (const bf16_t *)nullptr, (float *)nullptr, R, Cc, r, chunks, pg, rm);
    return hipGetLastError();
}

}  // namespace stl
