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
#include "stl_tile_items.h"

namespace stl {

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
    const int j = lane & 15, kq = lane >> 4;
    f32x4_t dacc[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) dacc[g] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    // wavefront w of block b takes items 4b + w, 4b + w + 4 * gridDim.x, ...
    encode_items<KC, OUTER>(A, E, P, Qp, R, Cc, r, chunks, pg, rm, (long)blockIdx.x * 4 + wave, (long)gridDim.x * 4,
                            (long)R * chunks, sT_all[OUTER ? wave : 0], slab_all[wave], dacc, lane);

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
