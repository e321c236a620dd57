// Tile-level linear maps of the STL operator: encode (step (i) of Algorithm 1), decode
// (step (iii)) and the two basis-gradient reductions.  All of these stream a matrix once
// through HBM; arithmetic is fp32.
#include "stl_kernels.h"
#include "stl_device.h"
#include "stl_tile_items.h"


namespace stl {

// ---------------------------------------------------------------------------------------
// encode:  P[p][I][L] = sum_q E[p][q] * A[4I + q/4][4L + q%4]        (planes of encoded tiles)
// One thread per tile; lanes run along L so that every row segment and every plane row is
// read / written contiguously by a wavefront.
// ---------------------------------------------------------------------------------------
// TB: type the basis is stored in (the storage type, or fp32 for a basis composed on the device).  R counts the tile
// rows this launch walks over (see RowMap).
template <typename T, typename TB>
__global__ __launch_bounds__(256) void encode_kernel(const T *__restrict__ A, const TB *__restrict__ E,
                                                     T *__restrict__ P, int R, int Cc, int r, int pg, RowMap rm)
{
    __shared__ float sE[64 * 16];
    const int tid = threadIdx.y * blockDim.x + threadIdx.x;
    for (int i = tid; i < r * 16; i += 256) sE[i] = Elem<TB>::ld(E + i);
    __syncthreads();

    const int L = blockIdx.x * blockDim.x + threadIdx.x;
    if (L >= Cc) return;
    const size_t ld = (size_t)Cc * 4;
    const size_t plane = (size_t)pg * Cc;
    // grid-stride over the tile rows: the grid's second extent is capped, any row count is covered
    for (int idx = blockIdx.y * blockDim.y + threadIdx.y; idx < R; idx += gridDim.y * blockDim.y) {
        const int I = rm.tile_row(idx), nv = rm.valid(I);
        const size_t r0 = rm.row0(I);
        float x[16];
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) x[a * 4 + b] = a < nv ? Elem<T>::ld(A + (r0 + a) * ld + (size_t)L * 4 + b) : 0.f;

        T *out = P + plane_row_base(I, pg, r, Cc) + L;
        for (int p = 0; p < r; ++p) {
            float s = 0.f;
#pragma unroll
            for (int q = 0; q < 16; ++q) s = fmaf(sE[p * 16 + q], x[q], s);
            Elem<T>::st(out + (size_t)p * plane, s);
        }
    }
}

// ---------------------------------------------------------------------------------------
// decode:  Cmat[4I + q/4][4J + q%4] = sum_p Dm[p][q] * P[p][I][J]     (+ optional GELU)
// ---------------------------------------------------------------------------------------
template <typename T, typename TB, bool GELU>
__global__ __launch_bounds__(256) void decode_kernel(const T *__restrict__ P, const TB *__restrict__ Dm,
                                                     T *__restrict__ Cmat, int R, int Cc, int r, int pg, RowMap rm)
{
    __shared__ float sD[64 * 16];
    const int tid = threadIdx.y * blockDim.x + threadIdx.x;
    for (int i = tid; i < r * 16; i += 256) sD[i] = Elem<TB>::ld(Dm + i);
    __syncthreads();

    const int J = blockIdx.x * blockDim.x + threadIdx.x;
    if (J >= Cc) return;
    const size_t plane = (size_t)pg * Cc;
    const size_t ld = (size_t)Cc * 4;
    // grid-stride over the tile rows, as in the encode
    for (int idx = blockIdx.y * blockDim.y + threadIdx.y; idx < R; idx += gridDim.y * blockDim.y) {
        const int I = rm.tile_row(idx), nv = rm.valid(I);
        const size_t r0 = rm.row0(I);
        const T *in = P + plane_row_base(I, pg, r, Cc) + J;
        float c[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) c[q] = 0.f;
        for (int p = 0; p < r; ++p) {
            const float y = Elem<T>::ld(in + (size_t)p * plane);
#pragma unroll
            for (int q = 0; q < 16; ++q) c[q] = fmaf(sD[p * 16 + q], y, c[q]);
        }
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                float v = c[a * 4 + b];
                if (GELU) v = gelu_erf(v);
                if (a < nv) Elem<T>::st(Cmat + (r0 + a) * ld + (size_t)J * 4 + b, v);
            }
    }
}

// ---------------------------------------------------------------------------------------
// basis gradients:  G[p][q] (+)= sum_{I,J} P[p][I][J] * V[4I + q/4][4J + q%4]
// (dD with P=Yhat, V=dC;  dE_X with P=dXhat, V=X).  Two deterministic stages: every block
// sums a fixed range of tiles in a fixed order into part[block][p][q]; the second stage
// adds the partials in block order.  No atomics, so results are bitwise reproducible.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void outer_partial_kernel(const T *__restrict__ P, const T *__restrict__ V,
                                                            float *__restrict__ part, int R, int Cc, int r,
                                                            int tiles_per_block, int pg, RowMap rm)
{
    // 256 threads: q = tid & 15, tile lane = tid >> 4 (16 tiles in flight); loop over planes.
    __shared__ float red[16][16];
    const int q = threadIdx.x & 15, tl = threadIdx.x >> 4;
    const size_t T_total = (size_t)R * Cc;
    const size_t t0 = (size_t)blockIdx.x * tiles_per_block;
    size_t t1 = t0 + tiles_per_block;
    if (t1 > T_total) t1 = T_total;
    const size_t ld = (size_t)Cc * 4;
    for (int p = 0; p < r; ++p) {
        float s = 0.f;
        for (size_t tile = t0 + tl; tile < t1; tile += 16) {
            const size_t J = tile % Cc;
            const int I = rm.tile_row((int)(tile / Cc));
            const float v = (q >> 2) < rm.valid(I) ? Elem<T>::ld(V + (rm.row0(I) + (q >> 2)) * ld + J * 4 + (q & 3)) : 0.f;
            const float y = Elem<T>::ld(P + plane_row_base(I, pg, r, Cc) + (size_t)p * pg * Cc + J);
            s = fmaf(y, v, s);
        }
        red[tl][q] = s;
        __syncthreads();
        if (tl == 0) {
            float tot = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) tot += red[i][q];
            part[((size_t)blockIdx.x * r + p) * 16 + q] = tot;
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(1024) void outer_final_kernel(const float *__restrict__ part, float *__restrict__ G,
                                                           int nblocks, int n_out, int accumulate,
                                                           const float *__restrict__ part1 = nullptr,
                                                           float *__restrict__ G1 = nullptr, int nblocks1 = 0)
{
    if (blockIdx.y == 1) {          // second sum of a launch that finishes two at once
        part = part1;
        G = G1;
        nblocks = nblocks1;
    }
    // 16 outputs per block of 1024 threads; 64 slices of the block range per output (up to 1024 partials: 16 loads per
    // thread, all in flight together), then a fixed-order sum over the slices.
    __shared__ float red[64][17];
    const int o = threadIdx.x & 15, sl = threadIdx.x >> 4;
    const int i = blockIdx.x * 16 + o;
    float s = 0.f;
    if (i < n_out)
#pragma unroll 16
        for (int b = sl; b < nblocks; b += 64) s += part[(size_t)b * n_out + i];
    red[sl][o] = s;
    __syncthreads();
    if (sl == 0 && i < n_out) {
        float tot = 0.f;
#pragma unroll
        for (int u = 0; u < 64; ++u) tot += red[u][o];
        G[i] = accumulate ? G[i] + tot : tot;
    }
}

// ---------------------------------------------------------------------------------------
// bf16 encode on the matrix cores.  The map "16 tile entries -> r planes" is a small dense
// contraction (K = 16); on the vector ALUs it costs as many cycles as the HBM transfer, on
// MFMA it is free and the kernel is bound by the stream through HBM alone.
//   v_mfma_f32_32x32x16_bf16:  rows = planes (E, 32 x 16), columns = tiles (tile entries, 16 x 32).
// A wavefront takes 128 consecutive tiles of one tile row: lane (j, h) loads rows 2h and 2h+1 of
// tiles 4j..4j+3 (32 contiguous bytes each); MFMA u works on tiles 4j+u, so that afterwards a lane
// holds 4 consecutive tiles of a plane and writes them with one 8-byte store.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void encode_mfma_kernel(const bf16_t *__restrict__ A, const bf16_t *__restrict__ E,
                                                          bf16_t *__restrict__ P, int R, int Cc, int r, int chunks, int pg,
                                                          RowMap rm)
{
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long item = (long)blockIdx.x * 4 + wave;          // (tile row, chunk of 128 tile columns)
    if (item >= (long)R * chunks) return;
    const int I = rm.tile_row((int)(item / chunks)), J0 = (int)(item % chunks) * 128;
    const int nv = rm.valid(I);
    const size_t r0 = rm.row0(I);
    const int j = lane & 31, h = lane >> 5;
    const size_t ld = (size_t)Cc * 4;
    const int Jl = J0 + 4 * j;                               // first of this lane's 4 tiles

    u32x4_t row[2][2];                                       // [row 2h / 2h+1][tiles (0,1) / (2,3)]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            u32x4_t z = {0u, 0u, 0u, 0u};
            if (Jl + 2 * c < Cc && 2 * h + a < nv)
                z = *reinterpret_cast<const u32x4_t *>(A + (r0 + 2 * h + a) * ld + (size_t)(Jl + 2 * c) * 4);
            row[a][c] = z;
        }

    const size_t plane = (size_t)pg * Cc, rowb = plane_row_base(I, pg, r, Cc);
    for (int g = 0; g < r; g += 32) {
        const int pl = g + j;
        u32x4_t ev = {0u, 0u, 0u, 0u};
        if (pl < r) ev = *reinterpret_cast<const u32x4_t *>(E + pl * 16 + 8 * h);
        const bf16x8_t ea = __builtin_bit_cast(bf16x8_t, ev);
        f32x16_t acc[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const u32x4_t bv = {row[0][u >> 1][2 * (u & 1)], row[0][u >> 1][2 * (u & 1) + 1],
                                row[1][u >> 1][2 * (u & 1)], row[1][u >> 1][2 * (u & 1) + 1]};
            f32x16_t zero;
#pragma unroll
            for (int v = 0; v < 16; ++v) zero[v] = 0.f;
            acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ea, __builtin_bit_cast(bf16x8_t, bv), zero, 0, 0, 0);
        }
        if (Jl < Cc) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int po = g + 8 * (v >> 2) + 4 * h + (v & 3);
                if (po < r) {
                    u32x2_t w = {pack_bf16x2(acc[0][v], acc[1][v]), pack_bf16x2(acc[2][v], acc[3][v])};
                    *reinterpret_cast<u32x2_t *>(P + rowb + (size_t)po * plane + Jl) = w;
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// bf16 basis gradients on the matrix cores:  G (r x 16) = P (r x T) . tileview(V) (T x 16),
// contraction over all T = R*Cc tiles, v_mfma_f32_16x16x32_bf16 (rows = planes, columns = the 16
// tile entries, K = 32 tiles).  P fragments come straight from HBM (8 consecutive tiles of a plane
// = 16 bytes); V is read coalesced and turned into "entry x tile" form through LDS.
// Stage 1 writes one partial per block in a fixed order; stage 2 adds them in block order.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void outer_mfma_kernel(const bf16_t *__restrict__ P, const bf16_t *__restrict__ V,
                                                         float *__restrict__ part, int R, int Cc, int r,
                                                         int tiles_per_block, int pg, RowMap rm)
{
    constexpr int PITCH = 64 + 8;                       // bf16 elements per LDS row (16-byte aligned rows)
    __shared__ __align__(16) bf16_t sV[4][16][PITCH];
    __shared__ float red[4][64 * 16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long T = (long)R * Cc;
    const long t0 = (long)blockIdx.x * tiles_per_block;
    long t1 = t0 + tiles_per_block;
    if (t1 > T) t1 = T;
    const size_t ld = (size_t)Cc * 4;
    const int q = lane & 15, kq = lane >> 4;
    const int ngroups = (r + 15) >> 4;

    f32x4_t acc[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) acc[g] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // operands of one 256-tile step of the block: this wavefront's 64 tiles of V (4 rows x 8 bytes per lane) and the
    // P fragments (8 consecutive tiles of a plane per lane).  The next step's operands are in flight while the
    // current step runs on the matrix cores.
    u32x2_t v[4];
    u32x4_t pa[2][4];
    auto fetch = [&](long base) {
        const long tb = base + wave * 64;
        const long tile = tb + lane;
        if (tile < t1) {
            const long idx = tile / Cc, J = tile - idx * Cc;
            const int I = rm.tile_row((int)idx), nv = rm.valid(I);
            const size_t r0 = rm.row0(I);
#pragma unroll
            for (int a = 0; a < 4; ++a)
                v[a] = a < nv ? *reinterpret_cast<const u32x2_t *>(V + (r0 + a) * ld + (size_t)J * 4) : u32x2_t{0u, 0u};
        } else {
#pragma unroll
            for (int a = 0; a < 4; ++a) v[a] = u32x2_t{0u, 0u};
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const long tk = tb + 32 * s + 8 * kq;        // 8 consecutive tiles of one tile row (Cc % 8 == 0): all in or all out
            const int Ik = (int)(tk / Cc);
            const size_t off = tk < t1 ? plane_row_base(rm.tile_row(Ik), pg, r, Cc) + (size_t)(tk - (long)Ik * Cc) : 0;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int pl = 16 * g + q;
                u32x4_t av = {0u, 0u, 0u, 0u};
                if (g < ngroups && pl < r && tk < t1) av = *reinterpret_cast<const u32x4_t *>(P + off + (size_t)pl * pg * Cc);
                pa[s][g] = av;
            }
        }
    };

    fetch(t0);
    for (long base = t0; base < t1; base += 256) {       // uniform trip count over the block
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            sV[wave][4 * a + 0][lane] = (bf16_t)(v[a][0] & 0xffffu);
            sV[wave][4 * a + 1][lane] = (bf16_t)(v[a][0] >> 16);
            sV[wave][4 * a + 2][lane] = (bf16_t)(v[a][1] & 0xffffu);
            sV[wave][4 * a + 3][lane] = (bf16_t)(v[a][1] >> 16);
        }
        u32x4_t pc[2][4];
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int g = 0; g < 4; ++g) pc[s][g] = pa[s][g];
        // sV[wave] is private to the wavefront and a wavefront's LDS operations execute in order: no workgroup barrier
        // (a barrier would also make the wavefront wait for the loads it is about to put in flight)
        if (base + 256 < t1) fetch(base + 256);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const bf16x8_t fb = *reinterpret_cast<const bf16x8_t *>(&sV[wave][q][32 * s + 8 * kq]);
#pragma unroll
            for (int g = 0; g < 4; ++g)
                if (g < ngroups)
                    acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, pc[s][g]), fb, acc[g], 0, 0, 0);
        }
    }
    // accumulator element e of group g: plane 16g + 4*(lane/16) + e, tile entry lane%16
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) red[wave][(16 * g + 4 * kq + e) * 16 + q] = acc[g][e];
    __syncthreads();
    for (int i = threadIdx.x; i < r * 16; i += 256)
        part[(size_t)blockIdx.x * r * 16 + i] = ((red[0][i] + red[1][i]) + red[2][i]) + red[3][i];
}

// ---------------------------------------------------------------------------------------
// bf16 decode on the matrix cores:  tile entries (16) x tiles = D^T (16 x r) . Yhat (r x tiles),
// v_mfma_f32_16x16x32_bf16 with rows = tile entries, columns = 16 tiles, K = planes.
// A wavefront takes 64 consecutive tiles of one tile row: the r plane segments (128 bytes each) are
// read coalesced into a private LDS slab [plane][tile]; the transposing ds_read_b64_tr_b16 hands
// every lane 4 consecutive planes of its tile (the MFMA B fragment).  The accumulator leaves each
// lane with one row of one output tile (4 entries = 8 bytes), so 16 lanes store 128 contiguous bytes.
// ---------------------------------------------------------------------------------------
// OUTER: the same pass also accumulates the basis gradient G (r x 16) += P (r x tiles) . tileview(V) (tiles x 16)
// (dE_X with P = dXhat, V = X while dX is decoded), so that the planes are read from HBM once for both results;
// every block writes one partial to `part`, added up in block order by outer_final_kernel.
template <bool GELU, int KC, bool OUTER>   // KC = number of 32-plane groups (1: r <= 32, 2: r <= 64)
__global__ __launch_bounds__(256) void decode_mfma_kernel(const bf16_t *__restrict__ P, const bf16_t *__restrict__ Dm,
                                                          bf16_t *__restrict__ Cmat, int R, int Cc, int r, int chunks,
                                                          const bf16_t *__restrict__ V, float *__restrict__ part, int pg,
                                                          RowMap rm)
{
    constexpr int ROWB = 128;                               // bytes per LDS row (64 tiles)
    __shared__ __align__(16) char slab_all[4][KC * 32 * ROWB];
    // OUTER: per wavefront the 64 tiles of V, tile-major [tile][16 entries] (32 bytes per tile)
    __shared__ __align__(16) char sT_all[OUTER ? 4 : 1][OUTER ? 64 * 32 : 16];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = lane & 15, kq = lane >> 4;
    f32x4_t oacc[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) oacc[g] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    // wavefront w of block b takes items 4b + w, 4b + w + 4 * gridDim.x, ...
    decode_items<GELU, KC, OUTER>(P, Dm, Cmat, R, Cc, r, chunks, V, pg, rm, (long)blockIdx.x * 4 + wave, (long)gridDim.x * 4,
                                  (long)R * chunks, sT_all[OUTER ? wave : 0], slab_all[wave], oacc, lane);
    if (OUTER) {
        // accumulator e of group g: plane 16g + 4*kq + e, tile entry j; fixed-order sum over the four wavefronts
        __syncthreads();
        float *red = reinterpret_cast<float *>(&slab_all[0][0]);      // 4 x (64 x 16) floats fit in the slabs
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e) red[wave * 1024 + (16 * g + 4 * kq + e) * 16 + j] = oacc[g][e];
        __syncthreads();
        for (int i = threadIdx.x; i < r * 16; i += 256)
            part[(size_t)blockIdx.x * r * 16 + i] = ((red[i] + red[1024 + i]) + red[2048 + i]) + red[3072 + i];
    }
}

// ---------------------------------------------------------------------------------------
// Images whose row count the tile size does not divide (Class-1 appendix, "More Details on STL Replacement in
// T2T-ViT", item 1): the nrho = rows mod 4 real rows of an image's last tile row are linear combinations of the 4
// padded output rows, out[rho] = sum_a fold[rho][a] y[a].  Since y[a][c] = sum_p Dm[p][4a+c] yhat[p], the fold is a
// decode with the composed decoder
//     Dp[p][4 rho + c] = sum_a fold[rho][a] Dm[p][4a + c]      (zero for rho >= nrho),
// and its adjoint an encode with the same Dp.  Dp is kept in fp32.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void fold_decoder_kernel(const T *__restrict__ Dm, const float *__restrict__ fold,
                                                           float *__restrict__ Dp, int r, int nrho)
{
    for (int i = threadIdx.x; i < r * 16; i += 256) {
        const int p = i >> 4, rho = (i >> 2) & 3, c = i & 3;
        float s = 0.f;
        if (rho < nrho)
#pragma unroll
            for (int a = 0; a < 4; ++a) s = fmaf(fold[rho * 4 + a], Elem<T>::ld(Dm + p * 16 + 4 * a + c), s);
        Dp[i] = s;
    }
}

// Gt[p][4 rho + c] = sum over the images' last tile rows of Yhat[p] * dC[rho][c] (rows rho >= nrho are zero) gives both
//     dD[p][4a + c]  += sum_rho fold[rho][a] Gt[p][4 rho + c]        (added to the part from the complete tile rows)
//     dfold[rho][a] (+)= sum_{p,c} Dm[p][4a + c] Gt[p][4 rho + c]    (fixed summation order)
template <typename T>
__global__ __launch_bounds__(256) void fold_grads_kernel(const float *__restrict__ Gt, const T *__restrict__ Dm,
                                                         const float *__restrict__ fold, float *__restrict__ dD,
                                                         float *__restrict__ dfold, int r, int nrho, int accumulate)
{
    if (dD)
        for (int i = threadIdx.x; i < r * 16; i += 256) {
            const int p = i >> 4, a = (i >> 2) & 3, c = i & 3;
            float s = 0.f;
            for (int rho = 0; rho < nrho; ++rho) s = fmaf(fold[rho * 4 + a], Gt[p * 16 + 4 * rho + c], s);
            dD[i] += s;
        }
    if (dfold && threadIdx.x < nrho * 4) {
        const int rho = threadIdx.x >> 2, a = threadIdx.x & 3;
        float s = 0.f;
        for (int p = 0; p < r; ++p)
#pragma unroll
            for (int c = 0; c < 4; ++c) s = fmaf(Elem<T>::ld(Dm + p * 16 + 4 * a + c), Gt[p * 16 + 4 * rho + c], s);
        dfold[threadIdx.x] = accumulate ? dfold[threadIdx.x] + s : s;
    }
}

hipError_t launch_fold_decoder(int dtype, const void *Dm, const float *fold, float *Dp, int r, int nrho, hipStream_t s)
{
    if (dtype == 0) hipLaunchKernelGGL(fold_decoder_kernel<float>, dim3(1), dim3(256), 0, s, (const float *)Dm, fold, Dp, r, nrho);
    else hipLaunchKernelGGL(fold_decoder_kernel<bf16_t>, dim3(1), dim3(256), 0, s, (const bf16_t *)Dm, fold, Dp, r, nrho);
    return hipGetLastError();
}

hipError_t launch_fold_grads(int dtype, const float *Gt, const void *Dm, const float *fold, float *dD, float *dfold, int r,
                             int nrho, int accumulate, hipStream_t s)
{
    if (dtype == 0)
        hipLaunchKernelGGL(fold_grads_kernel<float>, dim3(1), dim3(256), 0, s, Gt, (const float *)Dm, fold, dD, dfold, r, nrho,
                           accumulate);
    else
        hipLaunchKernelGGL(fold_grads_kernel<bf16_t>, dim3(1), dim3(256), 0, s, Gt, (const bf16_t *)Dm, fold, dD, dfold, r, nrho,
                           accumulate);
    return hipGetLastError();
}

// out[p][4a + b] (+)= in[p][4b + a]: vec of a transposed tile.  An encoder for B^T given as tiles of B, and the way back
// for its gradient (the map is its own inverse).
template <typename TI, typename TO>
__global__ __launch_bounds__(256) void transpose_basis_kernel(const TI *__restrict__ in, TO *__restrict__ out, int r, int accumulate)
{
    for (int i = threadIdx.x; i < r * 16; i += 256) {
        const int p = i >> 4, a = (i >> 2) & 3, b = i & 3;
        const float v = Elem<TI>::ld(in + p * 16 + 4 * b + a);
        Elem<TO>::st(out + i, accumulate ? Elem<TO>::ld(out + i) + v : v);
    }
}

hipError_t launch_transpose_basis(int dtype, const void *E, void *Et, int r, hipStream_t s)
{
    if (dtype == 0) hipLaunchKernelGGL((transpose_basis_kernel<float, float>), dim3(1), dim3(256), 0, s, (const float *)E, (float *)Et, r, 0);
    else hipLaunchKernelGGL((transpose_basis_kernel<bf16_t, bf16_t>), dim3(1), dim3(256), 0, s, (const bf16_t *)E, (bf16_t *)Et, r, 0);
    return hipGetLastError();
}

hipError_t launch_transpose_basis_grad(const float *Gt, float *G, int r, int accumulate, hipStream_t s)
{
    hipLaunchKernelGGL((transpose_basis_kernel<float, float>), dim3(1), dim3(256), 0, s, Gt, G, r, accumulate);
    return hipGetLastError();
}

// fp32 -> bf16 (round to nearest even), 8 elements per thread; n8 = number of 8-element groups, tail handled per element
__global__ __launch_bounds__(256) void cast_bf16_kernel(const float *__restrict__ in, bf16_t *__restrict__ out, size_t n)
{
    const size_t n8 = n / 8;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
        const f32x4_t a = reinterpret_cast<const f32x4_t *>(in)[2 * i], b = reinterpret_cast<const f32x4_t *>(in)[2 * i + 1];
        reinterpret_cast<u32x4_t *>(out)[i] = u32x4_t{pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(b[0], b[1]),
                                                      pack_bf16x2(b[2], b[3])};
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 7)) out[n8 * 8 + threadIdx.x] = f32_to_bf16(in[n8 * 8 + threadIdx.x]);
}

// ---------------------------------------------------------------------------------------
// host launchers
// ---------------------------------------------------------------------------------------
hipError_t launch_cast_bf16(const float *in, void *out, size_t n, hipStream_t s)
{
    size_t blocks = (n / 8 + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(cast_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, s, in, (bf16_t *)out, n);
    return hipGetLastError();
}

template <typename T, typename TB>
static hipError_t launch_encode_t(const void *A, const void *E, void *P, int Rs, int Cc, int r, int pg, const RowMap &rm,
                                  hipStream_t s)
{
    dim3 block(64, 4), grid((Cc + 63) / 64, (Rs + 3) / 4 > 32768 ? 32768 : (Rs + 3) / 4);   // the kernel strides over the rows
    hipLaunchKernelGGL((encode_kernel<T, TB>), grid, block, 0, s, (const T *)A, (const TB *)E, (T *)P, Rs, Cc, r, pg, rm);
    return hipGetLastError();
}

hipError_t launch_encode(int dtype, const void *A, const void *E, void *P, int R, int Cc, int r, int pg, hipStream_t s,
                         RowMap rm, bool basis_f32)
{
    if (pg <= 0) pg = R;
    const int Rs = rm.count(R);                             // tile rows this launch walks over
    if (Rs <= 0) return hipSuccess;
    if (dtype == 1 && (Cc % 8) == 0 && !basis_f32) return launch_encode_lines(A, E, P, R, Cc, r, pg, s, rm);
    if (dtype == 1 && (Cc % 4) == 0 && !basis_f32) {
        const int chunks = (Cc + 127) / 128;
        const long items = (long)Rs * chunks;
        hipLaunchKernelGGL(encode_mfma_kernel, dim3((unsigned)((items + 3) / 4)), dim3(256), 0, s, (const bf16_t *)A,
                           (const bf16_t *)E, (bf16_t *)P, Rs, Cc, r, chunks, pg, rm);
        return hipGetLastError();
    }
    if (dtype == 0) return launch_encode_t<float, float>(A, E, P, Rs, Cc, r, pg, rm, s);
    return basis_f32 ? launch_encode_t<bf16_t, float>(A, E, P, Rs, Cc, r, pg, rm, s)
                     : launch_encode_t<bf16_t, bf16_t>(A, E, P, Rs, Cc, r, pg, rm, s);
}

template <typename T, typename TB>
static hipError_t launch_decode_t(const void *P, const void *Dm, void *Cmat, int Rs, int Cc, int r, bool gelu, int pg,
                                  const RowMap &rm, hipStream_t s)
{
    dim3 block(64, 4), grid((Cc + 63) / 64, (Rs + 3) / 4 > 32768 ? 32768 : (Rs + 3) / 4);   // the kernel strides over the rows
    if (gelu)
        hipLaunchKernelGGL((decode_kernel<T, TB, true>), grid, block, 0, s, (const T *)P, (const TB *)Dm, (T *)Cmat, Rs, Cc, r,
                           pg, rm);
    else
        hipLaunchKernelGGL((decode_kernel<T, TB, false>), grid, block, 0, s, (const T *)P, (const TB *)Dm, (T *)Cmat, Rs, Cc, r,
                           pg, rm);
    return hipGetLastError();
}

hipError_t launch_decode(int dtype, const void *P, const void *Dm, void *Cmat, int R_all, int Cc, int r, bool gelu, int pg,
                         hipStream_t s, RowMap rm, bool basis_f32)
{
    if (pg <= 0) pg = R_all;
    const int R = rm.count(R_all);                          // tile rows this launch walks over
    if (R <= 0) return hipSuccess;
    if (dtype == 1 && (Cc % 8) == 0 && !basis_f32) {
        const int chunks = (Cc + 63) / 64;
        const long items = (long)R * chunks;
        long blocks = (items + 3) / 4;
        if (blocks > 8192) blocks = 8192;                   // grid-stride over (tile row, 64-tile chunk) items
        const dim3 grid((unsigned)blocks), block(256);
        const bf16_t *p = (const bf16_t *)P, *d = (const bf16_t *)Dm;
        bf16_t *c = (bf16_t *)Cmat;
        if (r <= 32) {
            if (gelu) hipLaunchKernelGGL((decode_mfma_kernel<true, 1, false>), grid, block, 0, s, p, d, c, R, Cc, r, chunks, nullptr, nullptr, pg, rm);
            else hipLaunchKernelGGL((decode_mfma_kernel<false, 1, false>), grid, block, 0, s, p, d, c, R, Cc, r, chunks, nullptr, nullptr, pg, rm);
        } else {
            if (gelu) hipLaunchKernelGGL((decode_mfma_kernel<true, 2, false>), grid, block, 0, s, p, d, c, R, Cc, r, chunks, nullptr, nullptr, pg, rm);
            else hipLaunchKernelGGL((decode_mfma_kernel<false, 2, false>), grid, block, 0, s, p, d, c, R, Cc, r, chunks, nullptr, nullptr, pg, rm);
        }
        return hipGetLastError();
    }
    if (dtype == 0) return launch_decode_t<float, float>(P, Dm, Cmat, R, Cc, r, gelu, pg, rm, s);
    return basis_f32 ? launch_decode_t<bf16_t, float>(P, Dm, Cmat, R, Cc, r, gelu, pg, rm, s)
                     : launch_decode_t<bf16_t, bf16_t>(P, Dm, Cmat, R, Cc, r, gelu, pg, rm, s);
}

hipError_t launch_outer_final(const float *part, float *G, int nb, int n_out, int accumulate, hipStream_t s)
{
    hipLaunchKernelGGL(outer_final_kernel, dim3((n_out + 15) / 16), dim3(1024), 0, s, part, G, nb, n_out, accumulate,
                       (const float *)nullptr, (float *)nullptr, 0);
    return hipGetLastError();
}

hipError_t launch_outer_final_pair(const float *part0, float *G0, int nb0, const float *part1, float *G1, int nb1, int n_out,
                                   int accumulate, hipStream_t s)
{
    hipLaunchKernelGGL(outer_final_kernel, dim3((n_out + 15) / 16, 2), dim3(1024), 0, s, part0, G0, nb0, n_out, accumulate, part1,
                       G1, nb1);
    return hipGetLastError();
}

bool decode_outer_eligible(int dtype, int Cc) { return dtype == 1 && (Cc % 8) == 0; }

int decode_outer_blocks(int R, int Cc)
{
    const long items = (long)R * ((Cc + 63) / 64);
    const long blocks = (items + 3) / 4;
    return (int)(blocks > 1024 ? 1024 : blocks);
}

hipError_t launch_decode_outer(const void *P, const void *Dm, void *Cmat, const void *V, float *G, float *part, int R_all,
                               int Cc, int r, int accumulate, int pg, hipStream_t s, RowMap rm, bool final_sum)
{
    if (pg <= 0) pg = R_all;
    const int R = rm.count(R_all);
    if (R <= 0) return hipErrorInvalidValue;
    const int chunks = (Cc + 63) / 64;
    const int nb = decode_outer_blocks(R, Cc);
    const bf16_t *p = (const bf16_t *)P, *d = (const bf16_t *)Dm, *v = (const bf16_t *)V;
    bf16_t *c = (bf16_t *)Cmat;
    if (r <= 32)
        hipLaunchKernelGGL((decode_mfma_kernel<false, 1, true>), dim3(nb), dim3(256), 0, s, p, d, c, R, Cc, r, chunks, v, part, pg, rm);
    else
        hipLaunchKernelGGL((decode_mfma_kernel<false, 2, true>), dim3(nb), dim3(256), 0, s, p, d, c, R, Cc, r, chunks, v, part, pg, rm);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !final_sum) return e;
    const int n_out = r * 16;
    return launch_outer_final(part, G, nb, n_out, accumulate, s);
}

static int outer_tiles_per_block(int64_t tiles)
{
    // at most 512 partials; blocks take whole 256-tile steps (4 wavefronts x 64 tiles)
    int64_t tpb = (tiles + 511) / 512;
    tpb = (tpb + 255) / 256 * 256;
    return (int)(tpb < 256 ? 256 : tpb);
}

int outer_reduce_blocks(int64_t tiles)
{
    const int tpb = outer_tiles_per_block(tiles);
    return (int)((tiles + tpb - 1) / tpb);
}

hipError_t launch_outer_reduce(int dtype, const void *P, const void *V, float *G, float *part, int R_all, int Cc, int r,
                               int accumulate, int pg, hipStream_t s, RowMap rm)
{
    if (pg <= 0) pg = R_all;
    const int R = rm.count(R_all);
    if (R <= 0) return hipErrorInvalidValue;
    const int64_t tiles = (int64_t)R * Cc;
    const int tpb = outer_tiles_per_block(tiles);
    const int nb = outer_reduce_blocks(tiles);
    if (dtype == 0)
        hipLaunchKernelGGL(outer_partial_kernel<float>, dim3(nb), dim3(256), 0, s, (const float *)P, (const float *)V,
                           part, R, Cc, r, tpb, pg, rm);
    else if (Cc % 8 == 0)
        hipLaunchKernelGGL(outer_mfma_kernel, dim3(nb), dim3(256), 0, s, (const bf16_t *)P, (const bf16_t *)V, part, R,
                           Cc, r, tpb, pg, rm);
    else
        hipLaunchKernelGGL(outer_partial_kernel<bf16_t>, dim3(nb), dim3(256), 0, s, (const bf16_t *)P,
                           (const bf16_t *)V, part, R, Cc, r, tpb, pg, rm);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int n_out = r * 16;
    return launch_outer_final(part, G, nb, n_out, accumulate, s);
}

}  // namespace stl
