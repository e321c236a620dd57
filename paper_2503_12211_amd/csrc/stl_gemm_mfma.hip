// Batched plane products on the CDNA4 matrix cores (step (ii) of Algorithm 1, Claim 3.4):
//     Out[p][i][j] (+)= sum_l A[p](i,l) * B[p](l,j)       bf16 x bf16 -> fp32, p < r planes.
//
// One workgroup owns a BM x BN block of one plane.  Both operands are staged in LDS in
// "row x 64 k-values" form (k contiguous), double buffered, 16-byte chunks XOR-swizzled so
// that fragment reads (ds_read_b128, 32 rows x 2 k-halves per wavefront) and staging writes
// spread over all banks.  An operand whose contiguous memory dimension is not the contraction
// index is transposed in registers on its way from HBM to LDS, so the MFMA loop is the same
// for the forward product and the two backward products.
// Wavefronts compute 32x32x16 MFMA fragments; accumulators stay in registers for the whole
// contraction.  Block ids are remapped so that consecutive blocks of one plane land on the
// same XCD (and share its L2).
#include "stl_kernels.h"
#include "stl_device.h"


namespace stl {

constexpr int BK = 64;  // contraction elements per LDS stage (one 128-byte LDS row)

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }

// byte offset of the 16-byte chunk c (0..7) of `row` inside one staged operand
__device__ __forceinline__ int lds_off(int row, int c) { return row * (BK * 2) + ((c ^ swz(row)) << 4); }

// where storage row `row` of plane p of an operand begins (rows in groups of pg, see plane_row_base)
struct Lay {
    int pg, batch, p;
    long ld;
    int row0;   // first stored row of this problem inside the stacked operand
    __device__ __forceinline__ size_t off(int row) const
    {
        return plane_row_base(row0 + row, pg, batch, (int)ld) + (size_t)p * pg * ld;
    }
};

// ---- HBM -> registers ------------------------------------------------------------------
// Direct operand: stored [row][l], l contiguous (leading dimension ld elements).
template <int ROWS, int NT>
struct DirectLoader {
    static constexpr int CH = ROWS * 8 / NT;  // 16-byte chunks per thread
    u32x4_t v[CH];
    __device__ __forceinline__ void load(const bf16_t *__restrict__ base, const Lay &lay, int row0, int rows_total, int k0,
                                         int Kl, int tid)
    {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int id = tid + j * NT, row = id >> 3, c = id & 7;
            const int gr = row0 + row, gk = k0 + c * 8;
            u32x4_t z = {0u, 0u, 0u, 0u};
            if (gr < rows_total && gk < Kl) z = *reinterpret_cast<const u32x4_t *>(base + lay.off(gr) + gk);
            v[j] = z;
        }
    }
    __device__ __forceinline__ void store(char *lds, int tid) const
    {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int id = tid + j * NT, row = id >> 3, c = id & 7;
            *reinterpret_cast<u32x4_t *>(lds + lds_off(row, c)) = v[j];
        }
    }
};

// Transposing operand: stored [l][row], row contiguous (leading dimension ld elements).
// A thread takes units of 4 l-values x 8 rows, swaps them in registers and writes 8 bytes
// (4 consecutive k) to each of 8 LDS rows.
template <int ROWS, int NT>
struct TransLoader {
    static constexpr int RG = ROWS / 8;                // row groups
    static constexpr int UNITS = (BK / 4) * RG / NT;   // units per thread
    u32x4_t v[UNITS][4];
    __device__ __forceinline__ void load(const bf16_t *__restrict__ base, const Lay &lay, int row0, int rows_total, int k0,
                                         int Kl, int tid)
    {
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            const int id = tid + u * NT, rg = id % RG, kq = id / RG;
            const int gr = row0 + rg * 8;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int gk = k0 + kq * 4 + kk;
                u32x4_t z = {0u, 0u, 0u, 0u};
                if (gr < rows_total && gk < Kl) z = *reinterpret_cast<const u32x4_t *>(base + lay.off(gk) + gr);
                v[u][kk] = z;
            }
        }
    }
    __device__ __forceinline__ void store(char *lds, int tid) const
    {
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            const int id = tid + u * NT, rg = id % RG, kq = id / RG;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                // element j of each of the four l-rows -> 4 consecutive k of LDS row rg*8+j
                const int d = j >> 1, sh = (j & 1) * 16;
                const uint32_t e0 = (v[u][0][d] >> sh) & 0xffffu, e1 = (v[u][1][d] >> sh) & 0xffffu;
                const uint32_t e2 = (v[u][2][d] >> sh) & 0xffffu, e3 = (v[u][3][d] >> sh) & 0xffffu;
                u32x2_t w = {e0 | (e1 << 16), e2 | (e3 << 16)};
                const int row = rg * 8 + j;
                *reinterpret_cast<u32x2_t *>(lds + lds_off(row, kq >> 1) + (kq & 1) * 8) = w;
            }
        }
    }
};

template <bool KMAJOR, int ROWS, int NT>
struct LoaderSel { typedef DirectLoader<ROWS, NT> type; };
template <int ROWS, int NT>
struct LoaderSel<true, ROWS, NT> { typedef TransLoader<ROWS, NT> type; };

// ---- kernel ----------------------------------------------------------------------------
// A_T: A stored [l][i];  B_T: B stored [l][j].  (false: stored [i][l] resp. [j][l].)
template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_T, bool B_T, typename TO, bool ACC>
__global__ __launch_bounds__(WAVES_M *WAVES_N * 64) void gemm_mfma_kernel(const bf16_t *__restrict__ A,
                                                                          const bf16_t *__restrict__ B,
                                                                          TO *__restrict__ Out, int Mi, int Nj, int Kl,
                                                                          int tiles_m, int tiles_n, int total, int a_pg,
                                                                          int b_pg, int o_pg, int batch)
{
    constexpr int NT = WAVES_M * WAVES_N * 64;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;
    extern __shared__ __align__(16) char smem[];

    // XCD-aware block order: hardware deals consecutive block ids round-robin to the 8 XCDs
    int bid = blockIdx.x;
    if ((total & 7) == 0) bid = (bid & 7) * (total >> 3) + (bid >> 3);
    const int per_plane = tiles_m * tiles_n;
    const int q = bid / per_plane;                    // (stacked problem, plane)
    const int rem = bid - q * per_plane;
    const int i0 = (rem / tiles_n) * BM, j0 = (rem % tiles_n) * BN;
    const int pb = q / batch, p = q - pb * batch;

    const Lay lda{a_pg, batch, p, A_T ? Mi : Kl, pb * (A_T ? Kl : Mi)}, ldb{b_pg, batch, p, B_T ? Nj : Kl, pb * (B_T ? Kl : Nj)},
        ldo{o_pg, batch, p, Nj, pb * Mi};

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    typename LoaderSel<A_T, BM, NT>::type la;
    typename LoaderSel<B_T, BN, NT>::type lb;

    f32x16_t acc[FM][FN];
#pragma unroll
    for (int a = 0; a < FM; ++a)
#pragma unroll
        for (int b = 0; b < FN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    const int nk = (Kl + BK - 1) / BK;
    la.load(A, lda, i0, Mi, 0, Kl, tid);
    lb.load(B, ldb, j0, Nj, 0, Kl, tid);
    la.store(smem, tid);
    lb.store(smem + A_BYTES, tid);
    __syncthreads();

    const int frow = lane & 31, fhalf = lane >> 5;
    for (int kt = 0; kt < nk; ++kt) {
        char *cur = smem + (kt & 1) * STAGE;
        char *nxt = smem + ((kt + 1) & 1) * STAGE;
        const bool more = kt + 1 < nk;
        if (more) {
            la.load(A, lda, i0, Mi, (kt + 1) * BK, Kl, tid);
            lb.load(B, ldb, j0, Nj, (kt + 1) * BK, Kl, tid);
        }
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8_t fa[FM], fb[FN];
#pragma unroll
            for (int a = 0; a < FM; ++a)
                fa[a] = *reinterpret_cast<const bf16x8_t *>(cur + lds_off(wm * WM + a * 32 + frow, ks * 2 + fhalf));
#pragma unroll
            for (int b = 0; b < FN; ++b)
                fb[b] = *reinterpret_cast<const bf16x8_t *>(cur + A_BYTES +
                                                            lds_off(wn * WN + b * 32 + frow, ks * 2 + fhalf));
#pragma unroll
            for (int a = 0; a < FM; ++a)
#pragma unroll
                for (int b = 0; b < FN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
        }
        if (more) {
            la.store(nxt, tid);
            lb.store(nxt + A_BYTES, tid);
        }
        __syncthreads();
    }

    // Epilogue.  Accumulator layout of a 32x32 fragment: column = lane % 32,
    // row = 8*(v/4) + 4*(lane/32) + v%4.  Each wavefront passes 32 rows x WN columns at a time
    // through its own LDS slab so that HBM sees whole 16-byte, row-contiguous stores.
    constexpr int ES = sizeof(TO);
    constexpr int PITCH = WN * ES + 16;                 // bytes per staged row (+16: spreads rows over banks)
    constexpr int LPR = WN * ES / 16;                   // lanes per row in the store phase
    constexpr int RPI = 64 / LPR;                       // rows per store instruction
    char *slab = smem + wave * (32 * PITCH);
    static_assert(32 * PITCH * WAVES_M * WAVES_N <= 2 * STAGE, "epilogue slab does not fit");
#pragma unroll
    for (int a = 0; a < FM; ++a) {
        __syncthreads();
#pragma unroll
        for (int b = 0; b < FN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int rr = 8 * (v >> 2) + 4 * fhalf + (v & 3), cc = b * 32 + frow;
                Elem<TO>::st(reinterpret_cast<TO *>(slab + rr * PITCH) + cc, acc[a][b][v]);
            }
        __syncthreads();
        const int gi_base = i0 + wm * WM + a * 32;
        const int gj = j0 + wn * WN + (lane % LPR) * (16 / ES);
#pragma unroll
        for (int it = 0; it < 32 / RPI; ++it) {
            const int rr = it * RPI + lane / LPR;
            const int gi = gi_base + rr;
            if (gi < Mi && gj < Nj) {
                u32x4_t w = *reinterpret_cast<const u32x4_t *>(slab + rr * PITCH + (lane % LPR) * 16);
                TO *o = Out + ldo.off(gi) + gj;
                if (ACC) {
                    const f32x4_t old = *reinterpret_cast<const f32x4_t *>(o);
                    f32x4_t nw = __builtin_bit_cast(f32x4_t, w);
                    nw += old;
                    *reinterpret_cast<f32x4_t *>(o) = nw;
                } else {
                    *reinterpret_cast<u32x4_t *>(o) = w;
                }
            }
        }
    }
}

// ---- host side ---------------------------------------------------------------------------
bool plane_gemm_mfma_eligible(const GemmDesc &g)
{
    if (g.Mi < 1 || g.Nj < 1 || g.Kl < 1 || g.batch < 1) return false;
    if (g.accumulate && !g.out_f32) return false;
    // instantiated operand forms: forward [i][l]x[l][j], input gradient [i][l]x[j][l] (storage out),
    // weight gradient [l][i]x[l][j] (fp32 out, or storage out for a run-time encoded second operand)
    if (g.a_kmajor ? !g.b_kmajor : g.out_f32) return false;
    // 16-byte global loads along each operand's contiguous dimension
    if (g.Mi % 8 || g.Nj % 8 || g.Kl % 8) return false;
    return true;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_T, bool B_T, typename TO, bool ACC>
static hipError_t launch_cfg(const GemmDesc &g, const void *A, const void *B, void *Out, hipStream_t s)
{
    auto kern = gemm_mfma_kernel<BM, BN, WAVES_M, WAVES_N, A_T, B_T, TO, ACC>;
    constexpr int smem = 2 * (BM + BN) * BK * 2;
    // once per instantiation (initialisation of a function-local static is thread-safe)
    static const hipError_t attr_err =
        hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (attr_err != hipSuccess) return attr_err;
    const int tiles_m = (g.Mi + BM - 1) / BM, tiles_n = (g.Nj + BN - 1) / BN;
    const long total = (long)tiles_m * tiles_n * g.batch * g.nb;
    if (total > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(WAVES_M * WAVES_N * 64), smem, s, (const bf16_t *)A,
                       (const bf16_t *)B, (TO *)Out, g.Mi, g.Nj, g.Kl, tiles_m, tiles_n, (int)total, g.a_rows_per_group(),
                       g.b_rows_per_group(), g.o_rows_per_group(), g.batch);
    return hipGetLastError();
}

template <bool A_T, bool B_T, typename TO, bool ACC>
static hipError_t launch_shape(const GemmDesc &g, const void *A, const void *B, void *Out, hipStream_t s)
{
    // large planes: 256 x 256 blocks, 8 wavefronts of 128 x 64; small ones: 128 x 128 blocks, 4 wavefronts of 64 x 64
    // (256x256 with 4 wavefronts of 128x128, 256x128 and 128x256 were measured and are not faster at any shape)
    if (g.Mi > 128 && g.Nj > 128) return launch_cfg<256, 256, 2, 4, A_T, B_T, TO, ACC>(g, A, B, Out, s);
    return launch_cfg<128, 128, 2, 2, A_T, B_T, TO, ACC>(g, A, B, Out, s);
}

hipError_t launch_plane_gemm_mfma(const GemmDesc &g, const void *A, const void *B, void *Out, hipStream_t s)
{
    if (g.out_f32) {
        if (g.a_kmajor && g.b_kmajor)
            return g.accumulate ? launch_shape<true, true, float, true>(g, A, B, Out, s)
                                : launch_shape<true, true, float, false>(g, A, B, Out, s);
        return hipErrorInvalidValue;  // only the weight-gradient product stores fp32
    }
    if (g.a_kmajor && g.b_kmajor) return launch_shape<true, true, bf16_t, false>(g, A, B, Out, s);
    if (!g.a_kmajor && g.b_kmajor) return launch_shape<false, true, bf16_t, false>(g, A, B, Out, s);
    if (!g.a_kmajor && !g.b_kmajor) return launch_shape<false, false, bf16_t, false>(g, A, B, Out, s);
    return hipErrorInvalidValue;
}

}  // namespace stl
