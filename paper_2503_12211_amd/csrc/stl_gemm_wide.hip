// Pipelined plane products whose first operand is stored [row][l] (the forward products Yhat[p] = Xhat[p] What[p] and
// the input-gradient products dXhat[p] = dYhat[p] What[p]^T), with that operand fetched as whole 128-byte lines.
//
// Same kernel as gemm_pipe_kernel in every other respect (256 x 256 block, eight wavefronts of 128 x 64, 32x32x16
// MFMA, persistent block list, next block's first loads in flight during the epilogue, wavefront-private epilogue
// slab), and the same products in the same order: results are bit-identical.  What differs is the path of the first
// operand into LDS (SrcWide / FragWide in stl_gemm_pipe.h): slots of 64 contraction elements that serve two stages
// each, filled half a slot per stage, three slots deep; the second operand keeps its ring of four 32-element stages.
// LDS: 3 x 32 KB + 4 x 16 KB = the whole 160 KB; the epilogue slabs lie in the third slot of the first operand,
// which is idle from the last stage of a block until the first stage of the next one has passed its barrier.
#include "stl_gemm_pipe.h"

namespace stl {

// B_T: second operand stored [l][j]; otherwise [j][l] (32-element stages, half lines, as in gemm_pipe_kernel).
// Requires Kl % 64 == 0.  One problem per launch (no stacking).
template <bool B_T>
__global__ __launch_bounds__(512) void gemm_pipe_wide_kernel(const bf16_t *__restrict__ A, const bf16_t *__restrict__ B,
                                                             bf16_t *__restrict__ Out, int Mi, int Nj, int Kl, int tiles_m,
                                                             int tiles_n, int total, int a_pg, int b_pg, int o_pg, int batch)
{
    using namespace pipe;
    constexpr int BM = 256, BN = 256, NW = 8, WAVES_N = 4, WM = 128, WN = 64, FM = 4, FN = 2, SWZ = 2, NSB = 4;
    constexpr int A_SLOT = BM * 128, B_STAGE = BN * BKS * 2, B_BASE = 3 * A_SLOT;
    constexpr int RP = 16, PITCH = WN * 2 + 16, SLAB = RP * PITCH;
    static_assert(B_BASE + NSB * B_STAGE == 160 * 1024 && NW * SLAB <= A_SLOT, "LDS map");
    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: LDS-DMA destinations stay in SGPRs
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    char *slab = smem + 2 * A_SLOT + wave * SLAB;
    const int per_plane = tiles_m * tiles_n;
    const int nks = Kl / BKS;                          // even
    const uint32_t smem_lds = (uint32_t)(uintptr_t)STL_LDS(smem);

    FragWide<BM> fa;
    Frag<B_T, SWZ, BN> fb;
    fa.init(wm * WM, lane);
    fb.init(wn * WN, lane);

    auto locate = [&](int v, int &p, int &i0, int &j0) {
        int lid = v;
        if ((total & 7) == 0 && (gridDim.x & 7) == 0) lid = (v & 7) * (total >> 3) + (v >> 3);
        p = lid / per_plane;
        const int rem = lid - p * per_plane;
        i0 = (rem / tiles_n) * BM;
        j0 = (rem % tiles_n) * BN;
    };

    SrcWide<BM, NW> sa;
    Src<B_T, SWZ, BN, NW> sb;
    // LDS addresses: first-operand slot of pair j, second-operand stage s
    auto a_slot = [&](int pair) { return (pair % 3) * A_SLOT; };
    auto b_slot = [&](int s) { return B_BASE + (s % NSB) * B_STAGE; };
    // Issue order of a block, per wavefront (H = half slot of the first operand, numbered 2 * pair + half; B = stage of
    // the second): H0 B0 H1 B1 H2 B2 H3 before the loop, then H(s+4) B(s+3) in iteration s -- four instructions per
    // iteration as long as both exist.
    auto start_block = [&](int v) {
        int p, i0, j0;
        locate(v, p, i0, j0);
        sa.init(A, Kl, i0, Mi, wave, lane, p, batch, a_pg, 0);
        sb.init(B, B_T ? Nj : Kl, j0, Nj, wave, lane, p, batch, b_pg, 0);
        sa.template issue_half<0>(smem_lds + a_slot(0), wave);
        sb.issue(smem_lds + b_slot(0), wave);
        sa.template issue_half<1>(smem_lds + a_slot(0), wave);
        sb.issue(smem_lds + b_slot(1), wave);
        if (nks > 2) {
            sa.template issue_half<0>(smem_lds + a_slot(1), wave);
            sb.issue(smem_lds + b_slot(2), wave);
            sa.template issue_half<1>(smem_lds + a_slot(1), wave);
        }
    };

    int v = blockIdx.x;
    if (v < total) start_block(v);

    for (; v < total; v += gridDim.x) {
        int p, i0, j0;
        locate(v, p, i0, j0);

        f32x16_t acc[FM][FN];
#pragma unroll
        for (int a = 0; a < FM; ++a)
#pragma unroll
            for (int b = 0; b < FN; ++b)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

        // Loads complete in the order they were issued.  Before the first fragments are read H0, B0, H1 must have
        // landed: everything but the last eight instructions (B1 H2 B2 H3) when the contraction has more than one
        // pair, everything but B1 otherwise.  (Stores of the previous epilogue may still be in flight: "at most N
        // outstanding" then over-waits, never under-waits.)
        if (nks > 2) wait_vmcnt<8>();
        else wait_vmcnt<2>();
        block_barrier();

        bf16x8_t va[2][FM], vb[2][FN];      // fragment double buffer: [k16-step parity]
#pragma unroll
        for (int a = 0; a < FM; ++a) va[0][a] = fa.read(smem + a_slot(0), a, 0, 0);
#pragma unroll
        for (int b = 0; b < FN; ++b) vb[0][b] = fb.read(smem + b_slot(0), b, 0);

        // One stage s = 2 * pair + SP (two k16-steps).  RA: half slot s + 4 of the first operand is fetched; RB: stage
        // s + 3 of the second.  At the top of iteration s everything issued up to iteration s - 2 must have landed
        // (stage s + 1 of both operands); what iteration s - 1 issued may still be in flight: WAIT instructions.
        auto stage = [&](int s, auto sp_c, auto ra_c, auto rb_c, auto wait_c) {
            constexpr int SP = decltype(sp_c)::value, WAIT = decltype(wait_c)::value;
            constexpr bool RA = decltype(ra_c)::value, RB = decltype(rb_c)::value;
            if constexpr (WAIT >= 0) wait_vmcnt<WAIT>();
            block_barrier();   // stage s+1 visible to all; nobody reads stage s-1 any more
            const int pair = s >> 1;
            const uint32_t dst_a = smem_lds + a_slot(pair + 2), dst_b = smem_lds + b_slot(s + NSB - 1);
            const char *cur_a = smem + a_slot(pair), *nxt_a = smem + a_slot(pair + SP);
            const char *nxt_b = smem + b_slot(s + 1), *cur_b = smem + b_slot(s);
            auto step = [&](auto par_c, const char *src_a, int sp_src, const char *src_b, int ks, auto a_side_c) {
                constexpr int par = decltype(par_c)::value;
                constexpr bool a_side = decltype(a_side_c)::value;
                static_for<0, FM * FN>([&](auto i_c) {
                    constexpr int i = decltype(i_c)::value, a = i / FN, b = i % FN;
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vb[par][b], va[par][a], acc[a][b], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    // one fragment fetch per MFMA slot, in the order the next step consumes them: B0, A0, B1, A1, A2, A3
                    if constexpr (i < FM + FN) {
                        if constexpr (i < 2 * FN) {
                            if constexpr ((i % 2) == 0) vb[par ^ 1][i / 2] = fb.read(src_b, i / 2, ks);
                            else va[par ^ 1][i / 2] = fa.read(src_a, i / 2, ks, sp_src);
                        } else {
                            va[par ^ 1][i - FN] = fa.read(src_a, i - FN, ks, sp_src);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if constexpr (i >= 2 && (i % 2) == 0) {
                        constexpr int j = (i - 2) / 2;       // DMA slot inside this step
                        if constexpr (a_side) {
                            if constexpr (RA && j < decltype(sa)::NI) sa.template issue_one<SP>(dst_a, wave, j);
                        } else {
                            if constexpr (RB && j < decltype(sb)::NI) sb.issue_one(dst_b, wave, j);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                });
            };
            // step 0 (fetch k16-step 1 of stage s; refill the first operand), step 1 (fetch k16-step 0 of stage s+1;
            // refill the second operand).  Stage s+1 lies in the same slot of the first operand when s is even.
            step(std::integral_constant<int, 0>{}, cur_a, SP, cur_b, 1, std::true_type{});
            step(std::integral_constant<int, 1>{}, nxt_a, SP ^ 1, nxt_b, 0, std::false_type{});
            if constexpr (RA) sa.template next_pair<SP>();
            if constexpr (RB) sb.next_stage();
        };
        using T_ = std::true_type;
        using F_ = std::false_type;
        using I0 = std::integral_constant<int, 0>;
        using I1 = std::integral_constant<int, 1>;
        using W4 = std::integral_constant<int, 4>;
        using W2 = std::integral_constant<int, 2>;
        using W0 = std::integral_constant<int, 0>;
        using WN_ = std::integral_constant<int, -1>;
        // stages s <= nks - 5 fetch both operands; s = nks - 4 (even) only the second; the last three nothing
        int s = 0;
        for (; s + 5 < nks; s += 2) {            // both stages of the pair at most nks - 5
            stage(s, I0{}, T_{}, T_{}, W4{});
            stage(s + 1, I1{}, T_{}, T_{}, W4{});
        }
        if (nks >= 4) {                          // s = nks - 4, nks - 3
            stage(s, I0{}, F_{}, T_{}, W4{});
            stage(s + 1, I1{}, F_{}, F_{}, W2{});
            s += 2;
        }
        stage(s, I0{}, F_{}, F_{}, W0{});        // s = nks - 2, nks - 1
        stage(s + 1, I1{}, F_{}, F_{}, WN_{});

        // every wavefront is done with the ring: refill it for the next block before storing this one
        block_barrier();
        if (v + (int)gridDim.x < total) start_block(v + gridDim.x);

        // Epilogue, as in gemm_pipe_kernel: accumulator e of fragment (a, b) is
        //   Out[row = 32a + lane%32][column = 32b + 8*(e/4) + 4*(lane/32) + e%4]
        bf16_t *outp = Out + (size_t)p * o_pg * Nj;
        const int frow = lane & 31, fhalf = lane >> 5;
        constexpr int LPR = WN * 2 / 16, RPI = 64 / LPR;
        static_for<0, FM>([&](auto a_c) {
            constexpr int a = decltype(a_c)::value;
            static_for<0, 32 / RP>([&](auto pass_c) {
                constexpr int pass = decltype(pass_c)::value;
                if ((frow / RP) == pass) {
                    char *rowp = slab + (frow % RP) * PITCH;
#pragma unroll
                    for (int b = 0; b < FN; ++b)
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const int cc = b * 32 + 8 * g + 4 * fhalf;
                            const u32x2_t w = {pack_bf16x2(acc[a][b][4 * g], acc[a][b][4 * g + 1]),
                                               pack_bf16x2(acc[a][b][4 * g + 2], acc[a][b][4 * g + 3])};
                            *reinterpret_cast<u32x2_t *>(rowp + cc * 2) = w;
                        }
                }
                asm volatile("" ::: "memory");
                const int gi_base = i0 + wm * WM + a * 32 + pass * RP;
                const size_t row_off = plane_row_base(gi_base < Mi ? gi_base : 0, o_pg, batch, Nj);
                const int gj = j0 + wn * WN + (lane % LPR) * 8;
#pragma unroll
                for (int it = 0; it < RP / RPI; ++it) {
                    const int rr = it * RPI + lane / LPR;
                    const int gi = gi_base + rr;
                    const u32x4_t w = *reinterpret_cast<const u32x4_t *>(slab + rr * PITCH + (lane % LPR) * 16);
                    if (gi < Mi && gj < Nj) *reinterpret_cast<u32x4_t *>(outp + row_off + (size_t)rr * Nj + gj) = w;
                }
                asm volatile("" ::: "memory");
            });
        });
    }
}

bool plane_gemm_wide_eligible(const GemmDesc &g)
{
    return plane_gemm_pipe_eligible(g) && !g.a_kmajor && !g.out_f32 && !g.accumulate && g.nb == 1 && g.Kl % 64 == 0;
}

static int wide_cu_count()
{
    static const int n = []() {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 256;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
        return cus;
    }();
    return n;
}

template <bool B_T>
static hipError_t launch_wide(const GemmDesc &g, const void *A, const void *B, void *Out, hipStream_t s)
{
    auto kern = gemm_pipe_wide_kernel<B_T>;
    constexpr int smem = 160 * 1024;
    static const hipError_t attr_err =
        hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (attr_err != hipSuccess) return attr_err;
    const int tiles_m = (g.Mi + 255) / 256, tiles_n = (g.Nj + 255) / 256;
    const long total = (long)tiles_m * tiles_n * g.batch;
    if (total > 0x7fffffffL) return hipErrorInvalidValue;
    const int cus = wide_cu_count();
    const unsigned grid = (unsigned)(total > cus ? cus : total);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(512), smem, s, (const bf16_t *)A, (const bf16_t *)B, (bf16_t *)Out, g.Mi, g.Nj, g.Kl,
                       tiles_m, tiles_n, (int)total, g.a_rows_per_group(), g.b_rows_per_group(), g.o_rows_per_group(), g.batch);
    return hipGetLastError();
}

hipError_t launch_plane_gemm_wide(const GemmDesc &g, const void *A, const void *B, void *Out, hipStream_t s)
{
    if (!plane_gemm_wide_eligible(g)) return hipErrorInvalidValue;
    return g.b_kmajor ? launch_wide<true>(g, A, B, Out, s) : launch_wide<false>(g, A, B, Out, s);
}

}  // namespace stl
