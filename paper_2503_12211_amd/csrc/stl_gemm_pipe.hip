// Pipelined batched plane products on the CDNA4 matrix cores (step (ii) of Algorithm 1, Claim 3.4):
//     Out[p][i][j] (+)= sum_l A[p](i,l) * B[p](l,j)       bf16 x bf16 -> fp32, p < r planes.
//
// Same blocking as the register-staged kernel (256 x 256 block of one plane per workgroup, eight
// wavefronts of 128 x 64, 32x32x16 MFMA), but HBM -> LDS goes through the LDS-DMA path
// (global_load_lds, 16 bytes per lane, no VGPR staging) into a ring of NS stages of 32 contraction
// elements each, issued NS-1 stages ahead of their use, so that an L2 / HBM miss has several
// MFMA stages of time to land.  Operands keep their memory orientation in LDS:
//   * contraction-contiguous operand ([row][l]): 64-byte LDS rows, fragments by ds_read_b128;
//   * contraction-major operand ([l][row]):      512-byte LDS rows, fragments by the transposing
//     ds_read_b64_tr_b16 (a 16-lane group turns 4 l-rows x 16 columns into 4 consecutive l per lane).
// An LDS-DMA instruction writes 64 lanes x 16 bytes contiguously, so bank swizzles are applied by
// permuting which global 16-byte chunk each lane fetches.
#include "stl_gemm_pipe.h"

namespace stl {

// A_T: A stored [l][i];  B_T: B stored [l][j].  Requires Kl % 32 == 0, Mi % 8 == 0, Nj % 8 == 0.
//
// Persistent: the grid is one workgroup per CU and every workgroup walks over its share of the
// (plane, block) list.  When a block's MFMA loop ends, the first ring stages of the NEXT block are put in
// flight before the epilogue starts, so the HBM/L2 latency of the refill and the store traffic of the
// epilogue overlap instead of adding up.  The epilogue goes through a wavefront-private LDS slab (no
// workgroup barrier): MFMA operands are passed as (B fragment, A fragment), which leaves every lane
// with 4 consecutive output columns of one row per accumulator quad, i.e. one 8- or 16-byte LDS write.
template <int WAVES_M, int WAVES_N, int NS, int SWZ, bool A_T, bool B_T, typename TO, bool ACC>
__global__ __launch_bounds__(WAVES_M *WAVES_N * 64) void gemm_pipe_kernel(const bf16_t *__restrict__ A, const bf16_t *__restrict__ B,
                                                        TO *__restrict__ Out, int Mi, int Nj, int Kl, int tiles_m,
                                                        int tiles_n, int total, int a_pg, int b_pg, int o_pg, int batch)
{
    using namespace pipe;
    constexpr int BM = 256, BN = 256, NW = WAVES_M * WAVES_N, WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int OPER_BYTES = BM * BKS * 2, STAGE_BYTES = (BM + BN) * BKS * 2;
    constexpr int DMA_PER_STAGE = (BM + BN) / 16 / NW;     // DMA instructions per wavefront and stage
    constexpr int ES = sizeof(TO);
    constexpr int RP = (ES == 2 ? 32 : 16) / (NS == 4 ? 2 : 1) / (WN / 64);   // rows staged per epilogue pass (LDS budget)
    constexpr int PITCH = WN * ES + 16;                     // bytes per staged row
    constexpr int SLAB = RP * PITCH;                        // per wavefront
    static_assert(NS == 3 || NS == 4, "ring depth");
    extern __shared__ __align__(16) char smem[];
    char *slab = smem + NS * STAGE_BYTES + (threadIdx.x >> 6) * SLAB;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: LDS-DMA destinations stay in SGPRs
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int per_plane = tiles_m * tiles_n;
    const int nks = Kl / BKS;
    const uint32_t smem_lds = (uint32_t)(uintptr_t)STL_LDS(smem);

    Frag<A_T, SWZ, BM> fa;
    Frag<B_T, SWZ, BN> fb;
    fa.init(wm * WM, lane);
    fb.init(wn * WN, lane);

    // block list: virtual block id v -> (plane, block row, block column); consecutive blocks of a plane are
    // dealt to one XCD (hardware deals workgroup ids round-robin over the 8 XCDs)
    auto locate = [&](int v, int &pb, int &p, int &i0, int &j0) {
        int lid = v;
        if ((total & 7) == 0 && (gridDim.x & 7) == 0) lid = (v & 7) * (total >> 3) + (v >> 3);
        const int q = lid / per_plane;               // (stacked problem, plane)
        const int rem = lid - q * per_plane;
        pb = q / batch;
        p = q - pb * batch;
        i0 = (rem / tiles_n) * BM;
        j0 = (rem % tiles_n) * BN;
    };

    Src<A_T, SWZ, BM, NW> sa;
    Src<B_T, SWZ, BN, NW> sb;
    auto start_block = [&](int v) {      // point the DMA sources at block v and put its first NS-1 stages in flight
        int pb, p, i0, j0;
        locate(v, pb, p, i0, j0);
        sa.init(A, A_T ? Mi : Kl, i0, Mi, wave, lane, p, batch, a_pg, pb * (A_T ? Kl : Mi));
        sb.init(B, B_T ? Nj : Kl, j0, Nj, wave, lane, p, batch, b_pg, pb * (B_T ? Kl : Nj));
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) {
            if (s < nks) {
                sa.issue(smem_lds + s * STAGE_BYTES, wave);
                sb.issue(smem_lds + s * STAGE_BYTES + OPER_BYTES, wave);
            }
        }
    };

    int v = blockIdx.x;
    if (v < total) start_block(v);

    for (; v < total; v += gridDim.x) {
        int pb, p, i0, j0;
        locate(v, pb, p, i0, j0);

        f32x16_t acc[FM][FN];
#pragma unroll
        for (int a = 0; a < FM; ++a)
#pragma unroll
            for (int b = 0; b < FN; ++b)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

        // Stage s+NS-1 is issued in iteration s; stage s+1 must have landed at the top of iteration s (fragments
        // are fetched one k16-step ahead, across the stage boundary).  Stores of the previous epilogue may still
        // be in flight: "at most N operations outstanding" then over-waits but never under-waits.
        if (nks > NS - 2) wait_vmcnt<DMA_PER_STAGE * (NS - 2)>();
        else wait_vmcnt<0>();
        block_barrier();

        bf16x8_t va[2][FM], vb[2][FN];      // fragment double buffer: [k16-step parity]
#pragma unroll
        for (int a = 0; a < FM; ++a) va[0][a] = fa.read(smem, a, 0);
#pragma unroll
        for (int b = 0; b < FN; ++b) vb[0][b] = fb.read(smem + OPER_BYTES, b, 0);

        // One stage (two k16-steps).  REFILL: stage s+NS-1 is fetched into the slot freed by stage s-1 -- a compile-time
        // switch, so that the loop over the stages that refill carries no test around the DMA instructions.
        auto stage = [&](int s, auto refill_c) {
            constexpr bool REFILL = decltype(refill_c)::value;
            if (s + 1 < nks) {
                if (REFILL || s + NS - 2 < nks) wait_vmcnt<DMA_PER_STAGE * (NS - 3)>();
                else wait_vmcnt<0>();
            }
            block_barrier();   // stage s+1 visible to all; nobody reads stage s-1 any more
            const uint32_t dst = smem_lds + ((s + NS - 1) % NS) * STAGE_BYTES;
            const char *cur = smem + (s % NS) * STAGE_BYTES;
            const char *nxt = smem + ((s + 1) % NS) * STAGE_BYTES;
            // One k16-step: MFMAs run on fragments fetched during the previous step while the fragments of the
            // following step are fetched (A fragments after the first MFMA, B fragments after the second) and
            // this wavefront's share of the refill DMA is issued one instruction at a time further down.  Issuing
            // the DMA in one burst right after the barrier backs up the vector-memory queue of all eight
            // wavefronts at once and holds their MFMAs behind it; the fences pin the interleaving.
            auto step = [&](auto par_c, const char *src, int ks, auto a_side_c) {
                constexpr int par = decltype(par_c)::value;
                constexpr bool a_side = decltype(a_side_c)::value;
                static_for<0, FM * FN>([&](auto i_c) {
                    constexpr int i = decltype(i_c)::value, a = i / FN, b = i % FN;
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vb[par][b], va[par][a], acc[a][b], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    // one fragment fetch per MFMA slot, in the order the next step consumes them: B0, A0, B1, A1, ...
                    // (eight wavefronts fetching all their fragments at once fill the LDS queue, and a wavefront
                    //  stuck issuing an LDS read cannot issue the independent MFMAs behind it)
                    if constexpr (i < FM + FN) {
                        constexpr int pairs = FM < FN ? FM : FN;
                        if constexpr (i < 2 * pairs) {
                            if constexpr ((i % 2) == 0) vb[par ^ 1][i / 2] = fb.read(src + OPER_BYTES, i / 2, ks);
                            else va[par ^ 1][i / 2] = fa.read(src, i / 2, ks);
                        } else if constexpr (FM > FN) {
                            va[par ^ 1][i - pairs] = fa.read(src, i - pairs, ks);
                        } else {
                            vb[par ^ 1][i - pairs] = fb.read(src + OPER_BYTES, i - pairs, ks);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if constexpr (REFILL && i >= 2 && (i % 2) == 0) {
                        constexpr int j = (i - 2) / 2;       // DMA slot inside this step
                        if constexpr (a_side) {
                            if constexpr (j < decltype(sa)::NI) sa.issue_one(dst, wave, j);
                        } else {
                            if constexpr (j < decltype(sb)::NI) sb.issue_one(dst + OPER_BYTES, wave, j);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                });
            };
            // step 0 of stage s (fetch step 1 of stage s; refill the A operand), then step 1 (fetch step 0 of stage
            // s+1 -- after the last stage that reads a stale ring slot whose values are never used; refill B)
            step(std::integral_constant<int, 0>{}, cur, 1, std::true_type{});
            step(std::integral_constant<int, 1>{}, nxt, 0, std::false_type{});
            if constexpr (REFILL) {
                sa.next_stage();
                sb.next_stage();
            }
        };
        const int n_refill = nks > NS - 1 ? nks - (NS - 1) : 0;
        for (int s = 0; s < n_refill; ++s) stage(s, std::true_type{});
        for (int s = n_refill; s < nks; ++s) stage(s, std::false_type{});

        // every wavefront is done with the ring: refill it for the next block before storing this one
        block_barrier();
        if (v + (int)gridDim.x < total) start_block(v + gridDim.x);

        // Epilogue.  With operands passed as (B fragment, A fragment) accumulator e of fragment (a, b) is
        //   Out[row = 32a + lane%32][column = 32b + 8*(e/4) + 4*(lane/32) + e%4].
        // output rows of one pass lie in one group of the output layout (groups are multiples of 32 rows, or everything)
        TO *outp = Out + (size_t)p * o_pg * Nj;
        const int frow = lane & 31, fhalf = lane >> 5;
        constexpr int LPR = WN * ES / 16;                   // lanes per row in the store phase
        constexpr int RPI = 64 / LPR;                       // rows per store instruction
        static_for<0, FM>([&](auto a_c) {
            constexpr int a = decltype(a_c)::value;
            static_for<0, 32 / RP>([&](auto pass_c) {
                constexpr int pass = decltype(pass_c)::value;
                if (RP == 32 || (frow / RP) == pass) {
                    char *rowp = slab + (frow % RP) * PITCH;
#pragma unroll
                    for (int b = 0; b < FN; ++b)
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const int cc = b * 32 + 8 * g + 4 * fhalf;
                            if (ES == 2) {
                                const u32x2_t w = {pack_bf16x2(acc[a][b][4 * g], acc[a][b][4 * g + 1]),
                                                   pack_bf16x2(acc[a][b][4 * g + 2], acc[a][b][4 * g + 3])};
                                *reinterpret_cast<u32x2_t *>(rowp + cc * 2) = w;
                            } else {
                                const f32x4_t w = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2],
                                                   acc[a][b][4 * g + 3]};
                                *reinterpret_cast<f32x4_t *>(rowp + cc * 4) = w;
                            }
                        }
                }
                // same wavefront wrote the slab; LDS operations of a wavefront complete in order
                asm volatile("" ::: "memory");
                const int gi_base = i0 + wm * WM + a * 32 + pass * RP;
                const size_t row_off = plane_row_base(pb * Mi + (gi_base < Mi ? gi_base : 0), o_pg, batch, Nj);
                const int gj = j0 + wn * WN + (lane % LPR) * (16 / ES);
#pragma unroll
                for (int it = 0; it < RP / RPI; ++it) {
                    const int rr = it * RPI + lane / LPR;
                    const int gi = gi_base + rr;
                    const u32x4_t w = *reinterpret_cast<const u32x4_t *>(slab + rr * PITCH + (lane % LPR) * 16);
                    if (gi < Mi && gj < Nj) {
                        TO *o = outp + row_off + (size_t)rr * Nj + gj;
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
                asm volatile("" ::: "memory");
            });
        });
    }
}

bool plane_gemm_pipe_eligible(const GemmDesc &g)
{
    if (!plane_gemm_mfma_eligible(g)) return false;
    if (g.Kl % pipe::BKS) return false;
    // a stage's 32 stored rows of an [l][row] operand stay inside one group; so do the rows of an epilogue pass
    if (g.a_kmajor && g.a_rows_per_group() % pipe::BKS) return false;
    if (g.b_kmajor && g.b_rows_per_group() % pipe::BKS) return false;
    if (g.o_pg > 0 && g.o_pg % 32) return false;
    // stacked problems: every problem's first stored row keeps those alignments; only the single-stage contraction
    // (attention-shaped products) is taken here, deeper stacked contractions go to the register-staged kernel
    if (g.nb > 1 && (g.Kl != pipe::BKS || (g.o_pg > 0 && g.Mi % 32))) return false;
    // a clamped edge chunk must still lie inside the operand
    if (g.Mi < 8 || g.Nj < 8) return false;
    return g.Mi > 128 && g.Nj > 128;
}

static int cu_count()
{
    static const int n = []() {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 256;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
        return cus;
    }();
    return n;
}

template <int WAVES_M, int WAVES_N, bool A_T, bool B_T, typename TO, bool ACC>
static hipError_t launch_pipe_cfg(const GemmDesc &g, const void *A, const void *B, void *Out, hipStream_t s)
{
    constexpr int NS = 4, SWZ = 2, NW = WAVES_M * WAVES_N, WN = 256 / WAVES_N;
    auto kern = gemm_pipe_kernel<WAVES_M, WAVES_N, NS, SWZ, A_T, B_T, TO, ACC>;
    constexpr int ES = sizeof(TO);
    constexpr int RP = (ES == 2 ? 32 : 16) / (NS == 4 ? 2 : 1) / (WN / 64);
    constexpr int smem = NS * 512 * pipe::BKS * 2 + NW * RP * (WN * ES + 16);
    static_assert(smem <= 160 * 1024, "LDS budget");
    // once per instantiation (initialisation of a function-local static is thread-safe)
    static const hipError_t attr_err =
        hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (attr_err != hipSuccess) return attr_err;
    const int tiles_m = (g.Mi + 255) / 256, tiles_n = (g.Nj + 255) / 256;
    const long total = (long)tiles_m * tiles_n * g.batch * g.nb;
    if (total > 0x7fffffffL) return hipErrorInvalidValue;
    // one workgroup per CU that walks the block list
    const int cus = cu_count();
    const unsigned grid = (unsigned)(total > cus ? cus : total);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NW * 64), smem, s, (const bf16_t *)A, (const bf16_t *)B, (TO *)Out, g.Mi, g.Nj,
                       g.Kl, tiles_m, tiles_n, (int)total, g.a_rows_per_group(), g.b_rows_per_group(), g.o_rows_per_group(), g.batch);
    return hipGetLastError();
}

// The [l][row] form of an operand is chosen per operand; the fp32 (weight-gradient) output exists for the
// doubly contraction-major form only, which is the only one the library asks for.
static hipError_t launch_pipe_form(const GemmDesc &g, const void *A, const void *B, void *Out, hipStream_t s)
{
    // eight wavefronts of 128 x 64 (four of 128 x 128 would read a third less from LDS per MFMA, but a single wavefront
    // per SIMD cannot cover its own LDS latency: measured slower)
    if (g.out_f32) {
        if (!(g.a_kmajor && g.b_kmajor)) return hipErrorInvalidValue;
        return g.accumulate ? launch_pipe_cfg<2, 4, true, true, float, true>(g, A, B, Out, s)
                            : launch_pipe_cfg<2, 4, true, true, float, false>(g, A, B, Out, s);
    }
    if (g.accumulate) return hipErrorInvalidValue;
    if (g.a_kmajor) {
        if (!g.b_kmajor) return hipErrorInvalidValue;
        return launch_pipe_cfg<2, 4, true, true, bf16_t, false>(g, A, B, Out, s);
    }
    if (g.b_kmajor) return launch_pipe_cfg<2, 4, false, true, bf16_t, false>(g, A, B, Out, s);
    return launch_pipe_cfg<2, 4, false, false, bf16_t, false>(g, A, B, Out, s);
}

hipError_t launch_plane_gemm_pipe(const GemmDesc &g, const void *A, const void *B, void *Out, hipStream_t s)
{
    // refuse here as well what plane_gemm_pipe_eligible excludes, so that a change of the dispatch rule cannot reach a
    // form of the kernel that no test covers (stacked problems with more than one contraction stage among them)
    if (!plane_gemm_pipe_eligible(g)) return hipErrorInvalidValue;
    return launch_pipe_form(g, A, B, Out, s);
}

}  // namespace stl
