// The forward pass (Algorithm 1: encode -> r plane products -> decode) as ONE persistent launch in which the
// HBM-bound tile maps run on some CUs while the matrix-core-bound plane products run on the others.
//
// The three steps of a row block (256 tile rows) depend on each other -- the plane products of row block b need its
// encoded rows, its decode needs all its r x (N / 256) product blocks -- but different row blocks are independent.
// The work of the whole call is cut into items,
//     E(b): encode of a share of row block b,   G(b): one 256 x 256 plane-product block of row block b,
//     D(b): decode of a share of row block b,
// and laid out as a list in which every item stands behind everything it depends on:
//     E(0) E(1) | G(0) E(2) | G(1) E(3) | G(2) D(0) E(4) | G(3) D(1) E(5) | ...  | D(nb-2) | D(nb-1)
// (round j holds G(j), D(j-2), E(j+2)).  One workgroup per CU takes items off the list with an atomic ticket, in
// order.  An item that depends on others waits on a counter of finished items (E(b) -> G(b), G(b) -> D(b)).  Waiting
// cannot deadlock: a ticket is only ever held by a running workgroup, and everything an item waits for has a smaller
// ticket, so the earliest unfinished item can always run.  (The wait is bounded all the same: after `spin_limit`
// polls a workgroup raises the error flag and goes on, so that every wavefront exits whatever happens.)
//
// While some CUs stream X -> Xhat or Yhat -> C at the full clock, the others multiply; the store bursts of the
// product blocks no longer coincide on all CUs either.  The list is kept per XCD (workgroup id mod 8, which is how
// the hardware deals workgroups to the XCDs): an XCD multiplies the planes p = xcd (mod 8), so the column blocks of
// a plane's row block share their Xhat rows in that XCD's L2.
//
// Visibility between workgroups on different XCDs (their L2s are not coherent with each other): what a later item
// reads -- Xhat and Yhat -- is stored THROUGH the writer's L2 to memory (store16<true>), and an item raises its counter
// (agent-scope atomic) only after all its stores have completed, so the data is in memory before anybody can learn
// that it exists.  A reader needs no invalidation: every item's output is a set of whole 128-byte lines that nobody
// reads, not even speculatively or as the other half of a line, before the item is finished (the lists, the guards
// in the item loops and the eligibility rule K, N multiples of 64 tiles see to that), and every launch starts with
// clean caches, so no cache can hold a stale copy of such a line.  (A write-back of the whole L2 per finished item
// and an invalidation per wait -- the agent-scope release and acquire fences -- were measured first: 0.37 ms for the
// benchmark forward against 0.25 ms with written-through stores and no fences.)
//
// Measured (bf16, m = 8192, k = n = 4096): this launch takes 0.25 ms at r = 32 and 0.17 ms at r = 8, the three separate
// launches 0.215 and 0.075 ms.  With every wait switched off (wrong results, timing only) it takes 0.208 and 0.086 ms,
// with the tile maps skipped as well 0.154 and 0.053 ms: the tile-map items cost as much wall time between the product
// blocks as they cost on their own.  A CU that runs a tile-map item does not multiply meanwhile (one workgroup per CU:
// the product code needs the whole LDS), and the items take nearly their stand-alone time although the other CUs leave
// most of the HBM bandwidth unused, so overlapping the HBM-bound and the matrix-core-bound work of this operator gains
// nothing on this GPU; the waits of the real list cost another 0.04-0.08 ms.  The variant is therefore selectable (STL_FLAG_PIPELINED) but never chosen automatically.
//
// Arithmetic, rounding and summation order are exactly those of the three separate kernels (same device functions,
// same block code): the results are bit-identical to the three-launch path.
#include "stl_gemm_pipe.h"
#include "stl_tile_items.h"

namespace stl {

namespace {

struct FwdPipe {
    const bf16_t *X, *E, *What, *Dm;
    bf16_t *Xhat, *Yhat, *C;
    int M, K, N, r;            // tile counts and planes
    int nrb, tiles_n;          // row blocks of 256 tile rows, column blocks of 256 tile columns
    int nG, nT;                // per XCD and row block: product blocks (ceil(r / 8) * tiles_n), encode items = decode items
    int enc_wi, dec_wi;        // wavefront items (tile row, 64-tile chunk) per encode / decode item
    unsigned *ctr;             // [0..7] tickets, [8] error flag, [16 + b] encode items done, [16 + nrb + b] product blocks done
    int spin_limit;
};

constexpr int kCtrTicket = 0, kCtrError = 8, kCtrBase = 16;

__global__ void pipeline_reset_kernel(unsigned *ctr, int n)
{
    for (int i = threadIdx.x; i < n; i += blockDim.x) ctr[i] = 0u;
}

}  // namespace

template <bool GELU>
__global__ __launch_bounds__(512) void forward_pipeline_kernel(const FwdPipe a)
{
    using namespace pipe;
    constexpr int NS = 4, SWZ = 2, BM = 256, BN = 256, NW = 8, WAVES_N = 4, WM = 128, WN = 64, FM = 4, FN = 2;
    constexpr int OPER_BYTES = BM * BKS * 2, STAGE_BYTES = (BM + BN) * BKS * 2;
    constexpr int DMA_PER_STAGE = (BM + BN) / 16 / NW;
    constexpr int RP = 16, PITCH = WN * 2 + 16, SLAB = RP * PITCH;     // epilogue staging per wavefront
    constexpr int PG = kPlaneGroup;
    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    char *slab = smem + NS * STAGE_BYTES + wave * SLAB;
    volatile int *mail = reinterpret_cast<volatile int *>(smem + NS * STAGE_BYTES + NW * SLAB);   // thread 0 -> workgroup
    char *tslab = smem + wave * 4096;                    // tile-map slab of this wavefront: lies in the (idle) ring
    const uint32_t smem_lds = (uint32_t)(uintptr_t)STL_LDS(smem);
    const int xcd = blockIdx.x & 7;
    const int Mi = a.M, Nj = a.N, Kl = a.K, nks = Kl / BKS, batch = a.r;
    const int per_round = a.nG + 2 * a.nT;
    const int total = (a.nrb + 4) * per_round;           // rounds -2 .. nrb + 1
    const int chunks_k = Kl / 64, chunks_n = (Nj + 63) / 64;
    const RowMap rm;

    Frag<false, SWZ, BM> fa;
    Frag<true, SWZ, BN> fb;
    fa.init(wm * WM, lane);
    fb.init(wn * WN, lane);
    Src<false, SWZ, BM, NW> sa;
    Src<true, SWZ, BN, NW> sb;

    // ---- the list -------------------------------------------------------------------------------------------------
    enum { K_NONE = 0, K_GEMM = 1, K_GEMM_EMPTY = 2, K_ENC = 3, K_DEC = 4 };
    struct Item { int kind, rb, p, bj, ti; };
    auto decode_ticket = [&](int t) {
        Item it{K_NONE, 0, 0, 0, 0};
        if (t >= total) return it;
        const int round = t / per_round - 2, idx = t - (round + 2) * per_round;
        if (idx < a.nG) {
            it.rb = round;
            if (round >= 0 && round < a.nrb) {
                it.p = 8 * (idx / a.tiles_n) + xcd;
                it.bj = idx % a.tiles_n;
                it.kind = it.p < a.r ? K_GEMM : K_GEMM_EMPTY;
            }
        } else if (idx < a.nG + a.nT) {
            it.rb = round - 2;
            it.ti = (idx - a.nG) * 8 + xcd;
            if (it.rb >= 0 && it.rb < a.nrb) it.kind = K_DEC;
        } else {
            it.rb = round + 2;
            it.ti = (idx - a.nG - a.nT) * 8 + xcd;
            if (it.rb >= 0 && it.rb < a.nrb) it.kind = K_ENC;
        }
        return it;
    };
    // next ticket of this XCD's list, the same value in every thread
    int grabs = 0;
    auto grab = [&]() {
        block_barrier();                                 // everybody has read the previous mail
#ifndef STL_PIPELINE_STATIC_TICKETS
        if (tid == 0) mail[0] = (int)__hip_atomic_fetch_add(a.ctr + kCtrTicket + xcd, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#else   // host build for the address check (threads run one after the other): the k-th grab of a workgroup is fixed
        mail[0] = (int)(blockIdx.x >> 3) + grabs * (int)(gridDim.x >> 3);
#endif
        ++grabs;
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        block_barrier();
        return __builtin_amdgcn_readfirstlane(mail[0]);          // uniform: lives in a scalar register
    };
    // counter[idx] >= target?  blocking: polls up to spin_limit times, then raises the error flag and gives up
    auto poll = [&](int idx, unsigned target, bool blocking) {
        block_barrier();
        if (tid == 0) {
            int ok = 0;
            const int tries = blocking ? a.spin_limit : 1;
            for (int i = 0; i < tries; ++i) {
                if (__hip_atomic_load(a.ctr + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target) { ok = 1; break; }
                __builtin_amdgcn_s_sleep(16);
            }
            if (!ok && blocking) __hip_atomic_fetch_or(a.ctr + kCtrError, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            mail[1] = ok;
        }
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        block_barrier();
        return __builtin_amdgcn_readfirstlane(mail[1]) != 0;
    };
    // this item is finished: all its (written-through) stores have completed before the counter moves
    auto signal = [&](int idx) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        block_barrier();
        if (tid == 0) __hip_atomic_fetch_add(a.ctr + idx, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    const unsigned enc_target = 8u * (unsigned)a.nT, gemm_target = 8u * (unsigned)a.nG;

    auto start_block = [&](const Item &it) {   // point the DMA sources at the block and put its first NS-1 stages in flight
        sa.init(a.Xhat, Kl, it.rb * BM, Mi, wave, lane, it.p, batch, PG, 0);
        sb.init(a.What, Nj, it.bj * BN, Nj, wave, lane, it.p, batch, Kl, 0);
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) {
            if (s < nks) {
                sa.issue(smem_lds + s * STAGE_BYTES, wave);
                sb.issue(smem_lds + s * STAGE_BYTES + OPER_BYTES, wave);
            }
        }
    };

    int t = grab();
    bool prefetched = false;
    while (t < total) {
        const Item it = decode_ticket(t);
        if (it.kind == K_GEMM) {
            if (!prefetched) {
                poll(kCtrBase + it.rb, enc_target, true);
                start_block(it);
            }
            const int i0 = it.rb * BM, j0 = it.bj * BN;
            f32x16_t acc[FM][FN];
#pragma unroll
            for (int x = 0; x < FM; ++x)
#pragma unroll
                for (int y = 0; y < FN; ++y)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[x][y][e] = 0.f;

            if (nks > NS - 2) wait_vmcnt<DMA_PER_STAGE * (NS - 2)>();
            else wait_vmcnt<0>();
            block_barrier();

            bf16x8_t va[2][FM], vb[2][FN];      // fragment double buffer: [k16-step parity]
#pragma unroll
            for (int x = 0; x < FM; ++x) va[0][x] = fa.read(smem, x, 0);
#pragma unroll
            for (int y = 0; y < FN; ++y) vb[0][y] = fb.read(smem + OPER_BYTES, y, 0);

            // one stage = two k16-steps; the same instruction order as the stand-alone plane-product kernel
            auto stage = [&](int s, auto refill_c) {
                constexpr bool REFILL = decltype(refill_c)::value;
                if (s + 1 < nks) {
                    if (REFILL || s + NS - 2 < nks) wait_vmcnt<DMA_PER_STAGE * (NS - 3)>();
                    else wait_vmcnt<0>();
                }
                block_barrier();
                const uint32_t dst = smem_lds + ((s + NS - 1) % NS) * STAGE_BYTES;
                const char *cur = smem + (s % NS) * STAGE_BYTES;
                const char *nxt = smem + ((s + 1) % NS) * STAGE_BYTES;
                auto step = [&](auto par_c, const char *src, int ks, auto a_side_c) {
                    constexpr int par = decltype(par_c)::value;
                    constexpr bool a_side = decltype(a_side_c)::value;
                    static_for<0, FM * FN>([&](auto i_c) {
                        constexpr int i = decltype(i_c)::value, x = i / FN, y = i % FN;
                        acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vb[par][y], va[par][x], acc[x][y], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                        if constexpr (i < FM + FN) {
                            constexpr int pairs = FM < FN ? FM : FN;
                            if constexpr (i < 2 * pairs) {
                                if constexpr ((i % 2) == 0) vb[par ^ 1][i / 2] = fb.read(src + OPER_BYTES, i / 2, ks);
                                else va[par ^ 1][i / 2] = fa.read(src, i / 2, ks);
                            } else {
                                va[par ^ 1][i - pairs] = fa.read(src, i - pairs, ks);
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        if constexpr (REFILL && i >= 2 && (i % 2) == 0) {
                            constexpr int j = (i - 2) / 2;
                            if constexpr (a_side) {
                                if constexpr (j < decltype(sa)::NI) sa.issue_one(dst, wave, j);
                            } else {
                                if constexpr (j < decltype(sb)::NI) sb.issue_one(dst + OPER_BYTES, wave, j);
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    });
                };
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

            // every wavefront is done with the ring.  Take the next ticket now: if it is a product block whose rows are
            // already encoded, its first stages go in flight before this block is stored.
            const int tn = grab();
            const Item nx = decode_ticket(tn);
            prefetched = false;
            if (nx.kind == K_GEMM && poll(kCtrBase + nx.rb, enc_target, false)) {
                start_block(nx);
                prefetched = true;
            }

            // Epilogue: accumulator e of fragment (x, y) is Out[row 32x + lane%32][column 32y + 8(e/4) + 4(lane/32) + e%4]
            bf16_t *outp = a.Yhat + (size_t)it.p * PG * Nj;
            const int frow = lane & 31, fhalf = lane >> 5;
            constexpr int LPR = WN * 2 / 16, RPI = 64 / LPR;
            static_for<0, FM>([&](auto x_c) {
                constexpr int x = decltype(x_c)::value;
                static_for<0, 32 / RP>([&](auto pass_c) {
                    constexpr int pass = decltype(pass_c)::value;
                    if ((frow / RP) == pass) {
                        char *rowp = slab + (frow % RP) * PITCH;
#pragma unroll
                        for (int y = 0; y < FN; ++y)
#pragma unroll
                            for (int g = 0; g < 4; ++g) {
                                const int cc = y * 32 + 8 * g + 4 * fhalf;
                                const u32x2_t w = {pack_bf16x2(acc[x][y][4 * g], acc[x][y][4 * g + 1]),
                                                   pack_bf16x2(acc[x][y][4 * g + 2], acc[x][y][4 * g + 3])};
                                *reinterpret_cast<u32x2_t *>(rowp + cc * 2) = w;
                            }
                    }
                    asm volatile("" ::: "memory");
                    const int gi_base = i0 + wm * WM + x * 32 + pass * RP;
                    const size_t row_off = plane_row_base(gi_base < Mi ? gi_base : 0, PG, batch, Nj);
                    const int gj = j0 + wn * WN + (lane % LPR) * 8;
#pragma unroll
                    for (int k = 0; k < RP / RPI; ++k) {
                        const int rr = k * RPI + lane / LPR;
                        const int gi = gi_base + rr;
                        const u32x4_t w = *reinterpret_cast<const u32x4_t *>(slab + rr * PITCH + (lane % LPR) * 16);
                        if (gi < Mi && gj < Nj) store16<true>(outp + row_off + (size_t)rr * Nj + gj, w);
                    }
                    asm volatile("" ::: "memory");
                });
            });
            signal(kCtrBase + a.nrb + it.rb);
            t = tn;
            continue;
        }
        prefetched = false;
        // the lane id as an opaque value: what the tile maps derive from it is computed per item and does not occupy
        // registers while product blocks run
        int tl = lane;
        asm volatile("" : "+v"(tl));
        if (it.kind == K_GEMM_EMPTY) {
            // a plane slot beyond r: nothing to multiply, but the decode of the row block counts the blocks
            signal(kCtrBase + a.nrb + it.rb);
        } else if (it.kind == K_ENC) {
            // wavefront items [first, end) of the encode: (tile row, 64-tile chunk) pairs of row block rb
            const long rb_first = (long)it.rb * BM * chunks_k;
            const long lim = (long)(it.rb + 1) * BM * chunks_k, all = (long)Mi * chunks_k;
            const long first = rb_first + (long)it.ti * a.enc_wi;
            long end = first + a.enc_wi;
            end = end < lim ? end : lim;
            end = end < all ? end : all;
            f32x4_t unused[4];
            encode_items<1, false, true, 4>(a.X, a.E, a.Xhat, nullptr, Mi, Kl, a.r, chunks_k, PG, rm, first + wave, NW, end, nullptr, tslab, unused, tl);
            signal(kCtrBase + it.rb);
        } else if (it.kind == K_DEC) {
            poll(kCtrBase + a.nrb + it.rb, gemm_target, true);
            const long rb_first = (long)it.rb * BM * chunks_n;
            const long lim = (long)(it.rb + 1) * BM * chunks_n, all = (long)Mi * chunks_n;
            const long first = rb_first + (long)it.ti * a.dec_wi;
            long end = first + a.dec_wi;
            end = end < lim ? end : lim;
            end = end < all ? end : all;
            f32x4_t unused[4];
            decode_items<GELU, 1, false, 4>(a.Yhat, a.Dm, a.C, Mi, Nj, a.r, chunks_n, nullptr, PG, rm, first + wave, NW, end, nullptr, tslab, unused, tl);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        t = grab();
    }
}

// ---- host side ----------------------------------------------------------------------------------------------------

bool forward_pipeline_eligible(int dtype, int M, int K, int N, int r)
{
    // bf16, at most 32 planes (one 32-plane group in the tile maps), whole 128-byte lines per item (K, N multiples of
    // 64 tiles), a contraction the ring takes, at least two row blocks to overlap, counters that fit their area
    return dtype == 1 && r >= 1 && r <= 32 && K % 64 == 0 && N % 64 == 0 && N >= 256 && M >= 512 && (M + 255) / 256 <= 4096;
}

size_t forward_pipeline_counter_bytes(int M) { return (size_t)(kCtrBase + 2 * ((M + 255) / 256)) * sizeof(unsigned); }

static int pipeline_cus()
{
    static const int n = []() {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 256;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8) return 256;
        return cus / 8 * 8;
    }();
    return n;
}

hipError_t launch_forward_pipeline(const void *X, const void *E, const void *What, const void *Dm, void *Xhat, void *Yhat,
                                   void *C, void *counters, int M, int K, int N, int r, bool gelu, hipStream_t s)
{
    if (!forward_pipeline_eligible(1, M, K, N, r)) return hipErrorInvalidValue;
    FwdPipe a{};
    a.X = (const bf16_t *)X; a.E = (const bf16_t *)E; a.What = (const bf16_t *)What; a.Dm = (const bf16_t *)Dm;
    a.Xhat = (bf16_t *)Xhat; a.Yhat = (bf16_t *)Yhat; a.C = (bf16_t *)C;
    a.M = M; a.K = K; a.N = N; a.r = r;
    a.nrb = (M + 255) / 256;
    a.tiles_n = (N + 255) / 256;
    a.nG = (r + 7) / 8 * a.tiles_n;
    a.nT = 8;                                           // 64 encode and 64 decode items per row block
    const int enc_all = 256 * (K / 64), dec_all = 256 * ((N + 63) / 64);
    a.enc_wi = (enc_all + 8 * a.nT - 1) / (8 * a.nT);
    a.dec_wi = (dec_all + 8 * a.nT - 1) / (8 * a.nT);
    a.ctr = (unsigned *)counters;
    a.spin_limit = 1 << 17;                             // about a thousand times the longest legitimate wait
    const int nctr = kCtrBase + 2 * a.nrb;
    hipLaunchKernelGGL(pipeline_reset_kernel, dim3(1), dim3(256), 0, s, a.ctr, nctr);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    constexpr int smem = 4 * 512 * pipe::BKS * 2 + 8 * 16 * (64 * 2 + 16) + 64;
    static_assert(smem <= 160 * 1024, "LDS budget");
    auto launch = [&](auto kern) {
        static const hipError_t attr_err =
            hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (attr_err != hipSuccess) return attr_err;
        hipLaunchKernelGGL(kern, dim3(pipeline_cus()), dim3(512), smem, s, a);
        return hipGetLastError();
    };
    return gelu ? launch(forward_pipeline_kernel<true>) : launch(forward_pipeline_kernel<false>);
}

}  // namespace stl
