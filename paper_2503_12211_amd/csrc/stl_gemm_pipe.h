// Building blocks of the LDS-DMA pipelined plane products: LDS-DMA source pointers, fragment addressing, swizzles,
// instruction-order fences and counted waits.  Shared by the plane-product kernel and by the kernel that runs the
// tile maps between its blocks.
#pragma once
#include "stl_kernels.h"
#include "stl_device.h"

#include <type_traits>

namespace stl {

namespace pipe {

constexpr int BKS = 32;                 // contraction elements per stage

typedef short v4i16_t __attribute__((ext_vector_type(4)));
#define STL_LDS(p) ((__attribute__((address_space(3))) char *)(p))

// Swizzles (16-byte chunk index XOR), chosen so that one access phase touches every bank once.  Measured with the
// SQ_LDS_BANK_CONFLICT counter: ds_read_b128 is served in four phases of 16 lanes, {0-3, 12-15, 20-23, 24-27},
// {4-11, 16-19, 28-31} and the same +32; for 64-byte rows read by lane = row, XOR with (row >> 2) & 3 is
// conflict-free (6 LDS cycles per instruction), (row >> 1) & 3 costs 4 extra cycles, no swizzle 12.
template <int SHIFT>
__device__ __forceinline__ int fswz(int row) { return (row >> SHIFT) & 3; }     // [row][l] operand, 4 chunks per row
__device__ __forceinline__ int gswz(int k) { return (k & 3) << 2; }              // [l][row] operand, 32 chunks per row

// LDS-DMA load, 16 bytes per lane: lane L's bytes land at lds_wave_base + 16*L (M0 carries the wave-uniform LDS
// address).  Issued as inline assembly on purpose: the main loop orders these loads against the fragment reads
// itself (vmcnt + barrier below); letting the compiler track them makes it drain every outstanding load before
// each LDS read, which removes the prefetch distance this kernel exists for.
__device__ __forceinline__ void dma16(const bf16_t *g, uint32_t lds_wave_base)
{
    const uint32_t l = __builtin_amdgcn_readfirstlane(lds_wave_base);
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(l) : "memory", "m0");
}

__device__ __forceinline__ void block_barrier() { asm volatile("s_barrier" ::: "memory"); }

// Per-thread global source pointers for the DMA instructions a wavefront issues per operand and stage.
// One operand stage is ROWS x 32 contraction elements = ROWS/16 KB = ROWS/16 instructions, dealt to NW wavefronts.
template <bool KMAJOR, int SWZ, int ROWS, int NW>
struct Src {
    static constexpr int NI = ROWS / 16 / NW;          // instructions per wavefront
    static constexpr int CPR = ROWS / 8;               // 16-byte chunks per LDS row of the [l][row] form
    const bf16_t *p[NI];
    long step;   // elements to advance per stage
    long jump;   // [l][row] form: extra elements when the next stage starts a new group of stored rows
    int kpos, pg;
    // base: the whole batched operand; plane p of `batch`; stored rows come in groups of pg (see plane_row_base), and a
    // stage's 32 stored rows of the [l][row] form never straddle two groups (pg % 32 == 0)
    // roff: first stored row of this problem inside the stacked operand (a multiple of 32 for the [l][row] form)
    __device__ __forceinline__ void init(const bf16_t *base, long ld, int row0, int rows_total, int wave, int lane, int plane,
                                         int batch, int pg_, int roff)
    {
        pg = pg_;
        kpos = roff % pg_;
        const size_t poff = (size_t)plane * pg * ld;
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int q = NI * wave + j;
            if (!KMAJOR) {
                const int row = 16 * q + (lane >> 2), c = (lane & 3) ^ fswz<SWZ>(row);
                int gr = row0 + row;
                gr = gr < rows_total ? gr : rows_total - 1;   // rows past the edge feed only discarded outputs
                p[j] = base + plane_row_base(roff + gr, pg, batch, (int)ld) + poff + 8 * c;
            } else {
                const int k = (64 / CPR) * q + lane / CPR, nc = (lane % CPR) ^ gswz(k);
                int gc = row0 + 8 * nc;
                gc = gc < rows_total ? gc : rows_total - 8;
                p[j] = base + plane_row_base(roff + k, pg, batch, (int)ld) + poff + gc;
            }
        }
        step = KMAJOR ? (long)BKS * ld : BKS;
        jump = KMAJOR ? (long)(batch - 1) * pg * ld : 0;
    }
    // instruction j of this wavefront's share (the main loop spreads them between MFMAs)
    __device__ __forceinline__ void issue_one(uint32_t oper_stage, int wave, int j)
    {
        dma16(p[j], oper_stage + (NI * wave + j) * 1024);
    }
    // after the last instruction of a stage: point at the next stage
    __device__ __forceinline__ void next_stage()
    {
        long adv = step;
        if (KMAJOR) {
            kpos += BKS;
            if (kpos == pg) {
                kpos = 0;
                adv += jump;
            }
        }
#pragma unroll
        for (int j = 0; j < NI; ++j) p[j] += adv;
    }
    __device__ __forceinline__ void issue(uint32_t oper_stage, int wave)   // LDS byte address of the operand stage
    {
#pragma unroll
        for (int j = 0; j < NI; ++j) dma16(p[j], oper_stage + (NI * wave + j) * 1024);
        next_stage();
    }
};


// ---- whole-line form of a [row][l] operand ------------------------------------------------------------------------------
// A [row][l] operand fetched 32 contraction elements at a time asks L2 for half a 128-byte line per row and stage, and
// for the other half one stage later: twice the requests for the same bytes (counted: TCC_REQ).  In the whole-line
// form an LDS slot holds 64 contraction elements of every row (128 bytes = one line per row, ROWS * 128 bytes per slot)
// and serves two stages; it is filled in two halves of ROWS / 2 rows, one half per stage, so that every stage still
// issues the same number of instructions.  Three slots: while pair j is multiplied, pair j+1 has landed and pair j+2
// is in flight.
// LDS: row stride 128 bytes; 16-byte chunk c of row `row` lies at chunk position c ^ ((row >> 1) & 7): the sixteen
// rows of one ds_read_b128 access phase ({0-3, 12-15, 20-23, 24-27} or {4-11, 16-19, 28-31}, see above) then fall
// on sixteen different (row parity, chunk position) pairs, i.e. on all 64 banks once.
__device__ __forceinline__ int wswz(int row) { return (row >> 1) & 7; }

template <int ROWS, int NW>
struct SrcWide {
    static constexpr int HALF = ROWS / 2;                   // rows per half slot
    static constexpr int NI = HALF / 8 / NW;                // instructions per wavefront and half (8 rows x 128 bytes each)
    static constexpr int SLOT_BYTES = ROWS * 128, HALF_BYTES = HALF * 128;
    const bf16_t *p[2][NI];
    __device__ __forceinline__ void init(const bf16_t *base, long ld, int row0, int rows_total, int wave, int lane, int plane,
                                         int batch, int pg, int roff)
    {
        const size_t poff = (size_t)plane * pg * ld;
#pragma unroll
        for (int hp = 0; hp < 2; ++hp)
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int q = NI * wave + j;
                const int row = HALF * hp + 8 * q + (lane >> 3), c = (lane & 7) ^ wswz(row);
                int gr = row0 + row;
                gr = gr < rows_total ? gr : rows_total - 1;   // rows past the edge feed only discarded outputs
                p[hp][j] = base + plane_row_base(roff + gr, pg, batch, (int)ld) + poff + 8 * c;
            }
    }
    // instruction j of half HP into the slot at LDS byte address `slot`
    template <int HP>
    __device__ __forceinline__ void issue_one(uint32_t slot, int wave, int j)
    {
        dma16(p[HP][j], slot + HP * HALF_BYTES + (NI * wave + j) * 1024);
    }
    template <int HP>
    __device__ __forceinline__ void next_pair()               // after the last instruction of half HP: 64 elements on
    {
#pragma unroll
        for (int j = 0; j < NI; ++j) p[HP][j] += 64;
    }
    template <int HP>
    __device__ __forceinline__ void issue_half(uint32_t slot, int wave)
    {
#pragma unroll
        for (int j = 0; j < NI; ++j) issue_one<HP>(slot, wave, j);
        next_pair<HP>();
    }
};

template <int ROWS>
struct FragWide {
    int off[2];     // [ks], for the first stage of a pair; the second stage's chunks are 4 further: off ^ 64
    __device__ __forceinline__ void init(int tile_row0, int lane)
    {
        const int h = lane >> 5, row = tile_row0 + (lane & 31);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) off[ks] = row * 128 + (((2 * ks + h) ^ wswz(row)) << 4);
    }
    // fragment f (32 rows further per f) of k16-step ks of stage parity sp, from the slot that holds the stage's pair
    __device__ __forceinline__ bf16x8_t read(const char *slot, int f, int ks, int sp) const
    {
        return *reinterpret_cast<const bf16x8_t *>(slot + (off[ks] ^ (sp << 6)) + f * 32 * 128);
    }
};

// Fragment addressing: byte offset inside one operand stage for MFMA rows (frag_row0 + lane%32), k16-step ks.
template <bool KMAJOR, int SWZ, int ROWS>
struct Frag {
    int off[2][2];   // [ks][kk]; kk only used for the transposing form
    __device__ __forceinline__ void init(int tile_row0, int lane)
    {
        const int h = lane >> 5;
        if (!KMAJOR) {
            const int row = tile_row0 + (lane & 31);
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                off[ks][0] = row * 64 + (((2 * ks + h) ^ fswz<SWZ>(row)) << 4);
                off[ks][1] = 0;
            }
        } else {
            const int i = lane & 15, blk = (lane >> 4) & 1;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    const int k = 16 * ks + 8 * h + 4 * kk + (i >> 2);
                    const int col = tile_row0 + 16 * blk + 4 * (i & 3);
                    off[ks][kk] = k * (ROWS * 2) + (((col >> 3) ^ gswz(k)) << 4) + ((col & 7) << 1);
                }
        }
    }
    // fragment f (32 rows further per f) of k16-step ks
    __device__ __forceinline__ bf16x8_t read(const char *oper_stage, int f, int ks) const
    {
        if (!KMAJOR) {
            return *reinterpret_cast<const bf16x8_t *>(oper_stage + off[ks][0] + f * 32 * 64);
        } else {
            // Fragment f starts 32 columns = 4 chunks further.  The wavefront's first column is a multiple of
            // 64, so chunk bits 2..3 of this lane's column are free and "+4f" is "^ (f<<2)", which commutes with
            // the swizzle XOR: in bytes, off ^ (f << 6).
            const v4i16_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) v4i16_t *)STL_LDS(oper_stage + (off[ks][0] ^ (f << 6))));
            const v4i16_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) v4i16_t *)STL_LDS(oper_stage + (off[ks][1] ^ (f << 6))));
            struct { v4i16_t a, b; } both = {lo, hi};
            return __builtin_bit_cast(bf16x8_t, both);
        }
    }
};

// Instruction order inside one k16-step: MFMAs whose operands were fetched a whole step ago are interleaved with
// the LDS reads of the following step (a few reads after each of the first MFMAs), so that no LDS latency sits
// in front of an MFMA and the reads of the wavefronts do not arrive at the LDS in one burst.
template <int NMFMA>
__device__ __forceinline__ void order_mfma_reads()
{
    if constexpr (NMFMA == 8) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    } else {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
    }
}

// compile-time loop: the body sees its index as a constant, so register arrays are never indexed dynamically
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else if constexpr (N == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
    else if constexpr (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else if constexpr (N == 6) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
    else if constexpr (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else if constexpr (N == 12) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
    else if constexpr (N == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    else static_assert(N == 0, "unsupported vmcnt");
}

}  // namespace pipe

}  // namespace stl
