// The 256 x 256 tile GEMM on four wavefronts: what its kernels share.  Included inside the
// translation unit's own namespace; the loop itself is gemm_w4_body.inc, included in the body
// of every kernel that runs it (the forward's expert GEMMs, the backward's row GEMMs), each
// with an epilogue of its own.
#pragma once

// ---------------------------------------------------------------- 256 x 256 GEMM, four wavefronts
// The same product as grouped_gemm_mfma_kernel for 256 x 256 output tiles, fp16 output and a
// contraction depth that is a multiple of 64, laid out for one wavefront per SIMD:
//  * four wavefronts of 128 x 128 (2 x 2): every operand fragment read from LDS feeds four
//    MFMAs (128 KB of LDS reads per 64-deep stage against 196 KB for eight wavefronts of
//    128 x 64); the 16 accumulators of a wavefront (256 registers) are pinned to AGPRs, which
//    leaves the 256 VGPRs to fragments and staging;
//  * TWO stages of global loads in flight in registers (2 x 64 VGPRs) beside the double-buffered
//    LDS tiles, through buffer loads whose per-lane byte offsets never change (the stage goes
//    into the scalar offset): no address arithmetic in the loop;
//  * one barrier per stage, and every memory instruction of a stage (32 LDS fragment reads,
//    16 LDS writes, 16 global loads per wavefront) issued singly between two MFMAs in a fixed
//    order: fragment reads one 16-deep step ahead, the LDS writes of the next stage spread
//    over the first three steps (all before the barrier), a register reloaded after it was
//    written.  The MFMAs are inline assembly so that the accumulators stay in AGPRs and the
//    order holds; nothing depends on an MFMA result before the loop ends.
//  * The tile leaves through LDS: every wavefront writes its 128 x 128 sub-tile to a patch of
//    its own and stores it as whole lines, 16 bytes per lane.
// Loads past the last stage fetch the last stage again (never used) instead of branching.
// Operand addresses are 32-bit byte offsets into two buffer resources (the tile's rows, or
// the whole token matrix when the rows are gathered through row_src; the expert's weight
// matrix), which the host checks fit.
#define MOE_LGKM0() asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory")
#define MOE_SB() __builtin_amdgcn_sched_barrier(0)
#define MOE_BAR()                                                                                 \
    do {                                                                                         \
        MOE_SB();                                                                                \
        __builtin_amdgcn_s_barrier();                                                            \
        MOE_SB();                                                                                \
    } while (0)

template <bool F16>
__device__ __forceinline__ void mfma_32x32x16_agpr(f32x16 &acc, const u32x4 &a, const u32x4 &b)
{
    if constexpr (F16)
        asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
    else
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

