// Score MFMAs as inline assembly with vector-register destinations (gfx950), shared by the
// prefill forward and backward kernels.
#pragma once
#include "plx_device.h"

namespace plx {

// The score MFMAs of the pipelined loop are emitted as inline assembly with VECTOR-register
// destinations: their results feed the exp arithmetic directly. (With the compiler's choice,
// accumulation registers, every score has to be copied out first, and such copies stall while
// MFMAs are in flight: measured +6 cycles per copy, ~100 copies per 64-key tile.) The compiler
// does not know these statements are MFMAs, so the two hazards it would otherwise cover are
// handled here: the first read of a finished score block is kept >= 16 issue slots behind its
// last MFMA (s_nop below; the ISA asks for 11 after an 8-pass MFMA), and operand order is
// pinned by the scheduling fences of the pipeline.
// An MFMA may not read a register that a vector-ALU instruction wrote less than two wait states
// before it (the hardware does not interlock this). For MFMAs the compiler knows about it keeps
// that distance itself; for these statements it cannot, and it does place copies directly in
// front of a statement's operands when it parks the Q/R fragments in accumulation registers.
// GUARD = true brings two wait states along. GUARD = false is for the steady-state loop, where
// the generated code has no such copy -- the build verifies that on the assembly it produced
// (asm_check.py) and fails otherwise.
// acc = A * B (first k-step) and acc += A * B, 32x32x16 bf16, all operands in vector registers.
template <bool GUARD>
__device__ __forceinline__ void mfma32_scores_first(f32x16 &acc, u32x4 a, u32x4 b) {
    // early clobber: the destination block must not share registers with A or B
    if constexpr (GUARD)
        asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "a"(b));
    else
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0 ; unguarded" : "=&v"(acc) : "v"(a), "a"(b));
}
template <bool GUARD>
__device__ __forceinline__ void mfma32_scores(f32x16 &acc, u32x4 a, u32x4 b) {
    if constexpr (GUARD)
        asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "a"(b));
    else
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0 ; unguarded" : "+v"(acc) : "v"(a), "a"(b));
}

}  // namespace plx
