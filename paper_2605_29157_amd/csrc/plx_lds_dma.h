// Direct global -> LDS tile loads for the gfx950 Parallax kernels (global_load_lds_dwordx4) and
// the wait + barrier that publishes the landed tiles.
#pragma once
#include "plx_device.h"

namespace plx {

// Tile loads go global -> LDS directly (global_load_lds_dwordx4: LDS address = M0 + 16 * lane).
// They are emitted as inline assembly: through the compiler builtin, the first LDS read after
// a tile load waits for that load to land (the compiler assumes every LDS read may alias the
// incoming tile), which exposes the full memory latency once per tile. In this kernel a tile
// in flight is never read before the workgroup barrier that publishes it, so the only wait
// needed is the explicit vmcnt(0) in front of that barrier (tile_barrier below).
// LANES < 64: only lanes 0..LANES-1 load (a shorter piece): EXEC is narrowed around the
// instruction.
template <int LANES = 64>
__device__ __forceinline__ void tile_load16(const void *gptr, uint32_t lds_byte_addr) {
    static_assert(LANES == 64 || LANES == 32 || LANES == 16, "piece sizes in use");
    const uint32_t m0v = __builtin_amdgcn_readfirstlane(lds_byte_addr);
    uint32_t saved_m0;  // M0 belongs to the compiler: put its value back
    uint64_t saved_exec;
    if constexpr (LANES < 64)
        asm volatile(
            "s_mov_b32 %0, m0\n\t"
            "s_mov_b64 %1, exec\n\t"
            "s_mov_b64 exec, %4\n\t"
            "s_mov_b32 m0, %3\n\t"
            "global_load_lds_dwordx4 %2, off\n\t"
            "s_mov_b64 exec, %1\n\t"
            "s_mov_b32 m0, %0"
            : "=&s"(saved_m0), "=&s"(saved_exec)
            : "v"(gptr), "s"(m0v), "n"((1ull << (LANES % 64)) - 1ull)
            : "memory");
    else
        asm volatile(
            "s_mov_b32 %0, m0\n\t"
            "s_mov_b32 m0, %2\n\t"
            "global_load_lds_dwordx4 %1, off\n\t"
            "s_mov_b32 m0, %0"
            : "=&s"(saved_m0)
            : "v"(gptr), "s"(m0v)
            : "memory");
}
// Same load with a wave-uniform tile base (scalar registers) plus a 32-bit per-lane byte offset:
// no per-lane 64-bit address arithmetic. The statement writes LDS, hence the memory clobber. M0
// is left modified and cannot be declared: this compiler treats M0 as a reserved register and
// answers an "m0" clobber with "may lead to undefined behaviour". What holds instead: nothing
// the compiler emits for these kernels touches M0 (no other LDS-DMA, no GWS / message /
// relative-index instructions), and the build verifies exactly that on the generated assembly
// of every file that includes this header (asm_check.py), failing otherwise.
template <bool QUARTER = false>
__device__ __forceinline__ void tile_load16_uniform(uint32_t lane_byte_off, const void *tile_base,
                                                    uint32_t lds_byte_addr) {
    uint64_t saved_exec;
    if constexpr (QUARTER)
        asm volatile(
            "s_mov_b64 %0, exec\n\t"
            "s_mov_b64 exec, 0xffff\n\t"
            "s_mov_b32 m0, %3\n\t"
            "global_load_lds_dwordx4 %1, %2\n\t"
            "s_mov_b64 exec, %0"
            : "=&s"(saved_exec)
            : "v"(lane_byte_off), "s"(tile_base), "s"(lds_byte_addr)
            : "memory");
    else
        asm volatile(
            "s_mov_b32 m0, %2\n\t"
            "global_load_lds_dwordx4 %0, %1"
            :
            : "v"(lane_byte_off), "s"(tile_base), "s"(lds_byte_addr)
            : "memory");
}
// The same load under a wave-uniform execution mask (`on` = -1: all lanes, 0: none): a loop body that issues
// the next tile's loads between its matrix instructions stays free of branches when there is no
// next tile to fetch -- with no lane enabled the instruction does nothing.
__device__ __forceinline__ void tile_load16_uniform_if(int32_t on, uint32_t lane_byte_off, const void *tile_base,
                                                       uint32_t lds_byte_addr) {
    on = __builtin_amdgcn_readfirstlane(on);  // (a scalar register, whatever the compiler kept it in)
    uint64_t saved_exec;
    asm volatile(
        "s_mov_b64 %0, exec\n\t"
        "s_mov_b32 exec_lo, %4\n\t"
        "s_mov_b32 exec_hi, %4\n\t"
        "s_mov_b32 m0, %3\n\t"
        "global_load_lds_dwordx4 %1, %2\n\t"
        "s_mov_b64 exec, %0"
        : "=&s"(saved_exec)
        : "v"(lane_byte_off), "s"(tile_base), "s"(lds_byte_addr), "s"(on)
        : "memory");
}
// Wait until at most PENDING of this wave's tile loads are still in flight (loads complete in
// issue order), then the workgroup barrier that publishes the landed tiles.
template <int PENDING = 0>
__device__ __forceinline__ void tile_barrier() {
    static_assert(PENDING >= 0 && PENDING < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PENDING) : "memory");
    __syncthreads();
}
__device__ __forceinline__ uint32_t lds_byte_address(const void *p) {
    typedef const char __attribute__((address_space(3))) * lds_cptr_t;
    return (uint32_t)(uintptr_t)(lds_cptr_t)p;
}

}  // namespace plx
