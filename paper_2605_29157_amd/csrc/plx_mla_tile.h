// The 64-key LDS tile of the latent-cache decode kernels (gfx950) and what both of them need
// around it.
#pragma once
#include "plx_device.h"

namespace plx {

constexpr int kMlaDC = 512, kMlaDR = 64, kMlaDK = kMlaDC + kMlaDR;
constexpr int kMlaTileKeys = 64;
constexpr int kMlaKSteps = kMlaDK / 32;      // 18 score k-steps of 32 dimensions, the last two on the rope part
constexpr int kMlaLatBlocks = kMlaDC / 128;  // column blocks of the latent part
constexpr int kMlaNDB = 128 / 16;            // 16-dimension output blocks per wave
constexpr int kMlaPvSteps = kMlaTileKeys / 32;         // 32-key k-steps of the second contraction
// A tile is stored as four latent column blocks [64 rows][16 chunks of 8 dimensions] followed by
// the rope block [64 rows][8 chunks], chunks permuted inside their row (lds_chunk_slot).
constexpr int kMlaBlkChunks = kMlaTileKeys * 16;       // 16-byte chunks of one column block
constexpr int kMlaRopeChunks = kMlaTileKeys * (kMlaDR / 8);
constexpr int kMlaTileChunks = kMlaLatBlocks * kMlaBlkChunks + kMlaRopeChunks;
constexpr int kMlaLoadsPerWave = kMlaTileChunks / 64 / 4;  // wave-wide 1 KB loads per tile and wave
constexpr int kRowGroups = kMlaTileKeys / 4;           // loads per latent column block (4 rows each)
static_assert(kMlaTileChunks % 256 == 0 && kMlaLoadsPerWave == 18, "four waves fill a tile with whole loads");

// Rounds four fp32 values to bf16 (one half of an MFMA B operand) and adds the ROUNDED values to
// acc, so that row sums and numerators use identical weights.
__device__ __forceinline__ u32x2 pack4_bf16_accumulate(float p0, float p1, float p2, float p3, float &acc) {
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    bf16x2 a, b;
    a[0] = (__bf16)p0, a[1] = (__bf16)p1;
    b[0] = (__bf16)p2, b[1] = (__bf16)p3;
    acc = __builtin_amdgcn_fdot2_f32_bf16(a, ones, acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(b, ones, acc, false);
    return u32x2{__builtin_bit_cast(uint32_t, a), __builtin_bit_cast(uint32_t, b)};
}

}  // namespace plx
