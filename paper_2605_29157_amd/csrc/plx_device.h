// Device-side helpers shared by the gfx950 Parallax kernels (types, MFMA wrappers, lane
// exchange, bf16 packing, LDS tile addressing). Wave size is 64 everywhere.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace plx {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegInf = -__builtin_inff();

// D(16x16) += A(16x32) * B(32x16), bf16 operands, fp32 accumulate.
// Operand layout (lane l): A holds row l%16, k-elements 8*(l/16)..+7; B holds column l%16,
// the same k-elements; the accumulator holds column l%16, rows 4*(l/16)..+3.
__device__ __forceinline__ f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// D(32x32) += A(32x16) * B(16x32). Lane l: A row l%32, k-elements 8*(l/32)..+7; B column l%32,
// same k-elements; accumulator register r holds column l%32, row 8*(r/4) + 4*(l/32) + r%4.
__device__ __forceinline__ f32x16 mfma32(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Two fp32 -> one dword of two bf16 (round to nearest even), low half = a.
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    bf16x2 v;
    v[0] = (__bf16)a;
    v[1] = (__bf16)b;
    return __builtin_bit_cast(uint32_t, v);
}

// The two bf16 halves of a packed dword, widened back to fp32 (exact).
__device__ __forceinline__ float bf16_lo_f32(uint32_t packed) {
    return __builtin_bit_cast(float, packed << 16);
}
__device__ __forceinline__ float bf16_hi_f32(uint32_t packed) {
    return __builtin_bit_cast(float, packed & 0xffff0000u);
}
// Round eight fp32 values to bf16 -- one MFMA operand -- and add the ROUNDED values to acc
// (v_dot2_f32_bf16 against (1, 1): one instruction per packed pair). The pairs are built as
// bf16 vectors first and only then viewed as dwords: taking a dword of an integer vector and
// viewing it as a bf16 pair is miscompiled by this toolchain (all four dot products read the
// same register).
__device__ __forceinline__ u32x4 pack8_bf16_accumulate(float p0, float p1, float p2, float p3,
                                                      float p4, float p5, float p6, float p7,
                                                      float &acc) {
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    bf16x2 a, b, c, d;
    a[0] = (__bf16)p0, a[1] = (__bf16)p1;
    b[0] = (__bf16)p2, b[1] = (__bf16)p3;
    c[0] = (__bf16)p4, c[1] = (__bf16)p5;
    d[0] = (__bf16)p6, d[1] = (__bf16)p7;
    acc = __builtin_amdgcn_fdot2_f32_bf16(a, ones, acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(b, ones, acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(c, ones, acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(d, ones, acc, false);
    return u32x4{__builtin_bit_cast(uint32_t, a), __builtin_bit_cast(uint32_t, b),
                 __builtin_bit_cast(uint32_t, c), __builtin_bit_cast(uint32_t, d)};
}

// Transposing LDS read (ds_read_b64_tr_b16). Within each group of 16 lanes, lane i receives
// element i%4 of the 8 bytes addressed by lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4. With lane i
// addressing row i/4, elements 4*(i%4)..+3 of a row-major [4 rows][16 elements] block, lane i
// therefore gets column i: the four rows' values of element i.
__device__ __forceinline__ u32x2 lds_read_tr16(const void *generic_lds_ptr) {
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr_t;
    const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)generic_lds_ptr);
    return __builtin_bit_cast(u32x2, v);
}

__device__ __forceinline__ float xor_shuffle(float v, int mask) { return __shfl_xor(v, mask, 64); }

// max / sum over the four 16-lane rows of a wave (lanes l, l^16, l^32, l^48)
__device__ __forceinline__ float rows_max(float v) {
    v = fmaxf(v, xor_shuffle(v, 16));
    return fmaxf(v, xor_shuffle(v, 32));
}
__device__ __forceinline__ float rows_sum(float v) {
    v += xor_shuffle(v, 16);
    return v + xor_shuffle(v, 32);
}
// Sum over aligned groups of N = 8 or 16 consecutive lanes, every lane of a group receiving the
// total, by data-parallel-primitive moves inside a 16-lane row (no LDS round trip as with a lane
// shuffle): pairs and quads by quad permutations, then the mirrored half-row and row.
template <int N>
__device__ __forceinline__ float lane_group_sum(float v) {
    static_assert(N == 8 || N == 16, "groups inside one 16-lane row");
    auto moved = [](float x, auto ctrl) {
        const int y = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value, 0xf, 0xf, true);
        return __builtin_bit_cast(float, y);
    };
    v += moved(v, std::integral_constant<int, 0xB1>{});   // quad_perm [1, 0, 3, 2]: lane ^ 1
    v += moved(v, std::integral_constant<int, 0x4E>{});   // quad_perm [2, 3, 0, 1]: lane ^ 2
    v += moved(v, std::integral_constant<int, 0x141>{});  // row_half_mirror: lane i <-> 7 - i of its half-row
    if constexpr (N == 16) v += moved(v, std::integral_constant<int, 0x140>{});  // row_mirror: i <-> 15 - i
    return v;
}

// max / sum over the two 32-lane halves of a wave
__device__ __forceinline__ float halves_max(float v) { return fmaxf(v, xor_shuffle(v, 32)); }
__device__ __forceinline__ float halves_sum(float v) { return v + xor_shuffle(v, 32); }

// LDS tiles hold rows of D bf16 as 16-byte chunks (8 elements). Chunk c of row `row` is stored
// at chunk slot row*CPR + (c ^ f(row)), CPR = D/8. f swaps the two low 2-bit fields of the row
// index (D = 128) so that all three access patterns spread evenly over the LDS banks:
// the coalesced row-wise write (16 lanes = one row), the K operand read (16 or 32 consecutive
// rows, one chunk) and the V^T operand read (4 consecutive rows x a few chunks).
template <int D>
__device__ __forceinline__ int lds_row_swizzle(int row) {
    if constexpr (D == 128) {
        return ((row & 3) << 2) | ((row >> 2) & 3);
    } else {  // D == 64: two rows share 256 bytes; permute on row/2
        const int y = (row >> 1) & 7;
        return ((y & 1) << 2) | ((y >> 1) & 3);
    }
}
template <int D>
__device__ __forceinline__ int lds_chunk_slot(int row, int chunk) {
    constexpr int CPR = D / 8;
    return row * CPR + (chunk ^ lds_row_swizzle<D>(row));
}

}  // namespace plx
