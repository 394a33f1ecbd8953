// Plain streaming kernels: a device-to-device copy (calibrates hardware byte counters against
// a known size) and a read-only stream (achievable HBM read bandwidth next to the attention
// kernels). 16 bytes per lane, grid-stride. And a register-only loop of bf16 MFMAs: the matrix
// rate the chip sustains when nothing else limits it (no memory, no LDS, no vector work).
#include "plx_device.h"
#include "plx_kernels.h"

namespace plx {

__global__ __launch_bounds__(256) void util_copy_kernel(u32x4 *dst, const u32x4 *src, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        dst[i] = src[i];
}

__global__ __launch_bounds__(256) void util_read_kernel(const u32x4 *src, size_t n, u32x4 *sink) {
    const size_t stride = (size_t)gridDim.x * blockDim.x * 4;
    u32x4 acc = {0u, 0u, 0u, 0u};
    // four independent 16-byte loads per lane and trip keep several KB per wave in flight
    for (size_t i = (size_t)blockIdx.x * blockDim.x * 4 + threadIdx.x; i < n; i += stride) {
        u32x4 a = src[i];
        u32x4 b = i + 256 < n ? src[i + 256] : u32x4{0u, 0u, 0u, 0u};
        u32x4 c = i + 512 < n ? src[i + 512] : u32x4{0u, 0u, 0u, 0u};
        u32x4 d = i + 768 < n ? src[i + 768] : u32x4{0u, 0u, 0u, 0u};
        acc ^= a ^ b ^ c ^ d;
    }
    // fold the workgroup into one value so the loads cannot be dropped
    __shared__ u32x4 part[256];
    part[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        u32x4 t = {0u, 0u, 0u, 0u};
        for (int j = 0; j < 256; ++j) t ^= part[j];
        sink[blockIdx.x] = t;
    }
}

// The same stream with a chosen grid and eight 16-byte loads per lane in flight (32 KB per
// workgroup and trip): few fat workgroups (one per compute unit) up to many thin ones.
__global__ __launch_bounds__(256) void util_read_grid_kernel(const u32x4 *src, size_t n, u32x4 *sink) {
    const size_t stride = (size_t)gridDim.x * 2048;
    const u32x4 zero = {0u, 0u, 0u, 0u};
    u32x4 acc = zero;
    for (size_t i = (size_t)blockIdx.x * 2048 + threadIdx.x; i < n; i += stride) {
        u32x4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = i + 256 * j < n ? src[i + 256 * j] : zero;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc ^= v[j];
    }
    __shared__ u32x4 part[256];
    part[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        u32x4 t = zero;
        for (int j = 0; j < 256; ++j) t ^= part[j];
        sink[blockIdx.x] = t;
    }
}

// Eight independent accumulation chains per wave: an MFMA never waits for the one before it, so
// one wave per SIMD keeps the matrix pipe full. Operands are fixed pseudo-random bf16 values in
// (-1, 1) (all-zero operands would draw less power than real data and flatter the clock).
__global__ __launch_bounds__(256) void util_mfma_kernel(int iters, float *sink) {
    const unsigned tid = threadIdx.x + blockIdx.x * 256u;
    u32x4 a[4], b[2];
#pragma unroll
    for (int j = 0; j < 6; ++j) {
        u32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            unsigned x = (tid * 6u + j) * 4u + e;
            x ^= x >> 16, x *= 0x7feb352du, x ^= x >> 15, x *= 0x846ca68bu, x ^= x >> 16;
            // two bf16 values: sign and 7 mantissa bits from the hash, exponent of [0.5, 1)
            v[e] = (x & 0x807f807fu) | 0x3f003f00u;
        }
        if (j < 4)
            a[j] = v;
        else
            b[j - 4] = v;
    }
    f32x16 acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = mfma32(a[j & 3], b[j >> 2], acc[j]);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[j][r];
    sink[tid] = s;
}

hipError_t launch_util_mfma(int workgroups, int iters, void *sink, hipStream_t stream) {
    hipLaunchKernelGGL(util_mfma_kernel, dim3((unsigned)workgroups), dim3(256), 0, stream, iters, (float *)sink);
    return hipGetLastError();
}

hipError_t launch_util_copy(void *dst, const void *src, size_t bytes, hipStream_t stream) {
    const size_t n = bytes / 16;
    if (n == 0) return hipSuccess;
    const size_t want = (n + 255) / 256;
    const unsigned blocks = (unsigned)(want < 8192 ? want : 8192);
    hipLaunchKernelGGL(util_copy_kernel, dim3(blocks), dim3(256), 0, stream, (u32x4 *)dst,
                       (const u32x4 *)src, n);
    return hipGetLastError();
}

hipError_t launch_util_read(const void *src, size_t bytes, void *sink, hipStream_t stream) {
    const size_t n = bytes / 16;
    hipLaunchKernelGGL(util_read_kernel, dim3(kReadSinkSlots), dim3(256), 0, stream,
                       (const u32x4 *)src, n, (u32x4 *)sink);
    return hipGetLastError();
}

hipError_t launch_util_read_grid(const void *src, size_t bytes, void *sink, int workgroups, hipStream_t stream) {
    hipLaunchKernelGGL(util_read_grid_kernel, dim3((unsigned)workgroups), dim3(256), 0, stream,
                       (const u32x4 *)src, bytes / 16, (u32x4 *)sink);
    return hipGetLastError();
}

}  // namespace plx
