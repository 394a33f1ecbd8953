// RMSNorm over the head dimension followed by rotary position embedding, for up to three
// tensors (q, rho, k of one layer) in ONE launch -- the operations the paper's language-model
// runs apply to q, k and rho in front of the attention call (experiment setup of Sec. 5 and the
// backbone appendix: RMSNorm on q, k, rho; RoPE with base 1e6). Standard formulas:
//     y = x / sqrt(mean_c(x_c^2) + eps) * gamma
//     (y_2i, y_2i+1) rotated by pos * theta^(-2i/d)   (adjacent pairs)
// HBM bound: every element is read once and written once, 16 bytes per lane; the lanes of one row
// (d * element size / 16 of them) share the sum of squares through lane shuffles. The angle is
// formed and reduced modulo 2 pi in double precision (pos * frequency reaches 1e5 and more, where
// fp32 would lose the fraction), sine and cosine are taken in single precision -- once per
// (position, pair), for all heads of all tensors.
#include "plx_device.h"
#include "plx_kernels.h"

namespace plx {

template <typename T>
struct Chunk;  // 16 bytes of a row
template <>
struct Chunk<__bf16> {
    static constexpr int E = 8;
    u32x4 raw;
    __device__ float get(int e) const { return (e & 1) ? bf16_hi_f32(raw[e >> 1]) : bf16_lo_f32(raw[e >> 1]); }
    __device__ void set_pair(int j, float a, float b) { raw[j] = pack_bf16(a, b); }
};
template <>
struct Chunk<float> {
    static constexpr int E = 4;
    f32x4 raw;
    __device__ float get(int e) const { return raw[e]; }
    __device__ void set_pair(int j, float a, float b) { raw[2 * j] = a, raw[2 * j + 1] = b; }
};

// A wave owns 64 / (lanes per row) consecutive positions of one sequence and walks over a chunk
// of the heads of every tensor at those positions: sine and cosine of a (position, pair) are
// computed once per wave. With many positions a wave takes all heads (the trigonometry is then
// done once per position); with few (a decode step has one row per sequence) the heads are
// dealt over more waves, because a wave that walks 40 heads alone is a chain of 10 dependent
// memory round trips (measured: 22 us for 8 x 16 x 1 rows, against 4 us in chunks of 4 heads).
template <typename T>
__global__ __launch_bounds__(256) void norm_rope_kernel(NormRopeParams p) {
    constexpr int E = Chunk<T>::E;
    constexpr int UNROLL = 4;                      // heads in flight per lane
    const int lpr = p.d / E;                       // lanes per row (a power of two <= 64)
    const int rows_per_wave = 64 / lpr;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lr = lane % lpr;                     // this lane's chunk of its row
    const int t_per_seq = (p.T + rows_per_wave - 1) / rows_per_wave;  // position groups per sequence
    const int64_t wid_all = (int64_t)blockIdx.x * 4 + wave;
    if (wid_all >= (int64_t)p.B * t_per_seq * p.head_chunks) return;   // whole waves only: no barrier below
    const int hchunk = (int)(wid_all % p.head_chunks);
    const int64_t wid = wid_all / p.head_chunks;
    const int b = (int)(wid / t_per_seq);
    const int t = (int)(wid % t_per_seq) * rows_per_wave + lane / lpr;
    const bool live = t < p.T;
    const int ld_t = live ? t : p.T - 1;

    float cs[E / 2], sn[E / 2];
    if (p.table != nullptr) {  // (uniform) from the caller's table: E floats = this lane's E / 2 pairs
        const int64_t pos = min(max((p.pos0 ? p.pos0[b] : 0) + ld_t, 0), p.n_pos - 1);
        const float *e = p.table + (pos * (p.d / 2) + lr * (E / 2)) * 2;
#pragma unroll
        for (int j = 0; j < E / 2; j += 2) {
            const f32x4 v = *(const f32x4 *)(e + 2 * j);
            cs[j] = v[0], sn[j] = v[1], cs[j + 1] = v[2], sn[j + 1] = v[3];
        }
    } else {
        const double pos = (double)((p.pos0 ? p.pos0[b] : 0) + ld_t);
        const double log2_theta = log2((double)p.theta);
#pragma unroll
        for (int j = 0; j < E / 2; ++j) {
            const int dim = lr * E + 2 * j;  // even dimension of the pair
            double ang = pos * exp2(-(double)dim / (double)p.d * log2_theta);
            ang -= floor(ang * 0.15915494309189535) * 6.283185307179586;  // modulo 2 pi
            sincosf((float)ang, &sn[j], &cs[j]);
        }
    }
    const float inv_d = 1.0f / (float)p.d;
    for (int i = 0; i < p.n_tensors; ++i) {
        const NormRopeTensor ten = p.t[i];
        float gam[E];
#pragma unroll
        for (int e = 0; e < E; ++e) gam[e] = ten.gamma[lr * E + e];
        const decltype(Chunk<T>::raw) *src = (const decltype(Chunk<T>::raw) *)ten.x;
        decltype(Chunk<T>::raw) *dst = (decltype(Chunk<T>::raw) *)ten.y;
        const int h_end = min(ten.H, (hchunk + 1) * p.heads_per_wave);
        for (int h0 = hchunk * p.heads_per_wave; h0 < h_end; h0 += UNROLL) {
            Chunk<T> c[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {  // all loads of the trip first
                const int h = min(h0 + u, h_end - 1);
                c[u].raw = src[(((int64_t)b * ten.H + h) * p.T + ld_t) * lpr + lr];
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                float ss = 0.f;
#pragma unroll
                for (int e = 0; e < E; ++e) ss = fmaf(c[u].get(e), c[u].get(e), ss);
                for (int off = 1; off < lpr; off <<= 1) ss += __shfl_xor(ss, off, 64);
                const float rinv = 1.0f / sqrtf(ss * inv_d + p.eps);
#pragma unroll
                for (int j = 0; j < E / 2; ++j) {
                    float y0 = c[u].get(2 * j) * rinv * gam[2 * j];
                    float y1 = c[u].get(2 * j + 1) * rinv * gam[2 * j + 1];
                    if (ten.rope) {
                        const float r0 = y0 * cs[j] - y1 * sn[j], r1 = y0 * sn[j] + y1 * cs[j];
                        y0 = r0, y1 = r1;
                    }
                    c[u].set_pair(j, y0, y1);
                }
                if (live && h0 + u < h_end)
                    dst[(((int64_t)b * ten.H + h0 + u) * p.T + t) * lpr + lr] = c[u].raw;
            }
        }
    }
}

// (cos, sin) of pos * theta^(-2i/d), one thread per (position, pair): the same double-precision
// angle reduction as above, so that the attention kernels that apply the rotation themselves
// (from this table) see the values this file's kernel would have used.
__global__ __launch_bounds__(256) void rope_table_kernel(float *table, int n_pos, int d, float theta) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int half = d / 2;
    if (idx >= (int64_t)n_pos * half) return;
    const int pos = (int)(idx / half), i = (int)(idx % half);
    double ang = (double)pos * exp2(-(double)(2 * i) / (double)d * log2((double)theta));
    ang -= floor(ang * 0.15915494309189535) * 6.283185307179586;  // modulo 2 pi
    float sn, cs;
    sincosf((float)ang, &sn, &cs);
    table[2 * idx] = cs;
    table[2 * idx + 1] = sn;
}

hipError_t launch_rope_table(float *table, int n_pos, int d, float theta, hipStream_t stream) {
    const int64_t blocks = ((int64_t)n_pos * (d / 2) + 255) / 256;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, table, n_pos, d, theta);
    return hipGetLastError();
}

hipError_t launch_norm_rope(const NormRopeParams &p_in, bool f32, hipStream_t stream) {
    NormRopeParams p = p_in;
    const int elems = f32 ? 4 : 8;
    const int rows_per_wave = 64 / (p.d / elems);
    const int64_t groups = (int64_t)p.B * ((p.T + rows_per_wave - 1) / rows_per_wave);
    // heads per wave: all of them when there are position groups enough to fill the chip
    // (about four waves per SIMD), else chunks, down to the four heads a wave has in flight
    int max_h = 1;
    for (int i = 0; i < p.n_tensors; ++i) max_h = p.t[i].H > max_h ? p.t[i].H : max_h;
    int hpw = max_h;
    while (hpw > 4 && groups * ((max_h + hpw - 1) / hpw) < 4096) hpw = (hpw + 1) / 2;
    hpw = (hpw + 3) / 4 * 4;
    p.heads_per_wave = hpw;
    p.head_chunks = (max_h + hpw - 1) / hpw;
    const int64_t waves = groups * p.head_chunks;
    const int64_t blocks = (waves + 3) / 4;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (f32)
        hipLaunchKernelGGL(norm_rope_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, stream, p);
    else
        hipLaunchKernelGGL(norm_rope_kernel<__bf16>, dim3((unsigned)blocks), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace plx
