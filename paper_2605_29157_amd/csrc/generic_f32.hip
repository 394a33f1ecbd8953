// fp32 Parallax forward for decode and prefill: a plain, untuned correctness path
// (one workgroup per query row, vector ALU only). It follows Algorithm 1 of the paper
// (Sec. 3.3) over key tiles of 256 with the running state (m, d1, d2, O1, O2) and closes with
// O1/d1 * (1 + d2/d1) - O2/d1. The tuned kernels are the bf16 MFMA ones.
#include "plx_device.h"
#include "plx_kernels.h"

namespace plx {

struct GenericParams {
    const float *q, *r, *k, *v;
    float *o;
    const int32_t *seq_lens;
    int32_t B, Hq, Hkv, G, Tq, Lk, d;
    int64_t qs[3], rs[3], ks[3], vs[3], os[3];
    float scale;
    int32_t causal, use_r;
    const int32_t *block_table;  // paged decode cache (see DecodeParams); NULL = contiguous
    int32_t page_size, table_stride, num_pages;
    int32_t tail_rows;  // decode with Tq rows: row i sees the keys before len_b - (Tq - 1 - i)
    int32_t window;     // > 0: a row sees only the last `window` of its keys
    float *vbar;        // row cache of the backward pass (prefill only), laid out like o; or NULL
    float *row_stats;   // [B, Hq, Tq, 2]: log-sum-exp (exp2 domain), ubar
};

constexpr int kGenThreads = 256;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__global__ __launch_bounds__(kGenThreads) void generic_f32_kernel(GenericParams p) {
    __shared__ float sq[256], sr[256], sp1[kGenThreads], sp2[kGenThreads];
    __shared__ float red[3][kGenThreads / 64];

    const int t = threadIdx.x, wv = t >> 6, ln = t & 63;
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int hk = h / p.G, d = p.d;
    int n_keys;
    if (p.causal)
        n_keys = i + 1 + (p.Lk - p.Tq);  // the query rows are the last Tq positions
    else
        n_keys = p.seq_lens ? min(max(p.seq_lens[b], 0), p.Lk) : p.Lk;
    if (p.tail_rows) n_keys = max(n_keys - (p.Tq - 1 - i), 0);
    const int j_first = (p.window > 0 && n_keys > p.window) ? n_keys - p.window : 0;

    const float *qrow = p.q + b * p.qs[0] + h * p.qs[1] + i * p.qs[2];
    const float *rrow = p.r ? p.r + b * p.rs[0] + h * p.rs[1] + i * p.rs[2] : nullptr;
    const bool paged = p.block_table != nullptr;
    const float *kb = p.k + (paged ? 0 : b * p.ks[0]) + hk * p.ks[1];
    const float *vb = p.v + (paged ? 0 : b * p.vs[0]) + hk * p.vs[1];
    // element offset of key j's row inside kb / vb (stride0 = page stride when paged)
    auto row_off = [&](int j, const int64_t *st) -> int64_t {
        if (!paged) return (int64_t)j * st[2];
        const int pg = min(max(p.block_table[(int64_t)b * p.table_stride + j / p.page_size], 0),
                           p.num_pages - 1);
        return (int64_t)pg * st[0] + (int64_t)(j % p.page_size) * st[2];
    };
    if (t < d) {
        sq[t] = qrow[t];
        sr[t] = (p.use_r && rrow) ? rrow[t] : 0.f;
    }
    __syncthreads();

    const float scale_log2 = p.scale * kLog2e;
    float m_run = kNegInf, d1 = 0.f, d2 = 0.f, o1 = 0.f, o2 = 0.f;  // o1/o2: dimension t

    for (int j0 = j_first; j0 < n_keys; j0 += kGenThreads) {
        const int j = j0 + t;
        const bool valid = j < n_keys;
        float s1 = kNegInf, s2 = 0.f;
        if (valid) {
            const float *kj = kb + row_off(j, p.ks);
            float a1 = 0.f, a2 = 0.f;
            for (int c = 0; c < d; ++c) {
                const float kv = kj[c];
                a1 = fmaf(sq[c], kv, a1);
                a2 = fmaf(sr[c], kv, a2);
            }
            s1 = a1 * scale_log2;
            s2 = a2;
        }
        float tm = wave_max(s1);
        if (ln == 0) red[0][wv] = tm;
        __syncthreads();
        tm = fmaxf(fmaxf(red[0][0], red[0][1]), fmaxf(red[0][2], red[0][3]));
        const float m_new = fmaxf(m_run, tm);  // finite: the tile has at least one valid key
        const float alpha = exp2f(m_run - m_new);
        m_run = m_new;
        const float p1 = valid ? exp2f(s1 - m_new) : 0.f;
        const float p2 = valid ? p1 * s2 : 0.f;
        sp1[t] = p1;
        sp2[t] = p2;
        const float w1 = wave_sum(p1), w2 = wave_sum(p2);
        if (ln == 0) {
            red[1][wv] = w1;
            red[2][wv] = w2;
        }
        __syncthreads();
        d1 = alpha * d1 + (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
        d2 = alpha * d2 + (red[2][0] + red[2][1]) + (red[2][2] + red[2][3]);
        if (t < d) {
            o1 *= alpha;
            o2 *= alpha;
            const int n = min(kGenThreads, n_keys - j0);
            for (int jj = 0; jj < n; ++jj) {
                const float vv = vb[row_off(j0 + jj, p.vs) + t];
                o1 = fmaf(sp1[jj], vv, o1);
                o2 = fmaf(sp2[jj], vv, o2);
            }
        }
        __syncthreads();  // sp1/sp2/red are rewritten by the next tile
    }

    if (t < d) {
        float out = 0.f;  // empty key set: zeros
        if (d1 > 0.f) out = (o1 / d1) * (1.f + d2 / d1) - o2 / d1;
        p.o[b * p.os[0] + h * p.os[1] + i * p.os[2] + t] = out;
        if (p.row_stats) p.vbar[b * p.os[0] + h * p.os[1] + i * p.os[2] + t] = d1 > 0.f ? o1 / d1 : 0.f;
    }
    if (p.row_stats && t == 0) {
        float *st = p.row_stats + (((int64_t)b * p.Hq + h) * p.Tq + i) * 2;
        st[0] = d1 > 0.f ? m_run + log2f(d1) : kNegInf;
        st[1] = d1 > 0.f ? d2 / d1 : 0.f;
    }
}

static hipError_t launch_generic(const GenericParams &g, hipStream_t stream) {
    const dim3 grid(g.Tq, g.Hq, g.B);
    hipLaunchKernelGGL(generic_f32_kernel, grid, dim3(kGenThreads), 0, stream, g);
    return hipGetLastError();
}

hipError_t launch_decode_f32(const DecodeParams &p, hipStream_t stream) {
    GenericParams g{};
    g.q = (const float *)p.q;
    g.r = (const float *)p.r;
    g.k = (const float *)p.k;
    g.v = (const float *)p.v;
    g.o = (float *)p.o;
    g.seq_lens = p.seq_lens;
    g.B = p.B, g.Hq = p.Hq, g.Hkv = p.Hkv, g.G = p.G, g.Tq = p.Tq, g.Lk = p.Lmax, g.d = p.d;
    g.qs[0] = g.rs[0] = g.os[0] = (int64_t)p.Hq * p.Tq * p.d;
    g.qs[1] = g.rs[1] = g.os[1] = (int64_t)p.Tq * p.d;
    g.qs[2] = g.rs[2] = g.os[2] = p.d;
    g.tail_rows = 1;
    g.ks[0] = p.ksb, g.ks[1] = p.ksh, g.ks[2] = p.ksl;
    g.vs[0] = p.vsb, g.vs[1] = p.vsh, g.vs[2] = p.vsl;
    g.scale = p.scale, g.causal = 0, g.use_r = p.use_r;
    g.window = p.window;
    g.block_table = p.block_table;
    g.page_size = p.page_size, g.table_stride = p.table_stride, g.num_pages = p.num_pages;
    return launch_generic(g, stream);
}

hipError_t launch_prefill_f32(const PrefillParams &p, hipStream_t stream) {
    GenericParams g{};
    g.q = (const float *)p.q;
    g.r = (const float *)p.r;
    g.k = (const float *)p.k;
    g.v = (const float *)p.v;
    g.o = (float *)p.o;
    g.seq_lens = nullptr;
    g.B = p.B, g.Hq = p.Hq, g.Hkv = p.Hkv, g.G = p.G, g.Tq = p.T, g.Lk = p.Tk, g.d = p.d;
    for (int a = 0; a < 3; ++a) {
        g.qs[a] = p.qs[a], g.rs[a] = p.rs[a], g.ks[a] = p.ks[a], g.vs[a] = p.vs[a];
        g.os[a] = p.os[a];
    }
    g.scale = p.scale, g.causal = p.causal, g.use_r = p.use_r;
    g.window = p.window;
    g.vbar = (float *)p.vbar, g.row_stats = p.row_stats;
    return launch_generic(g, stream);
}

// ---- fp32 backward (closed forms of the paper's App. D): plain, untuned correctness path ------
// Row kernel: one workgroup per query row; tau = dO.o and beta = dO.vbar first, then key tiles of
// 256 (one key per thread for p, u, a; one output dimension per thread for the sums over keys).
// It also leaves (lse, ubar, tau, beta) of its row in the workspace for the column kernel.
__global__ __launch_bounds__(kGenThreads) void generic_bwd_rows_f32_kernel(PrefillBwdParams p) {
    __shared__ float sq[256], sr[256], sg[256], s1s[kGenThreads], s2s[kGenThreads];
    __shared__ float red[2][kGenThreads / 64];
    const int t = threadIdx.x, wv = t >> 6, ln = t & 63;
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int hk = h / p.G, d = p.d, off = p.Tk - p.T;
    const int64_t row = ((int64_t)b * p.Hq + h) * p.T + i;
    const float *k = (const float *)p.k + ((int64_t)b * p.Hkv + hk) * p.Tk * d;
    const float *v = (const float *)p.v + ((int64_t)b * p.Hkv + hk) * p.Tk * d;
    float tau = 0.f, beta = 0.f;
    if (t < d) {
        sq[t] = ((const float *)p.q)[row * d + t];
        sr[t] = ((const float *)p.r)[row * d + t];
        sg[t] = ((const float *)p.d_o)[row * d + t];
        tau = sg[t] * ((const float *)p.o)[row * d + t];
        beta = sg[t] * ((const float *)p.vbar)[row * d + t];
    }
    tau = wave_sum(tau), beta = wave_sum(beta);
    if (ln == 0) red[0][wv] = tau, red[1][wv] = beta;
    __syncthreads();
    tau = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
    beta = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    const float lse = p.row_stats[2 * row], ubar = p.row_stats[2 * row + 1];
    if (t == 0) ((f32x4 *)p.row_cache)[row] = f32x4{lse, ubar, tau, beta};
    const float scale_log2 = p.scale * kLog2e;
    const int n_keys = p.causal ? min(i + 1 + off, p.Tk) : p.Tk;
    const int j_first = (p.window > 0 && n_keys > p.window) ? n_keys - p.window : 0;
    float dq = 0.f, dr = 0.f;  // dimension t
    for (int j0 = j_first; j0 < n_keys; j0 += kGenThreads) {
        const int j = j0 + t;
        float g1 = 0.f, g2 = 0.f;
        if (j < n_keys) {
            float a1 = 0.f, a2 = 0.f, a3 = 0.f;
            for (int c = 0; c < d; ++c) {
                const float kv = k[(int64_t)j * d + c];
                a1 = fmaf(sq[c], kv, a1);
                a2 = fmaf(sr[c], kv, a2);
                a3 = fmaf(sg[c], v[(int64_t)j * d + c], a3);
            }
            const float pr = exp2f(a1 * scale_log2 - lse);
            const float dlt = a3 - beta;
            g1 = pr * (a3 - tau + (ubar - a2) * dlt);
            g2 = -pr * dlt;
        }
        s1s[t] = g1, s2s[t] = g2;
        __syncthreads();
        if (t < d) {
            const int n = min(kGenThreads, n_keys - j0);
            for (int jj = 0; jj < n; ++jj) {
                const float kv = k[(int64_t)(j0 + jj) * d + t];
                dq = fmaf(s1s[jj], kv, dq);
                dr = fmaf(s2s[jj], kv, dr);
            }
        }
        __syncthreads();
    }
    if (t < d) {
        ((float *)p.dq)[row * d + t] = dq * p.scale;
        ((float *)p.dr)[row * d + t] = dr;
    }
}

// Column kernel: one workgroup per key; rows of every query head of the group in tiles of 256.
__global__ __launch_bounds__(kGenThreads) void generic_bwd_cols_f32_kernel(PrefillBwdParams p) {
    __shared__ float sk[256], sv[256], s1s[kGenThreads], s2s[kGenThreads], sws[kGenThreads];
    const int t = threadIdx.x;
    const int j = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
    const int d = p.d, off = p.Tk - p.T;
    const int64_t krow = ((int64_t)b * p.Hkv + hk) * p.Tk + j;
    if (t < d) {
        sk[t] = ((const float *)p.k)[krow * d + t];
        sv[t] = ((const float *)p.v)[krow * d + t];
    }
    __syncthreads();
    const float scale_log2 = p.scale * kLog2e;
    const int i_lo = p.causal ? max(j - off, 0) : 0;  // rows that see key j: i_lo .. i_end - 1
    const int i_end = p.window > 0 ? min(p.T, max(j - off + p.window, 0)) : p.T;
    float dk = 0.f, dv = 0.f;  // dimension t
    for (int g = 0; g < p.G; ++g) {
        const int64_t head = ((int64_t)b * p.Hq + hk * p.G + g) * p.T;
        const float *q = (const float *)p.q + head * d, *r = (const float *)p.r + head * d;
        const float *go = (const float *)p.d_o + head * d;
        for (int i0 = i_lo; i0 < i_end; i0 += kGenThreads) {
            const int i = i0 + t;
            float g1 = 0.f, g2 = 0.f, w = 0.f;
            if (i < i_end) {
                float a1 = 0.f, a2 = 0.f, a3 = 0.f;
                for (int c = 0; c < d; ++c) {
                    a1 = fmaf(q[(int64_t)i * d + c], sk[c], a1);
                    a2 = fmaf(r[(int64_t)i * d + c], sk[c], a2);
                    a3 = fmaf(go[(int64_t)i * d + c], sv[c], a3);
                }
                const f32x4 rc = ((const f32x4 *)p.row_cache)[head + i];  // (lse, ubar, tau, beta)
                const float pr = exp2f(a1 * scale_log2 - rc[0]);
                const float um = rc[1] - a2, dlt = a3 - rc[3];
                w = pr * (1.f + um);
                g1 = pr * (a3 - rc[2] + um * dlt) * p.scale;
                g2 = -pr * dlt;
            }
            s1s[t] = g1, s2s[t] = g2, sws[t] = w;
            __syncthreads();
            if (t < d) {
                const int n = min(kGenThreads, i_end - i0);
                for (int ii = 0; ii < n; ++ii) {
                    const int64_t e = (int64_t)(i0 + ii) * d + t;
                    dk = fmaf(s1s[ii], q[e], dk);
                    dk = fmaf(s2s[ii], r[e], dk);
                    dv = fmaf(sws[ii], go[e], dv);
                }
            }
            __syncthreads();
        }
    }
    if (t < d) {
        ((float *)p.dk)[krow * d + t] = dk;
        ((float *)p.dv)[krow * d + t] = dv;
    }
}

hipError_t launch_prefill_bwd_f32(const PrefillBwdParams &p, hipStream_t stream) {
    hipLaunchKernelGGL(generic_bwd_rows_f32_kernel, dim3(p.T, p.Hq, p.B), dim3(kGenThreads), 0, stream, p);
    hipLaunchKernelGGL(generic_bwd_cols_f32_kernel, dim3(p.Tk, p.Hkv, p.B), dim3(kGenThreads), 0, stream, p);
    return hipGetLastError();
}

}  // namespace plx
