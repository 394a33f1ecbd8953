// Host-side launch interface between the C ABI (parallax_api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace plx {

// Keys handled by one workgroup iteration of the bf16 decode kernel (4 waves x 32 keys).
constexpr int kDecodeBlockKeys = 128;

// RMSNorm + RoPE applied to q, rho as the attention kernels load them (gamma_q == nullptr: off).
struct QrPrep {
    const float *gamma_q, *gamma_r;  // [d]
    const float *table;              // [n_pos, d/2, 2] (cos, sin), or nullptr: RMSNorm only
    const int32_t *pos0;             // [B] or nullptr
    int32_t n_pos, rope_q, rope_r;
    float eps;
};

struct DecodeParams {
    const void *q, *r, *k, *v;
    void *o;
    const int32_t *seq_lens;
    float *ws;  // split partials: [B][Hq][S] records of (2d+4) floats
    int32_t B, Hq, Hkv, G, Lmax, d, S;
    int64_t ksb, ksh, ksl, vsb, vsh, vsl;  // element strides
    float scale;
    int32_t use_r;
    int32_t direct_out;  // 1: S == 1 and the split kernel writes o itself (no workspace)
    // paged cache: key j of sequence b is row j % page_size of page
    // block_table[b * table_stride + j / page_size]; ksb / vsb are then the page strides
    const int32_t *block_table;
    int32_t page_size, table_stride, num_pages;
    int32_t window;  // > 0: sliding window, a row at position pos sees keys pos - window + 1 .. pos
    int32_t *counters;  // in-kernel reduction: one arrival counter per (batch, kv head), zero on entry
    int32_t Tq;  // query rows per sequence (>= 1): the last Tq positions; q, r, o are [B, Hq, Tq, d]
    // bf16 split kernel, more than 16 columns: one launch handles the rows [row0, row0 + rows) of
    // the Tq (rows = 0: all of them)
    int32_t row0, rows;
    QrPrep prep;
};

struct PrefillParams {
    const void *q, *r, *k, *v;
    void *o;
    int32_t B, Hq, Hkv, G, T, Tk, d;  // T query rows, Tk keys
    int64_t qs[3], rs[3], ks[3], vs[3], os[3];  // element strides {batch, head, row}
    float scale;
    int32_t causal, use_r;
    int32_t window;  // > 0 (causal only): row at position pos sees keys pos - window + 1 .. pos
    // row cache for the backward pass, both or neither: vbar laid out like o, row_stats
    // [B, Hq, T, 2] fp32 = (log-sum-exp of the scaled scores in the exp2 domain, ubar)
    void *vbar;
    float *row_stats;
    // block-sparse (bf16, use_r, no window): row block rb of (batch sb, head sh) visits the key
    // tiles sparse_tile_idx[sparse_row_ptr[e] .. sparse_row_ptr[e + 1]), e = (sb * sparse_heads +
    // sh) * ceil(T / 128) + rb, ascending; sparse_batch / sparse_heads = 1 shares the lists
    const int32_t *sparse_row_ptr, *sparse_tile_idx;
    int32_t sparse_batch, sparse_heads;
    QrPrep prep;
};

// Decode over an MLA-style latent cache: one row [latent 512 | rope 64] per token shared by all
// heads (key = the row, value = its latent part); q, r [B, Hq, 576], o [B, Hq, 512] contiguous.
struct MlaDecodeParams {
    const void *q, *r, *ckv;
    void *o;
    const int32_t *seq_lens;
    float *ws;  // split partials: [B][Hq * Tq][S] records of (2 * 512 + 4) floats
    int32_t B, Hq, Lmax, S;
    int32_t Tq;      // query rows per head (q, r [B, Hq, Tq, 576]) at the last Tq positions
    int32_t window;  // > 0: a row sees its own position and the window - 1 before it
    int64_t csb, csl;  // element strides of the cache: batch (page, when paged), token
    float scale;
    int32_t direct_out;  // 1: S == 1, the kernel writes o itself
    // paged cache: token j of sequence b is row j % page_size of page
    // block_table[b * table_stride + j / page_size] of the pool
    const int32_t *block_table;
    int32_t page_size, table_stride, num_pages;
};

// Backward of the prefill forward: q-like tensors [B, Hq, T, d], k-like [B, Hkv, Tk, d].
struct PrefillBwdParams {
    const void *q, *r, *k, *v, *d_o;
    const void *o, *vbar;    // forward output and cached softmax value mean
    const float *row_stats;  // [B, Hq, T, 2] from the forward: (log-sum-exp in the exp2 domain, ubar)
    float *row_cache;        // workspace [B, Hq, T, 4]: row scalars (lse, ubar, tau, beta or combinations of them)
    void *dq, *dr, *dk, *dv;
    int32_t B, Hq, Hkv, G, T, Tk, d;
    float scale;
    int32_t causal;
    int32_t window;  // > 0 (causal only): a row sees its own position and the window - 1 before it
    // element strides {batch, head, row} of every tensor (innermost dimension contiguous)
    int64_t qs[3], rs[3], ks[3], vs[3], os[3], vbs[3], gs[3], dqs[3], drs[3], dks[3], dvs[3];
    // block-sparse (bf16, no window): the forward's lists per 128-row block (see PrefillParams) and
    // their transpose per 128-key block cb of (list batch sb, list head sh): entries
    // sparse_col_idx[sparse_col_ptr[e] .. sparse_col_ptr[e + 1]), e = (sb * sparse_heads + sh) *
    // ceil(Tk / 128) + cb, each 4 * row block + flags (bit t: the row block lists key tile 2 cb + t)
    const int32_t *sparse_row_ptr, *sparse_tile_idx, *sparse_col_ptr, *sparse_col_idx;
    int32_t sparse_batch, sparse_heads;
};

// RMSNorm + RoPE on up to three contiguous [B, H, T, d] tensors of one (B, T, d).
struct NormRopeTensor {
    const void *x;
    void *y;             // may be x
    const float *gamma;  // [d]
    int32_t H, rope;     // heads of this tensor; 0 = RMSNorm only
};
struct NormRopeParams {
    NormRopeTensor t[3];
    int32_t n_tensors, B, T, d;
    const int32_t *pos0;  // [B] position of row 0 of every sequence, or NULL = 0
    float eps, theta;
    const float *table;   // optional (cos, sin) per (position, pair); NULL = evaluate in the kernel
    int32_t n_pos;        // positions in the table
    int32_t heads_per_wave, head_chunks;  // set by the launcher
};

// Each returns hipSuccess or the launch error. No allocation, no synchronisation.
hipError_t launch_decode_bf16(const DecodeParams &p, hipStream_t stream);
hipError_t launch_decode_combine(const DecodeParams &p, hipStream_t stream);
hipError_t launch_prefill_bf16(const PrefillParams &p, hipStream_t stream);
hipError_t launch_prefill_bwd_bf16(const PrefillBwdParams &p, hipStream_t stream);
hipError_t launch_prefill_bwd_f32(const PrefillBwdParams &p, hipStream_t stream);
hipError_t launch_decode_f32(const DecodeParams &p, hipStream_t stream);
hipError_t launch_prefill_f32(const PrefillParams &p, hipStream_t stream);
hipError_t launch_norm_rope(const NormRopeParams &p, bool f32, hipStream_t stream);
hipError_t launch_rope_table(float *table, int n_pos, int d, float theta, hipStream_t stream);
hipError_t launch_decode_mla(const MlaDecodeParams &p, hipStream_t stream);
hipError_t launch_decode_mla_wide(const MlaDecodeParams &p, hipStream_t stream);  // the kernel launch only: more than 16 columns
hipError_t launch_util_copy(void *dst, const void *src, size_t bytes, hipStream_t stream);
hipError_t launch_util_read(const void *src, size_t bytes, void *sink, hipStream_t stream);
hipError_t launch_util_read_grid(const void *src, size_t bytes, void *sink, int workgroups, hipStream_t stream);
hipError_t launch_util_mfma(int workgroups, int iters, void *sink, hipStream_t stream);
constexpr int kReadSinkSlots = 4096;

}  // namespace plx
