/*
 * parallax.h -- C ABI of the MI355X (gfx950) Parallax attention forward library.
 *
 * Parallax (paper Sec. 3.1) extends softmax attention with a probe matrix R that has the
 * shape and head grouping of Q. For query row i with allowed key set J(i):
 *
 *     p_ij = softmax_j(scale * <q_i, k_j>)            scale = 1/h, natural exponential
 *     u_ij = <rho_i, k_j>                             (never scaled)
 *     o_i  = sum_j p_ij (1 + sum_j' p_ij' u_ij' - u_ij) v_j
 *          = o_softmax_i - Sigma_KV^(i) rho_i         (softmax-weighted KV covariance)
 *
 * The kernels evaluate it in one pass over K/V tiles with the running state
 * (m, d1, d2, O1, O2) of the paper's Algorithm 1 (Sec. 3.3) and finish with
 * O = O1/d1 * (1 + d2/d1) - O2/d1; decode splits the key range over workgroups and merges
 * the split partials with a log-sum-exp rescale (App. C, "in-kernel reduction" -- done here
 * by a separate combine kernel).
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller. The library never
 *     allocates, frees or keeps device memory.
 *   - Kernels are enqueued on the caller's hipStream_t (passed as void*, NULL = default
 *     stream). Calls return without synchronising; outputs are valid once the stream
 *     reaches that point.
 *   - Arguments are validated on the host before anything is launched: on a validation error
 *     (every status but PLX_ERR_LAUNCH) a negative plx_status is returned and nothing has been
 *     enqueued. PLX_ERR_LAUNCH means the HIP runtime refused a kernel launch; an entry point
 *     that enqueues several kernels may by then have enqueued the earlier ones, so treat its
 *     outputs and workspace as undefined. No call aborts or throws.
 *   - GQA: G = Hq / Hkv must be an integer; query head h reads KV head h / G.
 *   - Supported: dtype bf16 (MFMA kernels, d in {64, 128}, G <= 16) and fp32 (plain
 *     correctness kernels, d <= 256). Innermost dimension contiguous; base pointers and
 *     row strides 16-byte aligned. Output dtype = input dtype; all running state is fp32.
 */
#ifndef PARALLAX_H
#define PARALLAX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { PLX_BF16 = 0, PLX_F32 = 1 } plx_dtype;

typedef enum {
    PLX_OK = 0,
    PLX_ERR_NULL = -1,      /* a required pointer is NULL                          */
    PLX_ERR_SHAPE = -2,     /* non-positive size, Hq % Hkv != 0, unsupported d / G */
    PLX_ERR_DTYPE = -3,     /* unknown dtype                                       */
    PLX_ERR_ALIGN = -4,     /* pointer or stride not 16-byte aligned               */
    PLX_ERR_WORKSPACE = -5, /* split-KV workspace missing or too small             */
    PLX_ERR_LAUNCH = -6,    /* the HIP runtime refused a launch                    */
    PLX_ERR_SPLITS = -7,    /* num_splits outside [0, PLX_MAX_SPLITS]              */
    PLX_ERR_SCALE = -8,     /* scale is negative, infinite or NaN                  */
    PLX_ERR_SCRATCH = -9    /* parallax_decode_static: records exceed its scratch  */
} plx_status;

#define PLX_MAX_SPLITS 128
/* Split records (at d = 128: 1040 bytes each) that parallax_decode_static's scratch holds. */
#define PLX_STATIC_SCRATCH_RECORDS 16384

/*
 * RMSNorm + RoPE on the raw q and rho rows INSIDE the attention kernels (the paper's language-model
 * runs apply both in front of the attention call: Sec. 5 experiment setup, backbone appendix;
 * formulas as for parallax_norm_rope below): the rows are normalised, rotated and rounded to bf16 in
 * the kernel's prologue, so q and rho make no extra trip through HBM. K is prepared beforehand by
 * parallax_norm_rope (it is shared by all query heads and row blocks). bf16 only.
 *   q_gamma, r_gamma  [d] fp32 on the device, 16-byte aligned: RMSNorm weights; both non-NULL
 *                     switches the preparation on (r_gamma may be NULL when use_r == 0)
 *   eps               >= 0, under the root
 *   rope_table        NULL = RMSNorm only, else [rope_positions, d/2, 2] fp32 from
 *                     parallax_rope_table: (cos, sin) of pos * theta^(-2i/d)
 *   rope_q, rope_r    rotate q / rho (the paper: RoPE on q, k, optionally on rho)
 *   pos0              [B] int32 on the device or NULL (= 0): position of query row 0 of each
 *                     sequence (prefill: row i sits at pos0[b] + i; decode: NULL means the rows
 *                     are the last Tq positions, L_b - Tq + t, else pos0[b] + t); positions are
 *                     clamped to the table
 */
typedef struct {
    const float *q_gamma, *r_gamma;
    const float *rope_table;
    const int32_t *pos0;
    int32_t rope_positions;
    int32_t rope_q, rope_r;
    float eps;
} plx_qr_prep;

/*
 * Single-step decode (Algorithm 1 with one query row per head, Sec. 3.3; split-KV and merge,
 * App. C). The KV cache already contains the current token: key j of sequence b is allowed
 * iff j < L_b, L_b = seq_lens[b] (or Lmax when seq_lens is NULL).
 *
 *   q, r      [B, Hq, d]   contiguous
 *   k, v      [B, Hkv, Lmax, d] addressed as base + b*stride_b + h*stride_h + l*stride_l
 *             (strides in ELEMENTS, last dim contiguous)
 *   o         [B, Hq, d]   contiguous, written
 *   seq_lens  [B] int32 on the device, 0 <= L_b <= Lmax; rows with L_b = 0 (undefined in
 *             the paper: empty softmax) are written as zeros
 *   scale     multiplies q.k only (the probe score r.k is used as is); finite and >= 0
 *             (scale = 1/h for a bandwidth h > 0; 0 is the uniform-weight limit)
 *   use_r     1 = Parallax; 0 = softmax-only twin (r may be NULL, correction branch skipped)
 *   num_splits 0 = library heuristic, else the number of key-range splits to use
 *   workspace fp32 scratch for split partials, >= parallax_decode_workspace_bytes(...);
 *             may be NULL only when num_splits == 1
 *
 * Several query rows (Tq > 1; speculative rows or a short chunk, the causal set of Sec. 2.1 at
 * absolute positions): q, r, o are [B, Hq, Tq, d] and the rows are the LAST Tq positions of the
 * sequence, so row t sees key j iff j < L_b - (Tq - 1 - t). All rows of all heads of a GQA group
 * ride in one MFMA operand and share every K/V fetch as long as (Hq / Hkv) * Tq <= 16; with more
 * columns the bf16 path takes one launch per 16 / (Hq / Hkv) rows (each reads the cache again),
 * (bf16 GQA groups hold at most 16 heads). The workspace then needs Tq times
 * parallax_decode_workspace_bytes(...).
 *
 * Paged cache (block_table != NULL; the paper's Sec. 5 remark that cache layouts carry over --
 * same loop, different tile iterator): k, v point to a pool of pages
 *   [num_pages, Hkv, page_size, d] addressed as base + page*stride_b + h*stride_h + row*stride_l,
 * and key j of sequence b lives in page block_table[b*block_table_stride + j / page_size], row
 * j % page_size. block_table is int32 on the device; page_size >= 1;
 * block_table_stride * page_size >= Lmax. Entries are clamped to [0, num_pages) before use but
 * not otherwise checked. Lmax is the largest logical length (seq_lens bounds each sequence).
 *
 * Sliding window (window > 0; one of the sparsity patterns that Sec. 5 says carry over from
 * softmax attention -- the paper gives no formula, the usual one is taken): a query row at
 * position pos sees only the keys pos - window + 1 .. pos. The one decode row sits at position
 * L_b - 1 (row t of Tq at L_b - Tq + t). Key tiles outside the window are neither read nor
 * computed. 0 = no window.
 */
typedef struct {
    const void *q, *r;
    const void *k, *v;
    void *o;
    const int32_t *seq_lens;
    int32_t B, Hq, Hkv, Lmax, d;
    int64_t k_stride_b, k_stride_h, k_stride_l;
    int64_t v_stride_b, v_stride_h, v_stride_l;
    float scale;
    int32_t use_r;
    int32_t num_splits;
    void *workspace;
    size_t workspace_bytes;
    plx_dtype dtype;
    const int32_t *block_table; /* NULL = contiguous cache */
    int32_t page_size, block_table_stride, num_pages;
    int32_t Tq; /* query rows per sequence; 0 or 1 = one */
    int32_t window; /* sliding window in keys; 0 = none */
    int32_t *split_counters; /* parallax_decode_fused only: B*Hkv int32 on the device */
    plx_qr_prep prep; /* RMSNorm + RoPE on q, rho as they are loaded; all zero = q, rho used as given */
} plx_decode_args;

/* Bytes of workspace that is enough for any split count the library may pick or accept
 * for this shape: B*Hq*PLX_MAX_SPLITS records of (2d+4) floats (m, d1, d2, pad, O1[d], O2[d]). */
size_t parallax_decode_workspace_bytes(int32_t B, int32_t Hq, int32_t Hkv, int32_t Lmax, int32_t d);

/* The split count the heuristic picks for a shape on a device with num_cus compute units
 * (num_cus <= 0: ask the current device; 256 if none is visible). Pure host arithmetic. */
int32_t parallax_decode_num_splits(int32_t B, int32_t Hq, int32_t Hkv, int32_t Lmax, int32_t d,
                                   int32_t num_cus);

plx_status parallax_decode(const plx_decode_args *args, void *hip_stream);

/*
 * parallax_decode for callers that cannot allocate or pass a workspace -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc: the split records go to a
 * fixed array inside the library's code object instead (one copy per GPU, held until the
 * process ends; parallax_decode_static_scratch_bytes() = 17 039 360 bytes, i.e.
 * PLX_STATIC_SCRATCH_RECORDS records at d = 128). Same arguments, kernels and results as
 * parallax_decode (bit-identical for the same num_splits); args->workspace and
 * args->workspace_bytes are ignored. The call allocates nothing and calls no allocating
 * routine; the first call on a device looks the array's address up once.
 *   Limit: B * Hq * Tq * S * (2d + 4) * 4 bytes must fit the scratch (S = num_splits, or the
 *   heuristic's pick for num_splits = 0); otherwise PLX_ERR_SCRATCH and nothing is enqueued.
 *   S = 1 and fp32 calls use no scratch.
 *   Every call on a GPU shares that GPU's array: calls that may overlap on one device (two
 *   streams, two threads) race on it -- serialise them or give the others a workspace through
 *   parallax_decode. Nothing in the array has to start at zero (every record that is merged has
 *   been written by the same call), so stale contents of earlier calls are harmless.
 */
plx_status parallax_decode_static(const plx_decode_args *args, void *hip_stream);
size_t parallax_decode_static_scratch_bytes(void);

/*
 * The two halves of parallax_decode on their own (bf16 only), for callers that merge partials
 * themselves -- e.g. a KV cache sharded over devices, where every shard produces its partials
 * and one merge follows (App. C: the merge is an associative log-sum-exp rescale) -- and for
 * timing the two kernels separately.
 *   parallax_decode_partials: runs only the split kernel with S = num_splits (0 = heuristic) and
 *     ALWAYS writes the workspace, also for S = 1: record (b, hq, t, s) at float offset
 *     (((b*Hq + hq)*Tq + t)*S + s)*(2d+4) holds m (exp2 domain, -inf if the split saw no key),
 *     d1, d2, pad, O1[d], O2[d], all unnormalised. args->o is not touched and may be NULL.
 *   parallax_decode_combine: merges the S = num_splits (>= 1, required) records per (b, hq) of
 *     the workspace and writes args->o. Only o, B, Hq, Hkv, d, Tq, num_splits, workspace,
 *     workspace_bytes and dtype are read.
 */
plx_status parallax_decode_partials(const plx_decode_args *args, void *hip_stream);
plx_status parallax_decode_combine(const plx_decode_args *args, void *hip_stream);

/*
 * parallax_decode with the merge done inside the split kernel (the in-kernel reduction of
 * App. C): every workgroup writes its record, bumps an arrival counter of its (batch, kv head)
 * group, and the workgroup that arrives last merges the group's S records and writes o -- one
 * launch instead of two, nobody waits. bf16 only; same arguments as parallax_decode, plus
 *   split_counters  [B*Hkv] int32 on the device, 4-byte aligned. ALL ZERO when the call is
 *                   enqueued; the kernel puts every counter back to zero before it ends, so the
 *                   array is cleared once after allocation and then reused by later calls on the
 *                   same stream (any shape that fits). Calls that may overlap on the device need
 *                   counters (and workspaces) of their own. A launch that is aborted half-way
 *                   leaves counters undefined: clear them again.
 * The records are merged in the same order and with the same arithmetic as by
 * parallax_decode_combine: o is bit-identical to parallax_decode's for the same num_splits.
 * num_splits = 1 (given or picked) needs neither workspace nor counters.
 */
plx_status parallax_decode_fused(const plx_decode_args *args, void *hip_stream);

/*
 * Prefill forward over T query rows and Tkv keys per sequence (Algorithm 1, Sec. 3.3; forward
 * equation Sec. 3.1). Tkv = 0 means Tkv = T (the paper's square case).
 * causal != 0: the query rows are the LAST T positions of the Tkv-long sequence (a prefill
 * chunk behind an existing cache, or a few speculative rows): key j allowed iff
 * j <= i + (Tkv - T), diagonal included -- for Tkv = T that is j <= i and row 0 returns v_0.
 * Needs Tkv >= T. causal == 0: every key.
 * window > 0 (causal only): sliding window as for decode -- row i sees the keys
 * i + (Tkv - T) - window + 1 .. i + (Tkv - T); key tiles left of a row block's window are
 * skipped.
 *
 *   q, r, o   [B, Hq, T, d]    k, v  [B, Hkv, Tkv, d]
 *   *_stride  element strides {batch, head, row}; last dim contiguous
 */
typedef struct {
    const void *q, *r;
    const void *k, *v;
    void *o;
    int32_t B, Hq, Hkv, T, d;
    int64_t q_stride[3], r_stride[3], k_stride[3], v_stride[3], o_stride[3];
    float scale;
    int32_t causal;
    int32_t use_r;
    plx_dtype dtype;
    int32_t Tkv; /* keys per sequence; 0 = T */
    int32_t window; /* sliding window in keys (needs causal); 0 = none */
    /* Row cache for parallax_prefill_backward (App. D), both or neither (use_r):
     *   vbar       [B, Hq, T, d] like o (same strides): the softmax value mean O1 / d1
     *   row_stats  [B, Hq, T, 2] fp32 contiguous: log2 of sum_j exp(scale q.k_j) (i.e. the
     *              log-sum-exp in the exp2 domain) and ubar = sum_j p_j rho.k_j */
    void *vbar;
    float *row_stats;
    /* Block-sparse attention (one of the sparsity patterns Sec. 5 says carry over; bf16, use_r,
     * no window; the row cache may be asked for): softmax, ubar and the output run over the listed key tiles
     * only (intersected with the causal set when causal != 0). Blocks are the kernel's tiles:
     * 128 query rows x 64 keys. Row block rb of list-batch sb and list-head sh visits the key
     * tiles sparse_tile_idx[sparse_row_ptr[e] .. sparse_row_ptr[e + 1]),
     * e = (sb * sparse_heads + sh) * ceil(T / 128) + rb, in ASCENDING order, each at most once.
     * sparse_batch / sparse_heads are 1 (lists shared by all sequences / heads) or B / Hq. Both
     * arrays are int32 on the device; entries are clamped to existing tiles but not otherwise
     * checked (a list that does not ascend gives wrong results for its row block, never an access
     * outside the tensors); the arrays must not be written while the kernel runs. A row block
     * with an empty list (and any row none of whose listed keys is causal-visible) returns
     * zeros (and, in the row cache, vbar = 0, ubar = 0 and +infinity for the log-sum-exp, which
     * makes every probability of the row zero in the backward). NULL sparse_row_ptr = dense. */
    const int32_t *sparse_row_ptr;
    const int32_t *sparse_tile_idx;
    int32_t sparse_batch, sparse_heads;
    /* RMSNorm + RoPE on q, rho in the kernel's prologue (bf16, use_r, dense, no window, no row
     * cache); all zero = q, rho used as given */
    plx_qr_prep prep;
} plx_prefill_args;

plx_status parallax_prefill(const plx_prefill_args *args, void *hip_stream);

/*
 * Decode over an MLA-style latent cache (the closing discussion names multi-head latent
 * attention as structurally compatible; this is its absorbed-projection decode form). Every
 * cached token is ONE row [latent d_latent | rope part d_rope] shared by all heads: the key of
 * the token is the whole row, its value the latent part. With a = scale * q_h . c_j over all
 * d_latent + d_rope numbers, p = softmax_j(a), u_j = rho_h . c_j, ubar = sum_j p_j u_j:
 *     o_h = sum_j p_j (1 + ubar - u_j) c_j[:d_latent]          (forward definition, Sec. 3.1)
 * computed by Algorithm 1 with split-KV partials merged as in App. C. bf16 only,
 * d_latent = 512 and d_rope = 64.
 * Tq > 1 (0 means 1): every head has Tq query rows, which sit at the LAST Tq positions of the
 * cached sequence; row t sees the tokens 0 .. L_b - Tq + t (the rows of a speculative or chunked
 * decode step; with Tq = the prompt length, the causal prefill over the latent cache). window > 0:
 * a row sees its own position and the window - 1 before it only (Sec. 5's sliding-window remark).
 * A row that sees no token (L_b < Tq - t) returns zeros. q, r are then [B, Hq, Tq, 576] and o
 * [B, Hq, Tq, 512], contiguous; the workspace and split-count queries take Hq * Tq as their Hq.
 *   q, r       [B, Hq, 576] contiguous (already in the latent space), 16-byte aligned
 *   ckv        [B, Lmax, 576]: element strides ckv_stride_b / ckv_stride_l (multiples of 8,
 *              576 <= ckv_stride_l <= 2^23), last dimension contiguous
 *   o          [B, Hq, 512] contiguous (the value up-projection is the caller's)
 *   seq_lens   int32 [B] on the device or NULL (= Lmax); 0 gives a zero row
 *   num_splits 0 = heuristic, else 1 .. PLX_MAX_SPLITS
 *   workspace  fp32 scratch for num_splits > 1, >= parallax_decode_mla_workspace_bytes(B, Hq)
 *   block_table  NULL, or int32 [B, block_table_stride] on the device: the cache is then a pool
 *              ckv [num_pages, page_size, 576] (ckv_stride_b = page stride) and token j of
 *              sequence b is row j % page_size of page block_table[b][j / page_size]; entries
 *              are clamped to existing pages. block_table_stride * page_size >= Lmax. Any page
 *              size works; multiples of 64 are fetched page-wise, others row by row (slower).
 * Up to 16 (head, row) pairs per sequence run a memory-bound kernel (16 MFMA columns per
 * workgroup); more run a matrix-bound one (32 columns per workgroup, the workgroups of one
 * sequence placed so that they share an L2). Same results contract, same workspace format.
 * Validates on the host, enqueues one or two kernels on hip_stream, does not synchronise.
 */
typedef struct {
    const void *q, *r;
    const void *ckv;
    void *o;
    const int32_t *seq_lens;
    int32_t B, Hq, Lmax;
    int32_t d_latent, d_rope;
    int32_t num_splits;
    int64_t ckv_stride_b, ckv_stride_l;
    float scale;
    plx_dtype dtype;
    void *workspace;
    size_t workspace_bytes;
    const int32_t *block_table;
    int32_t page_size, num_pages, block_table_stride;
    int32_t Tq;     /* query rows per head; 0 = 1 */
    int32_t window; /* 0 = none */
} plx_decode_mla_args;

size_t parallax_decode_mla_workspace_bytes(int32_t B, int32_t Hq);
/* The split count the heuristic picks (num_cus <= 0: ask the device). */
int32_t parallax_decode_mla_num_splits(int32_t B, int32_t Hq, int32_t Lmax, int32_t num_cus);
plx_status parallax_decode_mla(const plx_decode_mla_args *args, void *hip_stream);

/*
 * Backward of parallax_prefill (closed-form gradients, App. D): given the upstream gradient d_o,
 * the forward's inputs, its output o and its row cache (vbar, row_stats), writes dq, dr
 * [B, Hq, T, d] and dk, dv [B, Hkv, Tkv, d]; the gradients of a KV head add up over the query
 * heads of its group. Every tensor 16-byte aligned with the head dimension innermost and
 * contiguous; *_stride are element strides {batch, head, row} as in plx_prefill_args, an all-zero
 * triple meaning the dense [B, H, T, d] layout (row_stats is always dense). bf16 (d = 64 or 128;
 * MFMA kernels) or fp32 (d <= 256, plain untuned path, vbar in fp32 too, dense layout only). causal, Tkv and window as in the forward (window > 0 needs causal != 0; the row cache
 * must come from a forward call with the same window).
 *   workspace  fp32 scratch, >= parallax_prefill_backward_workspace_bytes(B, Hq, T) = 16 bytes
 *              per query row (four row scalars built from lse, ubar, tau = dO.o, beta = dO.vbar;
 *              contents are private to the library)
 * Three kernels are enqueued (row scalars; dQ, dR; dK, dV); nothing is accumulated with atomics,
 * so results are deterministic and the outputs need no zeroing.
 */
typedef struct {
    const void *q, *r, *k, *v;
    const void *o, *vbar;
    const float *row_stats;
    const void *d_o;
    void *dq, *dr, *dk, *dv;
    int32_t B, Hq, Hkv, T, Tkv, d; /* Tkv = 0 means T */
    float scale;
    int32_t causal;
    plx_dtype dtype;
    int32_t window; /* 0 = none; W > 0: a row sees its own position and the W - 1 before it */
    void *workspace;
    size_t workspace_bytes;
    int64_t q_stride[3], r_stride[3], k_stride[3], v_stride[3], o_stride[3], vbar_stride[3], d_o_stride[3];
    int64_t dq_stride[3], dr_stride[3], dk_stride[3], dv_stride[3];
    /* Block-sparse (Sec. 5's sparsity remark x App. D; bf16, no window): all four arrays or none.
     * sparse_row_ptr / sparse_tile_idx / sparse_batch / sparse_heads: the forward's lists, as in
     * plx_prefill_args (the row cache must come from a forward call with the same lists). The
     * pass over the keys needs the same cells by columns: key block cb (128 keys = key tiles
     * 2 cb and 2 cb + 1) of list-batch sb and list-head sh is listed by the row blocks
     * sparse_col_idx[sparse_col_ptr[e] .. sparse_col_ptr[e + 1]) >> 2,
     * e = (sb * sparse_heads + sh) * ceil(Tkv / 128) + cb, each entry 4 * row block + flags, flag
     * bit t set iff that row block lists key tile 2 cb + t (at least one is). int32 on the
     * device, not written while the kernels run; row blocks are clamped to existing ones. The two
     * descriptions must name the same cells: if they differ, dq / dr follow the row lists and
     * dk / dv the column lists (wrong gradients, never an access outside the tensors). Row and
     * key blocks nobody lists get zero gradients. */
    const int32_t *sparse_row_ptr;
    const int32_t *sparse_tile_idx;
    const int32_t *sparse_col_ptr;
    const int32_t *sparse_col_idx;
    int32_t sparse_batch, sparse_heads;
} plx_prefill_bwd_args;

size_t parallax_prefill_backward_workspace_bytes(int32_t B, int32_t Hq, int32_t T);
plx_status parallax_prefill_backward(const plx_prefill_bwd_args *args, void *hip_stream);

/*
 * RMSNorm over the head dimension, then rotary position embedding, on up to three tensors of one
 * layer (q, rho, k) in one launch -- what the paper's language-model runs apply in front of the
 * attention call (Sec. 5 experiment setup, backbone appendix: RMSNorm on q, k and rho; RoPE with
 * base 1e6 on q, k and optionally rho). The paper gives no formulas; the standard ones are used:
 *     y = x / sqrt(mean_c(x_c^2) + eps) * gamma
 *     (y_2i, y_2i+1) rotated by pos * theta^(-2i/d), pos = pos0[b] + t   (adjacent pairs)
 *   tensors[i].x, .y  [B, H_i, T, d] contiguous, 16-byte aligned; y may be x (in place)
 *   tensors[i].gamma  [d] fp32 on the device
 *   tensors[i].rope   0 = RMSNorm only
 *   pos0              [B] int32 on the device (position of row 0; a decode step passes L_b - 1),
 *                     or NULL = 0
 *   d                 bf16: 64 or 128; fp32: 16, 32, 64, 128 or 256
 */
typedef struct {
    const void *x;
    void *y;
    const float *gamma;
    int32_t H;
    int32_t rope;
} plx_norm_rope_tensor;

typedef struct {
    plx_norm_rope_tensor tensors[3];
    int32_t n_tensors; /* 1..3 */
    int32_t B, T, d;
    const int32_t *pos0;
    float eps;   /* >= 0 */
    float theta; /* > 1 */
    plx_dtype dtype;
    /* Optional: (cos, sin) per (position, pair) from parallax_rope_table (same d and theta; fp32,
     * 16-byte aligned) instead of evaluating them in the kernel, positions clamped to
     * [0, table_positions). Worth it for decode steps (T = 1): the in-kernel evaluation forms the
     * angle in double precision, about 20 us of serial arithmetic that a long T amortises over
     * all heads but a single row does not. NULL = evaluate. */
    const float *rope_table;
    int32_t table_positions;
} plx_norm_rope_args;

plx_status parallax_norm_rope(const plx_norm_rope_args *args, void *hip_stream);

/* The rotation table of plx_qr_prep: table[(pos * d/2 + i) * 2 + {0, 1}] = cos, sin of
 * pos * theta^(-2i/d) for pos in [0, n_pos), i in [0, d/2) -- the angle reduced modulo 2 pi in double
 * precision, as parallax_norm_rope does. fp32 on the device, 16-byte aligned, n_pos * d floats;
 * d even, 2 <= d <= 256; theta > 1. Computed once per (d, theta, longest context). */
plx_status parallax_rope_table(float *table, int32_t n_pos, int32_t d, float theta, void *hip_stream);

const char *parallax_strerror(plx_status status);
int parallax_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PARALLAX_H */
