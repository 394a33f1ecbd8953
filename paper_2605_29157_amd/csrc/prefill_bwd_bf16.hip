// Parallax prefill backward for bf16 on gfx950 (closed-form gradients of the paper's App. D).
//
// With p_ij = exp2(S1_ij * scale * log2 e - lse_i), u_ij = rho_i.k_j, a_ij = dO_i.v_j and the
// row scalars ubar_i (cached by the forward), tau_i = dO_i.o_i, beta_i = dO_i.vbar_i:
//     g1_ij = p_ij [a_ij - tau_i + (ubar_i - u_ij)(a_ij - beta_i)],   g2_ij = -p_ij (a_ij - beta_i)
//     dQ_i = scale * sum_j g1_ij k_j      dR_i = sum_j g2_ij k_j
//     dK_j = scale * sum_i g1_ij q_i + sum_i g2_ij rho_i
//     dV_j = sum_i p_ij (1 + ubar_i - u_ij) dO_i
// As the appendix says, the two reduction directions make two passes:
//   * rows prepare: one wave per query row folds (lse, ubar) of the forward's row cache and
//     tau, beta into one float4 per row, (lse, 1 + ubar, beta - tau, beta): with delta = a - beta
//     and c = (1 + ubar) - u the bracket of g1 is delta * c + (beta - tau) and w = p * c, two
//     vector instructions per pair less than the textbook order;
//   * row pass (dQ, dR): a workgroup owns 128 query rows of one head (32 per wave), keeps their
//     Q, R, dO fragments in registers and streams K/V tiles of 64 keys. Scores are produced
//     transposed, as in the forward: S1^T = K Q^T, S2^T = K R^T, A^T = V dO^T, so a lane owns one
//     query row, the row scalars are per lane, and the accumulator registers of g1, g2 are
//     already the B operand of dQ^T += K^T g1^T, dR^T += K^T g2^T (K^T fragments by transposing
//     LDS reads);
//   * column pass (dK, dV): a workgroup owns 128 keys of one KV head (32 per wave), keeps their
//     K, V fragments in registers as B operands and streams Q, R, dO tiles of 64 rows of every
//     query head of the group. S1 = Q K^T, S2 = R K^T, A = dO V^T put a key in each lane and the
//     rows in its registers (row scalars come from LDS); the registers of p(1 + ubar - u), g1, g2
//     are the B operands of dV^T += dO^T W, dK^T += Q^T g1 + R^T g2 (transposing LDS reads of the
//     same tiles).
// Eleven contractions of 2d flops per (row, key) pair against the forward's four. Tiles go
// global -> LDS directly into a three-stage ring, one workgroup barrier per tile; both passes are
// software pipelines of hand-placed slots (one MFMA + its share of vector work), as in the forward.
// Every tensor is addressed through element strides {batch, head, row}; the workspace is dense.
// SPARSE (block lists over 128 query rows x 64 keys, the forward's cells): the row pass walks the
// forward's list of its row block; the column pass walks the TRANSPOSED list of its 128 keys --
// per query head of the group the row blocks that list one of its two key tiles, with two flag
// bits saying which: a wave whose key tile a row block does not list masks all its pairs. Both
// passes then run the masked form of their pipeline throughout.
#include "plx_device.h"
#include "plx_kernels.h"
#include <type_traits>

#include "plx_lds_dma.h"
#include "plx_mfma_asm.h"

namespace plx {

namespace {

constexpr int kTileRows = 64;  // rows (keys or query rows) per LDS tile
constexpr int kBlk = 32;       // rows per MFMA block

// Every tile is read both ways -- whole chunks of 32 consecutive rows (A / B operand of a score
// MFMA) and transposed, 4 consecutive rows x 4 chunks (A operand of an output MFMA) -- so rows are
// not padded but their chunks permuted (lds_chunk_slot): both patterns then spread over all banks.
template <int D>
struct BwdTile {
    static constexpr int CPR = D / 8;  // 16-byte chunks per row
    static constexpr int CHUNKS = kTileRows * CPR;
    static constexpr int NDMA = CHUNKS / 256;  // loads per wave and tile
    static_assert(CHUNKS % 256 == 0, "four waves fill a tile with whole 64-lane loads");
};

// Rows [row0, row0 + 64) of a row-major [n_rows][D] bf16 matrix -> LDS tile. A wave-wide load
// fills 64 consecutive LDS chunks, so every lane fetches the global chunk that belongs at its
// LDS position. Rows past the end re-read the last row (finite data; masked where it matters).
// Each wave fills a quarter.
template <int D>
__device__ __forceinline__ void load_tile64(const __bf16 *base, int64_t row_stride, int row0, int n_rows,
                                            uint32_t lds_tile_addr, int w, int lane) {
    using TL = BwdTile<D>;
#pragma unroll
    for (int i = 0; i < TL::NDMA; ++i) {
        const int c = (w * TL::NDMA + i) * 64 + lane;
        const int row = c / TL::CPR;
        const int chunk = (c % TL::CPR) ^ lds_row_swizzle<D>(row);
        const __bf16 *g = base + (int64_t)min(row0 + row, n_rows - 1) * row_stride + chunk * 8;
        tile_load16<64>(g, lds_tile_addr + (uint32_t)(w * TL::NDMA + i) * 1024u);
    }
}

// Per-lane chunk offsets of the two read patterns inside a 32-row block (they repeat every 16
// rows, so one set serves every block of every tile).
template <int D>
struct BwdLaneOffsets {
    static constexpr int CPR = D / 8, KSTEPS = D / 16, NDB = D / 32;
    int nt[KSTEPS];             // whole chunk 2*ks + h of row col: u32x4 index
    int tr_lo[NDB], tr_hi[NDB];  // transposing reads of rows tr_row / tr_row + 8: bf16 index

    __device__ __forceinline__ BwdLaneOffsets(int lane) {
        const int col = lane & 31, h = lane >> 5;
        const int f = lds_row_swizzle<D>(col);
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) nt[ks] = col * CPR + ((2 * ks + h) ^ f);
        // lane -> (row, chunk, half) inside a [4 rows][16 elements] group of a transposing read
        const int tr_row = 4 * h + ((lane & 15) >> 2);
        const int tr_half = (lane & 1) * 4;
        const int tr_chunk = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
#pragma unroll
        for (int n = 0; n < NDB; ++n) {
            tr_lo[n] = (tr_row * CPR + ((4 * n + tr_chunk) ^ lds_row_swizzle<D>(tr_row))) * 8 + tr_half;
            tr_hi[n] = ((tr_row + 8) * CPR + ((4 * n + tr_chunk) ^ lds_row_swizzle<D>(tr_row + 8))) * 8 + tr_half;
        }
    }
    // A operand with row = dim 32n + col, k-elements = rows 16j + 4h..+3 and 16j + 8 + 4h..+3 of
    // the 32-row block that starts at tile16
    __device__ __forceinline__ u32x4 transposed(const unsigned short *block16, int j, int n) const {
        const u32x2 lo = lds_read_tr16(block16 + 16 * j * CPR * 8 + tr_lo[n]);
        const u32x2 hi = lds_read_tr16(block16 + 16 * j * CPR * 8 + tr_hi[n]);
        return u32x4{lo[0], lo[1], hi[0], hi[1]};
    }
};

__device__ __forceinline__ u32x4 pack_group(const f32x16 &s, int j) {
    return u32x4{pack_bf16(s[8 * j + 0], s[8 * j + 1]), pack_bf16(s[8 * j + 2], s[8 * j + 3]),
                 pack_bf16(s[8 * j + 4], s[8 * j + 5]), pack_bf16(s[8 * j + 6], s[8 * j + 7])};
}

__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int r = 0; r < 16; ++r) z[r] = 0.f;
    return z;
}

}  // namespace

// ---- rows prepare: (lse, ubar, tau, beta) per query row ---------------------------------------
template <int D>
__global__ __launch_bounds__(256) void bwd_rows_prepare_kernel(PrefillBwdParams p) {
    // 16 bytes per lane: D / 8 lanes share a row, a workgroup takes 2048 / D rows
    constexpr int LPR = D / 8, ROWS = 256 / LPR;
    const int sub = threadIdx.x % LPR;
    const int64_t row = (int64_t)blockIdx.x * ROWS + threadIdx.x / LPR;
    const int64_t n_rows = (int64_t)p.B * p.Hq * p.T;
    const bool live = row < n_rows;  // (whole row groups; every lane takes part in the shuffles)
    const int64_t rr = live ? row : n_rows - 1;
    const int64_t bh = rr / p.T, t = rr - bh * p.T, b = bh / p.Hq, h = bh - b * p.Hq;
    const u32x4 g = ((const u32x4 *)((const __bf16 *)p.d_o + b * p.gs[0] + h * p.gs[1] + t * p.gs[2]))[sub];
    const u32x4 o = ((const u32x4 *)((const __bf16 *)p.o + b * p.os[0] + h * p.os[1] + t * p.os[2]))[sub];
    const u32x4 vb = ((const u32x4 *)((const __bf16 *)p.vbar + b * p.vbs[0] + h * p.vbs[1] + t * p.vbs[2]))[sub];
    float tau = 0.f, beta = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        tau += bf16_lo_f32(g[i]) * bf16_lo_f32(o[i]) + bf16_hi_f32(g[i]) * bf16_hi_f32(o[i]);
        beta += bf16_lo_f32(g[i]) * bf16_lo_f32(vb[i]) + bf16_hi_f32(g[i]) * bf16_hi_f32(vb[i]);
    }
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) {
        tau += __shfl_xor(tau, off, 64);
        beta += __shfl_xor(beta, off, 64);
    }
    if (live && sub == 0) {
        const f32x4 out = {p.row_stats[2 * row], 1.f + p.row_stats[2 * row + 1], beta - tau, beta};
        ((f32x4 *)p.row_cache)[row] = out;
    }
}

// ---- row pass: dQ, dR -------------------------------------------------------------------------
// Software pipeline over 32-key blocks, written as slots of ONE MFMA plus its share of vector
// work (the single wave of a SIMD issues in order, so vector instructions only run in the shadow
// of an MFMA that was issued before them):
//   phase 1 : the 3 * d/16 score MFMAs of the NEXT block (S1^T, S2^T, A^T alternate), while the
//             vector ALU turns the upper 16 keys of the CURRENT block into g1 / g2;
//   phase 2 : the output MFMAs of the CURRENT block (dQ^T, dR^T alternate), while the vector ALU
//             already turns the lower 16 keys of the NEXT block into its g1 / g2.
// Each slot that first uses an LDS fragment issues the read of the fragment needed three
// fragments later ([K, V of the next block | K^T of the current block | K, V of the block after]).
// WINDOW (sliding window, causal only): the key tiles before the window of the block's first row
// are skipped by moving the key origin; the leading tiles that some row sees only in part take
// the masked form of the pipeline, like the diagonal ones.
template <int D, bool CAUSAL, bool WINDOW = false, bool SPARSE = false>
__global__ __launch_bounds__(256, 1) void bwd_dq_dr_kernel(PrefillBwdParams p) {
    static_assert(CAUSAL || !WINDOW, "a sliding window is causal");
    static_assert(!(SPARSE && WINDOW), "block lists and a sliding window do not combine");
    using TL = BwdTile<D>;
    constexpr int CPR = TL::CPR, KSTEPS = D / 16, NDB = D / 32;
    constexpr int STAGES = 3, STAGE_CHUNKS = 2 * TL::CHUNKS;  // ring of [K tile | V tile]
    __shared__ u32x4 lds[STAGES * STAGE_CHUNKS];

    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int col = lane & 31, h = lane >> 5;
    const int T = p.T;
    const int nrb = (T + 127) / 128;
    // Work item: the row block is the slowest index, so that under a causal mask ALL heavy row
    // blocks are dispatched before any light one (with the row block as the fastest index every
    // head ends on its own light blocks while the last head's heavy ones have just started: the
    // tail cost 14 % of the pass). The (batch, kv head) pairs are dealt over the 8 XCDs by
    // workgroup id modulo 8, so that the heads of a GQA group share an L2.
    int rbi, hq, b;
    {
        const int id = blockIdx.x, pairs = p.B * p.Hkv, G = p.G;
        int pair, hg;
        if (pairs % 8 == 0) {
            const int x = id & 7, j = id >> 3, per = (pairs / 8) * G;
            rbi = j / per;
            const int rem = j - rbi * per;
            pair = (rem / G) * 8 + x;
            hg = rem % G;
        } else {
            const int per = pairs * G;
            rbi = id / per;
            const int rem = id - rbi * per;
            pair = rem / G;
            hg = rem % G;
        }
        b = pair / p.Hkv;
        hq = (pair - b * p.Hkv) * G + hg;
    }
    const int rb = CAUSAL ? nrb - 1 - rbi : rbi;  // heavy row blocks first
    // key tiles no row of this block sees (all keys before the window of its first row)
    const int kt_skip = WINDOW ? max(rb * 128 + (p.Tk - T) - p.window + 1, 0) / kTileRows : 0;
    const int Tk = p.Tk - kt_skip * kTileRows, off = Tk - T;  // keys from the first tile read on
    const int hk = hq / p.G;
    const int row0 = rb * 128 + w * 32, my_row = row0 + col;
    const int ld_row = min(my_row, T - 1);

    // B operands of the score MFMAs: column = query row, k-elements = the 8 dims of chunk 2*ks + h
    u32x4 qf[KSTEPS], rf[KSTEPS], gf[KSTEPS];
    {
        const __bf16 *qrow = (const __bf16 *)p.q + b * p.qs[0] + hq * p.qs[1] + ld_row * p.qs[2];
        const __bf16 *rrow = (const __bf16 *)p.r + b * p.rs[0] + hq * p.rs[1] + ld_row * p.rs[2];
        const __bf16 *grow = (const __bf16 *)p.d_o + b * p.gs[0] + hq * p.gs[1] + ld_row * p.gs[2];
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            qf[ks] = *(const u32x4 *)(qrow + 8 * (2 * ks + h));
            rf[ks] = *(const u32x4 *)(rrow + 8 * (2 * ks + h));
            gf[ks] = *(const u32x4 *)(grow + 8 * (2 * ks + h));
        }
    }
    const f32x4 rc = ((const f32x4 *)p.row_cache)[((int64_t)b * p.Hq + hq) * T + ld_row];
    const float neg_lse = -rc[0], one_ubar = rc[1], kappa = rc[2], beta = rc[3];  // (lse, 1 + ubar, beta - tau, beta)
    const float scale_log2 = p.scale * kLog2e;
    const BwdLaneOffsets<D> lo(lane);

    const __bf16 *kbase = (const __bf16 *)p.k + b * p.ks[0] + hk * p.ks[1] + (int64_t)kt_skip * kTileRows * p.ks[2];
    const __bf16 *vbase = (const __bf16 *)p.v + b * p.vs[0] + hk * p.vs[1] + (int64_t)kt_skip * kTileRows * p.vs[2];
    const uint32_t lds_base = lds_byte_address(lds);
    auto issue_tile = [&](int tile, int stage) __attribute__((always_inline)) {  // key tile -> ring stage
        load_tile64<D>(kbase, p.ks[2], tile * kTileRows, Tk, lds_base + (uint32_t)(stage * STAGE_CHUNKS) * 16u, w, lane);
        load_tile64<D>(vbase, p.vs[2], tile * kTileRows, Tk,
                       lds_base + (uint32_t)(stage * STAGE_CHUNKS + TL::CHUNKS) * 16u, w, lane);
    };
    // The steady-state loop spreads the loads of tile t + 2 over the MFMA slots of a step (as a
    // block at the top of an iteration they cost about a tenth of it): per-lane byte offsets
    // inside a complete tile, a wave-uniform tile base.
    uint32_t toffk[TL::NDMA], toffv[TL::NDMA];
#pragma unroll
    for (int i = 0; i < TL::NDMA; ++i) {
        const int c = (w * TL::NDMA + i) * 64 + lane;
        const int row = c / CPR;
        const int chunk = (c % CPR) ^ lds_row_swizzle<D>(row);
        toffk[i] = (uint32_t)(row * (int)p.ks[2] + chunk * 8) * 2u;
        toffv[i] = (uint32_t)(row * (int)p.vs[2] + chunk * 8) * 2u;
    }
    const char *dma_k = nullptr, *dma_v = nullptr;  // tile being fetched by the current step
    uint32_t dma_lds = 0;                           // this wave's first K chunk of its stage
    auto dma_slot = [&](int i) __attribute__((always_inline)) {  // load i of 2 * NDMA (K, then V)
        if (i < TL::NDMA)
            tile_load16_uniform<false>(toffk[i], dma_k, dma_lds + 1024u * i);
        else
            tile_load16_uniform<false>(toffv[i - TL::NDMA], dma_v,
                                       dma_lds + (uint32_t)TL::CHUNKS * 16u + 1024u * (i - TL::NDMA));
    };
    auto k_block = [&](int stage, int kb) __attribute__((always_inline)) { return (const u32x4 *)(lds + stage * STAGE_CHUNKS + kb * kBlk * CPR); };

    const int key_end = CAUSAL ? min(Tk, (rb + 1) * 128 + off) : Tk;
    // Block-sparse: ring position t holds key tile tile_at(t) of the row block's list (ascending,
    // caller's arrays, read as scalar loads; entries clamped to existing tiles; listed tiles past
    // the causal limit dropped) -- the list the forward walked.
    using const_i32 = const __attribute__((address_space(4))) int32_t;
    const_i32 *tile_list = nullptr;
    int n_list = 0;
    if constexpr (SPARSE) {
        const int sb = p.sparse_batch > 1 ? b : 0, sh = p.sparse_heads > 1 ? hq : 0;
        const int64_t e = ((int64_t)sb * p.sparse_heads + sh) * nrb + rb;
        const_i32 *row_ptr = (const_i32 *)(uintptr_t)p.sparse_row_ptr;
        const int first = row_ptr[e];
        tile_list = (const_i32 *)(uintptr_t)p.sparse_tile_idx + first;
        int lo_i = 0, hi_i = max(row_ptr[e + 1] - first, 0);
        while (lo_i < hi_i) {  // leading entries whose first key lies below key_end
            const int mid = (lo_i + hi_i) >> 1;
            if ((int64_t)max(tile_list[mid], 0) * kTileRows < key_end)
                lo_i = mid + 1;
            else
                hi_i = mid;
        }
        n_list = lo_i;
    }
    auto tile_at = [&](int i) __attribute__((always_inline)) {
        if constexpr (SPARSE)
            return min(max(tile_list[min(i, n_list - 1)], 0), (Tk - 1) / kTileRows);
        else
            return i;
    };
    const int n_tiles = SPARSE ? n_list : (key_end + kTileRows - 1) / kTileRows;
    const int lim_row = CAUSAL ? min(my_row + off, Tk - 1) : Tk - 1;  // last key this lane's row sees
    if constexpr (SPARSE) {
        if (n_tiles == 0) {  // (workgroup-uniform) a row block that lists nothing: zero gradients
            if (my_row < T) {
                __bf16 *dq_row = (__bf16 *)p.dq + b * p.dqs[0] + hq * p.dqs[1] + my_row * p.dqs[2];
                __bf16 *dr_row = (__bf16 *)p.dr + b * p.drs[0] + hq * p.drs[1] + my_row * p.drs[2];
#pragma unroll
                for (int c = 0; c < D / 16; ++c) {
                    *(u32x4 *)(dq_row + 8 * (2 * c + h)) = u32x4{0u, 0u, 0u, 0u};
                    *(u32x4 *)(dr_row + 8 * (2 * c + h)) = u32x4{0u, 0u, 0u, 0u};
                }
            }
            return;
        }
    }

    f32x16 dq[NDB], dr[NDB];
#pragma unroll
    for (int n = 0; n < NDB; ++n) dq[n] = dr[n] = zero16();

    // fragments in flight
    constexpr int NF1 = 2 * KSTEPS, NF2 = 2 * NDB, LA = 3;
    u32x4 f1[NF1], f2[NF2];
    auto load_f1 = [&](const u32x4 *kblk, int f) __attribute__((always_inline)) {  // even: K chunk, odd: V chunk of k-step f / 2
        f1[f] = (f & 1) ? kblk[TL::CHUNKS + lo.nt[f >> 1]] : kblk[lo.nt[f >> 1]];
    };
    auto load_f2 = [&](const u32x4 *kblk, int f) __attribute__((always_inline)) {
        f2[f] = lo.transposed((const unsigned short *)kblk, f / NDB, f % NDB);
    };
    auto prefetch = [&](int f, const u32x4 *next_blk, const u32x4 *cur_blk, const u32x4 *after_blk) __attribute__((always_inline)) {
        const int g = f + LA;
        if (g < NF1)
            load_f1(next_blk, g);
        else if (g < NF1 + NF2)
            load_f2(cur_blk, g - NF1);
        else
            load_f1(after_blk, g - NF1 - NF2);
    };

    // Element-wise work of the 8 score registers [r0, r0 + 8) of a block, as four stages in
    // consecutive slots so that a slot holds independent instructions only; the results replace
    // the scores: g1 in aa, g2 in s2. Register r holds key offset 8*(r/4) + r%4 (+ 4h, already
    // taken off lim). With a window a key counts iff 0 <= lim - offset < window: one unsigned compare.
    const unsigned wspan = WINDOW ? (unsigned)p.window : 0u;
    float dl[8];
    auto elem_stages = [&](auto masked_tag, f32x16 &s1, f32x16 &s2, f32x16 &aa, int r0, int slot, int slot0,
                           int n_slots, int lim) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int r = r0 + u;
            const int first = slot0 + u * (n_slots - 6 - slot0) / 7;
            if (slot == first) {
                s1[r] = fmaf(s1[r], scale_log2, neg_lse);
                dl[u] = aa[r] - beta;        // delta
                s2[r] = one_ubar - s2[r];    // 1 + ubar - u
            }
            if (slot == first + 1) {
                s1[r] = fast_exp2(s1[r]);             // p
                aa[r] = fmaf(s2[r], dl[u], kappa);    // a - tau + (ubar - u) delta
            }
            if constexpr (MASKED)
                if (slot == first + 2) {
                    if constexpr (WINDOW)
                        s1[r] = ((unsigned)(lim - (8 * (r >> 2) + (r & 3))) < wspan) ? s1[r] : 0.f;
                    else
                        s1[r] = (8 * (r >> 2) + (r & 3) <= lim) ? s1[r] : 0.f;
                }
            if (slot == first + 3) {
                aa[r] = s1[r] * aa[r];    // g1
                s2[r] = -(s1[r] * dl[u]);  // g2
            }
        }
    };

    // The score MFMAs are assembly statements with vector-register destinations (their results
    // feed the vector ALU; the compiler would put them in accumulation registers and copy every
    // one out). Each brings two wait states for its operands; the first vector read of a block
    // comes in slot 1 of phase 2, behind two more MFMAs: by then the block's last MFMA retired.
    u32x4 pg1[2], pg2[2];
    auto pipeline_step = [&](auto masked_tag, auto dma_tag, int key_base_cur, int key_base_next, const u32x4 *next_blk, const u32x4 *cur_blk, const u32x4 *after_blk,
                             f32x16 &c1, f32x16 &c2, f32x16 &ca, f32x16 &n1, f32x16 &n2, f32x16 &na) __attribute__((always_inline)) {
        const int lim_cur = lim_row - key_base_cur - 4 * h, lim_next = lim_row - key_base_next - 4 * h;
        constexpr int SLOTS1 = 3 * KSTEPS, SLOTS2 = 4 * NDB;
        constexpr bool DMA = decltype(dma_tag)::value;  // this step also fetches tile (dma_k, dma_v)
        static_assert(2 * TL::NDMA <= SLOTS1, "one tile load per slot");
#pragma unroll
        for (int sl = 0; sl < SLOTS1; ++sl) {
            const int ks = sl / 3, which = sl % 3;
            if constexpr (DMA)
                if (sl < 2 * TL::NDMA) dma_slot(sl);
            if (which == 0) {
                if (ks == 0) mfma32_scores_first<true>(n1, f1[2 * ks], qf[ks]);
                else mfma32_scores<true>(n1, f1[2 * ks], qf[ks]);
                prefetch(2 * ks, next_blk, cur_blk, after_blk);
            } else if (which == 1) {
                if (ks == 0) mfma32_scores_first<true>(n2, f1[2 * ks], rf[ks]);
                else mfma32_scores<true>(n2, f1[2 * ks], rf[ks]);
            } else {
                if (ks == 0) mfma32_scores_first<true>(na, f1[2 * ks + 1], gf[ks]);
                else mfma32_scores<true>(na, f1[2 * ks + 1], gf[ks]);
                prefetch(2 * ks + 1, next_blk, cur_blk, after_blk);
            }
            elem_stages(masked_tag, c1, c2, ca, 8, sl, 0, SLOTS1, lim_cur);
            if (sl == SLOTS1 - 2) pg1[1] = pack_group(ca, 1);
            if (sl == SLOTS1 - 1) pg2[1] = pack_group(c2, 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        u32x4 nb1 = {0u, 0u, 0u, 0u}, nb2 = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int sl = 0; sl < SLOTS2; ++sl) {
            const int j = sl / (2 * NDB), t = sl % (2 * NDB), n = t / 2, f = j * NDB + n;
            if (t % 2 == 0) {
                dq[n] = mfma32(f2[f], pg1[j], dq[n]);
                prefetch(NF1 + f, next_blk, cur_blk, after_blk);
            } else {
                dr[n] = mfma32(f2[f], pg2[j], dr[n]);
            }
            elem_stages(masked_tag, n1, n2, na, 0, sl, 1, SLOTS2, lim_next);
            if (sl == SLOTS2 - 2) nb1 = pack_group(na, 0);
            if (sl == SLOTS2 - 1) nb2 = pack_group(n2, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        pg1[0] = nb1;
        pg2[0] = nb2;
    };

    // Ring invariant at the top of iteration t: tiles t and (after the barrier) t + 1 are in
    // stages t % 3 and (t + 1) % 3; the barrier also proves that nobody reads tile t - 1 any more,
    // whose stage then receives tile t + 2.
    issue_tile(tile_at(0), 0);
    if (n_tiles > 1) issue_tile(tile_at(1), 1);
    if (n_tiles > 1)
        tile_barrier<2 * TL::NDMA>();  // tile 0 has landed (loads complete in order)
    else
        tile_barrier<0>();
    f32x16 a1, a2, a3, b1, b2, b3;
    {
        // prologue: scores of block (0, 0); its lower 16 keys -> g1 / g2; first fragments of (0, 1)
        const u32x4 *blk = k_block(0, 0);
        a1 = a2 = a3 = zero16();
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const u32x4 kf = blk[lo.nt[ks]], vf = blk[TL::CHUNKS + lo.nt[ks]];
            a1 = mfma32(kf, qf[ks], a1);
            a2 = mfma32(kf, rf[ks], a2);
            a3 = mfma32(vf, gf[ks], a3);
        }
#pragma unroll
        for (int sl = 0; sl < 12; ++sl)
            elem_stages(std::true_type{}, a1, a2, a3, 0, sl, 0, 12, lim_row - tile_at(0) * kTileRows - 4 * h);
        pg1[0] = pack_group(a3, 0);
        pg2[0] = pack_group(a2, 0);
#pragma unroll
        for (int f = 0; f < LA; ++f) load_f1(k_block(0, 1), f);
    }
    int stage = 0;
    auto tile_steps = [&](auto masked_tag, auto dma_tag, int t) __attribute__((always_inline)) {
        constexpr bool DMA = decltype(dma_tag)::value;
        const int next_stage = stage == STAGES - 1 ? 0 : stage + 1;
        const int free_stage = stage == 0 ? STAGES - 1 : stage - 1;
        tile_barrier<0>();  // tile t + 1 has landed; tile t - 1 is free
        if constexpr (DMA) {  // tile t + 2 is complete: fetched by the first step, slot by slot
            dma_lds = lds_base + (uint32_t)(free_stage * STAGE_CHUNKS + w * TL::NDMA * 64) * 16u;
        } else {
            if (t + 2 < n_tiles) issue_tile(tile_at(t + 2), free_stage);
        }
        const int key_base = tile_at(t) * kTileRows, key_base_after = tile_at(t + 1) * kTileRows;
        // block (t, 0) -> g, dQ / dR; scores of (t, 1); fragments of (t + 1, 0)
        pipeline_step(masked_tag, dma_tag, key_base, key_base + kBlk, k_block(stage, 1), k_block(stage, 0),
                      k_block(next_stage, 0), a1, a2, a3, b1, b2, b3);
        // block (t, 1) -> g, dQ / dR; scores of (t + 1, 0); fragments of (t + 1, 1)
        pipeline_step(masked_tag, std::false_type{}, key_base + kBlk, key_base_after, k_block(next_stage, 0),
                      k_block(stage, 1), k_block(next_stage, 1), b1, b2, b3, a1, a2, a3);
        stage = next_stage;
    };
    // tiles whose keys -- and those of the tile after (a step also prepares the lower half of the
    // next block) -- every row of the workgroup sees: no masks; then the diagonal / tail tiles.
    // The unmasked loop also stops two short of the last complete tile, so that the tile it
    // fetches exists completely.
    const int n_full = SPARSE ? 0 : min(CAUSAL ? (rb * 128 + off + 1) / kTileRows : Tk / kTileRows, Tk / kTileRows - 1);
    int t = 0;
    if constexpr (WINDOW) {
        // leading tiles that hold a key before the window of the block's last row
        const int n_left = min(n_tiles, max(rb * 128 + 128 + off - p.window + kTileRows - 1, 0) / kTileRows);
        for (; t < n_left; ++t) tile_steps(std::true_type{}, std::false_type{}, t);
    }
    const int64_t k_tile_bytes = (int64_t)kTileRows * 2 * p.ks[2], v_tile_bytes = (int64_t)kTileRows * 2 * p.vs[2];
    dma_k = (const char *)kbase + (t + 2) * k_tile_bytes;
    dma_v = (const char *)vbase + (t + 2) * v_tile_bytes;
    for (; t < n_full - 1; ++t) {
        tile_steps(std::false_type{}, std::true_type{}, t);
        dma_k += k_tile_bytes;
        dma_v += v_tile_bytes;
    }
    for (; t < n_tiles; ++t) tile_steps(std::true_type{}, std::false_type{}, t);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no tile load may land after the workgroup ends

    // dQ^T / dR^T register r of block n <-> dim 32n + 8*(r/4) + 4h + r%4 of row my_row
    if (my_row < T) {
        __bf16 *dq_row = (__bf16 *)p.dq + b * p.dqs[0] + hq * p.dqs[1] + my_row * p.dqs[2];
        __bf16 *dr_row = (__bf16 *)p.dr + b * p.drs[0] + hq * p.drs[1] + my_row * p.drs[2];
#pragma unroll
        for (int n = 0; n < NDB; ++n)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int dim = 32 * n + 8 * q4 + 4 * h;
                const u32x2 a = {pack_bf16(dq[n][4 * q4] * p.scale, dq[n][4 * q4 + 1] * p.scale),
                                 pack_bf16(dq[n][4 * q4 + 2] * p.scale, dq[n][4 * q4 + 3] * p.scale)};
                const u32x2 c = {pack_bf16(dr[n][4 * q4], dr[n][4 * q4 + 1]),
                                 pack_bf16(dr[n][4 * q4 + 2], dr[n][4 * q4 + 3])};
                *(u32x2 *)(dq_row + dim) = a;
                *(u32x2 *)(dr_row + dim) = c;
            }
    }
}

// ---- column pass: dK, dV ----------------------------------------------------------------------
// The same software pipeline over 32-row blocks of the streamed (Q, R, dO) tiles:
//   phase 1 : the 3 * d/16 score MFMAs of the NEXT row block (S1 = Q K^T, S2 = R K^T, A = dO V^T
//             alternate; the K, V fragments are the resident B operands), while the vector ALU
//             turns the upper 16 rows of the CURRENT block into w = p (1 + ubar - u), g1, g2;
//   phase 2 : the output MFMAs of the CURRENT block (dV^T += dO^T w, dK^T += Q^T g1, dK^T += R^T g2
//             alternate), while the vector ALU turns the lower 16 rows of the NEXT block.
// A lane owns a key, its registers the rows: the row scalars (lse, ubar, tau, beta) come from LDS,
// one float4 per register, read one slot ahead of their use.
// WINDOW: key j is seen by the rows [j - off, j - off + window) only; the row tiles past the
// last of them are not visited, those cut by the upper edge take the masked form.
template <int D, bool CAUSAL, bool WINDOW = false, bool SPARSE = false>
__global__ __launch_bounds__(256, 1) void bwd_dk_dv_kernel(PrefillBwdParams p) {
    static_assert(CAUSAL || !WINDOW, "a sliding window is causal");
    static_assert(!(SPARSE && WINDOW), "block lists and a sliding window do not combine");
    using TL = BwdTile<D>;
    constexpr int CPR = TL::CPR, KSTEPS = D / 16, NDB = D / 32;
    constexpr int STAGES = 3;
    constexpr int STAGE_CHUNKS = 3 * TL::CHUNKS + kTileRows;  // Q, R, dO tiles + one float4 per row
    __shared__ u32x4 lds[STAGES * STAGE_CHUNKS];

    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int col = lane & 31, h = lane >> 5;
    const int T = p.T, Tk = p.Tk, off = Tk - T, G = p.G;
    // Work item: the key block is the slowest index (causal: low key blocks see the most rows;
    // all of them come first, over every batch entry and head -- with the key block as the
    // fastest index the tail of the pass cost a quarter of it); (batch, kv head) pairs by
    // workgroup id modulo 8 onto the XCDs.
    int cb, hk, b;
    {
        const int id = blockIdx.x, pairs = p.B * p.Hkv;
        int pair;
        if (pairs % 8 == 0) {
            const int x = id & 7, j = id >> 3, per = pairs / 8;
            cb = j / per;
            pair = (j - cb * per) * 8 + x;
        } else {
            cb = id / pairs;
            pair = id - cb * pairs;
        }
        b = pair / p.Hkv;
        hk = pair - b * p.Hkv;
    }
    const int key0 = cb * 128 + w * 32, my_key = key0 + col;
    const int ld_key = min(my_key, Tk - 1);

    // B operands of the score MFMAs: column = key, k-elements = the 8 dims of chunk 2*ks + h
    u32x4 kf[KSTEPS], vf[KSTEPS];
    {
        const __bf16 *krow = (const __bf16 *)p.k + b * p.ks[0] + hk * p.ks[1] + ld_key * p.ks[2];
        const __bf16 *vrow = (const __bf16 *)p.v + b * p.vs[0] + hk * p.vs[1] + ld_key * p.vs[2];
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            kf[ks] = *(const u32x4 *)(krow + 8 * (2 * ks + h));
            vf[ks] = *(const u32x4 *)(vrow + 8 * (2 * ks + h));
        }
    }
    const float scale_log2 = p.scale * kLog2e, scale = p.scale;
    const BwdLaneOffsets<D> lo(lane);

    // row tiles that hold a row which sees a key of this block: rows i >= key - off
    const int rt_lo = CAUSAL ? max(cb * 128 - off, 0) / kTileRows : 0;
    const int n_rt = (T + kTileRows - 1) / kTileRows;
    // window: rows up to (last key of the block) - off + window - 1. A block no row sees at all
    // (keys before every window) still visits one tile, with every pair masked: zeros.
    const int rt_hi =
        WINDOW ? max(min(n_rt, (min(cb * 128 + 127, Tk - 1) - off + p.window + kTileRows - 1) / kTileRows), rt_lo + 1)
               : n_rt;
    const int per_head = rt_hi - rt_lo;
    int n_items = per_head * G;  // (head of the group, row tile)
    // Row tiles in which every (row, key) pair counts -- all rows exist and see every key of the
    // block, and the key block is complete -- need no masks. The items are taken in an order that
    // puts those of all heads first, so that the two forms of the pipeline are two loops.
    const int rt_full_lo = max(CAUSAL ? max(cb * 128 + 127 - off + kTileRows - 1, 0) / kTileRows : 0, rt_lo);
    // (window: the first key of the block is the first to drop out of a row's window)
    const int rt_full_hi =
        (cb + 1) * 128 <= Tk ? (WINDOW ? min(T, max(cb * 128 - off + p.window, 0)) : T) / kTileRows : 0;
    const int full_per_head = max(rt_full_hi - rt_full_lo, 0);
    const int n_full_items = full_per_head * G;
    const int rest_per_head = per_head - full_per_head;
    // Block-sparse: the items are, head after head of the group, the two row tiles of every row
    // block in the head's column list (entry = 4 * row block + flags; flag bit t: the row block
    // lists key tile 2 * cb + t). A cursor walks the lists; items are decoded in order, once each.
    using const_i32 = const __attribute__((address_space(4))) int32_t;
    const int n_cb = (Tk + 127) / 128, n_rb = (T + 127) / 128;
    auto col_list = [&](int g, int &first, int &end) __attribute__((always_inline)) {
        const int hq = hk * G + g;
        const int sb = p.sparse_batch > 1 ? b : 0, sh = p.sparse_heads > 1 ? hq : 0;
        const int64_t e = ((int64_t)sb * p.sparse_heads + sh) * n_cb + cb;
        const_i32 *col_ptr = (const_i32 *)(uintptr_t)p.sparse_col_ptr;
        first = col_ptr[e];
        end = max(col_ptr[e + 1], first);
    };
    int cur_g = 0, cur_pos = 0, cur_end = 0, cur_half = 0;  // the cursor: next item to decode
    if constexpr (SPARSE) {
        n_items = 0;
        for (int g = 0; g < G; ++g) {
            int first, end;
            col_list(g, first, end);
            n_items += 2 * (end - first);
        }
        cur_g = -1;
        while (cur_pos == cur_end && ++cur_g < G) col_list(cur_g, cur_pos, cur_end);  // first non-empty list
        if (n_items == 0) {  // (workgroup-uniform) nobody lists these keys: zero gradients
            if (my_key < Tk) {
                __bf16 *dk_row = (__bf16 *)p.dk + b * p.dks[0] + hk * p.dks[1] + my_key * p.dks[2];
                __bf16 *dv_row = (__bf16 *)p.dv + b * p.dvs[0] + hk * p.dvs[1] + my_key * p.dvs[2];
#pragma unroll
                for (int c = 0; c < D / 16; ++c) {
                    *(u32x4 *)(dk_row + 8 * (2 * c + h)) = u32x4{0u, 0u, 0u, 0u};
                    *(u32x4 *)(dv_row + 8 * (2 * c + h)) = u32x4{0u, 0u, 0u, 0u};
                }
            }
            return;
        }
    }
    // decodes the item under the cursor into (head of the group, row tile, flags) and moves on
    auto next_sparse_item = [&](int &g, int &rt, int &flags) __attribute__((always_inline)) {
        const int entry = ((const_i32 *)(uintptr_t)p.sparse_col_idx)[cur_pos];
        g = cur_g;
        rt = 2 * min(max(entry >> 2, 0), n_rb - 1) + cur_half;
        flags = entry & 3;
        cur_half ^= 1;
        if (cur_half == 0) {
            ++cur_pos;
            while (cur_pos == cur_end && ++cur_g < G) col_list(cur_g, cur_pos, cur_end);
        }
    };
    auto item_of = [&](int it, int &g, int &rt) __attribute__((always_inline)) {
        if (it < n_full_items) {
            g = it / full_per_head;
            rt = rt_full_lo + it % full_per_head;
        } else {
            const int j = it - n_full_items;
            g = j / rest_per_head;
            const int k = j % rest_per_head;  // the head's tiles before, then after, its full ones
            rt = rt_lo + k + (k >= rt_full_lo - rt_lo ? full_per_head : 0);
        }
    };

    const uint32_t lds_base = lds_byte_address(lds);
    auto issue_item_at = [&](int g, int rt, int stage) __attribute__((always_inline)) {
        const int hq = hk * G + g;
        const int64_t head = ((int64_t)b * p.Hq + hq) * T;
        const uint32_t s0 = lds_base + (uint32_t)(stage * STAGE_CHUNKS) * 16u;
        load_tile64<D>((const __bf16 *)p.q + b * p.qs[0] + hq * p.qs[1], p.qs[2], rt * kTileRows, T, s0, w, lane);
        load_tile64<D>((const __bf16 *)p.r + b * p.rs[0] + hq * p.rs[1], p.rs[2], rt * kTileRows, T,
                       s0 + (uint32_t)TL::CHUNKS * 16u, w, lane);
        load_tile64<D>((const __bf16 *)p.d_o + b * p.gs[0] + hq * p.gs[1], p.gs[2], rt * kTileRows, T,
                       s0 + (uint32_t)(2 * TL::CHUNKS) * 16u, w, lane);
        if (w == 0) {  // the rows' scalars, one float4 per lane
            const f32x4 *src = (const f32x4 *)p.row_cache + head + min(rt * kTileRows + lane, T - 1);
            tile_load16<64>(src, s0 + (uint32_t)(3 * TL::CHUNKS) * 16u);
        }
    };
    // The three items in flight: (head, row tile, flags) of item it, it + 1 and it + 2.
    int it_g[3] = {0, 0, 0}, it_rt[3] = {0, 0, 0}, it_flags[3] = {3, 3, 3};
    auto issue_item = [&](int it, int stage, int slot) __attribute__((always_inline)) {
        if constexpr (SPARSE)
            next_sparse_item(it_g[slot], it_rt[slot], it_flags[slot]);
        else
            item_of(it, it_g[slot], it_rt[slot]);
        issue_item_at(it_g[slot], it_rt[slot], stage);
    };
    constexpr int kItemLoads = 3 * TL::NDMA;  // per wave (wave 0 issues one more, last)
    // The unmasked loop spreads the loads of item it + 2 over the MFMA slots of a step: per-lane
    // byte offsets inside a complete tile, wave-uniform tile bases. (There every wave fetches the
    // 64 row scalars -- the same bytes to the same place -- so that the slots hold no branch.)
    uint32_t toffq[TL::NDMA], toffr[TL::NDMA], toffg[TL::NDMA];
#pragma unroll
    for (int i = 0; i < TL::NDMA; ++i) {
        const int c = (w * TL::NDMA + i) * 64 + lane;
        const int row = c / CPR;
        const int chunk = (c % CPR) ^ lds_row_swizzle<D>(row);
        toffq[i] = (uint32_t)(row * (int)p.qs[2] + chunk * 8) * 2u;
        toffr[i] = (uint32_t)(row * (int)p.rs[2] + chunk * 8) * 2u;
        toffg[i] = (uint32_t)(row * (int)p.gs[2] + chunk * 8) * 2u;
    }
    const char *dma_q = nullptr, *dma_r = nullptr, *dma_g = nullptr, *dma_rc = nullptr;
    uint32_t dma_lds = 0, dma_lds_rc = 0;
    auto set_dma_item = [&](int g, int rt, int stage) __attribute__((always_inline)) {
        const int hq = hk * G + g;
        const int64_t row0 = (int64_t)rt * kTileRows;
        dma_q = (const char *)p.q + (b * p.qs[0] + hq * p.qs[1] + row0 * p.qs[2]) * 2;
        dma_r = (const char *)p.r + (b * p.rs[0] + hq * p.rs[1] + row0 * p.rs[2]) * 2;
        dma_g = (const char *)p.d_o + (b * p.gs[0] + hq * p.gs[1] + row0 * p.gs[2]) * 2;
        dma_rc = (const char *)p.row_cache + (((int64_t)b * p.Hq + hq) * T + row0) * 16;
        dma_lds = lds_base + (uint32_t)(stage * STAGE_CHUNKS + w * TL::NDMA * 64) * 16u;
        dma_lds_rc = lds_base + (uint32_t)(stage * STAGE_CHUNKS + 3 * TL::CHUNKS) * 16u;
    };
    auto dma_slot = [&](int i) __attribute__((always_inline)) {  // load i of 3 * NDMA + 1
        if (i < TL::NDMA)
            tile_load16_uniform<false>(toffq[i], dma_q, dma_lds + 1024u * i);
        else if (i < 2 * TL::NDMA)
            tile_load16_uniform<false>(toffr[i - TL::NDMA], dma_r,
                                       dma_lds + (uint32_t)TL::CHUNKS * 16u + 1024u * (i - TL::NDMA));
        else if (i < 3 * TL::NDMA)
            tile_load16_uniform<false>(toffg[i - 2 * TL::NDMA], dma_g,
                                       dma_lds + (uint32_t)(2 * TL::CHUNKS) * 16u + 1024u * (i - 2 * TL::NDMA));
        else
            tile_load16_uniform<false>((uint32_t)lane * 16u, dma_rc, dma_lds_rc);
    };
    // Q-tile pointer of row block rbk of a stage; the R and dO tiles follow at + CHUNKS each
    auto q_block = [&](int stage, int rbk) __attribute__((always_inline)) {
        return (const u32x4 *)(lds + stage * STAGE_CHUNKS + rbk * kBlk * CPR);
    };
    auto row_scalars = [&](int stage, int rbk) __attribute__((always_inline)) {
        return (const f32x4 *)(lds + stage * STAGE_CHUNKS + 3 * TL::CHUNKS) + rbk * kBlk + 4 * h;
    };

    f32x16 dk[NDB], dv[NDB];
#pragma unroll
    for (int n = 0; n < NDB; ++n) dk[n] = dv[n] = zero16();

    // fragments in flight
    constexpr int NF1 = 3 * KSTEPS, NF2 = 6 * NDB, LA = 5;  // (5 against 3: 1 % on the config-4 pass)
    u32x4 f1[NF1], f2[NF2];
    auto load_f1 = [&](const u32x4 *qblk, int f) __attribute__((always_inline)) {  // (k-step, Q / R / dO chunk)
        f1[f] = qblk[(f % 3) * TL::CHUNKS + lo.nt[f / 3]];
    };
    auto load_f2 = [&](const u32x4 *qblk, int f) __attribute__((always_inline)) {  // (j, n, dO^T / Q^T / R^T)
        const int j = f / (3 * NDB), n = (f % (3 * NDB)) / 3, which = f % 3;
        const int tile = which == 0 ? 2 : which - 1;
        f2[f] = lo.transposed((const unsigned short *)(qblk + tile * TL::CHUNKS), j, n);
    };
    auto prefetch = [&](int f, const u32x4 *next_blk, const u32x4 *cur_blk, const u32x4 *after_blk)
                        __attribute__((always_inline)) {
        const int g = f + LA;
        if (g < NF1)
            load_f1(next_blk, g);
        else if (g < NF1 + NF2)
            load_f2(cur_blk, g - NF1);
        else
            load_f1(after_blk, g - NF1 - NF2);
    };

    // Element-wise work of the 8 score registers [r0, r0 + 8) of a block in five stages (row
    // scalars from LDS first); the results replace the scores: g1 / h in aa, g2 in s2, and
    // w = p (1 + ubar - u) in wv. Register r holds row offset 8*(r/4) + r%4 (+ 4h): with MASKED a
    // pair counts iff lo <= offset < lo + span (rows that exist and see this lane's key).
    f32x4 rcv[8];
    float dl[8], wodd = 0.f;
    uint32_t wp[4];  // w of the 8 registers, packed in pairs as they are produced
    auto elem_stages = [&](auto masked_tag, f32x16 &s1, f32x16 &s2, f32x16 &aa, const f32x4 *rows, int r0,
                           int slot, int slot0, int n_slots, int neg_lo, unsigned span)
                           __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int r = r0 + u;
            // (the row scalars are read two slots ahead of their use: an LDS read takes longer
            // than one MFMA slot)
            const int first = slot0 + u * (n_slots - 8 - slot0) / 7;
            if (slot == first) rcv[u] = rows[8 * (r >> 2) + (r & 3)];  // (lse, 1 + ubar, beta - tau, beta)
            if (slot == first + 2) {
                s1[r] = fmaf(s1[r], scale_log2, -rcv[u][0]);
                dl[u] = aa[r] - rcv[u][3];       // delta
                s2[r] = rcv[u][1] - s2[r];       // 1 + ubar - u
            }
            if (slot == first + 3) {
                s1[r] = fast_exp2(s1[r]);                // p
                aa[r] = fmaf(s2[r], dl[u], rcv[u][2]);   // a - tau + (ubar - u) delta
            }
            if constexpr (MASKED)
                if (slot == first + 4)
                    s1[r] = ((unsigned)(8 * (r >> 2) + (r & 3) + neg_lo) < span) ? s1[r] : 0.f;
            if (slot == first + 5) {
                const float wgt = s1[r] * s2[r];  // p (1 + ubar - u)
                if (u % 2 == 0)
                    wodd = wgt;
                else
                    wp[u / 2] = pack_bf16(wodd, wgt);
                aa[r] = (s1[r] * scale) * aa[r];    // g1 / h
                s2[r] = -(s1[r] * dl[u]);           // g2
            }
        }
    };
    auto pack_w = [&]() __attribute__((always_inline)) { return u32x4{wp[0], wp[1], wp[2], wp[3]}; };

    u32x4 pw[2], pg1[2], pg2[2];
    // rows of the block that starts at row_base which exist and see this lane's key:
    // offsets [lo, hi) relative to row_base + 4h
    auto row_window = [&](int row_base, int flags, int &neg_lo, unsigned &span) __attribute__((always_inline)) {
        // (block-sparse: a row block that does not list this wave's key tile -- none of its rows)
        const bool listed = !SPARSE || ((flags >> (w >> 1)) & 1) != 0;
        const int first_row = (my_key < Tk && listed) ? (CAUSAL ? max(my_key - off, 0) : 0) : T;  // no row at all
        const int end_row = WINDOW ? min(T, max(my_key - off + p.window, 0)) : T;
        const int lo_off = max(first_row - row_base - 4 * h, 0);
        const int hi_off = end_row - row_base - 4 * h;
        neg_lo = -lo_off;
        span = (unsigned)max(hi_off - lo_off, 0);
    };
    auto pipeline_step = [&](auto masked_tag, auto dma_tag, int row_base_cur, int flags_cur, int row_base_next,
                             int flags_next, const u32x4 *next_blk,
                             const u32x4 *cur_blk, const u32x4 *after_blk, const f32x4 *rows_cur,
                             const f32x4 *rows_next, f32x16 &c1, f32x16 &c2, f32x16 &ca, f32x16 &n1,
                             f32x16 &n2, f32x16 &na) __attribute__((always_inline)) {
        int nlo_c, nlo_n;
        unsigned span_c, span_n;
        row_window(row_base_cur, flags_cur, nlo_c, span_c);
        row_window(row_base_next, flags_next, nlo_n, span_n);
        constexpr int SLOTS1 = 3 * KSTEPS, SLOTS2 = 6 * NDB;
        constexpr bool DMA = decltype(dma_tag)::value;  // this step also fetches the item set_dma_item named
        static_assert(3 * TL::NDMA + 1 <= SLOTS1, "one tile load per slot");
#pragma unroll
        for (int sl = 0; sl < SLOTS1; ++sl) {
            const int ks = sl / 3, which = sl % 3;
            if constexpr (DMA)
                if (sl < 3 * TL::NDMA + 1) dma_slot(sl);
            f32x16 &dst = which == 0 ? n1 : which == 1 ? n2 : na;
            if (ks == 0)
                mfma32_scores_first<true>(dst, f1[sl], which == 2 ? vf[ks] : kf[ks]);
            else
                mfma32_scores<true>(dst, f1[sl], which == 2 ? vf[ks] : kf[ks]);
            prefetch(sl, next_blk, cur_blk, after_blk);
            elem_stages(masked_tag, c1, c2, ca, rows_cur, 8, sl, 0, SLOTS1, nlo_c, span_c);
            if (sl == SLOTS1 - 2) {
                pw[1] = pack_w();
                pg1[1] = pack_group(ca, 1);
            }
            if (sl == SLOTS1 - 1) pg2[1] = pack_group(c2, 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        u32x4 nw = {0u, 0u, 0u, 0u}, nb1 = {0u, 0u, 0u, 0u}, nb2 = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int sl = 0; sl < SLOTS2; ++sl) {
            const int j = sl / (3 * NDB), n = (sl % (3 * NDB)) / 3, which = sl % 3;
            if (which == 0)
                dv[n] = mfma32(f2[sl], pw[j], dv[n]);
            else if (which == 1)
                dk[n] = mfma32(f2[sl], pg1[j], dk[n]);
            else
                dk[n] = mfma32(f2[sl], pg2[j], dk[n]);
            prefetch(NF1 + sl, next_blk, cur_blk, after_blk);
            elem_stages(masked_tag, n1, n2, na, rows_next, 0, sl, 1, SLOTS2, nlo_n, span_n);
            if (sl == SLOTS2 - 2) {
                nw = pack_w();
                nb1 = pack_group(na, 0);
            }
            if (sl == SLOTS2 - 1) nb2 = pack_group(n2, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        pw[0] = nw;
        pg1[0] = nb1;
        pg2[0] = nb2;
    };

    // Ring invariant at the top of iteration it: items it and (after the barrier) it + 1 are in
    // stages it % 3 and (it + 1) % 3; the barrier also proves that nobody reads item it - 1 any
    // more, whose stage then receives item it + 2.
    issue_item(0, 0, 0);
    if (n_items > 1) issue_item(1, 1, 1);
    // item 0 has landed (loads complete in order; wave 0 has one more in flight per item)
    if (n_items > 1) {
        if (w == 0)
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kItemLoads + 1) : "memory");
        else
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kItemLoads) : "memory");
    } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();
    f32x16 a1, a2, a3, b1, b2, b3;
    {
        // prologue: scores of row block 0 of item 0; its lower 16 rows -> w, g1, g2
        const u32x4 *blk = q_block(0, 0);
        a1 = a2 = a3 = zero16();
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            a1 = mfma32(blk[lo.nt[ks]], kf[ks], a1);
            a2 = mfma32(blk[TL::CHUNKS + lo.nt[ks]], kf[ks], a2);
            a3 = mfma32(blk[2 * TL::CHUNKS + lo.nt[ks]], vf[ks], a3);
        }
        int nlo;
        unsigned span;
        row_window(it_rt[0] * kTileRows, it_flags[0], nlo, span);
#pragma unroll
        for (int sl = 0; sl < 16; ++sl)
            elem_stages(std::true_type{}, a1, a2, a3, row_scalars(0, 0), 0, sl, 0, 16, nlo, span);
        pw[0] = pack_w();
        pg1[0] = pack_group(a3, 0);
        pg2[0] = pack_group(a2, 0);
#pragma unroll
        for (int f = 0; f < LA; ++f) load_f1(q_block(0, 1), f);
    }
    int stage = 0;
    auto item_steps = [&](auto masked_tag, auto dma_tag, int it) __attribute__((always_inline)) {
        constexpr bool DMA = decltype(dma_tag)::value;
        const int next_stage = stage == STAGES - 1 ? 0 : stage + 1;
        const int free_stage = stage == 0 ? STAGES - 1 : stage - 1;
        tile_barrier<0>();  // item it + 1 has landed; item it - 1 is free
        // (items it, it + 1, it + 2 sit in slots 0, 1, 2 of the item record)
        if constexpr (DMA) {  // item it + 2 is a complete tile: fetched by the first step, slot by slot
            item_of(it + 2, it_g[2], it_rt[2]);
            set_dma_item(it_g[2], it_rt[2], free_stage);
        } else {
            if (it + 2 < n_items) issue_item(it + 2, free_stage, 2);
        }
        const int row_base = it_rt[0] * kTileRows, row_base_after = it_rt[1] * kTileRows;  // (past the end: never used)
        const int flags = it_flags[0], flags_after = it_flags[1];
        // row block 0 -> w, g; dV / dK; scores of row block 1; fragments of the next item
        pipeline_step(masked_tag, dma_tag, row_base, flags, row_base + kBlk, flags, q_block(stage, 1), q_block(stage, 0),
                      q_block(next_stage, 0), row_scalars(stage, 0), row_scalars(stage, 1), a1, a2, a3, b1, b2,
                      b3);
        // row block 1 -> w, g; dV / dK; scores of row block 0 of the next item
        pipeline_step(masked_tag, std::false_type{}, row_base + kBlk, flags, row_base_after, flags_after,
                      q_block(next_stage, 0), q_block(stage, 1),
                      q_block(next_stage, 1), row_scalars(stage, 1), row_scalars(next_stage, 0), b1, b2, b3, a1,
                      a2, a3);
        stage = next_stage;
#pragma unroll
        for (int j = 0; j < 2; ++j) it_g[j] = it_g[j + 1], it_rt[j] = it_rt[j + 1], it_flags[j] = it_flags[j + 1];
    };
    // a step also prepares the lower half of the next item's first block, and the unmasked loop
    // fetches item it + 2 as a complete tile: it stops two short of the last unmasked item
    int it = 0;
    if constexpr (!SPARSE)
        for (; it < n_full_items - 2; ++it) item_steps(std::false_type{}, std::true_type{}, it);
    for (; it < n_items; ++it) item_steps(std::true_type{}, std::false_type{}, it);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no tile load may land after the workgroup ends

    // dK^T / dV^T register r of block n <-> dim 32n + 8*(r/4) + 4h + r%4 of key my_key
    if (my_key < Tk) {
        __bf16 *dk_row = (__bf16 *)p.dk + b * p.dks[0] + hk * p.dks[1] + my_key * p.dks[2];
        __bf16 *dv_row = (__bf16 *)p.dv + b * p.dvs[0] + hk * p.dvs[1] + my_key * p.dvs[2];
#pragma unroll
        for (int n = 0; n < NDB; ++n)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int dim = 32 * n + 8 * q4 + 4 * h;
                const u32x2 a = {pack_bf16(dk[n][4 * q4], dk[n][4 * q4 + 1]),
                                 pack_bf16(dk[n][4 * q4 + 2], dk[n][4 * q4 + 3])};
                const u32x2 c = {pack_bf16(dv[n][4 * q4], dv[n][4 * q4 + 1]),
                                 pack_bf16(dv[n][4 * q4 + 2], dv[n][4 * q4 + 3])};
                *(u32x2 *)(dk_row + dim) = a;
                *(u32x2 *)(dv_row + dim) = c;
            }
    }
}

template <int D>
static hipError_t launch_bwd_d(const PrefillBwdParams &p, hipStream_t stream) {
    const long long n_rows = (long long)p.B * p.Hq * p.T;
    constexpr int kPrepRows = 2048 / D;  // rows per workgroup of the rows-prepare kernel
    const long long g0 = (n_rows + kPrepRows - 1) / kPrepRows;
    const long long g1 = (long long)((p.T + 127) / 128) * p.Hq * p.B;
    const long long g2 = (long long)((p.Tk + 127) / 128) * p.Hkv * p.B;
    if (g0 > 0x7fffffffLL || g1 > 0x7fffffffLL || g2 > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((bwd_rows_prepare_kernel<D>), dim3((unsigned)g0), dim3(256), 0, stream, p);
    if (p.sparse_row_ptr != nullptr) {  // block lists (no window; checked by the caller)
        if (p.causal) {
            hipLaunchKernelGGL((bwd_dq_dr_kernel<D, true, false, true>), dim3((unsigned)g1), dim3(256), 0, stream, p);
            hipLaunchKernelGGL((bwd_dk_dv_kernel<D, true, false, true>), dim3((unsigned)g2), dim3(256), 0, stream, p);
        } else {
            hipLaunchKernelGGL((bwd_dq_dr_kernel<D, false, false, true>), dim3((unsigned)g1), dim3(256), 0, stream, p);
            hipLaunchKernelGGL((bwd_dk_dv_kernel<D, false, false, true>), dim3((unsigned)g2), dim3(256), 0, stream, p);
        }
    } else if (p.causal && p.window > 0) {
        hipLaunchKernelGGL((bwd_dq_dr_kernel<D, true, true>), dim3((unsigned)g1), dim3(256), 0, stream, p);
        hipLaunchKernelGGL((bwd_dk_dv_kernel<D, true, true>), dim3((unsigned)g2), dim3(256), 0, stream, p);
    } else if (p.causal) {
        hipLaunchKernelGGL((bwd_dq_dr_kernel<D, true>), dim3((unsigned)g1), dim3(256), 0, stream, p);
        hipLaunchKernelGGL((bwd_dk_dv_kernel<D, true>), dim3((unsigned)g2), dim3(256), 0, stream, p);
    } else {
        hipLaunchKernelGGL((bwd_dq_dr_kernel<D, false>), dim3((unsigned)g1), dim3(256), 0, stream, p);
        hipLaunchKernelGGL((bwd_dk_dv_kernel<D, false>), dim3((unsigned)g2), dim3(256), 0, stream, p);
    }
    return hipGetLastError();
}

hipError_t launch_prefill_bwd_bf16(const PrefillBwdParams &p, hipStream_t stream) {
    return p.d == 128 ? launch_bwd_d<128>(p, stream) : launch_bwd_d<64>(p, stream);
}

}  // namespace plx
