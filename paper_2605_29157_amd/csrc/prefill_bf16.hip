// Causal / full Parallax prefill forward for bf16 on gfx950.
//
// What it computes: Algorithm 1 of the paper (Sec. 3.3) -- for a block of query rows, one pass
// over key tiles with the running state (m, d1, d2, O1, O2); S1 = Q K^T * scale (masked),
// S2 = R K^T (unscaled), P1 = exp2(S1 - m), P2 = P1 * S2, O1 += P1 V, O2 += P2 V; closing
// formula O1/d1 * (1 + d2/d1) - O2/d1. Causal: key j allowed iff j <= i (Sec. 3.1); with more
// keys than query rows the rows are the last positions of the sequence, j <= i + (Tk - T).
//
// Layout for CDNA4:
//   * one workgroup = 4 waves, one wave per SIMD, so a wave may use the whole 512-register
//     budget: O1^T, O2^T and the Q, R fragments live in the accumulation registers for the whole
//     pass -- an MFMA can take its B operand from there -- and the vector registers hold scores,
//     P and LDS fragments. A wave owns RW sub-blocks of 32 query rows: one at d = 128 (128 rows
//     per workgroup); two at d = 64 (256 rows per workgroup), where the accumulators of 64 rows
//     fit and every K / V^T fragment read from LDS then feeds four MFMAs instead of two, with
//     half as many tile barriers and workgroups per MFMA;
//   * every global read is a direct global -> LDS load of whole rows (global_load_lds_dwordx4:
//     no staging registers, no LDS write instructions): the wave's own Q and R rows once, then
//     K/V tiles of 64 keys into a three-stage ring, fetched two tiles ahead, one load per MFMA
//     slot of the pipeline. Rows are padded, not swizzled, so that every operand address is a
//     per-lane base plus a constant; one workgroup barrier per tile;
//   * scores are produced transposed with v_mfma_f32_32x32x16_bf16, S^T = K Q^T: each K
//     fragment read from LDS feeds two MFMAs (the q branch and the r branch). In the S^T
//     accumulator a lane owns ONE query row (column) and 16 of the 32 keys, so softmax
//     statistics are per lane, S1 and S2 of a (row, key) pair share lane and register, and the
//     accumulator registers are already the B operand of O^T += V^T P^T (V^T fragments come
//     from transposing LDS reads);
//   * key blocks of 32 are software-pipelined in slots of one MFMA plus its share of vector
//     work: the score MFMAs of block i+1 run under the exp arithmetic of block i, the PV MFMAs
//     of block i under the exp arithmetic of block i+1;
//   * row sums d1, d2: per-lane fp32 adds in tiles every row sees completely; in diagonal /
//     tail tiles MFMAs against a matrix of ones, i.e. sums of exactly the bf16 operands that
//     enter O1 / O2, so that rows with very few keys come out exact (row 0 returns v_0).
//
// The running max m of Algorithm 1 only has to keep exp2 in range: ANY per-row reference gives
// the same O after the final division. The fast pass therefore fixes m to the row maximum over
// the first key block and never rescales O1/O2 (no vector-ALU work on the 128 accumulator
// registers inside the loop). If a later score exceeds that reference by more than ~2^7 in the
// exp2 domain the sums overflow to inf/NaN; this is detected at the end of the pass and the
// workgroup redoes its rows with the textbook online update (max, alpha rescale) -- slower, and
// in practice never taken for attention logits, but it keeps the softmax safe for every input.
#include <type_traits>

#include "plx_device.h"
#include "plx_kernels.h"
#include "plx_lds_dma.h"
#include "plx_mfma_asm.h"

namespace plx {


constexpr int kBC = 64;   // keys per LDS tile
constexpr int kKB = 32;   // keys per inner block (one MFMA row block)



// RW: sub-blocks of 32 query rows per wave (the workgroup covers 128 * RW rows).
// PREP: RMSNorm + RoPE on the wave's Q and R rows in their LDS landing zones, before the MFMA
// fragments are read (the operations the paper's language-model runs put in front of the attention
// call: Sec. 5 experiment setup and the backbone appendix; same formulas and order of operations as
// norm_rope.hip, the rotation taken from a table of (cos, sin) per position and pair).
template <int D, bool USE_R, bool CAUSAL, bool WINDOW, bool STATS = false, bool SPARSE = false, int RW = 1,
          bool PREP = false>
__global__ __launch_bounds__(256, 1) void prefill_bf16_kernel(PrefillParams p) {
    static_assert(!PREP || (USE_R && !WINDOW && !STATS && !SPARSE), "q / rho preparation: dense forward only");
    static_assert(RW == 1 || (RW == 2 && D == 64), "two row sub-blocks per wave fit the registers at d = 64 only");
    static_assert(!SPARSE || RW == 1, "block-sparse lists are per 128 query rows");
    constexpr int WROWS = 32 * RW;  // query rows per wave
    constexpr int kBR = 4 * WROWS;  // query rows per workgroup
    static_assert(CAUSAL || !WINDOW, "a sliding window needs the rows' positions");
    static_assert(!STATS || USE_R, "the row cache is written for the backward pass only");
    static_assert(!SPARSE || !WINDOW, "block-sparse: its own tile iterator, no window");
    constexpr int CPR = D / 8;            // 16-byte chunks per row
    constexpr int KSTEPS = D / 16;        // k-steps of the score contraction
    constexpr int NDB = D / 32;           // 32-wide blocks of output dimensions
    constexpr int STAGES = 3;  // LDS ring; tiles are fetched STAGES - 1 ahead
    constexpr int kDist = STAGES - 1;
    // K rows are padded by one 16-byte chunk (16 consecutive rows, same chunk -> 16 different
    // bank groups), V rows by four chunks (the 4 consecutive rows of a transposing read land in
    // 4 different 64-byte bank groups). Tiles are filled by direct global->LDS loads: one
    // wave-wide instruction writes 64 consecutive chunks, so each lane fetches the global chunk
    // that belongs at its LDS position (padding positions re-fetch a neighbour), and both tiles
    // are rounded up to NDMA * 4 * 64 chunks.
    constexpr int KROW = CPR + 1, VROW = CPR + 4;  // row strides in chunks
    // Every wave fills a contiguous quarter of each tile: 16 * KROW chunks of K (CPR / 4 full
    // 64-lane loads and one 16-lane load), 16 * VROW chunks of V (CPR / 4 + 1 full loads).
    constexpr int K_WAVE_CHUNKS = 16 * KROW, V_WAVE_CHUNKS = 16 * VROW;
    constexpr int NDMA_K = CPR / 4 + 1, NDMA_V = CPR / 4 + 1;
    static_assert(K_WAVE_CHUNKS == 64 * (NDMA_K - 1) + 16 && V_WAVE_CHUNKS == 64 * NDMA_V, "split");
    constexpr int K_CHUNKS = kBC * KROW, V_CHUNKS = kBC * VROW;
    constexpr int kTileLoads = NDMA_K + NDMA_V;  // per wave and tile
    constexpr int STAGE_CHUNKS = K_CHUNKS + V_CHUNKS;

    // Behind the ring: one padded WROWS x D tile per wave. It receives the wave's Q rows at the
    // start and stages its output rows at the end. The R rows land in ring stage 2 where they
    // fit (RW = 1), else in a zone of their own behind the Q zone.
    constexpr int WAVE_TILE_CHUNKS = WROWS * KROW;
    constexpr int QZONE = STAGES * STAGE_CHUNKS;
    constexpr bool R_IN_RING = 4 * WAVE_TILE_CHUNKS <= STAGE_CHUNKS;
    static_assert(STAGES >= 3 && (R_IN_RING || RW > 1), "R rows land in ring stage 2");
    constexpr int RZONE = R_IN_RING ? 2 * STAGE_CHUNKS : QZONE + 4 * WAVE_TILE_CHUNKS;
    constexpr int LDS_CHUNKS = QZONE + (R_IN_RING ? 4 : 8) * WAVE_TILE_CHUNKS;
    static_assert(LDS_CHUNKS * 16 <= 160 * 1024, "LDS of one compute unit");
    __shared__ u32x4 lds[LDS_CHUNKS];  // [stage][K tile | V tile], Q (, R)

    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int col = lane & 31;  // MFMA column: query row within the wave's 32 rows
    const int h = lane >> 5;    // half-wave

    // ---- work item: heavy row blocks first; blocks of one (batch, kv head) share an XCD ----
    const int T = p.T, G = p.G;  // query rows
    const int nrb = (T + kBR - 1) / kBR;
    const int pairs = p.B * p.Hkv;
    int rbi, pair, hg;
    {
        const int id = blockIdx.x;
        if (pairs % 8 == 0) {
            const int x = id & 7, j = id >> 3;
            const int per = (pairs / 8) * G;
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
    }
    const int rb = CAUSAL ? nrb - 1 - rbi : rbi;
    // Sliding window: row i sees the keys i + off - window + 1 .. i + off. The key tiles before
    // the first key of the workgroup's first row are skipped by moving the K / V base; from
    // here on key positions, Tk and off are relative to that first tile.
    const int kt_skip = WINDOW ? max(rb * kBR + (p.Tk - T) - p.window + 1, 0) / kBC : 0;
    const int Tk = p.Tk - kt_skip * kBC;  // keys
    const int off = Tk - T;               // causal: row i sits at key position i + off
    const int b = pair / p.Hkv, hk = pair - b * p.Hkv;
    const int hq = hk * G + hg;

    const int row0 = rb * kBR + w * WROWS;  // first query row of this wave
    // this lane's query row in sub-block a (may be >= T)
    auto my_row = [&](int a) __attribute__((always_inline)) { return row0 + 32 * a + col; };

    // ---- Q / R rows of this wave: global -> LDS, whole rows (a lane fetching its own MFMA
    // fragments straight from global memory would touch 64 different rows per instruction).
    // Padded like a K tile; nobody else reads them, so no barrier is needed for them. Q lands
    // behind the ring, R in ring stage 2, which the tile loads do not reach before the first
    // loop iteration -- by then the fragments are in registers -- or behind the Q zone.
    constexpr int NDMA_Q = (WAVE_TILE_CHUNKS + 63) / 64;  // full loads (+ one 32-lane load)
    constexpr int Q_LAST_LANES = WAVE_TILE_CHUNKS - 64 * (NDMA_Q - 1);
    static_assert(Q_LAST_LANES == 32 || Q_LAST_LANES == 64, "split");
    // PREP: a wave-wide pass covers 64 / CPR rows (one 16-byte chunk = 4 pairs per lane); the
    // weights of this lane's chunk and the table entries of its rows are requested first of all,
    // so that they are there when the rows have landed.
    constexpr int PREP_RPI = 64 / CPR, PREP_NIT = WROWS / PREP_RPI;
    f32x4 prep_gq[2], prep_gr[2], prep_tab[PREP ? PREP_NIT : 1][2];
    if constexpr (PREP) {
        const int lr = lane % CPR, lrow = lane / CPR;
        prep_gq[0] = *(const f32x4 *)(p.prep.gamma_q + 8 * lr), prep_gq[1] = *(const f32x4 *)(p.prep.gamma_q + 8 * lr + 4);
        prep_gr[0] = *(const f32x4 *)(p.prep.gamma_r + 8 * lr), prep_gr[1] = *(const f32x4 *)(p.prep.gamma_r + 8 * lr + 4);
        if (p.prep.table != nullptr) {  // workgroup-uniform
            const int base = p.prep.pos0 ? p.prep.pos0[b] : 0;
#pragma unroll
            for (int it = 0; it < PREP_NIT; ++it) {
                const int grow = min(row0 + it * PREP_RPI + lrow, T - 1);
                const int64_t pos = min(max(base + grow, 0), p.prep.n_pos - 1);
                const float *e = p.prep.table + (pos * (D / 2) + 4 * lr) * 2;
                prep_tab[it][0] = *(const f32x4 *)e, prep_tab[it][1] = *(const f32x4 *)(e + 4);
            }
        }
    }
    const uint32_t lds_base = lds_byte_address(lds);
    {
        const __bf16 *qhead = (const __bf16 *)p.q + b * p.qs[0] + hq * p.qs[1];
        const __bf16 *rhead = (const __bf16 *)p.r + b * p.rs[0] + hq * p.rs[1];
        const uint32_t dq = lds_base + (uint32_t)(QZONE + w * WAVE_TILE_CHUNKS) * 16u;
        const uint32_t dr = lds_base + (uint32_t)(RZONE + w * WAVE_TILE_CHUNKS) * 16u;
#pragma unroll
        for (int i = 0; i < NDMA_Q; ++i) {
            const int c = 64 * i + lane;  // lanes >= 32 of a half last load: unused
            const int64_t grow = min(row0 + min(c / KROW, WROWS - 1), T - 1);
            const int pos = min(c % KROW, CPR - 1);
            const __bf16 *sq = qhead + grow * p.qs[2] + pos * 8;
            const __bf16 *sr = rhead + grow * p.rs[2] + pos * 8;
            if (i == NDMA_Q - 1 && Q_LAST_LANES == 32) {
                tile_load16<32>(sq, dq + 1024u * i);
                if constexpr (USE_R) tile_load16<32>(sr, dr + 1024u * i);
            } else {
                tile_load16<64>(sq, dq + 1024u * i);
                if constexpr (USE_R) tile_load16<64>(sr, dr + 1024u * i);
            }
        }
    }
    u32x4 qf[RW][KSTEPS], rf[RW][KSTEPS];

    const __bf16 *kbase = (const __bf16 *)p.k + b * p.ks[0] + hk * p.ks[1] + (int64_t)kt_skip * kBC * p.ks[2];
    const __bf16 *vbase = (const __bf16 *)p.v + b * p.vs[0] + hk * p.vs[1] + (int64_t)kt_skip * kBC * p.vs[2];

    const int key_end = CAUSAL ? min(Tk, (rb + 1) * kBR + off) : Tk;  // keys this workgroup may need
    // Block-sparse: the workgroup visits only the key tiles its row block lists (ascending tile
    // indices, caller's arrays); the ring position i and the key tile tile_at(i) then differ.
    // Entries are clamped to existing tiles, listed tiles past the causal limit are dropped.
    // (read through the constant address space: uniform, never written while the kernel runs, so the
    // reads are scalar loads that the tile loads in flight do not hold up)
    using const_i32 = const __attribute__((address_space(4))) int32_t;
    const_i32 *tile_list = nullptr;
    int n_list = 0;
    if constexpr (SPARSE) {
        const int sb = p.sparse_batch > 1 ? b : 0, sh = p.sparse_heads > 1 ? hq : 0;
        const int64_t e = ((int64_t)sb * p.sparse_heads + sh) * nrb + rb;
        const_i32 *row_ptr = (const_i32 *)(uintptr_t)p.sparse_row_ptr;
        const int first = row_ptr[e];
        tile_list = (const_i32 *)(uintptr_t)p.sparse_tile_idx + first;
        n_list = max(row_ptr[e + 1] - first, 0);
    }
    // number of leading list entries whose first key lies below `bound` (binary search: the list ascends)
    auto list_count = [&](int bound) __attribute__((always_inline)) {
        int lo = 0, hi = n_list;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if ((int64_t)max(tile_list[mid], 0) * kBC < bound)
                lo = mid + 1;
            else
                hi = mid;
        }
        return lo;
    };
    // all 64 keys of these leading entries exist and are visible to every row of the workgroup
    const int vis_end = CAUSAL ? min(rb * kBR + off + 1, Tk) : Tk;
    const int n_list_full = SPARSE ? list_count(vis_end - kBC + 1) : 0;
    if constexpr (SPARSE) n_list = list_count(key_end);
    // a row block that lists nothing runs one tile with every key masked: sums of zero, zeros out
    const bool no_tiles = SPARSE && n_list == 0;
    auto tile_at = [&](int i) __attribute__((always_inline)) {
        if constexpr (SPARSE)
            return no_tiles ? 0 : min(max(tile_list[min(i, n_list - 1)], 0), (Tk - 1) / kBC);
        else
            return i;
    };
    int n_tiles_ = SPARSE ? max(n_list, 1) : (key_end + kBC - 1) / kBC;
    // (block-sparse: the count is handed over as an opaque value. Knowing it is at least 1, the
    // compiler merges the pipeline prologue into the first loop iteration, and that one long
    // region needs more registers than the file holds.)
    if constexpr (SPARSE) asm volatile("" : "+s"(n_tiles_));
    const int n_tiles = n_tiles_;
    // leading tiles whose keys all exist and are visible to every row of the workgroup, less two
    // so that the tile prefetched two ahead inside that loop is always a complete one
    // (block-sparse: leading list entries; the entry prefetched two ahead is then not the last
    // one, the only one that may be the partial tile)
    const int n_full = SPARSE ? max(0, min(n_list_full, n_list - kDist))
                              : max(0, min(CAUSAL ? (rb * kBR + off + 1) / kBC : Tk / kBC, Tk / kBC - kDist));
    // sliding window: first key this lane's row sees, and the leading tiles that hold a key
    // some row of the workgroup does not see (its last row starts latest)
    int row_lo[RW];
#pragma unroll
    for (int a = 0; a < RW; ++a) row_lo[a] = WINDOW ? my_row(a) + off - p.window + 1 : 0;
    const int n_left = WINDOW ? min(n_tiles, max(rb * kBR + kBR + off - p.window + kBC - 1, 0) / kBC) : 0;

    // ---- global -> LDS tile loads (no staging registers, no LDS write instructions) --------
    // Load instruction i of wave w fills LDS chunks [64*(w + 4i), +64) of a tile; lane l owns
    // chunk g = 64*(w + 4i) + l = (row, pos) in the padded row-major layout.
    auto k_src = [&](int i, int &row, int &pos) __attribute__((always_inline)) {
        const int c = K_WAVE_CHUNKS * w + 64 * i + lane;  // lanes >= 16 of the last load: unused
        row = min(c / KROW, kBC - 1);
        pos = min(c % KROW, CPR - 1);
    };
    auto v_src = [&](int i, int &row, int &pos) __attribute__((always_inline)) {
        const int c = V_WAVE_CHUNKS * w + 64 * i + lane;
        row = c / VROW;
        pos = min(c % VROW, CPR - 1);
    };
    uint32_t koff[NDMA_K], voff[NDMA_V];  // byte offsets inside a tile whose 64 rows all exist
#pragma unroll
    for (int i = 0; i < NDMA_K; ++i) {
        int row, pos;
        k_src(i, row, pos);
        koff[i] = (uint32_t)(row * p.ks[2] + pos * 8) * 2u;
    }
#pragma unroll
    for (int i = 0; i < NDMA_V; ++i) {
        int row, pos;
        v_src(i, row, pos);
        voff[i] = (uint32_t)(row * p.vs[2] + pos * 8) * 2u;
    }
    const int64_t k_tile_bytes = (int64_t)(kBC * 2) * p.ks[2], v_tile_bytes = (int64_t)(kBC * 2) * p.vs[2];
    // LDS byte addresses of this wave's first K / V load of a stage
    auto stage_k_addr = [&](int stage) __attribute__((always_inline)) {
        return lds_base + (uint32_t)(stage * STAGE_CHUNKS + K_WAVE_CHUNKS * w) * 16u;
    };
    auto stage_v_addr = [&](int stage) __attribute__((always_inline)) {
        return lds_base + (uint32_t)(stage * STAGE_CHUNKS + K_CHUNKS + V_WAVE_CHUNKS * w) * 16u;
    };
    // load i of the tile at (tk, tv) into (dk, dv); tile rows all exist
    auto k_load = [&](int i, const char *tk, uint32_t dk) __attribute__((always_inline)) {
        if (i == NDMA_K - 1)
            tile_load16_uniform<true>(koff[i], tk, dk + 1024u * i);
        else
            tile_load16_uniform<false>(koff[i], tk, dk + 1024u * i);
    };
    auto v_load = [&](int i, const char *tv, uint32_t dv) __attribute__((always_inline)) {
        tile_load16_uniform<false>(voff[i], tv, dv + 1024u * i);
    };
    // tile kt with all 64 rows < T: uniform tile base + the precomputed lane offsets
    auto dma_full_tile = [&](int kt, int stage) __attribute__((always_inline)) {
        const char *tk = (const char *)kbase + kt * k_tile_bytes;
        const char *tv = (const char *)vbase + kt * v_tile_bytes;
#pragma unroll
        for (int i = 0; i < NDMA_K; ++i) k_load(i, tk, stage_k_addr(stage));
#pragma unroll
        for (int i = 0; i < NDMA_V; ++i) v_load(i, tv, stage_v_addr(stage));
    };
    // The steady-state loop spreads the loads of one tile over the MFMA slots of a pipeline step
    // (a block of 2 * NDMA loads at the top of an iteration would leave the matrix pipe idle
    // while they issue); these name the tile being fetched.
    const char *dma_tk = nullptr, *dma_tv = nullptr;
    uint32_t dma_dk = 0, dma_dv = 0;
    // any tile: rows past the last key re-read that key's row (finite data, masked where it matters)
    auto dma_tile = [&](int kt, int stage) __attribute__((always_inline)) {
        const uint32_t dk = stage_k_addr(stage), dv = stage_v_addr(stage);
#pragma unroll
        for (int i = 0; i < NDMA_K; ++i) {
            int row, pos;
            k_src(i, row, pos);
            const __bf16 *sk = kbase + (int64_t)min(kt * kBC + row, Tk - 1) * p.ks[2] + pos * 8;
            if (i == NDMA_K - 1)
                tile_load16<16>(sk, dk + 1024u * i);
            else
                tile_load16<64>(sk, dk + 1024u * i);
        }
#pragma unroll
        for (int i = 0; i < NDMA_V; ++i) {
            int row, pos;
            v_src(i, row, pos);
            const __bf16 *sv = vbase + (int64_t)min(kt * kBC + row, Tk - 1) * p.vs[2] + pos * 8;
            tile_load16<64>(sv, dv + 1024u * i);
        }
    };

    // S1^T, S2^T (32 keys x 32 rows per row sub-block) of key block kb of the tile in `stage`
    auto scores = [&](int stage, int kb, f32x16(&s1)[RW], f32x16(&s2)[RW]) __attribute__((always_inline)) {
        const u32x4 *tk = lds + stage * STAGE_CHUNKS + col * KROW + h;
#pragma unroll
        for (int a = 0; a < RW; ++a)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                s1[a][r] = 0.f;
                s2[a][r] = 0.f;
            }
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const u32x4 kf = tk[kb * kKB * KROW + 2 * ks];
#pragma unroll
            for (int a = 0; a < RW; ++a) {
                s1[a] = mfma32(kf, qf[a][ks], s1[a]);
                if constexpr (USE_R) s2[a] = mfma32(kf, rf[a][ks], s2[a]);
            }
        }
    };

    // accumulator register r of an S^T block <-> key key_base + 8*(r/4) + 4*h + r%4
    auto key_ok = [&](int key_base, int r, int a) __attribute__((always_inline)) {
        const int key = key_base + 8 * (r >> 2) + 4 * h + (r & 3);
        return key < Tk && (!CAUSAL || key <= my_row(a) + off) && (!WINDOW || key >= row_lo[a]) && !no_tiles;
    };

    // d1 / d2 are accumulated by MFMAs as well: Ones(32 x 16 keys) x P^T gives a block whose
    // every row is the column sum of the bf16-ROUNDED P over the keys, i.e. the row sums of
    // Algorithm 1 taken over exactly the numbers that enter O1 / O2 -- the effective attention
    // weights then sum to one exactly, and no vector-ALU work is spent on the sums (a dot-product
    // instruction would share the matrix pipeline and stall it; measured). One accumulator block
    // per row sub-block serves both sums: the A operand of the P1 sum is one in rows 0..15 and
    // zero below, that of the P2 sum the other way round, so rows 0..15 of the block hold d1
    // (register 0 of every lane) and rows 16..31 hold d2 (register 8).
    // Only the masked tiles take these MFMAs; the tiles every row sees completely add the
    // unrounded fp32 values on the vector ALU. (Measured at d = 64 with two row sub-blocks, where
    // the vector ALU has twice the work per MFMA: the MFMA sums in every tile -- a quarter more
    // matrix instructions -- cost what the removed adds saved and more, 537 against 514 us.)
    // With two row sub-blocks per wave the accumulation registers are taken (O1^T, O2^T, Q, R fill
    // three quarters of them and the rest backs the vector registers): the masked tiles then add
    // the rounded operands with dot-product instructions against (1, 1) instead, per lane like
    // vsum below (rsum).
    constexpr bool MFMA_SUMS = RW == 1;
    float m_ref[RW];
    f32x16 o1[RW][NDB], o2[RW][NDB], dacc[MFMA_SUMS ? RW : 1];
    float rsum1[RW] = {}, rsum2[RW] = {};                // !MFMA_SUMS: sums of rounded operands, this lane's keys
    float vsum1[RW][2] = {}, vsum2[RW][2] = {};          // per-lane partial row sums (this lane's keys)
    // Row cache only: fp32 sums of the UNROUNDED P1, P2 over the masked tiles as well. The backward
    // pass recomputes p and u in fp32 and forms 1 + ubar - u, which is 1 for a row with one key only
    // if ubar carries no bf16 rounding of P2; the output keeps the sums of the rounded operands.
    float msum1[RW][2] = {}, msum2[RW][2] = {};
#pragma unroll
    for (int a = 0; a < RW; ++a) m_ref[a] = kNegInf;
    const uint32_t one_top = col < 16 ? 0x3f803f80u : 0u, one_bot = col < 16 ? 0u : 0x3f803f80u;
    const u32x4 ones_top = {one_top, one_top, one_top, one_top}, ones_bot = {one_bot, one_bot, one_bot, one_bot};
    const float scale_log2 = p.scale * kLog2e;  // >= 0 (checked by the host)
    // What multiplies S1 in front of the exponential, per row sub-block. PREP: the 1 / rms of
    // the row's RMSNorm is a per-row scalar, so it is not applied to the q elements but rides on
    // this factor (and that of rho on the final O2, d2, which are linear in S2): r_gain.
    float row_scale[RW], r_gain[RW];
#pragma unroll
    for (int a = 0; a < RW; ++a) row_scale[a] = scale_log2, r_gain[a] = 1.f;

    // adds the bf16 values of a packed MFMA operand (this lane's 8 keys) to acc: one dot product
    // against (1, 1) per packed pair. Written as assembly: through the builtin, viewing a dword of
    // an integer vector as a bf16 pair is miscompiled by this toolchain (all four dot products
    // read the same register).
    auto add_rounded = [&](const u32x4 &pb, float &acc) __attribute__((always_inline)) {
#pragma unroll
        for (int e = 0; e < 4; ++e) asm("v_dot2c_f32_bf16_e32 %0, 0x3f803f80, %1" : "+v"(acc) : "v"(pb[e]));
    };

    // P1 = exp2(S1*scale - m_ref), P2 = P1*S2 for one key block, left as packed bf16 MFMA
    // operands (two groups of 16 keys).
    auto probs = [&](auto masked_tag, int key_base, f32x16(&s1)[RW], f32x16(&s2)[RW], u32x4(&pb1)[RW][2],
                     u32x4(&pb2)[RW][2]) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
#pragma unroll
        for (int a = 0; a < RW; ++a) {
            const float neg_m = m_ref[a] == kNegInf ? 0.f : -m_ref[a];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float p1 = fast_exp2(fmaf(s1[a][r], row_scale[a], neg_m));
                if constexpr (MASKED) p1 = key_ok(key_base, r, a) ? p1 : 0.f;
                s1[a][r] = p1;
                // s2 is finite (rows past the last key re-read it) and P1 = 0 where masked
                if constexpr (USE_R) s2[a][r] = p1 * s2[a][r];
                if constexpr (STATS) {
                    msum1[a][r & 1] += s1[a][r];
                    msum2[a][r & 1] += s2[a][r];
                }
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                // B operand k-element e <-> register 8j+e <-> key 16j + 8*(e/4) + 4h + e%4
                pb1[a][j] = u32x4{pack_bf16(s1[a][8 * j + 0], s1[a][8 * j + 1]), pack_bf16(s1[a][8 * j + 2], s1[a][8 * j + 3]),
                                  pack_bf16(s1[a][8 * j + 4], s1[a][8 * j + 5]), pack_bf16(s1[a][8 * j + 6], s1[a][8 * j + 7])};
                if constexpr (USE_R)
                    pb2[a][j] = u32x4{pack_bf16(s2[a][8 * j + 0], s2[a][8 * j + 1]), pack_bf16(s2[a][8 * j + 2], s2[a][8 * j + 3]),
                                      pack_bf16(s2[a][8 * j + 4], s2[a][8 * j + 5]), pack_bf16(s2[a][8 * j + 6], s2[a][8 * j + 7])};
            }
        }
    };

    // O1^T += V^T P1^T, O2^T += V^T P2^T for key block kb of the tile in `stage`.
    // A operand: row = dimension 32n + col, k-elements = the 8 keys of the B operand, fetched by
    // two transposing LDS reads (keys 16j+4h..+3 and 16j+8+4h..+3).
    const int tr_row = 4 * h + ((lane & 15) >> 2);
    const int tr_half = (lane & 1) * 4;
    const int tr_chunk = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
    const int tr_lane_off = (tr_row * VROW + tr_chunk) * 8 + tr_half;  // in bf16 elements
    auto accumulate = [&](int stage, int kb, const u32x4(&pb1)[RW][2], const u32x4(&pb2)[RW][2]) __attribute__((always_inline)) {
        const unsigned short *tv16 =
            (const unsigned short *)(lds + stage * STAGE_CHUNKS + K_CHUNKS) + tr_lane_off;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int n = 0; n < NDB; ++n) {
                const int off = ((kb * kKB + 16 * j) * VROW + 4 * n) * 8;
                const u32x2 lo = lds_read_tr16(tv16 + off);
                const u32x2 hi = lds_read_tr16(tv16 + off + 8 * VROW * 8);
                const u32x4 vt = {lo[0], lo[1], hi[0], hi[1]};
#pragma unroll
                for (int a = 0; a < RW; ++a) {
                    o1[a][n] = mfma32(vt, pb1[a][j], o1[a][n]);
                    if constexpr (USE_R) o2[a][n] = mfma32(vt, pb2[a][j], o2[a][n]);
                }
            }
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int a = 0; a < RW; ++a) {
                if constexpr (MFMA_SUMS) {
                    dacc[a] = mfma32(ones_top, pb1[a][j], dacc[a]);
                    if constexpr (USE_R) dacc[a] = mfma32(ones_bot, pb2[a][j], dacc[a]);
                } else {
                    add_rounded(pb1[a][j], rsum1[a]);
                    if constexpr (USE_R) add_rounded(pb2[a][j], rsum2[a]);
                }
            }
    };

    auto zero_state = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
#pragma unroll
            for (int a = 0; a < RW; ++a) {
                if constexpr (MFMA_SUMS) dacc[a][r] = 0.f;
#pragma unroll
                for (int n = 0; n < NDB; ++n) {
                    o1[a][n][r] = 0.f;
                    o2[a][n][r] = 0.f;
                }
            }
        }
#pragma unroll
        for (int a = 0; a < RW; ++a) rsum1[a] = rsum2[a] = 0.f;
    };

    // does this wave see any key of the block starting at key_base?
    auto block_visible = [&](int key_base) __attribute__((always_inline)) {
        return key_base < Tk && (!CAUSAL || key_base <= row0 + WROWS - 1 + off) &&
               (!WINDOW || key_base + kKB > row0 + off - p.window + 1);
    };

    u32x4 pb1[RW][2], pb2[RW][2];
#pragma unroll
    for (int a = 0; a < RW; ++a) pb2[a][0] = pb2[a][1] = u32x4{0u, 0u, 0u, 0u};

    // One step of the software pipeline over fully visible key blocks, written as slots of ONE
    // MFMA each followed by its share of vector-ALU work (measured on this chip: a wave can
    // issue about four vector instructions in the shadow of a 32x32x16 MFMA):
    //   phase 1 : score MFMAs of the NEXT block (S1 and S2 alternate), while the vector ALU
    //             turns the upper 16 keys of the CURRENT block into P1 / P2 (bf16 operands);
    //   phase 2 : PV and row-sum MFMAs of the CURRENT block, while the vector ALU already turns
    //             the lower 16 keys of the NEXT block into its P1 / P2.
    // Every fragment slot issues the LDS read of the fragment needed kLookAhead fragments later
    // ([K of next block | V^T of current block | K of the block after]). The scheduling fences
    // keep this order.
    constexpr int kLookAhead = 3;  // fragments read ahead of their MFMAs
    static_assert(2 * NDB == KSTEPS, "as many V^T fragments as K fragments per key block");
    u32x4 kf[KSTEPS], vt[KSTEPS];
    auto k_block_ptr = [&](int stage, int kb) __attribute__((always_inline)) {
        return (const u32x4 *)(lds + stage * STAGE_CHUNKS + col * KROW + h + kb * kKB * KROW);
    };
    auto v_block_ptr = [&](int stage, int kb) __attribute__((always_inline)) {
        return (const unsigned short *)(lds + stage * STAGE_CHUNKS + K_CHUNKS) + tr_lane_off +
               kb * kKB * VROW * 8;
    };
    auto load_kfrag = [&](const u32x4 *tk_block, int ks) __attribute__((always_inline)) {
        kf[ks] = tk_block[2 * ks];
    };
    auto load_vfrag = [&](const unsigned short *tv_block, int f) __attribute__((always_inline)) {
        const int j = f / NDB, n = f % NDB;  // key group of 16, dim block of 32
        const int off = (16 * j * VROW + 4 * n) * 8;
        const u32x2 lo = lds_read_tr16(tv_block + off);
        const u32x2 hi = lds_read_tr16(tv_block + off + 8 * VROW * 8);
        vt[f] = u32x4{lo[0], lo[1], hi[0], hi[1]};
    };
    auto prefetch = [&](int frag, const u32x4 *tk_next, const unsigned short *tv_cur,
                        const u32x4 *tk_after) __attribute__((always_inline)) {
        const int f = frag + kLookAhead;
        if (f < KSTEPS)
            load_kfrag(tk_next, f);
        else if (f < 2 * KSTEPS)
            load_vfrag(tv_cur, f - KSTEPS);
        else
            load_kfrag(tk_after, f - 2 * KSTEPS);
    };
    // exp / P2 of the 8 score registers [r0, r0+8) of a block, spread over the MFMA slots of a
    // phase as three separate stages (scale-and-shift, exp2, times S2) in consecutive slots: a
    // slot then holds independent instructions only, so the single wave of the SIMD never
    // waits on the latency of its own previous vector instruction.
    // With MASKED, `lim` is this lane's largest allowed key offset inside the block (its 4*h
    // already subtracted) and, with a sliding window, `lo` its smallest: register r holds key
    // offset 8*(r/4) + r%4.
    // last key this lane's row may see
    int row_lim[RW];
#pragma unroll
    for (int a = 0; a < RW; ++a) row_lim[a] = no_tiles ? -1 : (CAUSAL ? min(my_row(a) + off, Tk - 1) : Tk - 1);
    // The 8 * RW chains (row sub-block a, register r0 + u) of a phase, one after the other.
    auto exp_stages = [&](auto masked_tag, auto sums_tag, f32x16(&s1)[RW], f32x16(&s2)[RW], int r0, int slot,
                          int slot0, int n_slots, const float(&neg_m)[RW], const int(&lim)[RW], const int(&lo)[RW],
                          float(&acc1)[RW][2], float(&acc2)[RW][2]) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        constexpr bool SUMS = decltype(sums_tag)::value;  // a fourth stage adds P1, P2 to acc1, acc2
#pragma unroll
        for (int c = 0; c < 8 * RW; ++c) {
            const int a = c / 8, u = c % 8;
            const int r = r0 + u;
            // stages in slots first, first+1, first+2 (, first+3); none before slot0, none in
            // the last two
            const int first = slot0 + c * (n_slots - (SUMS ? 5 : 4) - slot0) / (8 * RW);
            if constexpr (SUMS)
                if (slot == first + 3) {
                    acc1[a][u & 1] += s1[a][r];
                    if constexpr (USE_R) acc2[a][u & 1] += s2[a][r];
                }
            if (slot == first) s1[a][r] = fmaf(s1[a][r], row_scale[a], neg_m[a]);
            if (slot == first + 1) {
                const float p1 = fast_exp2(s1[a][r]);
                const int key_off = 8 * (r >> 2) + (r & 3);
                const bool seen = !MASKED || (key_off <= lim[a] && (!WINDOW || key_off >= lo[a]));
                s1[a][r] = seen ? p1 : 0.f;
            }
            // P2: S2 is finite (rows past the last key re-read it) and P1 = 0 where masked
            if constexpr (USE_R)
                if (slot == first + 2) s2[a][r] = s1[a][r] * s2[a][r];
        }
    };
    auto pack_group = [&](const f32x16 &s, int j) __attribute__((always_inline)) {
        return u32x4{pack_bf16(s[8 * j + 0], s[8 * j + 1]), pack_bf16(s[8 * j + 2], s[8 * j + 3]),
                     pack_bf16(s[8 * j + 4], s[8 * j + 5]), pack_bf16(s[8 * j + 6], s[8 * j + 7])};
    };
    // Two row sub-blocks per wave: a step has twice the element-wise work per MFMA and the vector
    // ALU, not the matrix pipe, is what fills a slot. So the work is laid over ALL slots of the
    // step by absolute slot number g (phase 1 = [0, n1), phase 2 = [n1, n_slots)) instead of
    // phase by phase, one chain (scale-and-shift, exp2, times S2[, row-sum add]) starting per slot:
    //   U chains, upper key group of the CURRENT block (registers 8..15 of sc): chain c starts in
    //     slot c; they run over into phase 2, whose MFMAs need their operands from slot
    //     n1 + n2 / 2 on;
    //   L chains, lower key group of the NEXT block (registers 0..7 of sn): from the last slot of
    //     phase 1 (the scores of sub-block 0 are complete two slots earlier, those of sub-block 1
    //     when its chains start) to the end of the step;
    //   operands are packed pair by pair as soon as both chains of a pair are through, not as
    //     blocks of four at the end of a phase;
    //   the row-sum adds of the current block's lower key group (finished by the previous step)
    //     fill the slots at both ends of the step, where chains are still starting or already done.
    auto step_valu = [&](auto masked_tag, auto sums_tag, int g, int n1, int n_slots, f32x16(&sc1)[RW],
                         f32x16(&sc2)[RW], f32x16(&sn1)[RW], f32x16(&sn2)[RW], const float(&neg_m)[RW],
                         const int(&lim_cur)[RW], const int(&lo_cur)[RW], const int(&lim_next)[RW],
                         const int(&lo_next)[RW], float(&acc1)[RW][2], float(&acc2)[RW][2], u32x4(&nb1)[RW],
                         u32x4(&nb2)[RW]) __attribute__((always_inline)) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        constexpr bool ADDS = decltype(sums_tag)::value;
        constexpr int NCH = 8 * RW;
        const int l0 = n1 - 1, l_span = n_slots - 4 - l0;  // L chains start in [l0, l0 + l_span]
        // (the result of every stage passes through an empty volatile statement in the stage's
        // slot: such data dependences are what keeps a vector instruction from sinking over the
        // scheduling fences to the slot of its first use)
        auto pin = [](float x) __attribute__((always_inline)) {
            asm volatile("" : "+v"(x));
            return x;
        };

        // register r of a score block pair (b1, b2); r holds key offset 8*(r/4) + r%4
        auto chain = [&](f32x16 &b1, f32x16 &b2, int r, int start, float nm, float sc, int lim, int lo)
                         __attribute__((always_inline)) {
            if (g == start) b1[r] = pin(fmaf(b1[r], sc, nm));
            if (g == start + 1) {
                const float p1 = fast_exp2(b1[r]);
                const int key_off = 8 * (r >> 2) + (r & 3);
                const bool seen = !MASKED || (key_off <= lim && (!WINDOW || key_off >= lo));
                b1[r] = pin(seen ? p1 : 0.f);
            }
            // P2: S2 is finite (rows past the last key re-read it) and P1 = 0 where masked
            if constexpr (USE_R)
                if (g == start + 2) b2[r] = pin(b1[r] * b2[r]);
        };
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int a = c / 8, u = c % 8;
            const int us = c, ls = l0 + c * l_span / (NCH - 1);
            chain(sc1[a], sc2[a], 8 + u, us, neg_m[a], row_scale[a], lim_cur[a], lo_cur[a]);
            if constexpr (ADDS)
                if (g == us + 3) {
                    acc1[a][u & 1] = pin(acc1[a][u & 1] + sc1[a][8 + u]);
                    if constexpr (USE_R) acc2[a][u & 1] = pin(acc2[a][u & 1] + sc2[a][8 + u]);
                }
            chain(sn1[a], sn2[a], u, ls, neg_m[a], row_scale[a], lim_next[a], lo_next[a]);
            if (u & 1) {  // both chains of the pair (u - 1, u) are through: B operand dword u / 2
                if (g == us + 2) pb1[a][1][u / 2] = pack_bf16(sc1[a][8 + u - 1], sc1[a][8 + u]);
                if (g == ls + 2) nb1[a][u / 2] = pack_bf16(sn1[a][u - 1], sn1[a][u]);
                if constexpr (USE_R) {
                    if (g == us + 3) pb2[a][1][u / 2] = pack_bf16(sc2[a][8 + u - 1], sc2[a][8 + u]);
                    if (g == ls + 3) nb2[a][u / 2] = pack_bf16(sn2[a][u - 1], sn2[a][u]);
                }
            }
        }
        if constexpr (ADDS) {
            // 3, 2, 1 adds in the first three slots, the rest towards the end of the step
#pragma unroll
            for (int q = 0; q < NCH; ++q) {
                static_assert(NCH == 16, "slot table of the 16 lower-group adds");
                const int early[6] = {0, 0, 0, 1, 1, 2}, late[10] = {6, 5, 4, 3, 2, 2, 2, 1, 1, 1};
                const int at = q < 6 ? early[q] : n_slots - late[q - 6];
                if (g == at) {
                    const int a = q / 8, r = q % 8;
                    acc1[a][r & 1] = pin(acc1[a][r & 1] + sc1[a][r]);
                    if constexpr (USE_R) acc2[a][r & 1] = pin(acc2[a][r & 1] + sc2[a][r]);
                }
            }
        }
    };
    auto pipeline_step = [&](auto masked_tag, auto dma_tag, int key_base_cur, int key_base_next, const u32x4 *tk_next,
                             const unsigned short *tv_cur, const u32x4 *tk_after, f32x16(&sc1)[RW],
                             f32x16(&sc2)[RW], f32x16(&sn1)[RW], f32x16(&sn2)[RW]) __attribute__((always_inline)) {
        int lim_cur[RW], lim_next[RW], lo_cur[RW], lo_next[RW];  // current block, next block
        float neg_m[RW];
#pragma unroll
        for (int a = 0; a < RW; ++a) {
            lim_cur[a] = row_lim[a] - key_base_cur - 4 * h;
            lim_next[a] = row_lim[a] - key_base_next - 4 * h;
            lo_cur[a] = row_lo[a] - key_base_cur - 4 * h;
            lo_next[a] = row_lo[a] - key_base_next - 4 * h;
            neg_m[a] = -m_ref[a];
        }
        constexpr int SLOTS1 = 2 * KSTEPS * RW;      // phase 1: one slot per score MFMA
        constexpr bool DMA = decltype(dma_tag)::value;  // this step also fetches tile (dma_tk, dma_tv)
        constexpr bool MASKED = decltype(masked_tag)::value;
        // Row sums of the CURRENT block belong to this step. Masked steps (a row may see only a
        // few keys, so the sums must be those of the rounded operands exactly): two MFMAs against
        // ones per key group and row sub-block. Unmasked steps: vector adds of the fp32 values,
        // which stay in the score registers until the next step -- upper key group behind its
        // exp stages in phase 1, lower key group (finished by the previous step) during phase 2.
        constexpr bool SUMS = !MASKED;
        constexpr int PV = 2 * NDB * RW;                 // PV MFMAs per key group
        constexpr int GROUP2 = PV + (!SUMS && MFMA_SUMS ? 2 * RW : 0);  // phase 2, per key group: PV (+ row sums)
        constexpr int SLOTS2 = 2 * GROUP2;
        // (row cache: masked steps add the fp32 values as well, to sums of their own)
        constexpr bool ADDS = SUMS || STATS;
        const std::integral_constant<bool, ADDS> sums_tag{};
        float(&acc1)[RW][2] = SUMS ? vsum1 : msum1;
        float(&acc2)[RW][2] = SUMS ? vsum2 : msum2;
        static_assert(NDMA_K <= KSTEPS * RW && NDMA_V <= GROUP2, "one tile load per odd slot");
        u32x4 nb1[RW], nb2[RW];  // lower key group of the next block as operands
#pragma unroll
        for (int a = 0; a < RW; ++a) nb1[a] = nb2[a] = u32x4{0u, 0u, 0u, 0u};
        // ---- phase 1: scores of the next block | upper key group of the current block ------
        // slot = ((k-step, row sub-block), S1 | S2): a K fragment serves 2 * RW MFMAs in a row
#pragma unroll
        for (int sl = 0; sl < SLOTS1; ++sl) {
            const int ks = (sl / 2) / RW, a = (sl / 2) % RW;
            if (sl % 2 == 0) {
                if (ks == 0)
                    mfma32_scores_first<MASKED>(sn1[a], kf[ks], qf[a][ks]);
                else
                    mfma32_scores<MASKED>(sn1[a], kf[ks], qf[a][ks]);
                if (a == 0) prefetch(ks, tk_next, tv_cur, tk_after);
            } else if constexpr (USE_R) {
                if (ks == 0)
                    mfma32_scores_first<MASKED>(sn2[a], kf[ks], rf[a][ks]);
                else
                    mfma32_scores<MASKED>(sn2[a], kf[ks], rf[a][ks]);
            }
            if constexpr (DMA)
                if (sl % 2 == 1 && sl / 2 < NDMA_K) k_load(sl / 2, dma_tk, dma_dk);
            if constexpr (RW == 1) {
                exp_stages(masked_tag, sums_tag, sc1, sc2, 8, sl, 0, SLOTS1, neg_m, lim_cur, lo_cur, acc1, acc2);
                // upper key group -> operands, in the last two slots
                if (sl == SLOTS1 - 2) pb1[0][1] = pack_group(sc1[0], 1);
                if (sl == SLOTS1 - 1) {
                    if constexpr (USE_R) pb2[0][1] = pack_group(sc2[0], 1);
                }
            } else {
                step_valu(masked_tag, sums_tag, sl, SLOTS1, SLOTS1 + SLOTS2, sc1, sc2, sn1, sn2, neg_m, lim_cur, lo_cur,
                          lim_next, lo_next, acc1, acc2, nb1, nb2);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // ---- phase 2: PV + row sums of the current block | lower key group of the next block
        // The scores just issued are first read in slot 1, i.e. behind the PV MFMAs of slots 0
        // and 1. A wave issues in order and an MFMA is only accepted once the matrix pipe has
        // room, so by then the last score MFMA has retired: no wait states needed.
#pragma unroll
        for (int sl = 0; sl < SLOTS2; ++sl) {
            const int j = sl / GROUP2, t = sl % GROUP2;
            if (t < PV) {
                const int n = (t / 2) / RW, a = (t / 2) % RW, f = j * NDB + n;
                if (t % 2 == 0) {
                    o1[a][n] = mfma32(vt[f], pb1[a][j], o1[a][n]);
                    if (a == 0) prefetch(KSTEPS + f, tk_next, tv_cur, tk_after);
                } else if constexpr (USE_R) {
                    o2[a][n] = mfma32(vt[f], pb2[a][j], o2[a][n]);
                }
            } else if constexpr (MFMA_SUMS) {
                const int a = (t - PV) / 2;
                if ((t - PV) % 2 == 0)
                    dacc[a] = mfma32(ones_top, pb1[a][j], dacc[a]);
                else if constexpr (USE_R)
                    dacc[a] = mfma32(ones_bot, pb2[a][j], dacc[a]);
            }
            if constexpr (!SUMS && !MFMA_SUMS) {  // rounded operands of key group j, one operand per slot
                if (t < 2 * RW) {
                    if (t % 2 == 0)
                        add_rounded(pb1[t / 2][j], rsum1[t / 2]);
                    else if constexpr (USE_R)
                        add_rounded(pb2[t / 2][j], rsum2[t / 2]);
                }
            }
            if constexpr (DMA)
                if (sl % 2 == 1 && sl / 2 < NDMA_V) v_load(sl / 2, dma_tv, dma_dv);
            if constexpr (RW == 1) {
                exp_stages(masked_tag, std::false_type{}, sn1, sn2, 0, sl, 1, SLOTS2, neg_m, lim_next, lo_next, acc1,
                           acc2);
                if constexpr (ADDS) {
                    constexpr int PER = SLOTS2 / 8;  // lower key group of the current block
                    if (sl % PER == 0 && sl / PER < 8) {
                        const int r = sl / PER;
                        acc1[0][r & 1] += sc1[0][r];
                        if constexpr (USE_R) acc2[0][r & 1] += sc2[0][r];
                    }
                }
                if (sl == SLOTS2 - 2) nb1[0] = pack_group(sn1[0], 0);
                if (sl == SLOTS2 - 1) {
                    if constexpr (USE_R) nb2[0] = pack_group(sn2[0], 0);
                }
            } else {
                step_valu(masked_tag, sums_tag, SLOTS1 + sl, SLOTS1, SLOTS1 + SLOTS2, sc1, sc2, sn1, sn2, neg_m, lim_cur,
                          lo_cur, lim_next, lo_next, acc1, acc2, nb1, nb2);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int a = 0; a < RW; ++a) {
            pb1[a][0] = nb1[a];
            pb2[a][0] = nb2[a];
        }
    };

    // =========================== fast pass: fixed reference ================================
    // Ring invariant at the top of iteration kt: tiles kt and (after the barrier) kt+1 are in
    // stages kt % 3 and (kt+1) % 3 and visible to all waves. The barrier (every wave first waits
    // for its own tile loads) also proves that nobody reads tile kt-1 any more, whose stage then
    // receives tile kt+2: each tile load has a whole iteration to land.
    // load n of the first two tiles (tile 0 first, K before V), for issuing them one at a time
    auto initial_load = [&](int n) __attribute__((always_inline)) {
        const int t = n / kTileLoads, i = n % kTileLoads;
        if (Tk >= kDist * kBC) {  // workgroup-uniform: whole tiles, uniform base + lane offsets
            if (i < NDMA_K)
                k_load(i, (const char *)kbase + t * k_tile_bytes, stage_k_addr(t));
            else
                v_load(i - NDMA_K, (const char *)vbase + t * v_tile_bytes, stage_v_addr(t));
        } else {
            int row, pos;
            if (i < NDMA_K) {
                k_src(i, row, pos);
                const __bf16 *sk = kbase + (int64_t)min(t * kBC + row, Tk - 1) * p.ks[2] + pos * 8;
                if (i == NDMA_K - 1)
                    tile_load16<16>(sk, stage_k_addr(t) + 1024u * i);
                else
                    tile_load16<64>(sk, stage_k_addr(t) + 1024u * i);
            } else {
                v_src(i - NDMA_K, row, pos);
                const __bf16 *sv = vbase + (int64_t)min(t * kBC + row, Tk - 1) * p.vs[2] + pos * 8;
                tile_load16<64>(sv, stage_v_addr(t) + 1024u * (i - NDMA_K));
            }
        }
    };
    static_assert(kDist == 2, "the wait below leaves exactly tile 1 in flight");
    if constexpr (!PREP) {
        if constexpr (SPARSE) {  // (the clamping form only: it needs no per-lane offsets kept alive)
#pragma unroll
            for (int t = 0; t < kDist; ++t) dma_tile(tile_at(t), t);
        } else if (Tk >= kDist * kBC) {  // workgroup-uniform
#pragma unroll
            for (int t = 0; t < kDist; ++t) dma_full_tile(t, t);
        } else {
#pragma unroll
            for (int t = 0; t < kDist; ++t) dma_tile(t, t);
        }
        zero_state();
    } else {
        // Normalise, rotate and round this wave's Q and R rows where they landed (nobody else
        // reads them). Per row: sum of squares over the CPR lanes of the row, y = x / sqrt(mean
        // + eps) * gamma, then the adjacent pairs (2i, 2i + 1) turned by the row's angle.
        // (Issuing the loads of the first two key tiles between the row passes instead of in
        // front of them was tried: no faster.)
#pragma unroll
        for (int n = 0; n < kDist * kTileLoads; ++n) initial_load(n);
        zero_state();
        // this wave's Q and R rows (and the table entries) are there; the two tiles may still travel
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kDist * kTileLoads) : "memory");
        const int lr = lane % CPR, lrow = lane / CPR;
        u32x4 *zq = lds + QZONE + w * WAVE_TILE_CHUNKS, *zr = lds + RZONE + w * WAVE_TILE_CHUNKS;
        const float inv_d = 1.0f / (float)D;
        // sum of squares of the 8 bf16 values of a chunk (dot products of the packed pairs with
        // themselves), over the CPR lanes of the row; 1 / rms
        auto inv_rms = [&](const u32x4 &c) __attribute__((always_inline)) {
            float ss = 0.f;
#pragma unroll
            for (int e = 0; e < 3; ++e) asm("v_dot2c_f32_bf16_e32 %0, %1, %1" : "+v"(ss) : "v"(c[e]));
            // (the result of a dot product needs three wait states before another kind of
            // instruction reads it; the compiler does not see the instruction, so they are here)
            asm("v_dot2c_f32_bf16_e32 %0, %1, %1\n\ts_nop 2" : "+v"(ss) : "v"(c[3]));
            ss = lane_group_sum<CPR>(ss);  // the CPR lanes of a row are an aligned group
            return __builtin_amdgcn_rsqf(fmaf(ss, inv_d, p.prep.eps));
        };
        // gamma, then (unless ROT is off) the rotation of the four pairs; NOT the 1 / rms factor
        auto scale_rotate = [&](auto rot_tag, const u32x4 &c, const f32x4(&gam)[2], const f32x4(&tab)[2])
                                __attribute__((always_inline)) {
            u32x4 out;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float y0 = bf16_lo_f32(c[j]) * gam[j >> 1][2 * (j & 1)];
                float y1 = bf16_hi_f32(c[j]) * gam[j >> 1][2 * (j & 1) + 1];
                if constexpr (decltype(rot_tag)::value) {
                    const float cs = tab[j >> 1][2 * (j & 1)], sn = tab[j >> 1][2 * (j & 1) + 1];
                    const float r0 = y0 * cs - y1 * sn, r1 = y0 * sn + y1 * cs;
                    y0 = r0, y1 = r1;
                }
                out[j] = pack_bf16(y0, y1);
            }
            return out;
        };
        // The 1 / rms of a row goes to the padding chunk of the row (no fragment reads it), from
        // where the lane that owns the row in the MFMA layout picks it up below.
        auto prep_rows = [&](auto rot_q_tag, auto rot_r_tag) __attribute__((always_inline)) {
#pragma unroll
            for (int it = 0; it < PREP_NIT; ++it) {
                const int row = it * PREP_RPI + lrow, slot = row * KROW + lr;
                const u32x4 cq = zq[slot], cr = zr[slot];
                const float iq = inv_rms(cq), ir = inv_rms(cr);
                zq[slot] = scale_rotate(rot_q_tag, cq, prep_gq, prep_tab[it]);
                zr[slot] = scale_rotate(rot_r_tag, cr, prep_gr, prep_tab[it]);
                if (lr == 0) {
                    *(float *)&zq[row * KROW + CPR] = iq;
                    *(float *)&zr[row * KROW + CPR] = ir;
                }
            }
        };
        // (rotation switches are uniform over the launch: one specialised copy of the pass each)
        if (p.prep.rope_q != 0 && p.prep.rope_r != 0)
            prep_rows(std::true_type{}, std::true_type{});
        else if (p.prep.rope_q != 0)
            prep_rows(std::true_type{}, std::false_type{});
        else
            prep_rows(std::false_type{}, std::false_type{});
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int a = 0; a < RW; ++a) {
            row_scale[a] = scale_log2 * *(const float *)&zq[(32 * a + col) * KROW + CPR];
            r_gain[a] = *(const float *)&zr[(32 * a + col) * KROW + CPR];
        }
    }
    tile_barrier<kTileLoads>();  // Q, R and tile 0 have landed
    {
        // B operands: column = query row, k-elements = the 8 dims of chunk 2*ks + h
        const u32x4 *zq = lds + QZONE + w * WAVE_TILE_CHUNKS + col * KROW + h;
        const u32x4 *zr = lds + RZONE + w * WAVE_TILE_CHUNKS + col * KROW + h;
#pragma unroll
        for (int a = 0; a < RW; ++a)
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                qf[a][ks] = zq[32 * a * KROW + 2 * ks];
                if constexpr (USE_R) rf[a][ks] = zr[32 * a * KROW + 2 * ks];
            }
    }
    int stage = 0;
    f32x16 sa1[RW], sa2[RW], sb1[RW], sb2[RW];
    {
        // Pipeline prologue: scores of block (0, 0); reference = its row maximum (key 0 is
        // visible to every row); lower key group -> P. (Everything the loops read from registers
        // loaded out of global memory -- the Q, R fragments -- is consumed here first, so the
        // loops contain no wait on the vector-memory counter, which the tile loads in flight
        // would turn into a full memory round trip.)
        scores(0, 0, sa1, sa2);
#pragma unroll
        for (int f = 0; f < kLookAhead; ++f) load_kfrag(k_block_ptr(0, 1), f);
        int kb0 = tile_at(0) * kBC;  // 0 unless block-sparse
        if constexpr (SPARSE) asm volatile("" : "+s"(kb0));  // (opaque, for the same reason as n_tiles)
        float neg_m[RW];
        int lim0[RW], lo0[RW];
#pragma unroll
        for (int a = 0; a < RW; ++a) {
            float tmax = kNegInf;
#pragma unroll
            for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, key_ok(kb0, r, a) ? sa1[a][r] : kNegInf);
            tmax = halves_max(tmax);
            if constexpr (WINDOW || SPARSE) {
                // a row whose window starts behind this block takes the block's plain maximum: any
                // finite reference will do (the check after the loops catches one that was too far off)
                float tall = sa1[a][0];
#pragma unroll
                for (int r = 1; r < 16; ++r) tall = fmaxf(tall, sa1[a][r]);
                tall = halves_max(tall);
                tmax = tmax == kNegInf ? tall : tmax;
            }
            m_ref[a] = tmax * row_scale[a];
            neg_m[a] = -m_ref[a];
            lim0[a] = row_lim[a] - kb0 - 4 * h;
            lo0[a] = row_lo[a] - kb0 - 4 * h;
        }
#pragma unroll
        for (int sl = 0; sl < 12; ++sl)
            exp_stages(std::true_type{}, std::false_type{}, sa1, sa2, 0, sl, 0, 12, neg_m, lim0, lo0, msum1, msum2);
#pragma unroll
        for (int a = 0; a < RW; ++a) {
            pb1[a][0] = pack_group(sa1[a], 0);
            if constexpr (USE_R) pb2[a][0] = pack_group(sa2[a], 0);
        }
    }
    // kt: key tile in `stage`, kt_next: key tile in `next_stage` (kt + 1 unless block-sparse)
    auto tile_steps = [&](auto masked_tag, auto dma_tag, int kt, int kt_next, int stage, int next_stage) __attribute__((always_inline)) {
        // block (kt,0) -> P, PV; scores of (kt,1); K fragments of (kt_next,0); loads of the tile after
        pipeline_step(masked_tag, dma_tag, kt * kBC, kt * kBC + kKB, k_block_ptr(stage, 1),
                      v_block_ptr(stage, 0), k_block_ptr(next_stage, 0), sa1, sa2, sb1, sb2);
        // block (kt,1) -> P, PV; scores of (kt_next,0); K fragments of (kt_next,1)
        pipeline_step(masked_tag, std::false_type{}, kt * kBC + kKB, kt_next * kBC, k_block_ptr(next_stage, 0),
                      v_block_ptr(stage, 1), k_block_ptr(next_stage, 1), sb1, sb2, sa1, sa2);
    };
    // One tile of the pipeline with per-lane key masks. Blocks a wave cannot see at all
    // contribute exact zeros.
    auto masked_tile = [&](int kt) __attribute__((always_inline)) {
        const int next_stage = stage == STAGES - 1 ? 0 : stage + 1;
        const int free_stage = stage == 0 ? STAGES - 1 : stage - 1;
        tile_barrier();
        if (kt + kDist < n_tiles) {              // workgroup-uniform
            const int k2 = tile_at(kt + kDist);
            if (!SPARSE && (k2 + 1) * kBC <= Tk)  // the tile exists completely
                dma_full_tile(k2, free_stage);
            else
                dma_tile(k2, free_stage);
        }
        tile_steps(std::true_type{}, std::false_type{}, tile_at(kt), tile_at(kt + 1), stage, next_stage);
        stage = next_stage;
    };
    int kt = 0;
    // Sliding window: the leading tiles are cut by the left edge of some row's window.
    if constexpr (WINDOW)
        for (; kt < n_left; ++kt) masked_tile(kt);
    // Tiles whose keys -- and those of the tile after -- are visible to every row: no masks, a
    // branch-free body. (A step also prepares the lower half of the NEXT block, hence the -1.)
    dma_tk = (const char *)kbase + (kt + kDist) * k_tile_bytes;
    dma_tv = (const char *)vbase + (kt + kDist) * v_tile_bytes;
    for (; kt < n_full - 1; ++kt) {
        const int next_stage = stage == STAGES - 1 ? 0 : stage + 1;
        const int free_stage = stage == 0 ? STAGES - 1 : stage - 1;  // held tile kt - 1
        // tile kt + 1 has landed; the kDist - 2 tiles after it may still be in flight
        tile_barrier<(kDist - 2) * kTileLoads>();
        dma_dk = stage_k_addr(free_stage);  // tile kt + kDist <= T/64 - 1 in this loop: complete
        dma_dv = stage_v_addr(free_stage);
        if constexpr (SPARSE) {
            // (a list that does not ascend gives wrong results, but never a read past the last key)
            const int k2 = min(tile_at(kt + kDist), Tk / kBC - 1);
            dma_tk = (const char *)kbase + k2 * k_tile_bytes;
            dma_tv = (const char *)vbase + k2 * v_tile_bytes;
        }
        tile_steps(std::false_type{}, std::true_type{}, tile_at(kt), tile_at(kt + 1), stage, next_stage);
        if constexpr (!SPARSE) {
            dma_tk += k_tile_bytes;
            dma_tv += v_tile_bytes;
        }
        stage = next_stage;
    }
    // Remaining tiles (diagonal / tail): the same pipeline with per-lane key masks.
    for (; kt < n_tiles; ++kt) masked_tile(kt);
    // ---- closing formula into the wave's staging tile, and the check of the fast pass -------
    // O^T register r of block n <-> dim 32n + 8*(r/4) + 4h + r%4 of row my_row. A lane owns one
    // output ROW, so direct stores would scatter 8 bytes over 32 rows per instruction; the wave
    // instead transposes its 32 x D tile through LDS (its Q landing zone, which nobody else
    // touches) and later writes whole 256-byte rows, 16 bytes a lane.
    // The same pass over the accumulators decides whether the fixed reference held: an inf / NaN
    // anywhere in the sums or accumulators (the reference was too small) shows as a non-finite
    // row sum or output. Only then the workgroup redoes its rows with the online update below
    // and comes back here once more.
    constexpr int OROW = CPR + 1;  // padded row of the staging tile, in 16-byte chunks
    static_assert(OROW == KROW, "the staging tile is the wave's Q tile");
    u32x4 *otile = lds + QZONE + w * WAVE_TILE_CHUNKS;
    unsigned short *otile16 = (unsigned short *)otile;
    float inv[RW], dsum1[RW];
    auto stage_outputs = [&]() __attribute__((always_inline)) {
        float chk = 0.f;
#pragma unroll
        for (int a = 0; a < RW; ++a) {
            // Every row of the MFMA row-sum accumulators holds the sum over this lane's query row;
            // the per-lane partial sums cover this lane's keys only: add the other half-wave's.
            float dsum2;
            if constexpr (MFMA_SUMS) {
                dsum1[a] = dacc[a][0] + halves_sum(vsum1[a][0] + vsum1[a][1]);
                dsum2 = dacc[a][8] + halves_sum(vsum2[a][0] + vsum2[a][1]);
            } else {
                dsum1[a] = halves_sum(rsum1[a] + vsum1[a][0] + vsum1[a][1]);
                dsum2 = halves_sum(rsum2[a] + vsum2[a][0] + vsum2[a][1]);
            }
            if constexpr (PREP) dsum2 *= r_gain[a];
            inv[a] = dsum1[a] > 0.f ? 1.f / dsum1[a] : 0.f;  // empty key set: zeros
            const float gain = inv[a] * (1.f + dsum2 * inv[a]);
            const float inv2 = PREP ? inv[a] * r_gain[a] : inv[a];
            chk = fmaf(dsum1[a] + dsum2, 0.f, chk);  // inf or NaN -> NaN
#pragma unroll
            for (int n = 0; n < NDB; ++n)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    float y[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int r = 4 * q4 + i;
                        y[i] = o1[a][n][r] * gain - (USE_R ? o2[a][n][r] * inv2 : 0.f);
                        chk = fmaf(y[i], 0.f, chk);
                    }
                    const u32x2 packed = {pack_bf16(y[0], y[1]), pack_bf16(y[2], y[3])};
                    *(u32x2 *)(otile16 + (32 * a + col) * (OROW * 8) + 32 * n + 8 * q4 + 4 * h) = packed;
                }
        }
        return chk;
    };
    float chk = stage_outputs();
    if constexpr (WINDOW || SPARSE) {
        // the reference of a row may come from keys outside its window; if it was so far above
        // the row's own scores that the sum underflowed, take the exact path as well
        // (block-sparse: only for rows that do see a listed key -- the list is ascending, so that
        // is decided by its first tile)
#pragma unroll
        for (int a = 0; a < RW; ++a)
            if (my_row(a) < T && (!SPARSE || tile_at(0) * kBC <= row_lim[a]) && !(dsum1[a] > 1e-30f)) chk = 1.f;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // tile loads past the end have landed
    const bool overflow = __syncthreads_or(chk != 0.f);  // NaN != 0 is true; all waves agree

    // =========================== fallback: online max / rescale ============================
    if (overflow) {
        zero_state();
#pragma unroll
        for (int a = 0; a < RW; ++a) {
            vsum1[a][0] = vsum1[a][1] = vsum2[a][0] = vsum2[a][1] = 0.f;
            msum1[a][0] = msum1[a][1] = msum2[a][0] = msum2[a][1] = 0.f;
            m_ref[a] = kNegInf;
        }
        dma_tile(tile_at(0), 0);
        stage = 0;
        for (int t = 0; t < n_tiles; ++t) {
            const int next_stage = stage == STAGES - 1 ? 0 : stage + 1;
            tile_barrier();  // tile t has landed; tile t-2's stage is free for tile t+1
            dma_tile(tile_at(t + 1), next_stage);
#pragma unroll 1
            for (int kb = 0; kb < kBC / kKB; ++kb) {
                const int key_base = tile_at(t) * kBC + kb * kKB;
                if (!block_visible(key_base)) continue;
                scores(stage, kb, sa1, sa2);
#pragma unroll
                for (int a = 0; a < RW; ++a) {
                    float tmax = kNegInf;
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        tmax = fmaxf(tmax, key_ok(key_base, r, a) ? sa1[a][r] * row_scale[a] : kNegInf);
                    tmax = halves_max(tmax);
                    const float m_new = fmaxf(m_ref[a], tmax);
                    const float m_use = m_new == kNegInf ? 0.f : m_new;
                    const float alpha = fast_exp2(m_ref[a] - m_use);  // 0 while m_ref = -inf
                    m_ref[a] = m_new;
                    if constexpr (STATS) {
                        msum1[a][0] *= alpha, msum1[a][1] *= alpha;
                        msum2[a][0] *= alpha, msum2[a][1] *= alpha;
                    }
                    if constexpr (!MFMA_SUMS) rsum1[a] *= alpha, rsum2[a] *= alpha;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        if constexpr (MFMA_SUMS) dacc[a][r] *= alpha;
#pragma unroll
                        for (int n = 0; n < NDB; ++n) {
                            o1[a][n][r] *= alpha;
                            if constexpr (USE_R) o2[a][n][r] *= alpha;
                        }
                    }
                }
                probs(std::true_type{}, key_base, sa1, sa2, pb1, pb2);
                accumulate(stage, kb, pb1, pb2);
            }
            stage = next_stage;
        }
        tile_barrier();  // outstanding tile loads land before the workgroup may exit
        (void)stage_outputs();
    }

    // ---- epilogue: the staged rows go out as whole rows ------------------------------------
    {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __bf16 *obase = (__bf16 *)p.o + b * p.os[0] + hq * p.os[1];
        constexpr int RPI = 64 / CPR;  // rows covered by one wave-wide 16-byte store
#pragma unroll
        for (int i = 0; i < WROWS / RPI; ++i) {
            const int rr = i * RPI + lane / CPR, chunk = lane % CPR;
            const int row = row0 + rr;
            if (row < T) *(u32x4 *)(obase + (int64_t)row * p.os[2] + chunk * 8) = otile[rr * OROW + chunk];
        }
        if constexpr (STATS) {
            // Row cache for the backward pass (App. D): vbar_i = O1 / d1 through the same
            // staging tile, and per row the log-sum-exp of the scaled scores in the exp2 domain
            // (P1 = exp2(S1 * scale * log2 e - lse) needs no further division) and ubar = d2 / d1.
            // (from the fp32 sums of the unrounded P1, P2 -- see msum1 above)
#pragma unroll
            for (int a = 0; a < RW; ++a) {
                const float fsum1 = halves_sum(vsum1[a][0] + vsum1[a][1] + msum1[a][0] + msum1[a][1]);
                const float fsum2 = halves_sum(vsum2[a][0] + vsum2[a][1] + msum2[a][0] + msum2[a][1]);
                if (h == 0 && my_row(a) < T) {
                    float *st = p.row_stats + (((int64_t)b * p.Hq + hq) * T + my_row(a)) * 2;
                    // (a row with no visible key stores +inf: the backward's exp2(S1 - lse) is then
                    // zero for every pair of the row, whatever the mask arithmetic does)
                    st[0] = fsum1 > 0.f ? m_ref[a] + log2f(fsum1) : -kNegInf;
                    st[1] = fsum1 > 0.f ? fsum2 / fsum1 : 0.f;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int a = 0; a < RW; ++a)
#pragma unroll
                for (int n = 0; n < NDB; ++n)
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        const u32x2 packed = {pack_bf16(o1[a][n][4 * q4] * inv[a], o1[a][n][4 * q4 + 1] * inv[a]),
                                              pack_bf16(o1[a][n][4 * q4 + 2] * inv[a], o1[a][n][4 * q4 + 3] * inv[a])};
                        *(u32x2 *)(otile16 + (32 * a + col) * (OROW * 8) + 32 * n + 8 * q4 + 4 * h) = packed;
                    }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            __bf16 *vbase_out = (__bf16 *)p.vbar + b * p.os[0] + hq * p.os[1];
#pragma unroll
            for (int i = 0; i < WROWS / RPI; ++i) {
                const int rr = i * RPI + lane / CPR, chunk = lane % CPR;
                const int row = row0 + rr;
                if (row < T)
                    *(u32x4 *)(vbase_out + (int64_t)row * p.os[2] + chunk * 8) = otile[rr * OROW + chunk];
            }
        }
    }
}


// Block-sparse tile iterator (use_r, no window): lists per 128 query rows.
template <int D>
static hipError_t launch_prefill_sparse(const PrefillParams &p, hipStream_t stream) {
    const long long total = (long long)((p.T + 127) / 128) * p.Hq * p.B;
    if (total > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)total), block(256);
    if (p.row_stats != nullptr) {  // with the row cache of the backward pass
        if (p.causal)
            hipLaunchKernelGGL((prefill_bf16_kernel<D, true, true, false, true, true>), grid, block, 0, stream, p);
        else
            hipLaunchKernelGGL((prefill_bf16_kernel<D, true, false, false, true, true>), grid, block, 0, stream, p);
        return hipGetLastError();
    }
    if (p.causal)
        hipLaunchKernelGGL((prefill_bf16_kernel<D, true, true, false, false, true>), grid, block, 0, stream, p);
    else
        hipLaunchKernelGGL((prefill_bf16_kernel<D, true, false, false, false, true>), grid, block, 0, stream, p);
    return hipGetLastError();
}

// Dense kernels: RW = 2 (256 query rows per workgroup) at d = 64, RW = 1 at d = 128.
template <int D, int RW>
static hipError_t launch_prefill_dense(const PrefillParams &p, hipStream_t stream) {
    const int rows = 128 * RW;
    const long long total = (long long)((p.T + rows - 1) / rows) * p.Hq * p.B;
    if (total > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)total), block(256);
    if (p.prep.gamma_q != nullptr) {  // RMSNorm + RoPE on q, rho in the prologue (use_r, no window, no row cache)
        if (p.causal)
            hipLaunchKernelGGL((prefill_bf16_kernel<D, true, true, false, false, false, RW, true>), grid, block, 0, stream, p);
        else
            hipLaunchKernelGGL((prefill_bf16_kernel<D, true, false, false, false, false, RW, true>), grid, block, 0, stream, p);
        return hipGetLastError();
    }
    if (p.row_stats != nullptr && p.window > 0) {  // row cache + sliding window (causal, use_r)
        hipLaunchKernelGGL((prefill_bf16_kernel<D, true, true, true, true, false, RW>), grid, block, 0, stream, p);
    } else if (p.row_stats != nullptr) {  // with the row cache of the backward pass (use_r)
        if (p.causal)
            hipLaunchKernelGGL((prefill_bf16_kernel<D, true, true, false, true, false, RW>), grid, block, 0, stream, p);
        else
            hipLaunchKernelGGL((prefill_bf16_kernel<D, true, false, false, true, false, RW>), grid, block, 0, stream, p);
    } else if (p.window > 0) {  // causal only (checked by the caller)
        if (p.use_r)
            hipLaunchKernelGGL((prefill_bf16_kernel<D, true, true, true, false, false, RW>), grid, block, 0, stream, p);
        else
            hipLaunchKernelGGL((prefill_bf16_kernel<D, false, true, true, false, false, RW>), grid, block, 0, stream, p);
    } else if (p.use_r) {
        if (p.causal)
            hipLaunchKernelGGL((prefill_bf16_kernel<D, true, true, false, false, false, RW>), grid, block, 0, stream, p);
        else
            hipLaunchKernelGGL((prefill_bf16_kernel<D, true, false, false, false, false, RW>), grid, block, 0, stream, p);
    } else {
        if (p.causal)
            hipLaunchKernelGGL((prefill_bf16_kernel<D, false, true, false, false, false, RW>), grid, block, 0, stream, p);
        else
            hipLaunchKernelGGL((prefill_bf16_kernel<D, false, false, false, false, false, RW>), grid, block, 0, stream, p);
    }
    return hipGetLastError();
}

hipError_t launch_prefill_bf16(const PrefillParams &p, hipStream_t stream) {
    if (p.sparse_row_ptr != nullptr)
        return p.d == 128 ? launch_prefill_sparse<128>(p, stream) : launch_prefill_sparse<64>(p, stream);
    return p.d == 128 ? launch_prefill_dense<128, 1>(p, stream) : launch_prefill_dense<64, 2>(p, stream);
}

}  // namespace plx
