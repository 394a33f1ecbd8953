// Parallax attention over an MLA-style latent cache for MORE THAN 16 COLUMNS (bf16, gfx950): many
// heads on one GPU, several query rows per head, causal prefill over the latent cache.
//
// What it computes is what decode_mla_bf16.hip computes (Algorithm 1 of the paper, Sec. 3.3, over
// cached rows [latent 512 | rope 64] that are key and value at once; a (head, row) pair is one
// MFMA column with its own first and last token). With more than one group of 16 columns the step
// is no longer memory bound: every group walks the same tokens, so what counts is matrix work per
// byte read out of the LDS. This form therefore takes 32 columns per workgroup:
//   * two 64-key tiles in the LDS (the tile layout of the narrow form), filled by direct
//     global -> LDS loads one tile ahead, spread between the matrix instructions of the score
//     k-steps and the wait in front of the exchange. No register stages: the registers hold the
//     operands instead.
//   * scores: wave (kh, ch) takes the keys 32 kh .. 32 kh + 31 of the tile and the columns
//     16 ch .. 16 ch + 15, S^T = C [Q; R]^T over all 576 dimensions with
//     v_mfma_f32_16x16x32_bf16. Its q and rho fragments (144 registers) stay in registers; a K
//     fragment read from the LDS feeds two matrix instructions, the fragment pair of a k-step
//     four independent accumulation chains.
//   * P1 and P2 = P1 * S2 are published through the LDS in the B-operand order of the second
//     contraction, computed against the softmax reference the column has at that moment; the
//     tile maxima of the two waves that scored a column travel with them, and the reference
//     follows the maximum afterwards, in steps (see kRefSlack, kRefGuard);
//   * values: wave w owns the output dimensions 128 w .. 128 w + 127 and accumulates
//     O^T += V^T P^T over all 64 keys and all 32 columns with v_mfma_f32_32x32x16_bf16: a V^T
//     fragment (two transposing LDS reads) feeds two matrix instructions of twice the size.
// Two barriers per tile (the tile has landed; P and the maxima are published). A lane has two
// column identities: its score column (16 ch + lane % 16, rows of the score block are keys) and
// its output column (lane % 32); the softmax reference is kept for both, moved by the same rule
// from the same agreed tile maxima.
// Split partials and their merge are those of the narrow form.
#include "plx_device.h"
#include "plx_kernels.h"
#include "plx_lds_dma.h"
#include "plx_mla_tile.h"

namespace plx {

constexpr int kXcds = 8;            // accelerator dies of the chip, each with its own L2
constexpr int kGroupsPerXcdRun = 8;  // column groups of one (batch, split) that share an XCD
// The softmax reference of a column follows its running maximum only in steps: it moves when the
// maximum has risen more than this (log2 domain) above it. Weights then reach 2^kRefSlack at
// most -- nothing to fp32 sums or to bf16 operands, whose precision is relative -- and the
// 128 accumulation registers of a wave are rescaled a few times per sequence, not in nearly
// every tile (with 32 columns some maximum rises in most tiles; the rescale alone cost a quarter
// of the tile time).
constexpr float kRefSlack = 8.f;
// ... and weights computed before the tile's maximum is known may reach 2^kRefGuard (see the loop)
constexpr float kRefGuard = 64.f;

template <bool PAGED>
__global__ __launch_bounds__(256, 1) void decode_mla_wide_kernel(MlaDecodeParams p) {
    constexpr int CG = 32;              // columns of a workgroup
    constexpr int kPvSteps16 = kMlaTileKeys / 16;  // 16-key k-steps of the second contraction
    // [tile 0] [tile 1] [P1 | P2: 16-key step x lane] [tile maxima: wave x 16] [row sums: wave x 16 x 2]
    __shared__ u32x4 lds[2 * kMlaTileChunks + 2 * kPvSteps16 * 64 + 16 + 32];
    u32x4 *pbuf = lds + 2 * kMlaTileChunks;
    float *smax = (float *)(pbuf + 2 * kPvSteps16 * 64);
    float *dex = smax + 64;

    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int kh = w >> 1, ch = w & 1;  // the wave's half of the keys / of the columns (scores)
    const int c16 = lane & 15, g = lane >> 4;   // score phase: column 16 ch + c16, 16-lane row g
    const int c32 = lane & 31, hi = lane >> 5;  // second contraction: column c32, half hi
    // Workgroup -> (batch, split, column group). The hardware deals consecutive workgroup ids
    // round-robin over the 8 XCDs, each with an L2 of its own; the column groups of one (batch,
    // split) pair walk the same tokens, so up to kGroupsPerXcdRun of them get ids on ONE XCD, next
    // to each other in its sequence: run r = (chunk of groups, batch, split) executes on XCD r % 8
    // at the places (r / 8) kGroupsPerXcdRun + i. (Dealt the plain way, every group fetched its
    // tiles from memory itself: 128 heads read the cache four times.) The chunks are numbered
    // from the last one: with many rows per head those see the most tokens and start first.
    // Ids past the last run or group do nothing.
    const int S = p.S;
    const int n_cols = p.Hq * p.Tq;
    const int n_groups = (n_cols + CG - 1) / CG;
    const int run_len = min(n_groups, kGroupsPerXcdRun), n_chunks = (n_groups + run_len - 1) / run_len;
    const int units = p.B * S;
    const int xcd = blockIdx.x % kXcds, place = blockIdx.x / kXcds;
    const int run = (place / run_len) * kXcds + xcd;
    const int unit = run % units, chunk = n_chunks - 1 - run / units;
    const int cgroup = chunk * run_len + place % run_len;
    if (chunk < 0 || cgroup >= n_groups) return;
    const int split = unit % S, b = unit / S;
    const int scol = cgroup * CG + 16 * ch + c16, ocol = cgroup * CG + c32;  // in [0, Hq * Tq)
    const bool live_s = scol < n_cols, live_o = ocol < n_cols;

    int Lb = p.seq_lens ? p.seq_lens[b] : p.Lmax;
    Lb = min(max(Lb, 0), p.Lmax);
    // tokens [key_lo, key_end) of a column: row t of a head is at position Lb - Tq + t
    auto col_end = [&](int col, bool live) { return live ? max(Lb - p.Tq + (col % p.Tq) + 1, 0) : 0; };
    auto col_lo = [&](int end) { return p.window > 0 ? max(end - p.window, 0) : 0; };
    const int key_end = col_end(scol, live_s), key_lo = col_lo(key_end);  // of the score column
    // the workgroup's tiles: the union over its live columns (the same value in every wave)
    const int oend = col_end(ocol, live_o);
    int wg_end = oend, wg_lo = live_o && oend > 0 ? col_lo(oend) : 0x7fffffff;
#pragma unroll
    for (int off = 1; off < CG; off <<= 1) {
        wg_end = max(wg_end, __shfl_xor(wg_end, off, 64));
        wg_lo = min(wg_lo, __shfl_xor(wg_lo, off, 64));
    }
    wg_end = __builtin_amdgcn_readfirstlane(wg_end);
    wg_lo = __builtin_amdgcn_readfirstlane(min(wg_lo, wg_end));
    const int tile0 = wg_lo / kMlaTileKeys;
    const int n_tiles = (wg_end + kMlaTileKeys - 1) / kMlaTileKeys - tile0;
    const int tiles_per_split = (n_tiles + S - 1) / S;
    const int t_lo = tile0 + split * tiles_per_split;
    const int t_hi = min(t_lo + tiles_per_split, tile0 + n_tiles);

    // ---- B operands of the scores: q and rho of the score column (zero if it is dead), k-step s
    // = dimensions 32 s + 8 g .. + 7, resident for the whole kernel
    u32x4 qf[kMlaKSteps], rf[kMlaKSteps];
    {
        const int64_t row = ((int64_t)b * n_cols + (live_s ? scol : 0)) * kMlaDK;
        const __bf16 *qrow = (const __bf16 *)p.q + row;
        const __bf16 *rrow = (const __bf16 *)p.r + row;
        const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int s = 0; s < kMlaKSteps; ++s) {
            qf[s] = live_s ? *(const u32x4 *)(qrow + 32 * s + 8 * g) : z;
            rf[s] = live_s ? *(const u32x4 *)(rrow + 32 * s + 8 * g) : z;
        }
    }

    // ---- global -> LDS tile loads -------------------------------------------------------------
    // A load fills 64 consecutive chunk slots of the tile: four rows of a latent column block or
    // eight rows of the rope block; every lane fetches the global chunk that belongs at its slot.
    // Wave w brings in column block w (16 loads, rows 4 i .. 4 i + 3) and the rope rows
    // 16 w .. 16 w + 15 (2 loads). The chunk permutation of a latent row reads (row % 4, row / 4 % 4)
    // = (lane / 16, i % 4), that of a rope row (row / 2) % 8 = (4 j + lane / 16) % 8: four + two
    // per-lane byte offsets serve all 18 loads, the rest of an address is wave-uniform. A tile
    // whose 64 rows exist and lie in one piece is fetched that way; the last, partial tile of a
    // sequence (and a page size that is no multiple of 64) takes the per-row form, which re-reads
    // the sequence's last row for the rows past its end (finite data, masked below).
    const __bf16 *cbase = (const __bf16 *)p.ckv + (PAGED ? 0 : (int64_t)b * p.csb);
    using const_i32 = const __attribute__((address_space(4))) int32_t;
    const int32_t *table = PAGED ? p.block_table + (int64_t)b * p.table_stride : nullptr;
    const_i32 *table_c = (const_i32 *)(uintptr_t)table;  // scalar loads where the index is uniform
    const bool tiles_in_pages = !PAGED || p.page_size % kMlaTileKeys == 0;  // workgroup-uniform
    auto page_of = [&](int32_t entry) { return (int64_t)min(max(entry, 0), p.num_pages - 1); };
    auto tile_start = [&](int t) __attribute__((always_inline)) -> const char * {
        if constexpr (PAGED) {
            // (the division runs on the vector unit: hand the result back to scalar registers,
            // which is where the load statements take their base from)
            const int key = t * kMlaTileKeys;
            const int page_idx = __builtin_amdgcn_readfirstlane(key / p.page_size);
            const int in_page = __builtin_amdgcn_readfirstlane(key % p.page_size);
            return (const char *)(cbase + page_of(table_c[page_idx]) * p.csb + (int64_t)in_page * p.csl);
        } else {
            return (const char *)cbase + (int64_t)t * (kMlaTileKeys * 2) * p.csl;
        }
    };
    auto row_start = [&](int key) __attribute__((always_inline)) -> const __bf16 * {
        if constexpr (PAGED)
            return cbase + page_of(table[key / p.page_size]) * p.csb + (int64_t)(key % p.page_size) * p.csl;
        else
            return cbase + (int64_t)key * p.csl;
    };
    constexpr int kLatLoads = kRowGroups;  // 16 latent loads, then kMlaLoadsPerWave - 16 = 2 rope loads
    // load i of this wave: tile row of this lane and element of the cached row
    auto lane_row = [&](int i) { return i < kLatLoads ? 4 * i + (lane >> 4) : 8 * (2 * w + i - kLatLoads) + (lane >> 3); };
    auto lane_elem = [&](int i) {
        return i < kLatLoads ? 128 * w + (((lane & 15) ^ lds_row_swizzle<128>(lane_row(i))) * 8)
                             : kMlaDC + (((lane & 7) ^ lds_row_swizzle<64>(lane_row(i))) * 8);
    };
    // LDS byte address of load i of this wave in tile buffer buf
    const uint32_t lds_base = lds_byte_address(lds);
    auto load_dst = [&](int buf, int i) {
        const int slot0 = i < kLatLoads ? w * kMlaBlkChunks + 64 * i
                                        : kMlaLatBlocks * kMlaBlkChunks + 64 * (2 * w + i - kLatLoads);
        return lds_base + (uint32_t)(buf * kMlaTileChunks + slot0) * 16u;
    };
    const int csl32 = (int)p.csl;
    uint32_t lat_off[4], rope_off[2];  // the lane's part of the source byte offset
#pragma unroll
    for (int v = 0; v < 4; ++v) lat_off[v] = (uint32_t)((lane >> 4) * csl32 + lane_elem(v) - 128 * w) * 2u;
#pragma unroll
    for (int j = 0; j < 2; ++j) rope_off[j] = (uint32_t)((lane >> 3) * csl32 + lane_elem(kLatLoads + j) - kMlaDC) * 2u;
    // load i of a whole tile that starts at tile_base (a tile is addressed with 32-bit byte
    // offsets: the wave-uniform part of an offset is added to the lane's part, the base stays)
    // (`stride`: the token stride again, handed in as a value the compiler cannot see through --
    // with the plain one it keeps all 18 sums in registers across the loop, which it does not have)
    // (`lanes`: -1, or 0 = no load)
    auto issue_load = [&](const char *tile_base, int buf, int i, int stride, int32_t lanes) __attribute__((always_inline)) {
        if (i < kLatLoads)
            tile_load16_uniform_if(lanes, lat_off[i & 3] + (uint32_t)(4 * i * stride + 128 * w) * 2u, tile_base, load_dst(buf, i));
        else
            tile_load16_uniform_if(lanes, rope_off[i - kLatLoads] + (uint32_t)(8 * (2 * w + i - kLatLoads) * stride + kMlaDC) * 2u,
                                   tile_base, load_dst(buf, i));
    };
    // the whole tile as one block (prologue, partial tiles, tiles in several pieces)
    auto issue_tile = [&](int t, int buf) __attribute__((always_inline)) {
        const int tk0 = t * kMlaTileKeys;
        if (tiles_in_pages && tk0 + kMlaTileKeys <= Lb) {  // workgroup-uniform
            const char *tile_base = tile_start(t);
#pragma unroll
            for (int i = 0; i < kMlaLoadsPerWave; ++i) issue_load(tile_base, buf, i, csl32, -1);
        } else {
#pragma unroll
            for (int i = 0; i < kMlaLoadsPerWave; ++i)
                tile_load16<64>(row_start(min(tk0 + lane_row(i), Lb - 1)) + lane_elem(i), load_dst(buf, i));
        }
    };

    // per-lane LDS byte offsets inside a tile of the two read patterns (set up once).
    // K operand of score k-step s, row block rb: chunk 4 (s % 4) + g of row 32 kh + 16 rb + c16 in
    // column block s / 4 (+ 16 KB per block, + 4 KB per row block as immediates; the chunk
    // permutation reads bits 0 .. 3 of the row only), the two rope k-steps in the rope block.
    // V^T operand of the 32-dimension block n and the 16-key step kk: two transposing reads,
    // r = 0, 1, of the keys 16 kk + 8 hi + 4 r + (lane % 16) / 4, dimensions
    // 32 n + 16 (lane / 16 % 2) + 4 (lane % 4) .. + 3 of the wave's column block.
    const int krow = 32 * kh + c16;
    uint32_t k_off[4], k_off_rope[2], v_off[4][2];
#pragma unroll
    for (int j = 0; j < 4; ++j) k_off[j] = (uint32_t)lds_chunk_slot<128>(krow, 4 * j + g) * 16u;
#pragma unroll
    for (int j = 0; j < 2; ++j)
        k_off_rope[j] = (uint32_t)(kMlaLatBlocks * kMlaBlkChunks + lds_chunk_slot<64>(krow, 4 * j + g)) * 16u;
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int r = 0; r < 2; ++r)
            v_off[n][r] = (uint32_t)(w * kMlaBlkChunks + lds_chunk_slot<128>(8 * hi + 4 * r + (c16 >> 2),
                                                                             4 * n + 2 * (g & 1) + ((lane & 3) >> 1))) * 16u +
                          (uint32_t)(lane & 1) * 8u;

    // ---- running state ------------------------------------------------------------------------
    // score column: reference m_s and the row sums over this lane's keys; output column c32:
    // reference m_o and O^T, register i of block n = dimension 128 w + 32 n + 8 (i / 4) + 4 hi + i % 4
    float m_s = kNegInf, m_o = kNegInf, dsum1 = 0.f, dsum2 = 0.f;
    float rescale_s = 1.f, rescale_o = 1.f;  // owed to the sums since the references last moved
    f32x16 o1[4], o2[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int i = 0; i < 16; ++i) o1[n][i] = 0.f, o2[n][i] = 0.f;
    const float scale_log2 = p.scale * kLog2e;

    // One tile. If tile t + 1 is whole and lies in one piece, twelve of its 18 loads go between
    // the matrix instructions of the score k-steps (two of every three steps) and six in front of
    // the barrier that publishes P (under an execution mask, so the body has no branches);
    // otherwise they were issued as a block in front. (One load in every k-step asks the CU's
    // vector-memory path for exactly what it can deliver, and the waves queue up behind it: 3 %
    // slower. Later than the barrier the loads land too late.)
    // The LDS fragment reads run two steps ahead of the matrix instructions that use them (three
    // fragment sets in rotation); scheduling fences keep the compiler from sinking a read down to
    // its first use, which exposes the LDS latency once per step.
    constexpr int kScoreLoads = kMlaKSteps - kMlaKSteps / 3;  // 12
    if (t_lo < t_hi) issue_tile(t_lo, 0);
    for (int t = t_lo; t < t_hi; ++t) {
        const int buf = (t - t_lo) & 1;
        // tile t has landed and is visible; everybody is done with tile t - 1, whose buffer
        // receives tile t + 1 now
        tile_barrier<0>();
        const char *tile = (const char *)(lds + buf * kMlaTileChunks);
        const bool more = t + 1 < t_hi;
        const bool spread = more && tiles_in_pages && (t + 2) * kMlaTileKeys <= Lb;  // workgroup-uniform
        if (more && !spread) issue_tile(t + 1, buf ^ 1);
        const char *fill_base = spread ? tile_start(t + 1) : (const char *)cbase;
        const int32_t fill_lanes = __builtin_amdgcn_readfirstlane(spread ? -1 : 0);
        int stride_now = csl32;
        asm volatile("" : "+s"(stride_now));

        // ---- S1^T = C q^T, S2^T = C rho^T: keys 32 kh + 16 rb + 4 g + i, column 16 ch + c16 ----
        f32x4 s1[2], s2[2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) s1[rb] = f32x4{0.f, 0.f, 0.f, 0.f}, s2[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
        {
            u32x4 kf[3][2];  // [set = k-step % 3][row block]
            auto read_step = [&](int ks) __attribute__((always_inline)) {
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
                    kf[ks % 3][rb] = ks < kMlaLatBlocks * 4
                                         ? *(const u32x4 *)(tile + k_off[ks & 3] + (ks >> 2) * (kMlaBlkChunks * 16) + rb * (16 * 256))
                                         : *(const u32x4 *)(tile + k_off_rope[ks - kMlaLatBlocks * 4] + rb * (16 * 128));
            };
            read_step(0);
            read_step(1);
#pragma unroll
            for (int ks = 0; ks < kMlaKSteps; ++ks) {
                if (ks + 2 < kMlaKSteps) read_step(ks + 2);
                if (ks % 3 != 2) issue_load(fill_base, buf ^ 1, ks - ks / 3, stride_now, fill_lanes);  // loads 0 .. 11
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) {
                    s1[rb] = mfma16(kf[ks % 3][rb], qf[ks], s1[rb]);
                    s2[rb] = mfma16(kf[ks % 3][rb], rf[ks], s2[rb]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }

        // ---- P1, P2 of this lane's keys -> LDS in B-operand order, against the reference the
        // column has NOW: no agreement on the tile's maximum first (that cost a barrier and an LDS
        // round trip per tile). The tile maxima travel with P and are looked at behind the
        // barrier: if some column's maximum lies more than kRefGuard binades above its reference
        // (or the column has no reference yet: its first visible tile), the workgroup moves the
        // references and publishes P again before anybody uses it -- rare; otherwise the weights
        // stand (they are at most 2^kRefGuard) and the references move, in steps, for the next tile.
        // 16-key step kk = 2 kh + rb of the second contraction; k-elements 8 hi' .. 8 hi' + 7 of
        // the consuming lane (column, hi') are the keys 8 hi' + (0 .. 7) of the step, i.e. the
        // producing lanes g = 2 hi' (elements 0 .. 3) and g = 2 hi' + 1 (elements 4 .. 7).
        const int key0 = t * kMlaTileKeys + 32 * kh + 4 * g;  // this lane's keys: key0 + 16 rb + i
        float x[8];
        float tmax = kNegInf;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int key = key0 + 16 * (e >> 2) + (e & 3);
            x[e] = (key >= key_lo && key < key_end) ? s1[e >> 2][e & 3] * scale_log2 : kNegInf;
            tmax = fmaxf(tmax, x[e]);
        }
        float d1_tile, d2_tile;  // this lane's share of the tile's row sums, under the reference used
        auto publish = [&](float reference) __attribute__((always_inline)) {
            const float ref_use = reference == kNegInf ? 0.f : reference;
            d1_tile = 0.f, d2_tile = 0.f;
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                float p1[4], p2[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    p1[i] = fast_exp2(x[4 * rb + i] - ref_use);  // 0 if masked
                    p2[i] = x[4 * rb + i] == kNegInf ? 0.f : p1[i] * s2[rb][i];
                }
                const u32x2 pk1 = pack4_bf16_accumulate(p1[0], p1[1], p1[2], p1[3], d1_tile);
                const u32x2 pk2 = pack4_bf16_accumulate(p2[0], p2[1], p2[2], p2[3], d2_tile);
                u32x2 *dst = (u32x2 *)(pbuf + (2 * kh + rb) * 64 + 32 * (g >> 1) + 16 * ch + c16) + (g & 1);
                dst[0] = pk1;
                dst[2 * kPvSteps16 * 64] = pk2;  // P2 follows P1: 4 steps x 64 chunks = 512 half-chunks
            }
        };
        // a column's reference follows its maximum in steps of more than kRefSlack binades;
        // returns the factor that brings sums under the old reference to the new one
        auto move_reference = [&](float &reference, float tile_max) __attribute__((always_inline)) {
            const float moved = tile_max > reference + kRefSlack ? tile_max : reference;
            const float factor = fast_exp2(reference - (moved == kNegInf ? 0.f : moved));  // 0 from "none yet"
            reference = moved;
            return factor;
        };
        publish(m_s);
        tmax = rows_max(tmax);
        if (g == 0) smax[w * 16 + c16] = tmax;
        // the last six loads of the next tile: here the wave is about to wait anyway
#pragma unroll
        for (int i = kScoreLoads; i < kMlaLoadsPerWave; ++i) issue_load(fill_base, buf ^ 1, i, stride_now, fill_lanes);
        __syncthreads();
        // (wave 2 kh + ch holds column 16 ch + c16 at index 16 (2 kh + ch) + c16 = 32 kh + column)
        const float mt_s = fmaxf(smax[16 * ch + c16], smax[32 + 16 * ch + c16]);
        const float mt_o = fmaxf(smax[c32], smax[32 + c32]);
        // (every wave looks at all 32 columns through its output columns: the same decision in all)
        if (__any(mt_o > m_o + kRefGuard || (m_o == kNegInf && mt_o != kNegInf))) {
            rescale_s *= move_reference(m_s, mt_s);
            rescale_o *= move_reference(m_o, mt_o);
            publish(m_s);
            __syncthreads();
        }
        // the sums so far come under the columns' present references (moved at the end of the
        // tile before, or just now), then the tile joins them
        dsum1 = dsum1 * rescale_s + d1_tile;
        dsum2 = dsum2 * rescale_s + d2_tile;
        // The rescale works on the accumulation registers in place (assembly: written as plain
        // multiplications it made the compiler carry a second copy of all 128 accumulators in
        // vector registers around the loop, 128 moves per tile and as many registers short). The
        // matrix instructions that wrote these registers were issued a whole score phase ago,
        // the ones that read them follow behind the wait states below.
        if (!__all(rescale_o == 1.f)) {
#pragma unroll
            for (int n = 0; n < 4; ++n)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float a = o1[n][i], b2 = o2[n][i], ta, tb;
                    asm volatile(
                        "v_accvgpr_read_b32 %2, %0\n\t"
                        "v_accvgpr_read_b32 %3, %1\n\t"
                        "v_mul_f32 %2, %2, %4\n\t"
                        "v_mul_f32 %3, %3, %4\n\t"
                        "v_accvgpr_write_b32 %0, %2\n\t"
                        "v_accvgpr_write_b32 %1, %3"
                        : "+a"(a), "+a"(b2), "=&v"(ta), "=&v"(tb)
                        : "v"(rescale_o));
                    o1[n][i] = a, o2[n][i] = b2;
                }
            asm volatile("s_nop 7\n\ts_nop 7" ::: "memory");
        }
        // the references for the next tile (nothing moves right behind the slow path above); the
        // sums follow at this place of the next tile. Not behind the last tile: the record's
        // reference is the one its sums are under.
        rescale_s = 1.f, rescale_o = 1.f;
        if (more) {
            rescale_s = move_reference(m_s, mt_s);
            rescale_o = move_reference(m_o, mt_o);
        }

        // ---- O1^T += V^T P1^T, O2^T += V^T P2^T: dimensions 128 w .. 128 w + 127, 32 columns ---
        // step i = (16-key step kk = i / 4, dimension block n = i % 4): two transposing reads feed
        // two matrix instructions; the reads run two steps ahead
        {
            constexpr int kSteps = kPvSteps16 * 4;
            u32x2 vlo[3], vhi[3];
            u32x4 pb1[2], pb2[2];
            auto read_step = [&](int i) __attribute__((always_inline)) {
                const int kk = i >> 2, n = i & 3;
                if (n == 0) pb1[kk & 1] = pbuf[kk * 64 + lane], pb2[kk & 1] = pbuf[(kPvSteps16 + kk) * 64 + lane];
                vlo[i % 3] = lds_read_tr16(tile + v_off[n][0] + kk * (16 * 256));
                vhi[i % 3] = lds_read_tr16(tile + v_off[n][1] + kk * (16 * 256));
            };
            read_step(0);
            read_step(1);
#pragma unroll
            for (int i = 0; i < kSteps; ++i) {
                if (i + 2 < kSteps) read_step(i + 2);
                __builtin_amdgcn_sched_barrier(0);
                const int kk = i >> 2, n = i & 3;
                const u32x4 vt = {vlo[i % 3][0], vlo[i % 3][1], vhi[i % 3][0], vhi[i % 3][1]};
                o1[n] = mfma32(vt, pb1[kk & 1], o1[n]);
                o2[n] = mfma32(vt, pb2[kk & 1], o2[n]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    // ---- row sums of a column: over the rows of a wave, then over the two waves that scored it
    dsum1 = rows_sum(dsum1);
    dsum2 = rows_sum(dsum2);
    if (g == 0) {
        dex[(w * 16 + c16) * 2] = dsum1;
        dex[(w * 16 + c16) * 2 + 1] = dsum2;
    }
    __syncthreads();
    const float d1 = dex[c32 * 2] + dex[(32 + c32) * 2];
    const float d2 = dex[c32 * 2 + 1] + dex[(32 + c32) * 2 + 1];
    if (!live_o) return;
    const int64_t hq = (int64_t)b * n_cols + ocol;
    if (p.direct_out) {
        float inv = 0.f, gain = 0.f;  // empty key set: zeros
        if (d1 > 0.f) {
            inv = 1.f / d1;
            gain = inv * (1.f + d2 * inv);
        }
        __bf16 *orow = (__bf16 *)p.o + hq * kMlaDC + 128 * w + 4 * hi;
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                float y[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) y[i] = o1[n][4 * q4 + i] * gain - o2[n][4 * q4 + i] * inv;
                *(u32x2 *)(orow + 32 * n + 8 * q4) = u32x2{pack_bf16(y[0], y[1]), pack_bf16(y[2], y[3])};
            }
    } else {
        float *rec = p.ws + (hq * S + split) * (int64_t)(2 * kMlaDC + 4);
        if (w == 0 && hi == 0) *(f32x4 *)rec = f32x4{m_o, d1, d2, 0.f};
        float *r1 = rec + 4 + 128 * w + 4 * hi;
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                *(f32x4 *)(r1 + 32 * n + 8 * q4) =
                    f32x4{o1[n][4 * q4], o1[n][4 * q4 + 1], o1[n][4 * q4 + 2], o1[n][4 * q4 + 3]};
                *(f32x4 *)(r1 + kMlaDC + 32 * n + 8 * q4) =
                    f32x4{o2[n][4 * q4], o2[n][4 * q4 + 1], o2[n][4 * q4 + 2], o2[n][4 * q4 + 3]};
            }
    }
}

hipError_t launch_decode_mla_wide(const MlaDecodeParams &p, hipStream_t stream) {
    const int64_t n_groups = ((int64_t)p.Hq * p.Tq + 31) / 32, units = (int64_t)p.B * p.S;
    const int64_t run_len = n_groups < kGroupsPerXcdRun ? n_groups : kGroupsPerXcdRun;
    const int64_t runs = units * ((n_groups + run_len - 1) / run_len);
    const int64_t n_wgs = (runs + kXcds - 1) / kXcds * kXcds * run_len;
    if (n_wgs > 0x7fffffff) return hipErrorInvalidValue;
    const dim3 grid((unsigned)n_wgs);
    if (p.block_table)
        hipLaunchKernelGGL(decode_mla_wide_kernel<true>, grid, dim3(256), 0, stream, p);
    else
        hipLaunchKernelGGL(decode_mla_wide_kernel<false>, grid, dim3(256), 0, stream, p);
    return hipSuccess;
}

}  // namespace plx
