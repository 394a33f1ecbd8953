// Split-KV Parallax decode over an MLA-style latent cache (bf16, gfx950).
//
// What it computes: Algorithm 1 of the paper (Sec. 3.3) for one query row per head, where every
// cached token is ONE row c_j = [latent (512) | rope part (64)] shared by all heads: the key is
// the whole row, the value its latent part (the absorbed-projection decode form of multi-head
// latent attention, which the paper's closing discussion names as structurally compatible).
// q and rho arrive in the latent space ([B, Hq, Tq, 576]), the output is [B, Hq, Tq, 512].
// Tq > 1: the rows of a head sit at the last Tq positions of the sequence and row t sees the
// tokens up to its own (a speculative / chunked decode step, or the causal prefill over the
// latent cache with Tq = prompt length); `window` > 0 cuts a row's tokens to the last `window`.
// A (head, row) pair is simply one more MFMA column with its own first and last token: a
// workgroup's tile range is the union over its 16 columns.
//
// How it is laid out for CDNA4. With 16 heads per column group the step reads 1152 bytes per token
// for 70 kflop: still HBM bound, but the state of a column group -- O1^T, O2^T of 512 dimensions
// x 16 columns -- is four times that of the d = 128 decode kernel. So the four waves of a
// workgroup share each 64-key tile instead of streaming private ones:
//   * grid (split, group of 16 heads, batch). What buys bandwidth is bytes in flight: a tile
//     travels global -> registers -> LDS through TWO register stages per wave, so two 72 KB tiles
//     are on their way while a third is worked on (ordinary loads do not hold the issuing wave;
//     global -> LDS loads did, for 1.2 - 2.5 us per tile, with one tile in flight). The registers
//     for that come from keeping the q and rho fragments in LDS instead.
//   * scores: wave w takes keys 16w .. 16w+15 of the tile, S^T = C [Q;R]^T over all 576
//     dimensions (18 k-steps of v_mfma_f32_16x16x32_bf16);
//   * the tile maximum of a column is agreed on through LDS (one barrier), every wave then forms
//     P1, P2 = P1 * S2 of its 16 keys and publishes them, already packed as the B operand of the
//     second contraction, through LDS (second barrier);
//   * values: wave w owns the output dimensions 128w .. 128w+127 and accumulates
//     O^T += V^T P^T over all 64 keys, V^T fragments by transposing LDS reads of the same tile --
//     so no wave ever needs another wave's accumulators, and the tile is fetched once for both
//     contractions.
// The tile is stored as four 128-dimension column blocks plus the rope block, each with the XOR
// chunk swizzle of the d = 128 / d = 64 decode tiles, so the three access patterns (row-wise
// fill, K operand, V^T operand) are the ones those layouts were made for.
// Split partials use the record format of the d = 128 kernel (m, d1, d2, pad, O1[512], O2[512])
// and are merged by the same combine kernel (App. C).
#include "plx_device.h"
#include "plx_kernels.h"
#include "plx_mla_tile.h"

namespace plx {

// PAGED: the cache is a pool of pages behind a block table. A tile that lies inside one page
// (page size a multiple of 64) is fetched like a tile of a contiguous cache from its page;
// otherwise every lane looks up the page of its row.
template <bool PAGED>
__global__ __launch_bounds__(256, 1) void decode_mla_kernel(MlaDecodeParams p) {
    // [tile] [q fragments: k-step x lane] [rho fragments] [P1 | P2 as B operands] [tile maxima] [row sums]
    __shared__ u32x4 lds[kMlaTileChunks + 2 * kMlaKSteps * 64 + 128 * kMlaPvSteps + 16 + 32];
    u32x4 *qlds = lds + kMlaTileChunks;
    u32x4 *rlds = qlds + kMlaKSteps * 64;
    u32x4 *pbuf = rlds + kMlaKSteps * 64;               // P1: [k-step][64 lanes], then P2 likewise
    float *smax = (float *)(pbuf + 128 * kMlaPvSteps);  // [4 waves][16 columns]
    float *dex = smax + 64;                             // [4 waves][16 columns][2]

    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int c = lane & 15;  // MFMA column: (head, row) pair 16 * group + c, row fastest
    const int g = lane >> 4;  // 16-lane row of the wave
    const int split = blockIdx.x, hgroup = blockIdx.y, b = blockIdx.z;
    const int S = p.S;
    const int n_cols = p.Hq * p.Tq;
    const int head = hgroup * 16 + c;  // column index in [0, Hq * Tq)
    const bool live = head < n_cols;

    int Lb = p.seq_lens ? p.seq_lens[b] : p.Lmax;
    Lb = min(max(Lb, 0), p.Lmax);
    // tokens [key_lo, key_end) of this lane's column: row t of a head is at position Lb - Tq + t
    const int key_end = live ? max(Lb - p.Tq + (head % p.Tq) + 1, 0) : 0;
    const int key_lo = p.window > 0 ? max(key_end - p.window, 0) : 0;
    // the workgroup's tiles: the union over its live columns (the same value in every wave)
    int wg_end = key_end, wg_lo = live && key_end > 0 ? key_lo : 0x7fffffff;
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) {
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

    // ---- B operands: q and rho of the group's heads (zero in the dead columns) -> LDS, in the
    // order the MFMAs want them: entry [k-step s][lane (c, g)] = dims 32 s + 8 g .. + 7 of column c.
    // Wave w fills the k-steps w, w + 4, ...; everybody reads them back in every tile.
    {
        const int64_t row = ((int64_t)b * n_cols + (live ? head : 0)) * kMlaDK;
        const __bf16 *qrow = (const __bf16 *)p.q + row;
        const __bf16 *rrow = (const __bf16 *)p.r + row;
        const u32x4 z = {0u, 0u, 0u, 0u};
        for (int s = w; s < kMlaKSteps; s += 4) {
            qlds[s * 64 + lane] = live ? *(const u32x4 *)(qrow + 32 * s + 8 * g) : z;
            rlds[s * 64 + lane] = live ? *(const u32x4 *)(rrow + 32 * s + 8 * g) : z;
        }
    }

    // ---- global -> registers -> LDS tile path ------------------------------------------------
    // The LDS tile is four latent column blocks [64 rows][16 chunks] plus the rope block
    // [64 rows][8 chunks], chunks permuted inside their row (lds_chunk_slot).
    //  * dense cache (token stride = 576): a tile is 72 KB of consecutive memory and load idx
    //    (0..71) of the tile simply fetches its bytes [1024 idx, +1024) -- the access pattern of a
    //    plain copy; every lane then writes its chunk to the slot of its (row, chunk).
    //  * strided cache: load idx fetches the chunks of the 64 consecutive LDS slots [64 idx, +64)
    //    (four rows of a column block, or eight rows of the rope block), and the register -> LDS
    //    stores are consecutive.
    // Either way one per-lane offset per load is kept: the LDS slot (dense) or the global byte
    // offset (strided). A partial last tile re-reads the sequence's last row for the rows past
    // its end (finite data, masked below); its places are recomputed, not kept.
    const __bf16 *cbase = (const __bf16 *)p.ckv + (PAGED ? 0 : (int64_t)b * p.csb);
    const bool dense = p.csl == kMlaDK;  // workgroup-uniform
    // (the table is read through the constant address space where the index is uniform: scalar loads)
    using const_i32 = const __attribute__((address_space(4))) int32_t;
    const int32_t *table = PAGED ? p.block_table + (int64_t)b * p.table_stride : nullptr;
    const_i32 *table_c = (const_i32 *)(uintptr_t)table;
    const bool tiles_in_pages = !PAGED || p.page_size % kMlaTileKeys == 0;  // workgroup-uniform
    auto page_of = [&](int32_t entry) { return (int64_t)min(max(entry, 0), p.num_pages - 1); };
    // first byte of tile t when it lies in one piece
    auto tile_start = [&](int t) __attribute__((always_inline)) -> const char * {
        if constexpr (PAGED) {
            const int key = t * kMlaTileKeys;
            return (const char *)(cbase + page_of(table_c[key / p.page_size]) * p.csb +
                                  (int64_t)(key % p.page_size) * p.csl);
        } else {
            return (const char *)cbase + (int64_t)t * (kMlaTileKeys * 2) * p.csl;
        }
    };
    // row `key` of the sequence (per lane)
    auto row_start = [&](int key) __attribute__((always_inline)) -> const __bf16 * {
        if constexpr (PAGED)
            return cbase + page_of(table[key / p.page_size]) * p.csb + (int64_t)(key % p.page_size) * p.csl;
        else
            return cbase + (int64_t)key * p.csl;
    };
    auto slot_place = [&](int i, int &row, int &elem) __attribute__((always_inline)) {  // strided: load i of this wave
        const int idx = w * kMlaLoadsPerWave + i;  // wave-uniform
        if (idx < kMlaLatBlocks * kRowGroups) {
            row = 4 * (idx % kRowGroups) + (lane >> 4);
            elem = (idx / kRowGroups) * 128 + (((lane & 15) ^ lds_row_swizzle<128>(row)) * 8);
        } else {
            row = 8 * (idx - kMlaLatBlocks * kRowGroups) + (lane >> 3);
            elem = kMlaDC + (((lane & 7) ^ lds_row_swizzle<64>(row)) * 8);
        }
    };
    auto linear_place = [&](int i, int &row, int &chunk) __attribute__((always_inline)) {  // dense: load i of this wave
        const int q = (w * kMlaLoadsPerWave + i) * 64 + lane;  // 16-byte chunk of the tile
        row = q / (kMlaDK / 8);
        chunk = q - row * (kMlaDK / 8);
    };
    uint32_t off[kMlaLoadsPerWave];
#pragma unroll
    for (int i = 0; i < kMlaLoadsPerWave; ++i) {
        if (dense) {
            int row, chunk;
            linear_place(i, row, chunk);
            off[i] = chunk < 64 ? (uint32_t)((chunk >> 4) * kMlaBlkChunks + lds_chunk_slot<128>(row, chunk & 15)) * 16u
                                : (uint32_t)(kMlaLatBlocks * kMlaBlkChunks + lds_chunk_slot<64>(row, chunk - 64)) * 16u;
        } else {
            int row, elem;
            slot_place(i, row, elem);
            off[i] = (uint32_t)(row * (int)p.csl + elem) * 2u;
        }
    }
    const uint32_t wave_lin = (uint32_t)(w * kMlaLoadsPerWave * 64 + lane) * 16u;  // this lane's first chunk, both sides
    // The stage loads, the wait for them and the stage -> LDS stores are assembly statements:
    // left to the compiler, the wait in front of a stage's stores also covers the loads of the
    // OTHER stage, issued one tile later (its bookkeeping of loads in flight is pessimistic across
    // the loop edge), which takes away half of what is in flight. The stage registers are touched
    // by these statements only -- the build checks that on the generated code
    // (asm_check.find_foreign_uses_of_asm_loaded_registers): nothing else may read or move a
    // register whose load is still on its way. The stages live in accumulation registers (loads
    // and LDS stores take those directly on this chip), which the matrix instructions of this
    // kernel leave free. Loads complete in issue order, so "at most 18 in flight" means the older
    // stage has landed.
    u32x4 stg_a[kMlaLoadsPerWave], stg_b[kMlaLoadsPerWave];  // tiles t_lo + even / + odd
    auto load_stage = [&](u32x4 (&stg)[kMlaLoadsPerWave], int t) __attribute__((always_inline)) {
        const int tk0 = t * kMlaTileKeys;
        if (tiles_in_pages && tk0 + kMlaTileKeys <= Lb) {  // workgroup-uniform
            const char *tile_base = tile_start(t);
            if (dense) {
#pragma unroll
                for (int i = 0; i < kMlaLoadsPerWave; ++i)
                    asm volatile("global_load_dwordx4 %0, %1, %2" : "=a"(stg[i]) : "v"(wave_lin), "s"(tile_base + 1024 * i));
            } else {
#pragma unroll
                for (int i = 0; i < kMlaLoadsPerWave; ++i)
                    asm volatile("global_load_dwordx4 %0, %1, %2" : "=a"(stg[i]) : "v"(off[i]), "s"(tile_base));
            }
        } else {
#pragma unroll
            for (int i = 0; i < kMlaLoadsPerWave; ++i) {
                int row, elem;
                if (dense) {
                    linear_place(i, row, elem);
                    elem *= 8;
                } else {
                    slot_place(i, row, elem);
                }
                const __bf16 *src = row_start(min(tk0 + row, Lb - 1)) + elem;
                asm volatile("global_load_dwordx4 %0, %1, off" : "=a"(stg[i]) : "v"(src));
            }
        }
    };
    // Loads [i0, i1) of a COMPLETE tile (spread over the matrix work of the tile before: issued as
    // one block, the 72 loads of a tile keep the four waves in the issue stage for 1.2 - 1.6 us,
    // the time the texture path needs for 72 KB).
    auto load_piece = [&](u32x4 (&stg)[kMlaLoadsPerWave], const char *tile_base, int i0, int i1)
                          __attribute__((always_inline)) {
#pragma unroll
        for (int i = i0; i < i1; ++i) {
            if (dense)
                asm volatile("global_load_dwordx4 %0, %1, %2" : "=a"(stg[i]) : "v"(wave_lin), "s"(tile_base + 1024 * i));
            else
                asm volatile("global_load_dwordx4 %0, %1, %2" : "=a"(stg[i]) : "v"(off[i]), "s"(tile_base));
        }
    };
    const uint32_t lds_tile_addr = (uint32_t)(uintptr_t)(const char __attribute__((address_space(3))) *)lds;
    // `younger`: the other stage's 18 loads were issued after this stage's and may stay in flight
    auto store_stage = [&](const u32x4 (&stg)[kMlaLoadsPerWave], bool younger) __attribute__((always_inline)) {
        if (younger)
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kMlaLoadsPerWave) : "memory");
        else
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (dense) {
#pragma unroll
            for (int i = 0; i < kMlaLoadsPerWave; ++i)
                asm volatile("ds_write_b128 %0, %1" ::"v"(lds_tile_addr + off[i]), "a"(stg[i]) : "memory");
        } else {
            const uint32_t base = lds_tile_addr + wave_lin;
#pragma unroll
            for (int i = 0; i < kMlaLoadsPerWave; ++i)
                asm volatile("ds_write_b128 %0, %1 offset:%2" ::"v"(base), "a"(stg[i]), "n"(1024 * i) : "memory");
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the barrier that follows publishes the tile
    };
    // per-lane LDS byte offsets inside the tile of the two read patterns (set up once):
    // K operand of score k-step s: chunk 4 (s % 4) + g of row 16 w + c in column block s / 4
    // (+ 16 KB per block as an immediate), the two rope k-steps in the rope block; V^T operand of
    // dimension block n: rows 4 g + c / 4 (+ 16, 32, 48 rows as immediates: the chunk permutation
    // reads bits 0..3 of the row only)
    const int krow = 16 * w + c;
    uint32_t k_off[4], k_off_rope[2], v_off[kMlaNDB];
#pragma unroll
    for (int j = 0; j < 4; ++j) k_off[j] = (uint32_t)lds_chunk_slot<128>(krow, 4 * j + g) * 16u;
#pragma unroll
    for (int j = 0; j < 2; ++j)
        k_off_rope[j] = (uint32_t)(kMlaLatBlocks * kMlaBlkChunks + lds_chunk_slot<64>(krow, 4 * j + g)) * 16u;
#pragma unroll
    for (int n = 0; n < kMlaNDB; ++n)
        v_off[n] = (uint32_t)(w * kMlaBlkChunks + lds_chunk_slot<128>(4 * g + (c >> 2), 2 * n + ((c & 3) >> 1))) * 16u +
                   (uint32_t)(c & 1) * 8u;
    const char *tile = (const char *)lds;

    // ---- running state: column c; O^T rows = dimensions 128 w + 16 n + 4 g + i ---------------
    float m_run = kNegInf, dsum1 = 0.f, dsum2 = 0.f;  // sums: partial over this lane's keys
    f32x4 o1[kMlaNDB], o2[kMlaNDB];
#pragma unroll
    for (int n = 0; n < kMlaNDB; ++n) {
        o1[n] = f32x4{0.f, 0.f, 0.f, 0.f};
        o2[n] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const float scale_log2 = p.scale * kLog2e;

    // One tile: on entry it is in LDS (written by all waves, not yet published); `next` holds the
    // tile after it (in flight or landed), which is written to LDS at the end, and is then
    // refilled with the tile three ahead.
    // `fill` is the stage that was emptied at the end of the tile before: it receives tile t + 2.
    auto process_tile = [&](int t, u32x4 (&next)[kMlaLoadsPerWave], u32x4 (&fill)[kMlaLoadsPerWave])
                            __attribute__((always_inline)) {
        __syncthreads();  // tile t (and, the first time, the q / rho fragments) are visible
        // tile t + 2 sets off now: piece by piece between the matrix instructions if it is complete
        const bool refill = t > t_lo && t + 2 < t_hi;  // (the prologue has requested t_lo + 1 and t_lo + 2)
        const bool spread = refill && tiles_in_pages && (t + 3) * kMlaTileKeys <= Lb;  // workgroup-uniform
        const char *fill_base = spread ? tile_start(t + 2) : nullptr;
        if (refill && !spread) load_stage(fill, t + 2);

        // ---- S1^T = C q^T, S2^T = C rho^T for the keys 16 w .. 16 w + 15 of the tile ---------
        // (the fragment reads of three k-steps are issued together so that their latencies
        // overlap; two accumulation chains per product)
        f32x4 s1 = {0.f, 0.f, 0.f, 0.f}, s2 = {0.f, 0.f, 0.f, 0.f};
        f32x4 s1b = {0.f, 0.f, 0.f, 0.f}, s2b = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int part = 0; part < 6; ++part) {
            constexpr int HS = kMlaKSteps / 6;
            u32x4 kf[HS], qv[HS], rv[HS];
#pragma unroll
            for (int j = 0; j < HS; ++j) {
                const int ks = part * HS + j;
                kf[j] = ks < kMlaLatBlocks * 4 ? *(const u32x4 *)(tile + k_off[ks & 3] + (ks >> 2) * (kMlaBlkChunks * 16))
                                               : *(const u32x4 *)(tile + k_off_rope[ks - kMlaLatBlocks * 4]);
                qv[j] = qlds[ks * 64 + lane];
                rv[j] = rlds[ks * 64 + lane];
            }
            if (spread) load_piece(fill, fill_base, 2 * part, 2 * part + 2);
#pragma unroll
            for (int j = 0; j < HS; ++j) {
                if ((part * HS + j) & 1) {
                    s1b = mfma16(kf[j], qv[j], s1b);
                    s2b = mfma16(kf[j], rv[j], s2b);
                } else {
                    s1 = mfma16(kf[j], qv[j], s1);
                    s2 = mfma16(kf[j], rv[j], s2);
                }
            }
        }
        s1 += s1b;
        s2 += s2b;

        // ---- tile maximum of every column, agreed on by the four waves ------------------------
        const int key0 = t * kMlaTileKeys + 16 * w + 4 * g;  // this lane's keys: key0 + i
        float x[4];
        float tmax = kNegInf;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[i] = (key0 + i >= key_lo && key0 + i < key_end) ? s1[i] * scale_log2 : kNegInf;
            tmax = fmaxf(tmax, x[i]);
        }
        tmax = rows_max(tmax);
        if (g == 0) smax[w * 16 + c] = tmax;
        __syncthreads();
        const float m_tile = fmaxf(fmaxf(smax[c], smax[16 + c]), fmaxf(smax[32 + c], smax[48 + c]));
        const float m_new = fmaxf(m_run, m_tile);
        const float m_use = m_new == kNegInf ? 0.f : m_new;
        const float alpha = fast_exp2(m_run - m_use);  // 0 on the first live tile
        m_run = m_new;

        // ---- P1, P2 of this wave's keys -> LDS in B-operand order ----------------------------
        // k-step j of the second contraction covers the keys 32 j .. 32 j + 31 of the tile; its
        // k-element e of lane (c, g) is key 32 j + 16 (e / 4) + 4 g + e % 4: the first half comes
        // from wave 2 j, the second from wave 2 j + 1, each from the lane with the same (c, g).
        float p1[4], p2[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            p1[i] = fast_exp2(x[i] - m_use);  // 0 if masked
            p2[i] = x[i] == kNegInf ? 0.f : p1[i] * s2[i];
        }
        dsum1 *= alpha;
        dsum2 *= alpha;
        const u32x2 pk1 = pack4_bf16_accumulate(p1[0], p1[1], p1[2], p1[3], dsum1);
        const u32x2 pk2 = pack4_bf16_accumulate(p2[0], p2[1], p2[2], p2[3], dsum2);
        {
            u32x2 *dst = (u32x2 *)(pbuf + (w >> 1) * 64 + lane) + (w & 1);
            dst[0] = pk1;
            dst[128 * kMlaPvSteps] = pk2;  // P2 follows P1: 64 chunks = 128 half-chunks per k-step
        }
        __syncthreads();

        if (!__all(alpha == 1.f)) {
#pragma unroll
            for (int n = 0; n < kMlaNDB; ++n) {
                o1[n] *= alpha;
                o2[n] *= alpha;
            }
        }

        // ---- O1^T += V^T P1^T, O2^T += V^T P2^T for the dimensions 128 w .. 128 w + 127 --------
        // A operand: row = dimension 16 n + c of the wave's column block, k-elements = the keys of
        // the B operand, fetched with two transposing reads (keys 4g.. and 16 + 4g.. of the k-step).
#pragma unroll
        for (int j = 0; j < kMlaPvSteps; ++j) {
            const u32x4 pb1 = pbuf[j * 64 + lane], pb2 = pbuf[(kMlaPvSteps + j) * 64 + lane];
#pragma unroll
            for (int nh = 0; nh < kMlaNDB; nh += 4) {
                u32x2 vlo[4], vhi[4];
#pragma unroll
                for (int n = 0; n < 4; ++n) {
                    vlo[n] = lds_read_tr16(tile + v_off[nh + n] + j * (32 * 16 * 16));
                    vhi[n] = lds_read_tr16(tile + v_off[nh + n] + j * (32 * 16 * 16) + 16 * 16 * 16);
                }
                if (spread) {
                    const int piece = 2 * j + nh / 4;  // 0..3
                    load_piece(fill, fill_base, 12 + (piece * 6) / 4, 12 + ((piece + 1) * 6) / 4);
                }
#pragma unroll
                for (int n = 0; n < 4; ++n) {
                    const u32x4 vt = {vlo[n][0], vlo[n][1], vhi[n][0], vhi[n][1]};
                    o1[nh + n] = mfma16(vt, pb1, o1[nh + n]);
                    o2[nh + n] = mfma16(vt, pb2, o2[nh + n]);
                }
            }
        }

        // ---- everybody is done with tile t: the next one moves in, the one three ahead sets off
        if (t + 1 < t_hi) {
            __syncthreads();
            store_stage(next, t + 2 < t_hi);
        }
    };

    if (t_lo < t_hi) {
        load_stage(stg_a, t_lo);
        if (t_lo + 1 < t_hi) load_stage(stg_b, t_lo + 1);
        store_stage(stg_a, t_lo + 1 < t_hi);
        if (t_lo + 2 < t_hi) load_stage(stg_a, t_lo + 2);
    }
    for (int t = t_lo; t < t_hi; t += 2) {
        process_tile(t, stg_b, stg_a);
        if (t + 1 < t_hi) process_tile(t + 1, stg_a, stg_b);
    }

    // ---- row sums over the four waves; write the split partial or the output -----------------
    dsum1 = rows_sum(dsum1);
    dsum2 = rows_sum(dsum2);
    if (g == 0) {
        dex[(w * 16 + c) * 2] = dsum1;
        dex[(w * 16 + c) * 2 + 1] = dsum2;
    }
    __syncthreads();
    float d1 = 0.f, d2 = 0.f;
#pragma unroll
    for (int ww = 0; ww < 4; ++ww) {
        d1 += dex[(ww * 16 + c) * 2];
        d2 += dex[(ww * 16 + c) * 2 + 1];
    }
    if (!live) return;
    const int64_t hq = (int64_t)b * n_cols + head;
    if (p.direct_out) {
        float inv = 0.f, gain = 0.f;  // empty key set: zeros
        if (d1 > 0.f) {
            inv = 1.f / d1;
            gain = inv * (1.f + d2 * inv);
        }
        __bf16 *orow = (__bf16 *)p.o + hq * kMlaDC + 128 * w + 4 * g;
#pragma unroll
        for (int n = 0; n < kMlaNDB; ++n) {
            const f32x4 y = o1[n] * gain - o2[n] * inv;
            *(u32x2 *)(orow + 16 * n) = u32x2{pack_bf16(y[0], y[1]), pack_bf16(y[2], y[3])};
        }
    } else {
        float *rec = p.ws + (hq * S + split) * (int64_t)(2 * kMlaDC + 4);
        if (w == 0 && g == 0) *(f32x4 *)rec = f32x4{m_run, d1, d2, 0.f};
        float *r1 = rec + 4 + 128 * w + 4 * g;
#pragma unroll
        for (int n = 0; n < kMlaNDB; ++n) {
            *(f32x4 *)(r1 + 16 * n) = o1[n];
            *(f32x4 *)(r1 + kMlaDC + 16 * n) = o2[n];
        }
    }
}


hipError_t launch_decode_mla(const MlaDecodeParams &p, hipStream_t stream) {
    // more than one group of 16 columns: the step is matrix bound -- the 32-column form
    if (p.Hq * p.Tq > 16) {
        const hipError_t err = launch_decode_mla_wide(p, stream);
        if (err != hipSuccess) return err;
    } else {
        const dim3 grid(p.S, 1, p.B);
        if (p.block_table)
            hipLaunchKernelGGL(decode_mla_kernel<true>, grid, dim3(256), 0, stream, p);
        else
            hipLaunchKernelGGL(decode_mla_kernel<false>, grid, dim3(256), 0, stream, p);
    }
    if (!p.direct_out) {
        DecodeParams c{};
        c.ws = p.ws, c.o = p.o, c.B = p.B, c.Hq = p.Hq * p.Tq, c.Tq = 1, c.S = p.S, c.d = kMlaDC;
        const hipError_t err = launch_decode_combine(c, stream);
        if (err != hipSuccess) return err;
    }
    return hipGetLastError();
}

}  // namespace plx
