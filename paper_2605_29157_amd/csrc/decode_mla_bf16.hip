// Split-KV Parallax decode over an MLA-style latent cache (bf16, gfx950).
//
// What it computes: Algorithm 1 of the paper (Sec. 3.3) for one query row per head, where every
// cached token is ONE row c_j = [latent (512) | rope part (64)] shared by all heads: the key is
// the whole row, the value its latent part (the absorbed-projection decode form of multi-head
// latent attention, which the paper's closing discussion names as structurally compatible).
// q and rho arrive in the latent space ([B, Hq, 576]), the output is [B, Hq, 512].
//
// How it is laid out for CDNA4. With 16 heads per column group the step reads 1152 bytes per token
// for 70 kflop: still HBM bound, but the state of a column group -- O1^T, O2^T of 512 dimensions
// x 16 columns -- is four times that of the d = 128 decode kernel. So the four waves of a
// workgroup share each 64-key tile instead of streaming private ones:
//   * grid (split, group of 16 heads, batch); tiles go global -> LDS directly (no staging
//     registers), double buffered, 72 KB each, one tile ahead; the loads of the next tile are
//     spread over the score MFMAs of the current one;
//   * scores: wave w takes keys 16w .. 16w+15 of the tile, S^T = C [Q;R]^T over all 576
//     dimensions (18 k-steps of v_mfma_f32_16x16x32_bf16 against q and rho fragments that stay in
//     registers);
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
#include "plx_lds_dma.h"

namespace plx {

namespace {

constexpr int kMlaDC = 512, kMlaDR = 64, kMlaDK = kMlaDC + kMlaDR;
constexpr int kMlaKSteps = kMlaDK / 32;      // 18 score k-steps, the last two on the rope part
constexpr int kMlaLatBlocks = kMlaDC / 128;  // column blocks of the latent part
constexpr int kMlaNDB = 128 / 16;            // 16-dimension output blocks per wave

// Rounds four fp32 values to bf16 (one half of an MFMA B operand) and adds the ROUNDED values to
// acc, so that row sums and numerators use identical weights.
__device__ __forceinline__ u32x2 pack4_bf16_accumulate(float p0, float p1, float p2, float p3, float &acc) {
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    bf16x2 a, b;
    a[0] = (__bf16)p0, a[1] = (__bf16)p1;
    b[0] = (__bf16)p2, b[1] = (__bf16)p3;
    acc = __builtin_amdgcn_fdot2_f32_bf16(a, ones, acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(b, ones, acc, false);
    return u32x2{__builtin_bit_cast(uint32_t, a), __builtin_bit_cast(uint32_t, b)};
}

}  // namespace

// Timing instrumentation for kernel analysis (off in the product build): wave 0 of workgroup 0 adds
// up the wall-clock time (10 ns units) between the phase boundaries of its iterations.
#ifdef PLX_MLA_TIMING
__device__ unsigned long long plx_mla_stamps[8];
#define MLA_STAMP(slot)                                  \
    do {                                                 \
        const unsigned long long now_ = wall_clock64();  \
        acc_[slot] += now_ - last_;                      \
        last_ = now_;                                    \
    } while (0)
#else
#define MLA_STAMP(slot) ((void)0)
#endif

// TK keys per tile: 64 (two buffers, all four waves score 16 keys each; the one in use) or 32
// (ring of four buffers, waves 0 and 1 score: more tiles in flight, but the per-tile chain of
// barriers and LDS exchanges is paid twice as often -- measured 25 % slower).
template <int TK>
__global__ __launch_bounds__(256, 1) void decode_mla_kernel(MlaDecodeParams p) {
    constexpr int kMlaTileKeys = TK;
    constexpr int kMlaBufs = 128 / TK;        // tile buffers: what the LDS holds
    constexpr int kMlaScoreWaves = TK / 16;   // waves that compute scores (16 keys each)
    constexpr int kMlaPvSteps = TK / 32;      // k-steps of the second contraction
    constexpr int kMlaBlkChunks = kMlaTileKeys * 16;  // 16-byte chunks of one column block
    constexpr int kMlaRopeChunks = kMlaTileKeys * (kMlaDR / 8);
    constexpr int kMlaBufChunks = kMlaLatBlocks * kMlaBlkChunks + kMlaRopeChunks;
    constexpr int kMlaLoadsPerWave = kMlaBufChunks / 64 / 4;  // wave-wide 1 KB loads per tile and wave
    constexpr int kRowGroups = TK / 4;        // loads per latent column block (4 rows each)
    static_assert(TK == 32 || TK == 64, "tile sizes in use");
    static_assert(kMlaBufChunks % 256 == 0, "four waves fill a tile with whole loads");
    // [ring of tile buffers] [P1 | P2 as B operands: 64 lanes each] [tile maxima] [row sums]
    __shared__ u32x4 lds[kMlaBufs * kMlaBufChunks + 128 * kMlaPvSteps + 4 * kMlaScoreWaves + 8 * kMlaScoreWaves];
    u32x4 *pbuf = lds + kMlaBufs * kMlaBufChunks;  // P1: [k-step][64 lanes], then P2 likewise
    float *smax = (float *)(pbuf + 128 * kMlaPvSteps);  // [scoring waves][16 columns]
    float *dex = smax + 16 * kMlaScoreWaves;            // [scoring waves][16 columns][2]

    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int c = lane & 15;  // MFMA column: head 16 * group + c
    const int g = lane >> 4;  // 16-lane row of the wave
    const int split = blockIdx.x, hgroup = blockIdx.y, b = blockIdx.z;
    const int S = p.S;
    const int head = hgroup * 16 + c;
    const bool live = head < p.Hq;

    int Lb = p.seq_lens ? p.seq_lens[b] : p.Lmax;
    Lb = min(max(Lb, 0), p.Lmax);
    const int n_tiles = (Lb + kMlaTileKeys - 1) / kMlaTileKeys;
    const int tiles_per_split = (n_tiles + S - 1) / S;
    const int t_lo = split * tiles_per_split;
    const int t_hi = min(t_lo + tiles_per_split, n_tiles);
    const int key_hi = min(t_hi * kMlaTileKeys, Lb);

    // ---- B operands: q and rho of the group's heads, zero in the dead columns ---------------
    u32x4 qf[kMlaKSteps], rf[kMlaKSteps];
    {
        const int64_t row = ((int64_t)b * p.Hq + (live ? head : 0)) * kMlaDK;
        const __bf16 *qrow = (const __bf16 *)p.q + row;
        const __bf16 *rrow = (const __bf16 *)p.r + row;
        const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int s = 0; s < kMlaKSteps; ++s) {
            qf[s] = live ? *(const u32x4 *)(qrow + 32 * s + 8 * g) : z;
            rf[s] = live ? *(const u32x4 *)(rrow + 32 * s + 8 * g) : z;
        }
    }

    // ---- global -> LDS tile loads -------------------------------------------------------------
    // Load idx (0..35) of a tile fills the 64 consecutive chunk slots [64 idx, 64 idx + 64): four
    // rows of a latent column block (idx < 32: block idx / 8, rows 4 (idx % 8) ..) or eight rows
    // of the rope block. Every lane fetches the global chunk that belongs at its slot. Rows past
    // the sequence end re-read its last row (finite data, masked below).
    // A tile whose 32 rows all exist is fetched through a wave-uniform tile base plus per-lane
    // byte offsets computed once (no address arithmetic in the loop); the last, partial tile of a
    // sequence takes the clamping form.
    const __bf16 *cbase = (const __bf16 *)p.ckv + (int64_t)b * p.csb;
    const uint32_t lds_base = lds_byte_address(lds);
    int ld_row[kMlaLoadsPerWave], ld_elem[kMlaLoadsPerWave];
    uint32_t ld_off[kMlaLoadsPerWave];
#pragma unroll
    for (int i = 0; i < kMlaLoadsPerWave; ++i) {
        const int idx = w * kMlaLoadsPerWave + i;  // wave-uniform
        if (idx < kMlaLatBlocks * kRowGroups) {
            ld_row[i] = 4 * (idx % kRowGroups) + (lane >> 4);
            ld_elem[i] = (idx / kRowGroups) * 128 + (((lane & 15) ^ lds_row_swizzle<128>(ld_row[i])) * 8);
        } else {
            ld_row[i] = 8 * (idx - kMlaLatBlocks * kRowGroups) + (lane >> 3);
            ld_elem[i] = kMlaDC + (((lane & 7) ^ lds_row_swizzle<64>(ld_row[i])) * 8);
        }
        ld_off[i] = (uint32_t)(ld_row[i] * (int)p.csl + ld_elem[i]) * 2u;
    }
    const int64_t tile_bytes = (int64_t)kMlaTileKeys * 2 * p.csl;
    auto issue_tile = [&](int t, int buf) __attribute__((always_inline)) {
        const int tk0 = t * kMlaTileKeys;
        const uint32_t dst = lds_base + (uint32_t)(buf * kMlaBufChunks + w * kMlaLoadsPerWave * 64) * 16u;
        if (tk0 + kMlaTileKeys <= Lb) {  // workgroup-uniform
            const char *tile_base = (const char *)cbase + t * tile_bytes;
#pragma unroll
            for (int i = 0; i < kMlaLoadsPerWave; ++i) tile_load16_uniform<false>(ld_off[i], tile_base, dst + 1024u * i);
        } else {
#pragma unroll
            for (int i = 0; i < kMlaLoadsPerWave; ++i) {
                const int key = min(tk0 + ld_row[i], Lb - 1);
                tile_load16<64>(cbase + (int64_t)key * p.csl + ld_elem[i], dst + 1024u * i);
            }
        }
    };
    // The loads of a COMPLETE next tile are spread over the score MFMAs of the current one (a
    // wave-wide load occupies the wave for as long as the texture path needs for its kilobyte;
    // issued as a block, a tile's loads cost a third of an iteration): these name that tile.
    const char *dma_base = nullptr;
    uint32_t dma_dst = 0;
    // per-lane LDS byte offsets inside a tile buffer of the two read patterns (set up once):
    // K operand of score k-step s: chunk 4 (s % 4) + g of row 16 w + c in column block s / 4
    // (+ 8 KB per block as an immediate), the two rope k-steps in the rope block; V^T operand of
    // dimension block n: rows 4 g + c / 4 (and + 16: + 4 KB, the swizzle does not see bit 4)
    const int krow = 16 * (w % kMlaScoreWaves) + c;
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
    // (rows r, r + 16, r + 32, r + 48 of a tile share the chunk permutation: it reads bits 0..3)

    // ---- running state: column c; O^T rows = dimensions 128 w + 16 n + 4 g + i ---------------
    float m_run = kNegInf, dsum1 = 0.f, dsum2 = 0.f;  // sums: partial over this lane's keys
    f32x4 o1[kMlaNDB], o2[kMlaNDB];
#pragma unroll
    for (int n = 0; n < kMlaNDB; ++n) {
        o1[n] = f32x4{0.f, 0.f, 0.f, 0.f};
        o2[n] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const float scale_log2 = p.scale * kLog2e;

#pragma unroll
    for (int i = 0; i < kMlaBufs - 1; ++i)
        if (t_lo + i < t_hi) issue_tile(t_lo + i, i);
    const bool scorer = w < kMlaScoreWaves;  // wave-uniform
#ifdef PLX_MLA_TIMING
    unsigned long long acc_[8] = {0, 0, 0, 0, 0, 0, 0, 0}, last_ = wall_clock64();
#endif
    int buf = 0;
    for (int t = t_lo; t < t_hi; ++t, buf = (buf + 1) & (kMlaBufs - 1)) {
        // Tile t has landed (loads complete in issue order; up to kMlaBufs - 2 younger tiles stay
        // in flight) and is visible; every wave is past its reads of tile t - 1, whose buffer
        // then receives tile t + kMlaBufs - 1.
        const int younger = t_hi - 1 - t;  // workgroup-uniform
        if (kMlaBufs >= 4 && younger >= 2)
            tile_barrier<(kMlaBufs >= 4 ? 2 : 0) * kMlaLoadsPerWave>();
        else if (kMlaBufs >= 3 && younger == 1)
            tile_barrier<(kMlaBufs >= 3 ? 1 : 0) * kMlaLoadsPerWave>();
        else
            tile_barrier<0>();
        MLA_STAMP(0);  // wait for the tile + barrier
        bool spread = false;  // workgroup-uniform
        if (t + kMlaBufs - 1 < t_hi) {
            const int tn = t + kMlaBufs - 1, bn = (buf + kMlaBufs - 1) & (kMlaBufs - 1);
            spread = kMlaScoreWaves == 4 && (tn + 1) * kMlaTileKeys <= Lb;
            if (spread) {
                dma_base = (const char *)cbase + tn * tile_bytes;
                dma_dst = lds_base + (uint32_t)(bn * kMlaBufChunks + w * kMlaLoadsPerWave * 64) * 16u;
            } else {
                issue_tile(tn, bn);
            }
        }
        const char *tile = (const char *)(lds + buf * kMlaBufChunks);

        // ---- S1^T = C q^T, S2^T = C rho^T for the keys 16 w .. 16 w + 15 of the tile ---------
        // (all fragment reads of a half first, so that their latencies overlap; two accumulation
        // chains per product, so that an MFMA does not wait for the one before it)
        f32x4 s1 = {0.f, 0.f, 0.f, 0.f}, s2 = {0.f, 0.f, 0.f, 0.f};
        if (scorer) {
            f32x4 s1b = {0.f, 0.f, 0.f, 0.f}, s2b = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                constexpr int HS = kMlaKSteps / 2;
                u32x4 kf[HS];
#pragma unroll
                for (int j = 0; j < HS; ++j) {
                    const int ks = half * HS + j;
                    kf[j] = ks < kMlaLatBlocks * 4
                                ? *(const u32x4 *)(tile + k_off[ks & 3] + (ks >> 2) * (kMlaBlkChunks * 16))
                                : *(const u32x4 *)(tile + k_off_rope[ks - kMlaLatBlocks * 4]);
                }
                if (spread) {
#pragma unroll
                    for (int j = 0; j < HS; ++j) {
                        const int ks = half * HS + j;
                        if (ks < kMlaLoadsPerWave) tile_load16_uniform<false>(ld_off[ks], dma_base, dma_dst + 1024u * ks);
                        if (j & 1) {
                            s1b = mfma16(kf[j], qf[ks], s1b);
                            s2b = mfma16(kf[j], rf[ks], s2b);
                        } else {
                            s1 = mfma16(kf[j], qf[ks], s1);
                            s2 = mfma16(kf[j], rf[ks], s2);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < HS; ++j) {
                        const int ks = half * HS + j;
                        if (j & 1) {
                            s1b = mfma16(kf[j], qf[ks], s1b);
                            s2b = mfma16(kf[j], rf[ks], s2b);
                        } else {
                            s1 = mfma16(kf[j], qf[ks], s1);
                            s2 = mfma16(kf[j], rf[ks], s2);
                        }
                    }
                }
            }
            s1 += s1b;
            s2 += s2b;
        }

        MLA_STAMP(1);  // (block issue of the loads) + scores
        // ---- tile maximum of every column, agreed on by the four waves ------------------------
        const int key0 = t * kMlaTileKeys + 16 * w + 4 * g;  // this lane's keys: key0 + i
        float x[4];
        float tmax = kNegInf;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[i] = scorer && key0 + i < key_hi ? s1[i] * scale_log2 : kNegInf;
            tmax = fmaxf(tmax, x[i]);
        }
        tmax = rows_max(tmax);
        if (scorer && g == 0) smax[w * 16 + c] = tmax;
        MLA_STAMP(2);  // mask, wave maximum
        __syncthreads();
        MLA_STAMP(3);  // barrier
        float m_tile = smax[c];
#pragma unroll
        for (int ww = 1; ww < kMlaScoreWaves; ++ww) m_tile = fmaxf(m_tile, smax[16 * ww + c]);
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
        if (scorer) {
            u32x2 *dst = (u32x2 *)(pbuf + (w >> 1) * 64 + lane) + (w & 1);
            dst[0] = pk1;
            dst[128 * kMlaPvSteps] = pk2;  // P2 follows P1: 64 chunks = 128 half-chunks per k-step
        }
        MLA_STAMP(4);  // softmax, P
        __syncthreads();
        MLA_STAMP(5);  // barrier

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
            u32x2 vlo[kMlaNDB], vhi[kMlaNDB];
#pragma unroll
            for (int n = 0; n < kMlaNDB; ++n) {
                vlo[n] = lds_read_tr16(tile + v_off[n] + j * (32 * 16 * 16));
                vhi[n] = lds_read_tr16(tile + v_off[n] + j * (32 * 16 * 16) + 16 * 16 * 16);
            }
#pragma unroll
            for (int n = 0; n < kMlaNDB; ++n) {
                const u32x4 vt = {vlo[n][0], vlo[n][1], vhi[n][0], vhi[n][1]};
                o1[n] = mfma16(vt, pb1, o1[n]);
                o2[n] = mfma16(vt, pb2, o2[n]);
            }
        }
        MLA_STAMP(6);  // rescale + second contraction
    }
#ifdef PLX_MLA_TIMING
    if (tid == 0 && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0)
        for (int i = 0; i < 8; ++i) plx_mla_stamps[i] = acc_[i];
#endif

    // ---- row sums over the four waves; write the split partial or the output -----------------
    dsum1 = rows_sum(dsum1);
    dsum2 = rows_sum(dsum2);
    if (scorer && g == 0) {
        dex[(w * 16 + c) * 2] = dsum1;
        dex[(w * 16 + c) * 2 + 1] = dsum2;
    }
    __syncthreads();
    float d1 = 0.f, d2 = 0.f;
#pragma unroll
    for (int ww = 0; ww < kMlaScoreWaves; ++ww) {
        d1 += dex[(ww * 16 + c) * 2];
        d2 += dex[(ww * 16 + c) * 2 + 1];
    }
    if (!live) return;
    const int64_t hq = (int64_t)b * p.Hq + head;
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

#ifdef PLX_MLA_TIMING
extern "C" int parallax_debug_read_mla_stamps(void *host_dst, size_t bytes) {
    return (int)hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(plx_mla_stamps), bytes, 0, hipMemcpyDeviceToHost);
}
#endif

hipError_t launch_decode_mla(const MlaDecodeParams &p, hipStream_t stream) {
    const dim3 grid(p.S, (p.Hq + 15) / 16, p.B);
    hipLaunchKernelGGL(decode_mla_kernel<64>, grid, dim3(256), 0, stream, p);
    if (!p.direct_out) {
        DecodeParams c{};
        c.ws = p.ws, c.o = p.o, c.B = p.B, c.Hq = p.Hq, c.Tq = 1, c.S = p.S, c.d = kMlaDC;
        const hipError_t err = launch_decode_combine(c, stream);
        if (err != hipSuccess) return err;
    }
    return hipGetLastError();
}

}  // namespace plx
