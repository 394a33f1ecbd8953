// Causal / full Parallax prefill forward for bf16 on gfx950.
//
// What it computes: Algorithm 1 of the paper (Sec. 3.3) -- for a block of query rows, one pass
// over key tiles with the running state (m, d1, d2, O1, O2); S1 = Q K^T * scale (masked),
// S2 = R K^T (unscaled), P1 = exp2(S1 - m), P2 = P1 * S2, O1 += P1 V, O2 += P2 V; closing
// formula O1/d1 * (1 + d2/d1) - O2/d1. Causal: key j allowed iff j <= i (Sec. 3.1).
//
// Layout for CDNA4:
//   * one workgroup = 4 waves = 128 query rows of one query head (32 rows per wave, one wave
//     per SIMD, so a wave may use the whole 512-register budget: O1^T, O2^T and the Q, R
//     fragments stay in registers for the whole pass);
//   * K/V tiles of 64 keys are fetched coalesced (16 lanes = one 256-byte row), parked in
//     registers while the previous tile is being consumed, and written to a double-buffered,
//     XOR-swizzled LDS tile: one workgroup barrier per tile;
//   * scores are produced transposed with v_mfma_f32_32x32x16_bf16, S^T = K Q^T: each K
//     fragment read from LDS feeds two MFMAs (the q branch and the r branch). In the S^T
//     accumulator a lane owns ONE query row (column) and 16 of the 32 keys, so the softmax
//     statistics are per lane (one exchange with the other half-wave for the max), S1 and S2
//     of a (row, key) pair share lane and register, and the accumulator registers are already
//     the B operand of O^T += V^T P^T;
//   * the running max is updated lazily: the reference m of a row moves only when a tile's
//     maximum exceeds it by more than 2^8, so O1/O2 are rescaled on few tiles. Any reference
//     gives the same result after the final division; P stays <= 2^8 in fp32 / bf16 range.
#include "plx_device.h"
#include "plx_kernels.h"

namespace plx {

constexpr int kBR = 128;        // query rows per workgroup
constexpr int kBC = 64;         // keys per LDS tile
constexpr int kKB = 32;         // keys per inner block (one MFMA row block)
constexpr float kLazyTau = 8.f; // log2 of the largest P tolerated before re-referencing

template <int D, bool USE_R, bool CAUSAL>
__global__ __launch_bounds__(256, 1) void prefill_bf16_kernel(PrefillParams p) {
    constexpr int CPR = D / 8;                  // 16-byte chunks per row
    constexpr int KSTEPS = D / 16;              // k-steps of the score contraction
    constexpr int NDB = D / 32;                 // 32-wide blocks of output dimensions
    constexpr int TILE_CHUNKS = kBC * CPR;
    constexpr int NLD = TILE_CHUNKS / 256;      // staging loads per thread, tile and tensor

    __shared__ u32x4 lds[2 * 2 * TILE_CHUNKS];  // [stage][K|V][tile]

    const int tid = threadIdx.x;
    const int w = tid >> 6, lane = tid & 63;
    const int col = lane & 31;  // MFMA column: query row within the wave's 32 rows
    const int h = lane >> 5;    // half-wave

    // ---- work item: heavy row blocks first; blocks of one (batch, kv head) share an XCD ----
    const int T = p.T, G = p.G;
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
    const int b = pair / p.Hkv, hk = pair - b * p.Hkv;
    const int hq = hk * G + hg;

    const int row0 = rb * kBR + w * 32;          // first query row of this wave
    const int my_row = row0 + col;               // this lane's query row (may be >= T)
    const int ld_qrow = min(my_row, T - 1);

    // ---- Q^T / R^T B operands: column = query row, k-elements = 8 dims of chunk 2*ks + h ----
    u32x4 qf[KSTEPS], rf[KSTEPS];
    {
        const __bf16 *qrow = (const __bf16 *)p.q + b * p.qs[0] + hq * p.qs[1] + ld_qrow * p.qs[2];
        const __bf16 *rrow = (const __bf16 *)p.r + b * p.rs[0] + hq * p.rs[1] + ld_qrow * p.rs[2];
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            qf[ks] = *(const u32x4 *)(qrow + 8 * (2 * ks + h));
            if constexpr (USE_R) rf[ks] = *(const u32x4 *)(rrow + 8 * (2 * ks + h));
        }
    }

    const __bf16 *kbase = (const __bf16 *)p.k + b * p.ks[0] + hk * p.ks[1];
    const __bf16 *vbase = (const __bf16 *)p.v + b * p.vs[0] + hk * p.vs[1];

    const int key_end = CAUSAL ? min(T, (rb + 1) * kBR) : T;  // keys this block may need
    const int n_tiles = (key_end + kBC - 1) / kBC;

    u32x4 kst[NLD], vst[NLD];
    auto issue_loads = [&](int kt) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int idx = i * 256 + tid;
            const int key = min(kt * kBC + idx / CPR, T - 1);  // clamp: finite data, masked below
            const int chunk = idx % CPR;
            kst[i] = *(const u32x4 *)(kbase + (int64_t)key * p.ks[2] + chunk * 8);
            vst[i] = *(const u32x4 *)(vbase + (int64_t)key * p.vs[2] + chunk * 8);
        }
    };
    auto stage_to_lds = [&](int stage) {
        u32x4 *dk = lds + stage * (2 * TILE_CHUNKS);
        u32x4 *dv = dk + TILE_CHUNKS;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int idx = i * 256 + tid;
            const int slot = lds_chunk_slot<D>(idx / CPR, idx % CPR);
            dk[slot] = kst[i];
            dv[slot] = vst[i];
        }
    };

    // ---- running state ---------------------------------------------------------------------
    float m_ref = kNegInf, dsum1 = 0.f, dsum2 = 0.f;
    f32x16 o1[NDB], o2[NDB];
#pragma unroll
    for (int n = 0; n < NDB; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            o1[n][r] = 0.f;
            o2[n][r] = 0.f;
        }
    const float scale_log2 = p.scale * kLog2e;

    issue_loads(0);
    stage_to_lds(0);
    __syncthreads();

    for (int kt = 0; kt < n_tiles; ++kt) {
        const bool more = kt + 1 < n_tiles;
        if (more) issue_loads(kt + 1);

        const u32x4 *tk = lds + (kt & 1) * (2 * TILE_CHUNKS);
        const u32x4 *tv = tk + TILE_CHUNKS;
        const unsigned short *tv16 = (const unsigned short *)tv;

#pragma unroll
        for (int kb = 0; kb < kBC / kKB; ++kb) {
            const int key_base = kt * kBC + kb * kKB;
            // wave-uniform: nothing of this key block is visible to the wave's rows
            if (key_base >= T || (CAUSAL && key_base > row0 + 31)) continue;
            const bool need_mask = (key_base + kKB > T) || (CAUSAL && key_base + kKB - 1 > row0);

            // ---- S1^T, S2^T (32 keys x 32 rows) --------------------------------------------
            f32x16 s1, s2;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                s1[r] = 0.f;
                s2[r] = 0.f;
            }
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                const u32x4 kf = tk[lds_chunk_slot<D>(kb * kKB + col, 2 * ks + h)];
                s1 = mfma32(kf, qf[ks], s1);
                if constexpr (USE_R) s2 = mfma32(kf, rf[ks], s2);
            }

            // ---- online softmax; register r <-> key key_base + 8*(r/4) + 4*h + r%4 ---------
            float tmax = kNegInf;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float x = s1[r] * scale_log2;
                if (need_mask) {
                    const int key = key_base + 8 * (r >> 2) + 4 * h + (r & 3);
                    const bool ok = key < T && (!CAUSAL || key <= my_row);
                    x = ok ? x : kNegInf;
                }
                s1[r] = x;
                tmax = fmaxf(tmax, x);
            }
            tmax = halves_max(tmax);
            if (__any(tmax > m_ref + kLazyTau)) {  // also true on the first block (m_ref = -inf)
                const float m_new = fmaxf(m_ref, tmax);
                const float m_use = m_new == kNegInf ? 0.f : m_new;
                const float alpha = fast_exp2(m_ref - m_use);
                m_ref = m_new;
                dsum1 *= alpha;
                dsum2 *= alpha;
#pragma unroll
                for (int n = 0; n < NDB; ++n)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        o1[n][r] *= alpha;
                        if constexpr (USE_R) o2[n][r] *= alpha;
                    }
            }
            const float m_use = m_ref == kNegInf ? 0.f : m_ref;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                s1[r] = fast_exp2(s1[r] - m_use);  // P1, exactly 0 for masked keys
                // P2: s2 is finite (clamped loads) and P1 = 0 where masked
                if constexpr (USE_R) s2[r] = s1[r] * s2[r];
            }

            // ---- O1^T += V^T P1^T, O2^T += V^T P2^T: two groups of 16 keys -------------------
            // P1, P2 are rounded to bf16 once (MFMA operands) and d1, d2 add the ROUNDED values,
            // so the effective attention weights sum to one exactly.
            const int tr_key = kb * kKB + 4 * h + ((lane & 15) >> 2);  // row this lane addresses
            const int tr_half = (lane & 1) * 4;
            const int tr_chunk = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                // B operand k-element e <-> accumulator register 8j+e <-> key 16j + 8*(e/4) + 4h + e%4
                const u32x4 pb1 = {pack_bf16(s1[8 * j + 0], s1[8 * j + 1]),
                                   pack_bf16(s1[8 * j + 2], s1[8 * j + 3]),
                                   pack_bf16(s1[8 * j + 4], s1[8 * j + 5]),
                                   pack_bf16(s1[8 * j + 6], s1[8 * j + 7])};
                dsum1 += sum_bf16x8(pb1);
                u32x4 pb2 = {0u, 0u, 0u, 0u};
                if constexpr (USE_R) {
                    pb2 = u32x4{pack_bf16(s2[8 * j + 0], s2[8 * j + 1]),
                                pack_bf16(s2[8 * j + 2], s2[8 * j + 3]),
                                pack_bf16(s2[8 * j + 4], s2[8 * j + 5]),
                                pack_bf16(s2[8 * j + 6], s2[8 * j + 7])};
                    dsum2 += sum_bf16x8(pb2);
                }
#pragma unroll
                for (int n = 0; n < NDB; ++n) {
                    // A operand: row = dimension 32n + col, k-elements = the same 8 keys, by two
                    // transposing LDS reads (keys 16j+4h..+3 and 16j+8+4h..+3)
                    const int chunk = 4 * n + tr_chunk;
                    const u32x2 lo = lds_read_tr16(
                        tv16 + lds_chunk_slot<D>(tr_key + 16 * j, chunk) * 8 + tr_half);
                    const u32x2 hi = lds_read_tr16(
                        tv16 + lds_chunk_slot<D>(tr_key + 16 * j + 8, chunk) * 8 + tr_half);
                    const u32x4 vt = {lo[0], lo[1], hi[0], hi[1]};
                    o1[n] = mfma32(vt, pb1, o1[n]);
                    if constexpr (USE_R) o2[n] = mfma32(vt, pb2, o2[n]);
                }
            }
        }

        if (more) stage_to_lds((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue: O^T register r of block n <-> dim 32n + 8*(r/4) + 4h + r%4, row my_row ----
    dsum1 = halves_sum(dsum1);
    dsum2 = halves_sum(dsum2);
    if (my_row < T) {
        const float inv = dsum1 > 0.f ? 1.f / dsum1 : 0.f;
        const float gain = inv * (1.f + dsum2 * inv);
        __bf16 *orow = (__bf16 *)p.o + b * p.os[0] + hq * p.os[1] + my_row * p.os[2];
#pragma unroll
        for (int n = 0; n < NDB; ++n)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                float y[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int r = 4 * q4 + i;
                    y[i] = o1[n][r] * gain - (USE_R ? o2[n][r] * inv : 0.f);
                }
                u32x2 packed = {pack_bf16(y[0], y[1]), pack_bf16(y[2], y[3])};
                *(u32x2 *)(orow + 32 * n + 8 * q4 + 4 * h) = packed;
            }
    }
}

template <int D>
static hipError_t launch_prefill_d(const PrefillParams &p, hipStream_t stream) {
    const int nrb = (p.T + kBR - 1) / kBR;
    const long long total = (long long)nrb * p.Hq * p.B;
    if (total > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)total), block(256);
    if (p.use_r) {
        if (p.causal)
            hipLaunchKernelGGL((prefill_bf16_kernel<D, true, true>), grid, block, 0, stream, p);
        else
            hipLaunchKernelGGL((prefill_bf16_kernel<D, true, false>), grid, block, 0, stream, p);
    } else {
        if (p.causal)
            hipLaunchKernelGGL((prefill_bf16_kernel<D, false, true>), grid, block, 0, stream, p);
        else
            hipLaunchKernelGGL((prefill_bf16_kernel<D, false, false>), grid, block, 0, stream, p);
    }
    return hipGetLastError();
}

hipError_t launch_prefill_bf16(const PrefillParams &p, hipStream_t stream) {
    return p.d == 128 ? launch_prefill_d<128>(p, stream) : launch_prefill_d<64>(p, stream);
}

}  // namespace plx
