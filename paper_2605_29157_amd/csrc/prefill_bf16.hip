// Causal / full Parallax prefill forward for bf16 on gfx950.
//
// What it computes: Algorithm 1 of the paper (Sec. 3.3) -- for a block of query rows, one pass
// over key tiles with the running state (m, d1, d2, O1, O2); S1 = Q K^T * scale (masked),
// S2 = R K^T (unscaled), P1 = exp2(S1 - m), P2 = P1 * S2, O1 += P1 V, O2 += P2 V; closing
// formula O1/d1 * (1 + d2/d1) - O2/d1. Causal: key j allowed iff j <= i (Sec. 3.1).
//
// Layout for CDNA4:
//   * one workgroup = 4 waves = 128 query rows of one query head (32 rows per wave, one wave
//     per SIMD, so a wave may use the whole 512-register budget: O1^T, O2^T live in the
//     accumulation registers and the Q, R fragments in vector registers for the whole pass);
//   * K/V tiles of 64 keys are fetched coalesced (16 lanes = one 256-byte row), parked in
//     registers for one tile time, and written to a three-stage LDS ring whose rows are padded
//     (not swizzled) so that every operand address is a per-lane base plus a constant: one
//     workgroup barrier per tile;
//   * scores are produced transposed with v_mfma_f32_32x32x16_bf16, S^T = K Q^T: each K
//     fragment read from LDS feeds two MFMAs (the q branch and the r branch). In the S^T
//     accumulator a lane owns ONE query row (column) and 16 of the 32 keys, so softmax
//     statistics are per lane, S1 and S2 of a (row, key) pair share lane and register, and the
//     accumulator registers are already the B operand of O^T += V^T P^T (V^T fragments come
//     from transposing LDS reads);
//   * key blocks of 32 are software-pipelined: the score MFMAs of block i+1 are issued before
//     the softmax arithmetic of block i, so matrix cores and vector ALU overlap inside a wave.
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

namespace plx {

constexpr int kBR = 128;  // query rows per workgroup
constexpr int kBC = 64;   // keys per LDS tile
constexpr int kKB = 32;   // keys per inner block (one MFMA row block)

#ifndef PLX_PF_SCHED
#define PLX_PF_SCHED 0
#endif
#if PLX_PF_SCHED == 0
#define PLX_PF_SCHED_HINT() ((void)0)
#else
#define PLX_PF_SCHED_HINT() __builtin_amdgcn_iglp_opt(PLX_PF_SCHED - 1)
#endif

template <int D, bool USE_R, bool CAUSAL>
__global__ __launch_bounds__(256, 1) void prefill_bf16_kernel(PrefillParams p) {
    constexpr int CPR = D / 8;            // 16-byte chunks per row
    constexpr int KSTEPS = D / 16;        // k-steps of the score contraction
    constexpr int NDB = D / 32;           // 32-wide blocks of output dimensions
    constexpr int NLD = kBC * CPR / 256;  // staging loads per thread, tile and tensor
    constexpr int STAGES = 3;
    // K rows are padded by one 16-byte chunk (16 consecutive rows, same chunk -> 16 different
    // bank groups), V rows by four chunks (the 4 consecutive rows of a transposing read land in
    // 4 different 64-byte bank groups).
    constexpr int KROW = CPR + 1, VROW = CPR + 4;  // row strides in chunks
    constexpr int K_CHUNKS = kBC * KROW, V_CHUNKS = kBC * VROW;
    constexpr int STAGE_CHUNKS = K_CHUNKS + V_CHUNKS;

    __shared__ u32x4 lds[STAGES * STAGE_CHUNKS];  // [stage][K tile | V tile]

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

    const int row0 = rb * kBR + w * 32;  // first query row of this wave
    const int my_row = row0 + col;       // this lane's query row (may be >= T)
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

    const int key_end = CAUSAL ? min(T, (rb + 1) * kBR) : T;  // keys this workgroup may need
    const int n_tiles = (key_end + kBC - 1) / kBC;
    // leading tiles whose keys are all < T and visible to every row of the workgroup, less two
    // so that the tile prefetched two ahead inside that loop is always a complete one
    const int n_full = max(0, min(CAUSAL ? 2 * rb : T / kBC, T / kBC - 2));

    const int st_row = tid / CPR, st_chunk = tid % CPR;  // this thread's place in a staging pass
    u32x4 kst[NLD], vst[NLD];
    auto issue_loads = [&](int kt) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            // rows past T re-read row T-1: finite data, masked where it matters
            const int key = min(kt * kBC + i * (256 / CPR) + st_row, T - 1);
            kst[i] = *(const u32x4 *)(kbase + (int64_t)key * p.ks[2] + st_chunk * 8);
            vst[i] = *(const u32x4 *)(vbase + (int64_t)key * p.vs[2] + st_chunk * 8);
        }
    };
    // same for a tile whose 64 rows all exist: uniform 64-bit tile base + 32-bit per-thread
    // offset, so the loop spends no vector ALU on addresses (the host bounds the row strides)
    const uint32_t st_off_k = (uint32_t)(st_row * p.ks[2] + st_chunk * 8) * 2u;
    const uint32_t st_off_v = (uint32_t)(st_row * p.vs[2] + st_chunk * 8) * 2u;
    const uint32_t st_step_k = (uint32_t)((256 / CPR) * p.ks[2]) * 2u;
    const uint32_t st_step_v = (uint32_t)((256 / CPR) * p.vs[2]) * 2u;
    auto issue_loads_full_tile = [&](int kt) {
        const char *tk = (const char *)kbase + (int64_t)kt * (kBC * 2) * p.ks[2];
        const char *tv = (const char *)vbase + (int64_t)kt * (kBC * 2) * p.vs[2];
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            kst[i] = *(const u32x4 *)(tk + (st_off_k + i * st_step_k));
            vst[i] = *(const u32x4 *)(tv + (st_off_v + i * st_step_v));
        }
    };
    auto stage_to_lds = [&](int stage) {
        u32x4 *dk = lds + stage * STAGE_CHUNKS + st_row * KROW + st_chunk;
        u32x4 *dv = lds + stage * STAGE_CHUNKS + K_CHUNKS + st_row * VROW + st_chunk;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            dk[i * (256 / CPR) * KROW] = kst[i];
            dv[i * (256 / CPR) * VROW] = vst[i];
        }
    };

    // S1^T, S2^T (32 keys x 32 rows) of key block kb of the tile in `stage`
    auto scores = [&](int stage, int kb, f32x16 &s1, f32x16 &s2) {
        const u32x4 *tk = lds + stage * STAGE_CHUNKS + col * KROW + h;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            s1[r] = 0.f;
            s2[r] = 0.f;
        }
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const u32x4 kf = tk[kb * kKB * KROW + 2 * ks];
            s1 = mfma32(kf, qf[ks], s1);
            if constexpr (USE_R) s2 = mfma32(kf, rf[ks], s2);
        }
    };

    // accumulator register r of an S^T block <-> key key_base + 8*(r/4) + 4*h + r%4
    auto key_ok = [&](int key_base, int r) {
        const int key = key_base + 8 * (r >> 2) + 4 * h + (r & 3);
        return key < T && (!CAUSAL || key <= my_row);
    };

    float m_ref = kNegInf, dsum1 = 0.f, dsum2 = 0.f;
    f32x16 o1[NDB], o2[NDB];
    const float scale_log2 = p.scale * kLog2e;  // >= 0 (checked by the host)

    // P1 = exp2(S1*scale - m_ref), P2 = P1*S2 for one key block, left as packed bf16 MFMA
    // operands (two groups of 16 keys). d1 / d2 add the ROUNDED values, so the effective
    // attention weights sum to one exactly.
    auto probs = [&](auto masked_tag, int key_base, f32x16 &s1, f32x16 &s2, u32x4(&pb1)[2],
                     u32x4(&pb2)[2]) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        const float neg_m = m_ref == kNegInf ? 0.f : -m_ref;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float p1 = fast_exp2(fmaf(s1[r], scale_log2, neg_m));
            if constexpr (MASKED) p1 = key_ok(key_base, r) ? p1 : 0.f;
            s1[r] = p1;
            // s2 is finite (rows past T re-read row T-1) and P1 = 0 where masked
            if constexpr (USE_R) s2[r] = p1 * s2[r];
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            // B operand k-element e <-> register 8j+e <-> key 16j + 8*(e/4) + 4h + e%4
            pb1[j] = u32x4{pack_bf16(s1[8 * j + 0], s1[8 * j + 1]), pack_bf16(s1[8 * j + 2], s1[8 * j + 3]),
                           pack_bf16(s1[8 * j + 4], s1[8 * j + 5]), pack_bf16(s1[8 * j + 6], s1[8 * j + 7])};
            dsum1 = add_bf16x8(dsum1, pb1[j]);
            if constexpr (USE_R) {
                pb2[j] = u32x4{pack_bf16(s2[8 * j + 0], s2[8 * j + 1]), pack_bf16(s2[8 * j + 2], s2[8 * j + 3]),
                               pack_bf16(s2[8 * j + 4], s2[8 * j + 5]), pack_bf16(s2[8 * j + 6], s2[8 * j + 7])};
                dsum2 = add_bf16x8(dsum2, pb2[j]);
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
    auto accumulate = [&](int stage, int kb, const u32x4(&pb1)[2], const u32x4(&pb2)[2]) {
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
                o1[n] = mfma32(vt, pb1[j], o1[n]);
                if constexpr (USE_R) o2[n] = mfma32(vt, pb2[j], o2[n]);
            }
    };

    auto zero_state = [&]() {
        dsum1 = 0.f;
        dsum2 = 0.f;
#pragma unroll
        for (int n = 0; n < NDB; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                o1[n][r] = 0.f;
                o2[n][r] = 0.f;
            }
    };

    // does this wave see any key of the block starting at key_base / is every key visible?
    auto block_visible = [&](int key_base) {
        return key_base < T && (!CAUSAL || key_base <= row0 + 31);
    };
    auto block_full = [&](int key_base) {
        return key_base + kKB <= T && (!CAUSAL || key_base + kKB - 1 <= row0);
    };

    u32x4 pb1[2], pb2[2];
    pb2[0] = pb2[1] = u32x4{0u, 0u, 0u, 0u};

    // =========================== fast pass: fixed reference ================================
    zero_state();
    issue_loads(0);
    stage_to_lds(0);
    issue_loads(1);  // tiles past the end re-read the last row and are never consumed
    __syncthreads();
    {   // reference = row maximum over the first key block (key 0 is visible to every row)
        f32x16 t1, t2;
        scores(0, 0, t1, t2);
        float tmax = kNegInf;
#pragma unroll
        for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, key_ok(0, r) ? t1[r] : kNegInf);
        m_ref = halves_max(tmax) * scale_log2;
    }

    int stage = 0;
    f32x16 sa1, sa2, sb1, sb2;
    if (n_full > 0) scores(0, 0, sa1, sa2);
    int kt = 0;
    // tiles in which every key is visible to every row: software-pipelined, branch-free body
    for (; kt < n_full; ++kt) {
        const int next_stage = stage == STAGES - 1 ? 0 : stage + 1;
        scores(stage, 1, sb1, sb2);
        probs(std::false_type{}, 0, sa1, sa2, pb1, pb2);
        accumulate(stage, 0, pb1, pb2);
        stage_to_lds(next_stage);  // unconditional: no branch in this loop body
        issue_loads_full_tile(kt + 2);
        PLX_PF_SCHED_HINT();
        __syncthreads();
        scores(next_stage, 0, sa1, sa2);  // unused after the last full tile
        probs(std::false_type{}, 0, sb1, sb2, pb1, pb2);
        accumulate(stage, 1, pb1, pb2);
        PLX_PF_SCHED_HINT();
        stage = next_stage;
    }
    // diagonal / tail tiles: per-wave visibility and masks
    for (; kt < n_tiles; ++kt) {
        const int next_stage = stage == STAGES - 1 ? 0 : stage + 1;
#pragma unroll
        for (int kb = 0; kb < kBC / kKB; ++kb) {
            const int key_base = kt * kBC + kb * kKB;
            if (!block_visible(key_base)) continue;  // wave-uniform
            scores(stage, kb, sa1, sa2);
            if (block_full(key_base))
                probs(std::false_type{}, key_base, sa1, sa2, pb1, pb2);
            else
                probs(std::true_type{}, key_base, sa1, sa2, pb1, pb2);
            accumulate(stage, kb, pb1, pb2);
        }
        stage_to_lds(next_stage);
        issue_loads(kt + 2);
        __syncthreads();
        stage = next_stage;
    }

    // overflow check: any inf/NaN in the sums means the fixed reference was too small
    float chk = dsum1 * 0.f + dsum2 * 0.f;
#pragma unroll
    for (int n = 0; n < NDB; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            chk = fmaf(o1[n][r], 0.f, chk);
            if constexpr (USE_R) chk = fmaf(o2[n][r], 0.f, chk);
        }
    const bool overflow = __syncthreads_or(chk != 0.f);  // NaN != 0 is true; all waves agree

    // =========================== fallback: online max / rescale ============================
    if (overflow) {
        zero_state();
        m_ref = kNegInf;
        issue_loads(0);
        for (int t = 0; t < n_tiles; ++t) {
            stage_to_lds(0);
            if (t + 1 < n_tiles) issue_loads(t + 1);
            __syncthreads();
#pragma unroll 1
            for (int kb = 0; kb < kBC / kKB; ++kb) {
                const int key_base = t * kBC + kb * kKB;
                if (!block_visible(key_base)) continue;
                scores(0, kb, sa1, sa2);
                float tmax = kNegInf;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    tmax = fmaxf(tmax, key_ok(key_base, r) ? sa1[r] * scale_log2 : kNegInf);
                tmax = halves_max(tmax);
                const float m_new = fmaxf(m_ref, tmax);
                const float m_use = m_new == kNegInf ? 0.f : m_new;
                const float alpha = fast_exp2(m_ref - m_use);  // 0 while m_ref = -inf
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
                probs(std::true_type{}, key_base, sa1, sa2, pb1, pb2);
                accumulate(0, kb, pb1, pb2);
            }
            __syncthreads();
        }
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
