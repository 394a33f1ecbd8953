// Split-KV Parallax decode for bf16 K/V caches on gfx950, plus the combine kernel.
//
// What it computes: Algorithm 1 of the paper (Sec. 3.3) for one query row per head -- running
// state (m, d1, d2, O1, O2) over key tiles, S2 = R K^T unscaled, P2 = P1 * S2 -- with the key
// range of each sequence cut into S splits whose unnormalised partials are merged by a
// log-sum-exp rescale and finished with O1/d1 * (1 + d2/d1) - O2/d1 (App. C).
//
// How it is laid out for CDNA4 (not the paper's Hopper prototype):
//   * grid (split, kv head, batch), 4 waves per workgroup. Every wave streams its own 32-key
//     tiles (wave w takes tiles w, w+4, ... of the split) with private running state, so the
//     main loop has no workgroup barrier; the four states are merged through LDS at the end.
//   * K and V rows are fetched with 16-byte-per-lane loads in which 16 consecutive lanes cover
//     one 256-byte row (fully coalesced), parked in registers one tile ahead, then written to
//     a per-wave LDS tile with an XOR chunk swizzle and re-read in MFMA operand order.
//   * scores are produced transposed, S^T = K [Q;R]^T, with v_mfma_f32_16x16x32_bf16: the K
//     fragment is the A operand and is used twice (once against the q columns, once against
//     the r columns), the G query heads of the GQA group are the live columns. The accumulator
//     layout of S^T (lane = column, 4 consecutive keys per lane) is already the B-operand
//     layout of the second contraction O^T = V^T P^T, so P1 and P2 = P1*S2 never leave their
//     lane; only the running max needs a cross-lane exchange.
//   * all state is fp32; P1 and P2 are rounded to bf16 only as MFMA operands.
#include "plx_device.h"
#include "plx_kernels.h"

namespace plx {

constexpr int kTileKeys = 32;  // keys per wave tile
constexpr int kWaves = 4;      // waves per workgroup
static_assert(kTileKeys * kWaves == kDecodeBlockKeys, "block tile = waves x wave tile");

// Merge the S split partials of one (batch, query head, query row): m* = max_s m_s, weights
// exp2(m_s - m*), then the closing formula of Algorithm 1 (App. C). 256 threads laid out as
// [split lane][dimension lane x float4]: every thread folds the records s = split lane,
// split lane + SL, ... into a private state with all loads of a trip issued together, then the SL
// private states are merged through shared memory (MergeScratch). Deterministic: no float
// atomics, a fixed order.
struct MergeState {
    float m, d1, d2;
    f32x4 a1, a2;
};

__device__ __forceinline__ void merge_into(MergeState &st, float ms, float d1, float d2, f32x4 a1,
                                           f32x4 a2) {
    const float m_new = fmaxf(st.m, ms);
    const float m_use = m_new == kNegInf ? 0.f : m_new;
    const float w_old = fast_exp2(st.m - m_use);  // exp2(-inf) = 0 for an empty side
    const float w_new = fast_exp2(ms - m_use);
    st.m = m_new;
    st.d1 = w_old * st.d1 + w_new * d1;
    st.d2 = w_old * st.d2 + w_new * d2;
    st.a1 = w_old * st.a1 + w_new * a1;
    st.a2 = w_old * st.a2 + w_new * a2;
}

__device__ __forceinline__ void record_store(float *p, float x) {
    __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int D>
struct MergeScratch {
    static constexpr int DL = D / 4;     // lanes over the head dimension (float4 each)
    static constexpr int SL = 256 / DL;  // lanes over splits
    float hdr[SL][4];
    f32x4 a1[SL][DL], a2[SL][DL];
};

// Four floats of a record. COHERENT: as device-scope atomic loads, which are served from the
// point where the eight XCDs' private L2 caches agree -- for records that other workgroups of
// the SAME launch wrote with record_store's device-scope stores.
template <bool COHERENT>
__device__ __forceinline__ f32x4 record_load4(const float *p) {
    if constexpr (COHERENT) {
        union { unsigned long long u[2]; f32x4 f; } x;
        x.u[0] = __hip_atomic_load((const unsigned long long *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        x.u[1] = __hip_atomic_load((const unsigned long long *)p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return x.f;
    } else {
        return *(const f32x4 *)p;
    }
}

// Merges NROW output rows at once (their loads are all in flight together). rec0[i]: the S
// records of row i; out_row[i]: its D bf16 outputs. All 256 threads take part (one
// __syncthreads inside); sm holds NROW scratch areas.
template <int D, bool COHERENT, int NROW>
__device__ __forceinline__ void merge_records(const float *const (&rec0)[NROW], int S,
                                              __bf16 *const (&out_row)[NROW], int tid,
                                              MergeScratch<D> *sm) {
    constexpr int DL = MergeScratch<D>::DL, SL = MergeScratch<D>::SL;
    constexpr int REC = 2 * D + 4;
    // records per thread and trip: with D = 128 a trip covers 64 records (32 per row for two
    // rows), so that up to 64 splits are merged with every load in flight at once
    constexpr int U = NROW == 1 ? 8 : 4;
    const int sl = tid / DL, dl = tid % DL;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};

    MergeState st[NROW];
#pragma unroll
    for (int i = 0; i < NROW; ++i) st[i] = MergeState{kNegInf, 0.f, 0.f, zero, zero};
    for (int base = 0; base < S; base += U * SL) {
        f32x4 hdr[NROW][U], a1[NROW][U], a2[NROW][U];
#pragma unroll
        for (int i = 0; i < NROW; ++i)
#pragma unroll
            for (int u = 0; u < U; ++u) {  // issue every load of the trip before using any
                const int s = base + u * SL + sl;
                const bool ok = s < S;
                const float *rec = rec0[i] + (int64_t)(ok ? s : 0) * REC;
                hdr[i][u] = ok ? record_load4<COHERENT>(rec) : f32x4{kNegInf, 0.f, 0.f, 0.f};
                a1[i][u] = ok ? record_load4<COHERENT>(rec + 4 + 4 * dl) : zero;
                a2[i][u] = ok ? record_load4<COHERENT>(rec + 4 + D + 4 * dl) : zero;
            }
#pragma unroll
        for (int i = 0; i < NROW; ++i)
#pragma unroll
            for (int u = 0; u < U; ++u)
                merge_into(st[i], hdr[i][u][0], hdr[i][u][1], hdr[i][u][2], a1[i][u], a2[i][u]);
    }
#pragma unroll
    for (int i = 0; i < NROW; ++i) {
        if (dl == 0) {
            sm[i].hdr[sl][0] = st[i].m;
            sm[i].hdr[sl][1] = st[i].d1;
            sm[i].hdr[sl][2] = st[i].d2;
        }
        sm[i].a1[sl][dl] = st[i].a1;
        sm[i].a2[sl][dl] = st[i].a2;
    }
    __syncthreads();
    if (sl < NROW) {  // split lane i finishes row i
        const MergeScratch<D> &my = sm[sl];
        MergeState tot{kNegInf, 0.f, 0.f, zero, zero};
#pragma unroll
        for (int j = 0; j < SL; ++j)
            merge_into(tot, my.hdr[j][0], my.hdr[j][1], my.hdr[j][2], my.a1[j][dl], my.a2[j][dl]);
        f32x4 out = zero;  // empty key set: zeros
        if (tot.d1 > 0.f) {
            const float inv = 1.f / tot.d1;
            out = tot.a1 * (inv * (1.f + tot.d2 * inv)) - tot.a2 * inv;
        }
        const u32x2 packed = {pack_bf16(out[0], out[1]), pack_bf16(out[2], out[3])};
        __bf16 *dst = out_row[0];
#pragma unroll
        for (int i = 1; i < NROW; ++i) dst = sl == i ? out_row[i] : dst;
        *(u32x2 *)(dst + 4 * dl) = packed;
    }
}

// RANGE: the launch covers the query rows [row0, row0 + rows) of Tq only (calls with more than 16
// columns); its own instantiation, so that the one-launch kernel stays as it is.
// PREP: RMSNorm + RoPE on the q / rho rows after they are loaded (own instantiations as well).
template <int D, bool USE_R, bool PAGED, bool RANGE = false, bool PREP = false>
__global__ __launch_bounds__(256, 2) void decode_bf16_kernel(DecodeParams p) {
    constexpr int CPR = D / 8;            // 16-byte chunks per K/V row
    constexpr int KPI = 64 / CPR;         // rows covered by one wave-wide 16-byte load
    constexpr int NLD = kTileKeys / KPI;  // loads per lane per tile and tensor
    constexpr int KSTEPS = D / 32;        // MFMA k-steps over the head dimension
    constexpr int NDB = D / 16;           // 16-wide blocks of output dimensions
    constexpr int TILE_CHUNKS = kTileKeys * CPR;

    // K/V tiles of the four waves; reused at the end for the merge of their states, which for 16
    // live columns needs 768 bytes more than the tiles
    __shared__ u32x4 lds[kWaves * 2 * TILE_CHUNKS + 48];

    const int tid = threadIdx.x;
    const int w = tid >> 6, lane = tid & 63;
    const int c = lane & 15;   // MFMA column: (query row t, head of the GQA group), live if c < GC
    const int g = lane >> 4;   // 16-lane row of the wave
    const int split = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
    const int G = p.G, S = p.S;
    // With Tq query rows per sequence (the last Tq positions: speculative rows, a short chunk)
    // column c = t * G + head: all rows of all heads of the group share every K/V fetch.
    // A launch may cover only the rows [row0, row0 + Tq) of Tq_all (more than 16 columns take
    // several launches): the rows behind them shorten what this launch sees of the sequence.
    const int Tq_all = p.Tq, row0 = RANGE ? p.row0 : 0;
    const int Tq = RANGE ? p.rows : Tq_all, GC = G * Tq;
    const int col_t = c / G, col_h = c - col_t * G;

    int Lb = p.seq_lens ? p.seq_lens[b] : p.Lmax;
    Lb = min(max(Lb, 0), p.Lmax);
    if constexpr (RANGE) Lb = max(Lb - (Tq_all - row0 - Tq), 0);
    const int n_bt = (Lb + kDecodeBlockKeys - 1) / kDecodeBlockKeys;
    // sliding window: a row at position pos sees the keys pos - window + 1 .. pos, so the block
    // tiles before the first key of the earliest row (position Lb - Tq) are never read and the
    // splits divide what is left
    const int bt_first = p.window > 0 ? max(Lb - Tq + 1 - p.window, 0) / kDecodeBlockKeys : 0;
    const int bt_per_split = (n_bt - bt_first + S - 1) / S;
    const int key_lo = (bt_first + split * bt_per_split) * kDecodeBlockKeys;
    const int key_hi = min(key_lo + bt_per_split * kDecodeBlockKeys, Lb);

    // ---- B operands: q and r rows of the group's heads, zero in the dead columns ----------
    const bool live = c < GC;
    u32x4 qf[KSTEPS], rf[KSTEPS];
    {
        const int64_t row =
            (((int64_t)b * p.Hq + (int64_t)hk * G + (live ? col_h : 0)) * Tq_all + row0 + (live ? col_t : 0)) * D;
        const __bf16 *qrow = (const __bf16 *)p.q + row;
        const __bf16 *rrow = (const __bf16 *)p.r + row;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            const u32x4 z = {0u, 0u, 0u, 0u};
            qf[s] = live ? *(const u32x4 *)(qrow + 8 * (4 * s + g)) : z;
            if constexpr (USE_R) rf[s] = live ? *(const u32x4 *)(rrow + 8 * (4 * s + g)) : z;
        }
    }

    // paged cache: the batch stride is the page stride and is applied per row below
    const __bf16 *kbase = (const __bf16 *)p.k + (PAGED ? 0 : (int64_t)b * p.ksb) + (int64_t)hk * p.ksh;
    const __bf16 *vbase = (const __bf16 *)p.v + (PAGED ? 0 : (int64_t)b * p.vsb) + (int64_t)hk * p.vsh;
    u32x4 *ldsK = lds + w * (2 * TILE_CHUNKS);
    u32x4 *ldsV = ldsK + TILE_CHUNKS;
    const unsigned short *ldsV16 = (const unsigned short *)ldsV;

    const int ld_row = lane / CPR, ld_chunk = lane % CPR;  // this lane's place in a load
    u32x4 kst[NLD], vst[NLD];
    // paged cache: page numbers of this lane's rows, looked up one tile before the rows
    // themselves are fetched so that the table read is off the critical path
    int32_t pg[NLD];
    const int32_t *table = PAGED ? p.block_table + (int64_t)b * p.table_stride : nullptr;
    auto lookup_pages = [&](int tk0) {
        if constexpr (PAGED) {
#pragma unroll
            for (int i = 0; i < NLD; ++i) pg[i] = table[min(tk0 + i * KPI + ld_row, Lb - 1) / p.page_size];
        }
    };
    auto issue_loads = [&](int tk0) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            // rows past the sequence end re-read its last row (finite data, masked below)
            const int key = min(tk0 + i * KPI + ld_row, Lb - 1);
            int64_t koff = (int64_t)key * p.ksl, voff = (int64_t)key * p.vsl;
            if constexpr (PAGED) {
                const int64_t page = min(max(pg[i], 0), p.num_pages - 1);
                const int row = key % p.page_size;
                koff = page * p.ksb + (int64_t)row * p.ksl;
                voff = page * p.vsb + (int64_t)row * p.vsl;
            }
            kst[i] = *(const u32x4 *)(kbase + koff + ld_chunk * 8);
            vst[i] = *(const u32x4 *)(vbase + voff + ld_chunk * 8);
        }
    };

    if constexpr (PREP && PAGED) {  // (the first tile's page numbers travel with the weights)
        const int tk_first = key_lo + w * kTileKeys;
        if (tk_first < key_hi) lookup_pages(tk_first);
    }
    // ---- RMSNorm + RoPE on the q / rho rows in their operand registers (the operations the
    // paper's language-model runs apply in front of the attention call; formulas of
    // norm_rope.hip, rotation from the (cos, sin) table). The weights and table entries are
    // requested and used HERE, in front of the first tile's loads, when the memory system is
    // still idle: behind them they queue up behind the tile traffic of the whole chip (measured:
    // +19 us on a 30 us step), and with a tile parked in registers the arithmetic does not fit
    // the register file (spills, whose reloads queue up the same way).
    f32x4 prep_gq[KSTEPS][2], prep_gr[KSTEPS][2], prep_tab[KSTEPS][2];
    if constexpr (PREP) {
        const QrPrep &pr = p.prep;
        int Lfull = p.seq_lens ? p.seq_lens[b] : p.Lmax;
        Lfull = min(max(Lfull, 0), p.Lmax);
        const int t = row0 + (live ? col_t : 0);
        const int64_t pos = min(max(pr.pos0 ? pr.pos0[b] + t : Lfull - Tq_all + t, 0), max(pr.n_pos - 1, 0));
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            const int dim = 8 * (4 * s + g);
            prep_gq[s][0] = *(const f32x4 *)(pr.gamma_q + dim), prep_gq[s][1] = *(const f32x4 *)(pr.gamma_q + dim + 4);
            if constexpr (USE_R)
                prep_gr[s][0] = *(const f32x4 *)(pr.gamma_r + dim), prep_gr[s][1] = *(const f32x4 *)(pr.gamma_r + dim + 4);
            if (pr.table != nullptr) {  // (uniform)
                const float *e = pr.table + (pos * (D / 2) + dim / 2) * 2;
                prep_tab[s][0] = *(const f32x4 *)e, prep_tab[s][1] = *(const f32x4 *)(e + 4);
            }
        }
    }

    // Lane (c, g) holds dims 8 (4 s + g) .. + 7 of column c's row for every k-step s, so the row's
    // sum of squares is this lane's plus those of the three lanes c + 16, 32, 48.
    if constexpr (PREP) {
        const QrPrep &pr = p.prep;
        auto prepare = [&](u32x4(&f)[KSTEPS], const f32x4(&gam)[KSTEPS][2], bool rot) {
            float ss = 0.f;
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float lo = bf16_lo_f32(f[s][e]), hi = bf16_hi_f32(f[s][e]);
                    ss = fmaf(lo, lo, ss);
                    ss = fmaf(hi, hi, ss);
                }
            ss = rows_sum(ss);
            const float rinv = 1.0f / sqrtf(ss * (1.0f / (float)D) + pr.eps);
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
                const f32x4 g0 = gam[s][0], g1 = gam[s][1];
                const f32x4 ident = {1.f, 0.f, 1.f, 0.f};
                const f32x4 t0 = rot ? prep_tab[s][0] : ident, t1 = rot ? prep_tab[s][1] : ident;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float gm0 = j < 2 ? g0[2 * j] : g1[2 * j - 4], gm1 = j < 2 ? g0[2 * j + 1] : g1[2 * j - 3];
                    const float y0 = bf16_lo_f32(f[s][j]) * rinv * gm0, y1 = bf16_hi_f32(f[s][j]) * rinv * gm1;
                    const float cs = j < 2 ? t0[2 * j] : t1[2 * j - 4], sn = j < 2 ? t0[2 * j + 1] : t1[2 * j - 3];
                    f[s][j] = live ? pack_bf16(y0 * cs - y1 * sn, y0 * sn + y1 * cs) : 0u;
                }
            }
        };
        prepare(qf, prep_gq, pr.rope_q != 0);
        if constexpr (USE_R) prepare(rf, prep_gr, pr.rope_r != 0);
    }

    // ---- running state (per lane: column c, partial over this lane's keys) ----------------
    float m_run = kNegInf, dsum1 = 0.f, dsum2 = 0.f;
    f32x4 o1[NDB], o2[NDB];
#pragma unroll
    for (int n = 0; n < NDB; ++n) {
        o1[n] = f32x4{0.f, 0.f, 0.f, 0.f};
        o2[n] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const float scale_log2 = p.scale * kLog2e;
    // last-positions alignment: row t of Tq sees the keys before position Lb - (Tq - 1 - t)
    // ... and, with a sliding window, not before position (its own) - window + 1. Both bounds in
    // one unsigned compare: key - col_lo < col_span, with key = tk + 16*sub + i + 4*g.
    const int col_end = Lb - (Tq - 1 - (live ? col_t : Tq - 1));
    const int col_lo = p.window > 0 ? max(col_end - p.window, 0) : 0;
    const int lane_rel = 4 * g - col_lo;
    const unsigned col_span = (unsigned)max(min(key_hi, col_end) - col_lo, 0);

    int tk = key_lo + w * kTileKeys;
    if constexpr (PREP) {
        // The first tile's loads must not be issued before the preparation above is through (the
        // compiler would hoist them: then the block's registers do not fit beside the parked
        // tile, and the reloads of what it spills wait in line behind the tile loads). An empty
        // statement makes the first key depend on the prepared operands.
        asm volatile("" : "+v"(tk) : "v"(qf[KSTEPS - 1][3]), "v"(rf[KSTEPS - 1][3]));
    }
    if (tk < key_hi) {
        if constexpr (!(PREP && PAGED)) lookup_pages(tk);
        issue_loads(tk);
        if (tk + kWaves * kTileKeys < key_hi) lookup_pages(tk + kWaves * kTileKeys);
    }
    for (; tk < key_hi; tk += kWaves * kTileKeys) {
        // registers -> swizzled LDS tile (private to this wave)
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int slot = lds_chunk_slot<D>(i * KPI + ld_row, ld_chunk);
            ldsK[slot] = kst[i];
            ldsV[slot] = vst[i];
        }
        const int tk_next = tk + kWaves * kTileKeys;
        if (tk_next < key_hi) {
            issue_loads(tk_next);
            if (tk_next + kWaves * kTileKeys < key_hi) lookup_pages(tk_next + kWaves * kTileKeys);
        }
        // lanes exchange data through LDS inside one wave: LDS executes a wave's accesses in
        // order, the fence only stops the compiler from moving reads above the writes
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---- S1^T = K q^T, S2^T = K r^T : 2 sub-tiles of 16 keys ---------------------------
        f32x4 s1[2], s2[2];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            s1[sub] = f32x4{0.f, 0.f, 0.f, 0.f};
            s2[sub] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < KSTEPS; ++s) {
                const u32x4 kf = ldsK[lds_chunk_slot<D>(16 * sub + c, 4 * s + g)];
                s1[sub] = mfma16(kf, qf[s], s1[sub]);
                if constexpr (USE_R) s2[sub] = mfma16(kf, rf[s], s2[sub]);
            }
        }

        // ---- online softmax on this lane's 8 keys (key = tk + 16*sub + 4*g + i) ------------
        float x[2][4];
        float tmax = kNegInf;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool seen = (unsigned)(tk + 16 * sub + i + lane_rel) < col_span;
                x[sub][i] = seen ? s1[sub][i] * scale_log2 : kNegInf;
                tmax = fmaxf(tmax, x[sub][i]);
            }
        tmax = rows_max(tmax);
        const float m_new = fmaxf(m_run, tmax);
        const float m_use = m_new == kNegInf ? 0.f : m_new;
        const float alpha = fast_exp2(m_run - m_use);  // 0 on the first live tile
        m_run = m_new;
        // P1, P2 are rounded to bf16 once (they are MFMA operands) and the row sums d1, d2 add
        // the ROUNDED values: numerators and denominators then use identical weights, so the
        // effective attention weights still sum to one exactly.
        // B operand k-element e of lane (c, g) is key 4g+e (e<4) or 16+4g+(e-4): exactly the
        // keys this lane already holds from the two S^T accumulators.
        float p1[2][4];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int i = 0; i < 4; ++i) p1[sub][i] = fast_exp2(x[sub][i] - m_use);  // 0 if masked
        dsum1 *= alpha;
        const u32x4 pb1 = pack8_bf16_accumulate(p1[0][0], p1[0][1], p1[0][2], p1[0][3], p1[1][0],
                                                p1[1][1], p1[1][2], p1[1][3], dsum1);
        u32x4 pb2 = {0u, 0u, 0u, 0u};
        if constexpr (USE_R) {
            float p2[2][4];
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    p2[sub][i] = x[sub][i] == kNegInf ? 0.f : p1[sub][i] * s2[sub][i];
            dsum2 *= alpha;
            pb2 = pack8_bf16_accumulate(p2[0][0], p2[0][1], p2[0][2], p2[0][3], p2[1][0], p2[1][1],
                                        p2[1][2], p2[1][3], dsum2);
        }

        if (!__all(alpha == 1.f)) {
#pragma unroll
            for (int n = 0; n < NDB; ++n) {
                o1[n] *= alpha;
                if constexpr (USE_R) o2[n] *= alpha;
            }
        }

        // ---- O1^T += V^T P1^T, O2^T += V^T P2^T -------------------------------------------
        // A operand: row = output dimension 16n + c, k-elements = the same 8 keys, fetched
        // with two transposing LDS reads (keys 4g..4g+3 and 16+4g..16+4g+3).
        {
            const int tr_key = 4 * g + (c >> 2);          // row this lane addresses
            const int tr_half = (c & 1) * 4;              // element offset inside the chunk
#pragma unroll
            for (int n = 0; n < NDB; ++n) {
                const int chunk = 2 * n + ((c & 3) >> 1);
                const u32x2 lo = lds_read_tr16(ldsV16 + lds_chunk_slot<D>(tr_key, chunk) * 8 + tr_half);
                const u32x2 hi =
                    lds_read_tr16(ldsV16 + lds_chunk_slot<D>(16 + tr_key, chunk) * 8 + tr_half);
                const u32x4 vt = {lo[0], lo[1], hi[0], hi[1]};
                o1[n] = mfma16(vt, pb1, o1[n]);
                if constexpr (USE_R) o2[n] = mfma16(vt, pb2, o2[n]);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }

    // ---- wave partial -> LDS; merge the 4 waves; write the split partial or the output ----
    dsum1 = rows_sum(dsum1);
    dsum2 = rows_sum(dsum2);
    __syncthreads();  // every wave is done with its tile buffers
    float *mrg = (float *)lds;
    float *mrg_m = mrg;                        // [kWaves][16]
    float *mrg_d1 = mrg + kWaves * 16;         // [kWaves][16]
    float *mrg_d2 = mrg + 2 * kWaves * 16;     // [kWaves][16]
    float *mrg_o1 = mrg + 3 * kWaves * 16;     // [kWaves][GC][D]
    float *mrg_o2 = mrg_o1 + kWaves * GC * D;  // [kWaves][GC][D]
    if (live) {
        if (g == 0) {
            mrg_m[w * 16 + c] = m_run;
            mrg_d1[w * 16 + c] = dsum1;
            mrg_d2[w * 16 + c] = dsum2;
        }
#pragma unroll
        for (int n = 0; n < NDB; ++n)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int dim = 16 * n + 4 * g + i;  // accumulator row of O^T
                mrg_o1[(w * GC + c) * D + dim] = o1[n][i];
                mrg_o2[(w * GC + c) * D + dim] = USE_R ? o2[n][i] : 0.f;
            }
    }
    __syncthreads();

    const bool fused = p.counters != nullptr;
    for (int idx = tid; idx < GC * D; idx += 256) {
        const int hh = idx / D, dim = idx - hh * D;  // hh: column (t, head)
        float m_star = kNegInf;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) m_star = fmaxf(m_star, mrg_m[ww * 16 + hh]);
        float d1 = 0.f, d2 = 0.f, a1 = 0.f, a2 = 0.f;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) {
            const float mw = mrg_m[ww * 16 + hh];
            const float wt = mw == kNegInf ? 0.f : fast_exp2(mw - m_star);
            d1 += wt * mrg_d1[ww * 16 + hh];
            d2 += wt * mrg_d2[ww * 16 + hh];
            a1 += wt * mrg_o1[(ww * GC + hh) * D + dim];
            a2 += wt * mrg_o2[(ww * GC + hh) * D + dim];
        }
        const int ot = hh / G, oh = hh - ot * G;
        // output / workspace row of (batch, query head, query row)
        const int64_t hq = ((int64_t)b * p.Hq + (int64_t)hk * G + oh) * Tq_all + row0 + ot;
        if (p.direct_out) {
            float out = 0.f;  // empty key set: zeros
            if (d1 > 0.f) {
                const float inv = 1.f / d1;
                out = a1 * inv * (1.f + d2 * inv) - a2 * inv;
            }
            ((__bf16 *)p.o)[hq * D + dim] = (__bf16)out;
        } else {
            float *rec = p.ws + (hq * S + split) * (int64_t)(2 * D + 4);
            if (fused) {  // device-scope stores: written through to where every XCD sees them
                if (dim == 0) {
                    record_store(rec + 0, m_star);
                    record_store(rec + 1, d1);
                    record_store(rec + 2, d2);
                    record_store(rec + 3, 0.f);
                }
                record_store(rec + 4 + dim, a1);
                record_store(rec + 4 + D + dim, a2);
            } else {
                if (dim == 0) {
                    rec[0] = m_star;
                    rec[1] = d1;
                    rec[2] = d2;
                    rec[3] = 0.f;
                }
                rec[4 + dim] = a1;
                rec[4 + D + dim] = a2;
            }
        }
    }

    // ---- in-kernel reduction (App. C): the last split of a (batch, kv head) group to arrive
    // merges the group's records itself; nobody waits on anybody. The XCDs have private L2
    // caches, and a device-scope release / acquire fence pair would write back and invalidate a
    // whole L2 per workgroup (measured: the step takes four times as long). Instead only the
    // records travel at device scope: written with device-scope stores above (written through to
    // where every XCD sees them), read back with device-scope loads by the workgroup that reads
    // S - 1 from the group's arrival counter. What orders the record stores before the counter
    // update is spelled out here, not left to how a workgroup barrier happens to be lowered:
    // every thread waits until its own stores have been acknowledged (vmcnt counts stores on
    // this chip), then the barrier collects all threads, then one thread bumps the counter with
    // a device-scope atomic. The merger also puts the counter back to zero for the next launch.
    if (fused) {
        __shared__ int is_last;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) {
            const int arrived = __hip_atomic_fetch_add(p.counters + (int64_t)b * p.Hkv + hk, 1,
                                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            is_last = arrived == S - 1;
        }
        __syncthreads();
        if (is_last) {
            MergeScratch<D> *sm = reinterpret_cast<MergeScratch<D> *>(lds);
            auto row_of = [&](int cc) {  // output / workspace row of column cc = (t, head)
                const int ot = cc / G, oh = cc - ot * G;
                return ((int64_t)b * p.Hq + (int64_t)hk * G + oh) * Tq_all + row0 + ot;
            };
            constexpr int64_t REC = 2 * D + 4;
            int cc = 0;
            for (; cc + 2 <= GC; cc += 2) {  // two rows at a time: their loads overlap
                const int64_t h0 = row_of(cc), h1 = row_of(cc + 1);
                const float *const recs[2] = {p.ws + h0 * S * REC, p.ws + h1 * S * REC};
                __bf16 *const outs[2] = {(__bf16 *)p.o + h0 * D, (__bf16 *)p.o + h1 * D};
                merge_records<D, true, 2>(recs, S, outs, tid, sm);
                __syncthreads();  // the scratch is reused by the next rows
            }
            if (cc < GC) {
                const int64_t h0 = row_of(cc);
                const float *const recs[1] = {p.ws + h0 * S * REC};
                __bf16 *const outs[1] = {(__bf16 *)p.o + h0 * D};
                merge_records<D, true, 1>(recs, S, outs, tid, sm);
            }
            if (tid == 0) p.counters[(int64_t)b * p.Hkv + hk] = 0;
        }
    }
}

template <int D>
__global__ __launch_bounds__(256) void decode_combine_kernel(DecodeParams p) {
    __shared__ MergeScratch<D> sm;
    const int64_t hq = (int64_t)blockIdx.y * p.Hq * p.Tq + blockIdx.x;  // (batch, head, query row)
    const float *const recs[1] = {p.ws + hq * p.S * (int64_t)(2 * D + 4)};
    __bf16 *const outs[1] = {(__bf16 *)p.o + hq * D};
    merge_records<D, false, 1>(recs, p.S, outs, threadIdx.x, &sm);
}

template <int D, bool USE_R>
static void launch_decode_variant(const DecodeParams &p, dim3 grid, hipStream_t stream) {
    if (p.prep.gamma_q != nullptr) {  // q / rho prepared in the kernel (the row-range form serves every call)
        DecodeParams pr = p;
        if (pr.rows == 0) pr.row0 = 0, pr.rows = pr.Tq;
        if (p.block_table)
            hipLaunchKernelGGL((decode_bf16_kernel<D, USE_R, true, true, true>), grid, dim3(256), 0, stream, pr);
        else
            hipLaunchKernelGGL((decode_bf16_kernel<D, USE_R, false, true, true>), grid, dim3(256), 0, stream, pr);
    } else if (p.rows > 0) {  // a range of the query rows
        if (p.block_table)
            hipLaunchKernelGGL((decode_bf16_kernel<D, USE_R, true, true>), grid, dim3(256), 0, stream, p);
        else
            hipLaunchKernelGGL((decode_bf16_kernel<D, USE_R, false, true>), grid, dim3(256), 0, stream, p);
    } else if (p.block_table) {
        hipLaunchKernelGGL((decode_bf16_kernel<D, USE_R, true>), grid, dim3(256), 0, stream, p);
    } else {
        hipLaunchKernelGGL((decode_bf16_kernel<D, USE_R, false>), grid, dim3(256), 0, stream, p);
    }
}

hipError_t launch_decode_bf16(const DecodeParams &p, hipStream_t stream) {
    const dim3 grid(p.S, p.Hkv, p.B);
    if (p.d == 128) {
        if (p.use_r)
            launch_decode_variant<128, true>(p, grid, stream);
        else
            launch_decode_variant<128, false>(p, grid, stream);
    } else {
        if (p.use_r)
            launch_decode_variant<64, true>(p, grid, stream);
        else
            launch_decode_variant<64, false>(p, grid, stream);
    }
    return hipGetLastError();
}

hipError_t launch_decode_combine(const DecodeParams &p, hipStream_t stream) {
    const dim3 grid(p.Hq * p.Tq, p.B);
    if (p.d == 512)  // records of the latent-cache kernel
        hipLaunchKernelGGL((decode_combine_kernel<512>), grid, dim3(256), 0, stream, p);
    else if (p.d == 128)
        hipLaunchKernelGGL((decode_combine_kernel<128>), grid, dim3(256), 0, stream, p);
    else
        hipLaunchKernelGGL((decode_combine_kernel<64>), grid, dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace plx
