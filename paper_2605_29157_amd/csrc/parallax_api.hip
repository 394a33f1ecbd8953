// C ABI of the Parallax attention library: argument validation, split heuristic, dispatch.
// Everything is checked on the host before the first launch; no call allocates or synchronises.
#include "../../include/parallax.h"
#include "../../include/parallax_util.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <mutex>

#include "plx_kernels.h"

// Split workspace of parallax_decode_static, the decode entry point for callers that cannot
// allocate: every GPU the library runs on holds its own copy of this array from the moment the
// code object is loaded until the process ends. In host code the name below is only a handle
// for hipGetSymbolAddress; kernels and copies get the per-device address it returns.
#define PLX_STATIC_SCRATCH_FLOATS (PLX_STATIC_SCRATCH_RECORDS * (2 * 128 + 4))
static __device__ __align__(256) float scratch[PLX_STATIC_SCRATCH_FLOATS];

namespace {

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int elem_size(plx_dtype t) { return t == PLX_BF16 ? 2 : 4; }

bool stride_aligned(int64_t stride_elems, plx_dtype t) {
    return ((stride_elems * elem_size(t)) & 15) == 0;
}

plx_status check_common(plx_dtype dtype, int32_t B, int32_t Hq, int32_t Hkv, int32_t len,
                        int32_t d) {
    if (dtype != PLX_BF16 && dtype != PLX_F32) return PLX_ERR_DTYPE;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || len <= 0 || d <= 0) return PLX_ERR_SHAPE;
    if (B > 65535 || Hq > 65535) return PLX_ERR_SHAPE;
    if (Hq % Hkv != 0) return PLX_ERR_SHAPE;
    if (dtype == PLX_BF16) {
        if (d != 64 && d != 128) return PLX_ERR_SHAPE;
        if (Hq / Hkv > 16) return PLX_ERR_SHAPE;  // one MFMA operand holds a group's heads as 16 columns
    } else {
        if (d > 256 || d % 4 != 0) return PLX_ERR_SHAPE;
    }
    return PLX_OK;
}

constexpr int kMaxDevices = 64;

// Compute units of the current device, asked once per device (the split heuristics run on every
// call). 256 when no device answers.
int query_num_cus() {
    static std::atomic<int> cached[kMaxDevices];
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    const bool slot = dev >= 0 && dev < kMaxDevices;
    if (slot && (cus = cached[dev].load(std::memory_order_relaxed)) > 0) return cus;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        cus <= 0)
        return 256;
    if (slot) cached[dev].store(cus, std::memory_order_relaxed);
    return cus;
}

// The in-kernel q / rho preparation of a call: validated and copied, or left switched off.
plx_status take_prep(const plx_qr_prep &a, plx_dtype dtype, bool use_r, plx::QrPrep *out) {
    *out = plx::QrPrep{};
    const bool any = a.q_gamma || a.r_gamma || a.rope_table || a.pos0 || a.rope_q || a.rope_r;
    if (!any) return PLX_OK;
    if (dtype != PLX_BF16) return PLX_ERR_DTYPE;
    if (!a.q_gamma || (use_r && !a.r_gamma)) return PLX_ERR_NULL;
    if (!(a.eps >= 0.f && a.eps <= 3.0e38f)) return PLX_ERR_SCALE;
    // (the kernels fetch the weights four at a time)
    if (!aligned16(a.q_gamma) || !aligned16(a.r_gamma) || (reinterpret_cast<uintptr_t>(a.pos0) & 3u))
        return PLX_ERR_ALIGN;
    if (a.rope_table) {
        if (!aligned16(a.rope_table)) return PLX_ERR_ALIGN;
        if (a.rope_positions < 1) return PLX_ERR_SHAPE;
    } else if (a.rope_q || a.rope_r) {
        return PLX_ERR_NULL;
    }
    out->gamma_q = a.q_gamma, out->gamma_r = use_r ? a.r_gamma : a.q_gamma;
    out->table = a.rope_table, out->pos0 = a.pos0, out->n_pos = a.rope_positions;
    out->rope_q = a.rope_table && a.rope_q, out->rope_r = a.rope_table && a.rope_r;
    out->eps = a.eps;
    return PLX_OK;
}

size_t ws_bytes(int64_t B, int64_t Hq, int64_t S, int64_t d) {
    return (size_t)(B * Hq * S * (2 * d + 4)) * sizeof(float);
}

// Device address of `scratch` on the current device, looked up once per device (each GPU has
// its own copy of the array at its own address) and kept for the life of the process.
std::mutex g_scratch_mutex;
float *g_scratch_ptr[kMaxDevices];

plx_status static_scratch_of_current_device(float **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PLX_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return PLX_ERR_LAUNCH;
        g_scratch_ptr[dev] = static_cast<float *>(ptr);
    }
    *out = g_scratch_ptr[dev];
    return PLX_OK;
}

}  // namespace

extern "C" {

size_t parallax_decode_workspace_bytes(int32_t B, int32_t Hq, int32_t Hkv, int32_t Lmax,
                                       int32_t d) {
    (void)Hkv;
    (void)Lmax;
    if (B <= 0 || Hq <= 0 || d <= 0) return 0;
    return ws_bytes(B, Hq, PLX_MAX_SPLITS, d);
}

int32_t parallax_decode_num_splits(int32_t B, int32_t Hq, int32_t Hkv, int32_t Lmax, int32_t d,
                                   int32_t num_cus) {
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Lmax <= 0 || d <= 0) return 1;
    if (num_cus <= 0) num_cus = query_num_cus();
    // A model of the launch, fitted to sweeps of S on MI355X. The dispatcher deals the W = pairs * S
    // workgroups round-robin over the compute units, so with W = k * CUs + n2 some units get k and
    // n2 of them k + 1; the memory system shares its bandwidth (~5.9 TB/s with two or more
    // workgroups per unit in flight, ~5.65 with one) equally among the busy units, and a unit
    // cannot take more than ~44 GB/s however many workgroups it holds. All units run until those
    // with k workgroups are through (t1), the n2 others then finish their last workgroup with the
    // bandwidth the rest has freed (t2):
    //     x  = min(44, HBM / CUs) GB/s,          t1 = k * bytes_per_workgroup / x
    //     x2 = min(44, HBM / n2)  GB/s,          t2 = bytes_per_workgroup / x2   (n2 > 0)
    // plus about 3 us for a unit's first workgroup, 0.75 us for each further one and 5 us for the
    // merge launch when S > 1. Measured us for 12 sequences x 16384 keys (96 pairs): S = 1 188,
    // 2 137, 3 175, 4 146, 5 141, 6 152 -- a count that leaves a small remainder over a multiple
    // of the unit count costs up to a quarter, which is what the model is for (the first rule
    // here, "fill two workgroups per unit, rounded up", lost 9 - 19 % at 3, 5, 6, 10, 12 and 20
    // sequences). Over sweeps of S on 20 shapes the chosen count is within 4 % of the best (one shape: 6 %). The
    // count with the smallest estimate wins, the larger one among near-ties with as many rounds;
    // at least two 128-key block tiles per split, and no split below 1024 keys at all (the merge
    // kernel then costs more than the shorter loop saves).
    const int64_t pairs = (int64_t)B * Hkv;
    const double total_mb = (double)pairs * (double)Lmax * (double)d * 4.0 / 1.0e6;  // K and V, bf16
    const int64_t n_bt = ((int64_t)Lmax + plx::kDecodeBlockKeys - 1) / plx::kDecodeBlockKeys;
    int64_t cap = n_bt >= 8 ? n_bt / 2 : 1;
    if (cap > PLX_MAX_SPLITS) cap = PLX_MAX_SPLITS;
    const double cu_rate = 44.0e-3;  // MB per us
    auto cost_of = [&](int64_t s) {
        const int64_t w = pairs * s, k = w / num_cus, n2 = w - k * num_cus;
        const int64_t per_cu = k + (n2 > 0 ? 1 : 0);
        const double hbm_rate = per_cu >= 2 ? 5900.0e-3 : 5650.0e-3;
        const double mb = total_mb / (double)w;
        const double x = cu_rate < hbm_rate / num_cus ? cu_rate : hbm_rate / num_cus;
        double t = (double)k * mb / x;
        if (n2 > 0) t += mb / (cu_rate < hbm_rate / (double)n2 ? cu_rate : hbm_rate / (double)n2);
        return t + 3.0 + 0.75 * (double)(per_cu - 1) + (s > 1 ? 5.0 : 0.0);
    };
    int64_t best = 1;
    for (int64_t s = 2; s <= cap; ++s)
        if (cost_of(s) < cost_of(best)) best = s;
    const int64_t best_rounds = (pairs * best + num_cus - 1) / num_cus;
    const double limit = 1.02 * cost_of(best);
    for (int64_t s = best + 1; s <= cap && (pairs * s + num_cus - 1) / num_cus == best_rounds; ++s)
        if (cost_of(s) <= limit) best = s;
    return (int32_t)best;
}

namespace {

// Validation shared by the decode entry points; fills the launch parameters.
plx_status prepare_decode(const plx_decode_args *a, bool need_inputs, bool need_out,
                          plx::DecodeParams *out) {
    if (!a) return PLX_ERR_NULL;
    if (need_inputs && (!a->q || !a->k || !a->v)) return PLX_ERR_NULL;
    if (need_inputs && a->use_r && !a->r) return PLX_ERR_NULL;
    if (need_out && !a->o) return PLX_ERR_NULL;
    plx_status st = check_common(a->dtype, a->B, a->Hq, a->Hkv, need_inputs ? a->Lmax : 1, a->d);
    if (st != PLX_OK) return st;
    if (a->num_splits < 0 || a->num_splits > PLX_MAX_SPLITS) return PLX_ERR_SPLITS;
    if (a->Tq < 0 || a->Tq > 65535) return PLX_ERR_SHAPE;
    if (a->window < 0) return PLX_ERR_SHAPE;
    const int32_t Tq = a->Tq ? a->Tq : 1;
    // (16 MFMA columns per launch: more rows take several launches; check_common bounds the group size)
    if (need_inputs && !(a->scale >= 0.f && a->scale <= 3.0e38f)) return PLX_ERR_SCALE;
    if (need_out && !aligned16(a->o)) return PLX_ERR_ALIGN;
    if (((int64_t)a->d * elem_size(a->dtype)) % 16 != 0) return PLX_ERR_ALIGN;
    if (need_inputs) {
        if (!aligned16(a->q) || !aligned16(a->k) || !aligned16(a->v) || (a->r && !aligned16(a->r)))
            return PLX_ERR_ALIGN;
        if (a->seq_lens && (reinterpret_cast<uintptr_t>(a->seq_lens) & 3u)) return PLX_ERR_ALIGN;
        const int64_t strides[6] = {a->k_stride_b, a->k_stride_h, a->k_stride_l,
                                    a->v_stride_b, a->v_stride_h, a->v_stride_l};
        for (int64_t s : strides) {
            if (s < 0) return PLX_ERR_SHAPE;
            if (!stride_aligned(s, a->dtype)) return PLX_ERR_ALIGN;
        }
        if (a->k_stride_l < a->d || a->v_stride_l < a->d) return PLX_ERR_SHAPE;
        if (a->block_table) {
            if (reinterpret_cast<uintptr_t>(a->block_table) & 3u) return PLX_ERR_ALIGN;
            if (a->page_size < 1 || a->num_pages < 1 || a->block_table_stride < 1)
                return PLX_ERR_SHAPE;
            if ((int64_t)a->block_table_stride * a->page_size < a->Lmax) return PLX_ERR_SHAPE;
        }
    }
    plx::DecodeParams p{};
    p.q = a->q, p.r = a->use_r ? a->r : a->q, p.k = a->k, p.v = a->v, p.o = a->o;
    p.seq_lens = a->seq_lens;
    p.B = a->B, p.Hq = a->Hq, p.Hkv = a->Hkv, p.G = a->Hq / a->Hkv, p.Lmax = a->Lmax, p.d = a->d;
    p.ksb = a->k_stride_b, p.ksh = a->k_stride_h, p.ksl = a->k_stride_l;
    p.vsb = a->v_stride_b, p.vsh = a->v_stride_h, p.vsl = a->v_stride_l;
    p.scale = a->scale, p.use_r = a->use_r ? 1 : 0;
    p.Tq = Tq;
    p.window = a->window;
    if (need_inputs && a->block_table) {
        p.block_table = a->block_table;
        p.page_size = a->page_size, p.table_stride = a->block_table_stride;
        p.num_pages = a->num_pages;
    }
    if (need_inputs) {
        st = take_prep(a->prep, a->dtype, a->use_r != 0, &p.prep);
        if (st != PLX_OK) return st;
    }
    *out = p;
    return PLX_OK;
}

// Heuristic split count of a call: with a sliding window only the keys inside it are read.
int32_t pick_splits(const plx_decode_args *a, int32_t Tq) {
    int64_t len = a->Lmax;
    if (a->window > 0 && (int64_t)a->window + Tq - 1 < len) len = (int64_t)a->window + Tq - 1;
    return parallax_decode_num_splits(a->B, a->Hq, a->Hkv, (int32_t)len, a->d, 0);
}

plx_status attach_workspace(const plx_decode_args *a, int32_t S, plx::DecodeParams *p) {
    if (!a->workspace || !aligned16(a->workspace)) return PLX_ERR_WORKSPACE;
    if (a->workspace_bytes < ws_bytes(a->B, (int64_t)a->Hq * p->Tq, S, a->d)) return PLX_ERR_WORKSPACE;
    p->ws = static_cast<float *>(a->workspace);
    return PLX_OK;
}

// The split records of a call go to the library's static scratch instead of a caller's
// workspace; a call whose records do not fit is refused.
plx_status attach_static_scratch(const plx_decode_args *a, int32_t S, plx::DecodeParams *p) {
    if (ws_bytes(a->B, (int64_t)a->Hq * p->Tq, S, a->d) > sizeof(float) * PLX_STATIC_SCRATCH_FLOATS)
        return PLX_ERR_SCRATCH;
    return static_scratch_of_current_device(&p->ws);
}

// The bf16 split kernel has 16 MFMA columns (heads of the GQA group x query rows): a call with
// more takes one launch per 16 / G rows. Every launch reads the cache again; they share the
// split workspace and one combine.
hipError_t launch_split_passes(const plx::DecodeParams &p, hipStream_t stream) {
    if (p.G * p.Tq <= 16) return plx::launch_decode_bf16(p, stream);
    const int32_t per = 16 / p.G;
    for (int32_t row0 = 0; row0 < p.Tq; row0 += per) {
        plx::DecodeParams q = p;
        q.row0 = row0;
        q.rows = p.Tq - row0 < per ? p.Tq - row0 : per;
        const hipError_t err = plx::launch_decode_bf16(q, stream);
        if (err != hipSuccess) return err;
    }
    return hipSuccess;
}

}  // namespace

namespace {

plx_status decode_two_kernels(const plx_decode_args *a, bool static_scratch, void *hip_stream) {
    plx::DecodeParams p{};
    plx_status st = prepare_decode(a, true, true, &p);
    if (st != PLX_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    if (a->dtype == PLX_F32) {
        p.S = 1;
        p.r = a->r;
        return plx::launch_decode_f32(p, stream) == hipSuccess ? PLX_OK : PLX_ERR_LAUNCH;
    }

    int32_t S = a->num_splits;
    if (S == 0) S = pick_splits(a, p.Tq);
    p.S = S;
    p.direct_out = S == 1;
    if (S > 1) {
        st = static_scratch ? attach_static_scratch(a, S, &p) : attach_workspace(a, S, &p);
        if (st != PLX_OK) return st;
    }
    if (launch_split_passes(p, stream) != hipSuccess) return PLX_ERR_LAUNCH;
    if (S > 1 && plx::launch_decode_combine(p, stream) != hipSuccess) return PLX_ERR_LAUNCH;
    return PLX_OK;
}

}  // namespace

plx_status parallax_decode(const plx_decode_args *a, void *hip_stream) {
    return decode_two_kernels(a, false, hip_stream);
}

plx_status parallax_decode_static(const plx_decode_args *a, void *hip_stream) {
    return decode_two_kernels(a, true, hip_stream);
}

size_t parallax_decode_static_scratch_bytes(void) { return sizeof(float) * PLX_STATIC_SCRATCH_FLOATS; }

plx_status parallax_decode_fused(const plx_decode_args *a, void *hip_stream) {
    plx::DecodeParams p{};
    plx_status st = prepare_decode(a, true, true, &p);
    if (st != PLX_OK) return st;
    if (a->dtype != PLX_BF16) return PLX_ERR_DTYPE;
    int32_t S = a->num_splits;
    if (S == 0) S = pick_splits(a, p.Tq);
    p.S = S;
    p.direct_out = S == 1;
    if (S > 1) {
        st = attach_workspace(a, S, &p);
        if (st != PLX_OK) return st;
        if (!a->split_counters || (reinterpret_cast<uintptr_t>(a->split_counters) & 3u))
            return PLX_ERR_WORKSPACE;
        p.counters = a->split_counters;
    }
    return launch_split_passes(p, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? PLX_OK : PLX_ERR_LAUNCH;
}

plx_status parallax_decode_partials(const plx_decode_args *a, void *hip_stream) {
    plx::DecodeParams p{};
    plx_status st = prepare_decode(a, true, false, &p);
    if (st != PLX_OK) return st;
    if (a->dtype != PLX_BF16) return PLX_ERR_DTYPE;
    int32_t S = a->num_splits;
    if (S == 0) S = pick_splits(a, p.Tq);
    p.S = S;
    p.direct_out = 0;
    st = attach_workspace(a, S, &p);
    if (st != PLX_OK) return st;
    return launch_split_passes(p, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? PLX_OK : PLX_ERR_LAUNCH;
}

plx_status parallax_decode_combine(const plx_decode_args *a, void *hip_stream) {
    plx::DecodeParams p{};
    plx_status st = prepare_decode(a, false, true, &p);
    if (st != PLX_OK) return st;
    if (a->dtype != PLX_BF16) return PLX_ERR_DTYPE;
    if (a->num_splits < 1) return PLX_ERR_SPLITS;
    p.S = a->num_splits;
    st = attach_workspace(a, p.S, &p);
    if (st != PLX_OK) return st;
    return plx::launch_decode_combine(p, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? PLX_OK
               : PLX_ERR_LAUNCH;
}

plx_status parallax_prefill(const plx_prefill_args *a, void *hip_stream) {
    if (!a) return PLX_ERR_NULL;
    if (!a->q || !a->k || !a->v || !a->o) return PLX_ERR_NULL;
    if (a->use_r && !a->r) return PLX_ERR_NULL;
    plx_status st = check_common(a->dtype, a->B, a->Hq, a->Hkv, a->T, a->d);
    if (st != PLX_OK) return st;
    if (a->Tkv < 0) return PLX_ERR_SHAPE;
    const int32_t Tk = a->Tkv ? a->Tkv : a->T;
    if (a->causal && Tk < a->T) return PLX_ERR_SHAPE;
    if (a->window < 0 || (a->window > 0 && !a->causal)) return PLX_ERR_SHAPE;
    if (!(a->scale >= 0.f && a->scale <= 3.0e38f)) return PLX_ERR_SCALE;
    if (!aligned16(a->q) || !aligned16(a->k) || !aligned16(a->v) || !aligned16(a->o) ||
        (a->r && !aligned16(a->r)))
        return PLX_ERR_ALIGN;
    if (((int64_t)a->d * elem_size(a->dtype)) % 16 != 0) return PLX_ERR_ALIGN;
    const int64_t *sets[5] = {a->q_stride, a->r_stride, a->k_stride, a->v_stride, a->o_stride};
    for (int t = 0; t < 5; ++t) {
        if (t == 1 && !a->use_r) continue;
        for (int j = 0; j < 3; ++j) {
            if (sets[t][j] < 0) return PLX_ERR_SHAPE;
            if (!stride_aligned(sets[t][j], a->dtype)) return PLX_ERR_ALIGN;
        }
        if (sets[t][2] < a->d) return PLX_ERR_SHAPE;
        // the bf16 kernel addresses a 64-row tile with 32-bit byte offsets
        if (a->dtype == PLX_BF16 && sets[t][2] > (1 << 23)) return PLX_ERR_SHAPE;
    }

    plx::PrefillParams p{};
    p.q = a->q, p.r = a->use_r ? a->r : a->q, p.k = a->k, p.v = a->v, p.o = a->o;
    p.B = a->B, p.Hq = a->Hq, p.Hkv = a->Hkv, p.G = a->Hq / a->Hkv, p.T = a->T, p.Tk = Tk, p.d = a->d;
    for (int j = 0; j < 3; ++j) {
        p.qs[j] = a->q_stride[j];
        p.rs[j] = a->use_r ? a->r_stride[j] : a->q_stride[j];
        p.ks[j] = a->k_stride[j];
        p.vs[j] = a->v_stride[j];
        p.os[j] = a->o_stride[j];
    }
    p.scale = a->scale, p.causal = a->causal ? 1 : 0, p.use_r = a->use_r ? 1 : 0;
    p.window = a->window;
    if ((a->sparse_row_ptr != nullptr) != (a->sparse_tile_idx != nullptr)) return PLX_ERR_NULL;
    if (a->sparse_row_ptr) {
        if (a->dtype != PLX_BF16) return PLX_ERR_DTYPE;
        if (!a->use_r || a->window > 0) return PLX_ERR_SHAPE;
        if ((a->sparse_batch != 1 && a->sparse_batch != a->B) ||
            (a->sparse_heads != 1 && a->sparse_heads != a->Hq))
            return PLX_ERR_SHAPE;
        if ((reinterpret_cast<uintptr_t>(a->sparse_row_ptr) | reinterpret_cast<uintptr_t>(a->sparse_tile_idx)) & 3u)
            return PLX_ERR_ALIGN;
        p.sparse_row_ptr = a->sparse_row_ptr, p.sparse_tile_idx = a->sparse_tile_idx;
        p.sparse_batch = a->sparse_batch, p.sparse_heads = a->sparse_heads;
    }
    st = take_prep(a->prep, a->dtype, a->use_r != 0, &p.prep);
    if (st != PLX_OK) return st;
    if (p.prep.gamma_q && (!a->use_r || a->window > 0 || a->sparse_row_ptr || a->row_stats || a->vbar))
        return PLX_ERR_SHAPE;
    if ((a->vbar != nullptr) != (a->row_stats != nullptr)) return PLX_ERR_NULL;
    if (a->row_stats) {
        if (!a->use_r) return PLX_ERR_SHAPE;
        if (!aligned16(a->vbar) || (reinterpret_cast<uintptr_t>(a->row_stats) & 7u)) return PLX_ERR_ALIGN;
        p.vbar = a->vbar, p.row_stats = a->row_stats;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t err = a->dtype == PLX_F32 ? plx::launch_prefill_f32(p, stream)
                                         : plx::launch_prefill_bf16(p, stream);
    return err == hipSuccess ? PLX_OK : PLX_ERR_LAUNCH;
}

size_t parallax_decode_mla_workspace_bytes(int32_t B, int32_t Hq) {
    if (B <= 0 || Hq <= 0) return 0;
    return (size_t)B * Hq * PLX_MAX_SPLITS * (2 * 512 + 4) * sizeof(float);
}

int32_t parallax_decode_mla_num_splits(int32_t B, int32_t Hq, int32_t Lmax, int32_t num_cus) {
    if (B <= 0 || Hq <= 0 || Lmax <= 0) return 1;
    if (num_cus <= 0) num_cus = query_num_cus();
    // One workgroup per compute unit is resident (tile, q / rho fragments and the two register
    // stages fill its LDS and registers), so a launch runs in ROUNDS of num_cus workgroups. A
    // workgroup costs about 10 us to start and finish plus, per 64-key tile, 3.2 us when the chip
    // is full (72 KB x 256 per 3.2 us is what the memory delivers) and no less than 2.4 us (the
    // tile's chain of phases) when W < num_cus workgroups share the memory; merging splits costs
    // one more launch (about 6 us). The split count is the one with the smallest
    //     (rounds - 1) * (tiles * 3.2 + 10) + (tiles * max(2.4, 3.2 * W_last / num_cus) + 10) + (S > 1 ? 6 : 0)
    // with at least 256 keys per split. Against sweeps of S on MI355X (model / measured us):
    // 64 pairs of (sequence, column group) x L = 16384: S = 4 221 / 226 (8: 242); 96 pairs: S = 2
    // 323 / 344 (3, a round and an eighth: 501 / 505); 160 pairs x L = 8192: S = 3 284 / 289 (2:
    // 384 / 392, 1: 317 / 334); 256 pairs: unsplit 829 / 813 (2: 836, 4: 864); 40 pairs x
    // L = 32768: S = 14 362 / 356, 7: 434 / 424, 4: 323 / 340.
    // More than 16 columns take the 32-column kernel, which is bound by its matrix work and the
    // LDS, not by the memory: 2.6 us per tile when every unit holds a workgroup, 2.3 us at least.
    const bool wide = Hq > 16;
    const double t_full = wide ? 2.6 : 3.2, t_least = wide ? 2.3 : 2.4;
    const int64_t pairs = (int64_t)B * (wide ? (Hq + 31) / 32 : 1);
    const int64_t n_tiles = ((int64_t)Lmax + 63) / 64;
    int64_t cap = n_tiles >= 8 ? n_tiles / 4 : 1;
    if (cap > PLX_MAX_SPLITS) cap = PLX_MAX_SPLITS;
    auto cost_of = [&](int64_t s) {
        const int64_t rounds = (pairs * s + num_cus - 1) / num_cus;
        const int64_t tiles = (n_tiles + s - 1) / s;
        const double w_last = (double)(pairs * s - (rounds - 1) * num_cus) / (double)num_cus;
        const double t_last = t_full * w_last > t_least ? t_full * w_last : t_least;
        return (double)(rounds - 1) * ((double)tiles * t_full + 10.0) + ((double)tiles * t_last + 10.0) +
               (s > 1 ? 6.0 : 0.0);
    };
    int64_t best = 1;
    for (int64_t s = 2; s <= cap; ++s)
        if (cost_of(s) < cost_of(best)) best = s;
    // (among counts with as many rounds that the model cannot tell apart, the larger: a fuller
    // round measured a few per cent better than the model gives it credit for)
    const int64_t best_rounds = (pairs * best + num_cus - 1) / num_cus;
    const double limit = 1.02 * cost_of(best);
    for (int64_t s = best + 1; s <= cap && (pairs * s + num_cus - 1) / num_cus == best_rounds; ++s)
        if (cost_of(s) <= limit) best = s;
    return (int32_t)best;
}

plx_status parallax_decode_mla(const plx_decode_mla_args *a, void *hip_stream) {
    if (!a) return PLX_ERR_NULL;
    if (!a->q || !a->r || !a->ckv || !a->o) return PLX_ERR_NULL;
    if (a->dtype != PLX_BF16) return PLX_ERR_DTYPE;
    if (a->B <= 0 || a->Hq <= 0 || a->Lmax <= 0) return PLX_ERR_SHAPE;
    if (a->d_latent != 512 || a->d_rope != 64) return PLX_ERR_SHAPE;
    if (a->Tq < 0 || a->window < 0) return PLX_ERR_SHAPE;
    const int32_t Tq = a->Tq ? a->Tq : 1;
    const int64_t n_cols = (int64_t)a->Hq * Tq;  // (head, row) pairs: the kernel's columns
    if (a->B > 65535 || (n_cols + 15) / 16 > 65535) return PLX_ERR_SHAPE;  // grid dimensions
    if (!(a->scale >= 0.f && a->scale <= 3.0e38f)) return PLX_ERR_SCALE;
    if (!aligned16(a->q) || !aligned16(a->r) || !aligned16(a->ckv) || !aligned16(a->o)) return PLX_ERR_ALIGN;
    if (a->seq_lens && (reinterpret_cast<uintptr_t>(a->seq_lens) & 3u)) return PLX_ERR_ALIGN;
    // (a 64-token tile is addressed with 32-bit byte offsets)
    if (a->ckv_stride_b < 0 || a->ckv_stride_l < 576 || a->ckv_stride_l > (1 << 23)) return PLX_ERR_SHAPE;
    if (!stride_aligned(a->ckv_stride_b, a->dtype) || !stride_aligned(a->ckv_stride_l, a->dtype))
        return PLX_ERR_ALIGN;
    if (a->num_splits < 0 || a->num_splits > PLX_MAX_SPLITS) return PLX_ERR_SPLITS;
    if (a->block_table) {
        if (reinterpret_cast<uintptr_t>(a->block_table) & 3u) return PLX_ERR_ALIGN;
        if (a->page_size < 1 || a->num_pages < 1 || a->block_table_stride < 1) return PLX_ERR_SHAPE;
        if ((int64_t)a->block_table_stride * a->page_size < a->Lmax) return PLX_ERR_SHAPE;
    }

    plx::MlaDecodeParams p{};
    p.q = a->q, p.r = a->r, p.ckv = a->ckv, p.o = a->o, p.seq_lens = a->seq_lens;
    p.B = a->B, p.Hq = a->Hq, p.Lmax = a->Lmax;
    p.Tq = Tq, p.window = a->window;
    p.csb = a->ckv_stride_b, p.csl = a->ckv_stride_l;
    p.scale = a->scale;
    if (a->block_table) {
        p.block_table = a->block_table;
        p.page_size = a->page_size, p.table_stride = a->block_table_stride, p.num_pages = a->num_pages;
    }
    int32_t S = a->num_splits;
    if (S == 0) S = parallax_decode_mla_num_splits(a->B, (int32_t)n_cols, a->Lmax, 0);
    p.S = S;
    p.direct_out = S == 1;
    if (S > 1) {
        if (!a->workspace || !aligned16(a->workspace)) return PLX_ERR_WORKSPACE;
        if (a->workspace_bytes < (size_t)a->B * n_cols * S * (2 * 512 + 4) * sizeof(float)) return PLX_ERR_WORKSPACE;
        p.ws = static_cast<float *>(a->workspace);
    }
    return plx::launch_decode_mla(p, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? PLX_OK
                                                                                         : PLX_ERR_LAUNCH;
}

size_t parallax_prefill_backward_workspace_bytes(int32_t B, int32_t Hq, int32_t T) {
    if (B <= 0 || Hq <= 0 || T <= 0) return 0;
    return (size_t)B * Hq * T * 4 * sizeof(float);
}

plx_status parallax_prefill_backward(const plx_prefill_bwd_args *a, void *hip_stream) {
    if (!a) return PLX_ERR_NULL;
    const void *ptrs[12] = {a->q, a->r, a->k, a->v, a->o, a->vbar, a->row_stats, a->d_o,
                            a->dq, a->dr, a->dk, a->dv};
    for (const void *ptr : ptrs) {
        if (!ptr) return PLX_ERR_NULL;
        if (!aligned16(ptr)) return PLX_ERR_ALIGN;
    }
    plx_status st = check_common(a->dtype, a->B, a->Hq, a->Hkv, a->T, a->d);
    if (st != PLX_OK) return st;
    if (a->Tkv < 0) return PLX_ERR_SHAPE;
    const int32_t Tk = a->Tkv ? a->Tkv : a->T;
    if (a->causal && Tk < a->T) return PLX_ERR_SHAPE;
    if (a->window < 0 || (a->window > 0 && !a->causal)) return PLX_ERR_SHAPE;
    if (a->dtype == PLX_F32 && (a->T > 65535 || Tk > 0x7fffffff / 2)) return PLX_ERR_SHAPE;
    if ((int64_t)a->B * a->Hq * a->T > 0x7fffffffLL || (int64_t)a->B * a->Hkv * Tk > 0x7fffffffLL)
        return PLX_ERR_SHAPE;
    if (!(a->scale >= 0.f && a->scale <= 3.0e38f)) return PLX_ERR_SCALE;
    if (!a->workspace || !aligned16(a->workspace) ||
        a->workspace_bytes < parallax_prefill_backward_workspace_bytes(a->B, a->Hq, a->T))
        return PLX_ERR_WORKSPACE;

    plx::PrefillBwdParams p{};
    p.q = a->q, p.r = a->r, p.k = a->k, p.v = a->v, p.d_o = a->d_o, p.o = a->o, p.vbar = a->vbar;
    p.row_stats = a->row_stats, p.row_cache = static_cast<float *>(a->workspace);
    p.dq = a->dq, p.dr = a->dr, p.dk = a->dk, p.dv = a->dv;
    p.B = a->B, p.Hq = a->Hq, p.Hkv = a->Hkv, p.G = a->Hq / a->Hkv, p.T = a->T, p.Tk = Tk, p.d = a->d;
    p.scale = a->scale, p.causal = a->causal ? 1 : 0;
    // a window that reaches back past the first key is no window
    p.window = (a->window > 0 && a->window < Tk) ? a->window : 0;
    {
        // strides: an all-zero triple is the dense layout; otherwise as in the forward
        const int64_t *given[11] = {a->q_stride, a->r_stride, a->k_stride, a->v_stride, a->o_stride, a->vbar_stride,
                                    a->d_o_stride, a->dq_stride, a->dr_stride, a->dk_stride, a->dv_stride};
        int64_t *dst[11] = {p.qs, p.rs, p.ks, p.vs, p.os, p.vbs, p.gs, p.dqs, p.drs, p.dks, p.dvs};
        for (int t = 0; t < 11; ++t) {
            const bool key_side = t == 2 || t == 3 || t == 9 || t == 10;
            const int64_t H = key_side ? a->Hkv : a->Hq, rows = key_side ? Tk : a->T;
            const int64_t dense[3] = {H * rows * a->d, rows * a->d, a->d};
            const bool zero = given[t][0] == 0 && given[t][1] == 0 && given[t][2] == 0;
            for (int j = 0; j < 3; ++j) {
                const int64_t s = zero ? dense[j] : given[t][j];
                if (s < 0) return PLX_ERR_SHAPE;
                if (!stride_aligned(s, a->dtype)) return PLX_ERR_ALIGN;
                if (a->dtype == PLX_F32 && s != dense[j]) return PLX_ERR_SHAPE;  // plain path: dense only
                dst[t][j] = s;
            }
            // (a 64-row tile is addressed with 32-bit byte offsets)
            if (dst[t][2] < a->d || dst[t][2] > (1 << 23)) return PLX_ERR_SHAPE;
        }
    }
    {
        const void *lists[4] = {a->sparse_row_ptr, a->sparse_tile_idx, a->sparse_col_ptr, a->sparse_col_idx};
        int given = 0;
        for (const void *l : lists) given += l != nullptr;
        if (given != 0 && given != 4) return PLX_ERR_NULL;
        if (given) {
            if (a->dtype != PLX_BF16) return PLX_ERR_DTYPE;
            if (a->window > 0) return PLX_ERR_SHAPE;
            if ((a->sparse_batch != 1 && a->sparse_batch != a->B) ||
                (a->sparse_heads != 1 && a->sparse_heads != a->Hq))
                return PLX_ERR_SHAPE;
            for (const void *l : lists)
                if (reinterpret_cast<uintptr_t>(l) & 3u) return PLX_ERR_ALIGN;
            p.sparse_row_ptr = a->sparse_row_ptr, p.sparse_tile_idx = a->sparse_tile_idx;
            p.sparse_col_ptr = a->sparse_col_ptr, p.sparse_col_idx = a->sparse_col_idx;
            p.sparse_batch = a->sparse_batch, p.sparse_heads = a->sparse_heads;
        }
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const hipError_t err = a->dtype == PLX_F32 ? plx::launch_prefill_bwd_f32(p, stream)
                                               : plx::launch_prefill_bwd_bf16(p, stream);
    return err == hipSuccess ? PLX_OK : PLX_ERR_LAUNCH;
}

plx_status parallax_norm_rope(const plx_norm_rope_args *a, void *hip_stream) {
    if (!a) return PLX_ERR_NULL;
    if (a->dtype != PLX_BF16 && a->dtype != PLX_F32) return PLX_ERR_DTYPE;
    if (a->n_tensors < 1 || a->n_tensors > 3 || a->B <= 0 || a->T <= 0) return PLX_ERR_SHAPE;
    const bool f32 = a->dtype == PLX_F32;
    const int32_t d = a->d;
    if (f32 ? !(d == 16 || d == 32 || d == 64 || d == 128 || d == 256) : !(d == 64 || d == 128))
        return PLX_ERR_SHAPE;
    if (!(a->eps >= 0.f && a->eps <= 3.0e38f) || !(a->theta > 1.f && a->theta <= 3.0e38f))
        return PLX_ERR_SCALE;
    if (a->pos0 && (reinterpret_cast<uintptr_t>(a->pos0) & 3u)) return PLX_ERR_ALIGN;
    plx::NormRopeParams p{};
    for (int i = 0; i < a->n_tensors; ++i) {
        const plx_norm_rope_tensor &t = a->tensors[i];
        if (!t.x || !t.y || !t.gamma) return PLX_ERR_NULL;
        if (!aligned16(t.x) || !aligned16(t.y) || (reinterpret_cast<uintptr_t>(t.gamma) & 3u))
            return PLX_ERR_ALIGN;
        if (t.H <= 0 || (int64_t)a->B * t.H * a->T > 0x7fffffffLL) return PLX_ERR_SHAPE;
        p.t[i].x = t.x, p.t[i].y = t.y, p.t[i].gamma = t.gamma, p.t[i].H = t.H, p.t[i].rope = t.rope ? 1 : 0;
    }
    p.n_tensors = a->n_tensors, p.B = a->B, p.T = a->T, p.d = d;
    p.pos0 = a->pos0, p.eps = a->eps, p.theta = a->theta;
    if (a->rope_table) {
        if (!aligned16(a->rope_table)) return PLX_ERR_ALIGN;
        if (a->table_positions < 1) return PLX_ERR_SHAPE;
        p.table = a->rope_table, p.n_pos = a->table_positions;
    }
    return plx::launch_norm_rope(p, f32, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? PLX_OK
               : PLX_ERR_LAUNCH;
}

plx_status parallax_rope_table(float *table, int32_t n_pos, int32_t d, float theta, void *hip_stream) {
    if (!table) return PLX_ERR_NULL;
    if (!aligned16(table)) return PLX_ERR_ALIGN;
    if (n_pos < 1 || d < 2 || d > 256 || d % 2 != 0) return PLX_ERR_SHAPE;
    if (!(theta > 1.f && theta <= 3.0e38f)) return PLX_ERR_SCALE;
    return plx::launch_rope_table(table, n_pos, d, theta, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? PLX_OK
               : PLX_ERR_LAUNCH;
}

plx_status parallax_util_copy(void *dst, const void *src, size_t bytes, void *hip_stream) {
    if (!dst || !src) return PLX_ERR_NULL;
    if (bytes % 16 != 0) return PLX_ERR_SHAPE;
    if (!aligned16(dst) || !aligned16(src)) return PLX_ERR_ALIGN;
    return plx::launch_util_copy(dst, src, bytes, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? PLX_OK
               : PLX_ERR_LAUNCH;
}

plx_status parallax_util_read(const void *src, size_t bytes, void *sink, void *hip_stream) {
    if (!src || !sink) return PLX_ERR_NULL;
    if (bytes % 16 != 0) return PLX_ERR_SHAPE;
    if (!aligned16(src) || !aligned16(sink)) return PLX_ERR_ALIGN;
    return plx::launch_util_read(src, bytes, sink, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? PLX_OK
               : PLX_ERR_LAUNCH;
}

plx_status parallax_util_read_grid(const void *src, size_t bytes, void *sink, int32_t workgroups,
                                   void *hip_stream) {
    if (!src || !sink) return PLX_ERR_NULL;
    if (bytes % 16 != 0 || workgroups < 1 || workgroups > plx::kReadSinkSlots) return PLX_ERR_SHAPE;
    if (!aligned16(src) || !aligned16(sink)) return PLX_ERR_ALIGN;
    return plx::launch_util_read_grid(src, bytes, sink, workgroups, static_cast<hipStream_t>(hip_stream)) ==
                   hipSuccess
               ? PLX_OK
               : PLX_ERR_LAUNCH;
}

int32_t parallax_util_read_sink_slots(void) { return plx::kReadSinkSlots; }

plx_status parallax_util_mfma(int32_t workgroups, int32_t iters, void *sink, void *hip_stream) {
    if (!sink) return PLX_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(sink) & 3u) return PLX_ERR_ALIGN;
    if (workgroups < 1 || workgroups > 65536 || iters < 1 || iters > (1 << 24)) return PLX_ERR_SHAPE;
    return plx::launch_util_mfma(workgroups, iters, sink, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? PLX_OK
               : PLX_ERR_LAUNCH;
}

const char *parallax_strerror(plx_status status) {
    switch (status) {
        case PLX_OK: return "ok";
        case PLX_ERR_NULL: return "a required pointer is NULL";
        case PLX_ERR_SHAPE: return "unsupported or inconsistent shape / stride";
        case PLX_ERR_DTYPE: return "unknown dtype";
        case PLX_ERR_ALIGN: return "pointer or stride is not 16-byte aligned";
        case PLX_ERR_WORKSPACE: return "split-KV workspace missing, misaligned or too small";
        case PLX_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
        case PLX_ERR_SPLITS: return "num_splits outside [0, PLX_MAX_SPLITS]";
        case PLX_ERR_SCALE: return "scale must be finite and non-negative";
        case PLX_ERR_SCRATCH:
            return "the split records of this call do not fit parallax_decode_static's fixed scratch "
                   "(use fewer splits, a smaller batch, or parallax_decode with a workspace)";
    }
    return "unknown status";
}

int parallax_version(void) { return 100; }

}  // extern "C"
