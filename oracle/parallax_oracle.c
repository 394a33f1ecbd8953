/*
 * Parallax attention forward -- CPU ORACLE (test infrastructure, not product code).
 *
 * Slow, plain, double-precision evaluation of the *definition* of the Parallax
 * output (paper Sec. 3.1, forward equation in its re-weighted softmax form, which
 * the paper restates in App. D and in Sec. 4.4 as the per-token weight s_ij):
 *
 *     a_j  = scale * <q_i, k_j>                 (kernel weight exp(q.k/h), scale = 1/h, Sec. 2.1)
 *     p_j  = softmax_j(a_j)  over the allowed keys J(i)
 *     u_j  = <rho_i, k_j>                       (probe score, NOT scaled: Alg. 1 S2 = R K^T)
 *     ubar = sum_j p_j u_j
 *     o_i  = sum_j p_j (1 + ubar - u_j) v_j
 *
 * t_ij = rho^T (k_j - q_i) in the paper differs from u_j by the j-independent
 * rho^T q_i, which cancels in (tbar - t_ij) = (ubar - u_j).
 *
 * Allowed key set J(i): causal => keys at positions <= the query's position (diagonal
 * included, Sec. 2.1 D_i). With Tq query rows over Lk >= Tq keys the queries are the LAST Tq
 * positions of the sequence (chunked prefill), so row i sits at position i + (Lk - Tq) and
 * sees j <= i + (Lk - Tq); Tq == Lk is the paper's square case j <= i.
 * Otherwise j < len_b, with len_b = seq_lens[b] or Lk when seq_lens is NULL.
 * Sliding window (one of the sparsity patterns Sec. 5 says carry over from softmax attention;
 * the paper gives no formula, the usual one is taken): with window W > 0 a query at position
 * pos sees only the W positions pos - W + 1 .. pos, i.e. of its n allowed keys the last
 * min(n, W). Defined where the query's position is: causal, or a single query row (decode,
 * position len_b - 1).
 * GQA: query head h reads KV head h / (Hq/Hkv); R is shaped and grouped like Q (App. E).
 *
 * No tiling, no online softmax, no fusion: three plain passes per row. Only tests,
 * the smoke check and the benchmark's cpu_baseline leg may use this file; it shares
 * no code with the HIP library.
 *
 * Pins (tests/test_oracle_pins.py): hand-worked two-key example, brute-force weight
 * matrices, R=0 -> library softmax attention, affine equivariance in V, key-translation
 * invariance, scale=0 closed form via cumulative sums, one/two-key closed forms,
 * values affine in keys, the exact-LLA identity with a solved probe, and split-merge
 * associativity of the streaming form.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* One output row. kmat, vmat: [n_keys][d] row-major doubles (only the allowed keys). */
static void plx_row(const double *q, const double *rho, const double *kmat, const double *vmat,
                    int64_t n_keys, int d, double scale, double *o, double *a, double *u)
{
    for (int c = 0; c < d; ++c) o[c] = 0.0;
    if (n_keys <= 0) return; /* undefined in the paper (omega = 0); documented as zeros */

    double amax = -INFINITY;
    for (int64_t j = 0; j < n_keys; ++j) {
        const double *kj = kmat + j * (int64_t)d;
        double s1 = 0.0, s2 = 0.0;
        for (int c = 0; c < d; ++c) {
            s1 += q[c] * kj[c];
            s2 += rho[c] * kj[c];
        }
        a[j] = scale * s1;
        u[j] = s2;
        if (a[j] > amax) amax = a[j];
    }
    double omega = 0.0;
    for (int64_t j = 0; j < n_keys; ++j) {
        a[j] = exp(a[j] - amax); /* a[] now holds w_j */
        omega += a[j];
    }
    double ubar = 0.0;
    for (int64_t j = 0; j < n_keys; ++j) {
        a[j] /= omega; /* a[] now holds p_j */
        ubar += a[j] * u[j];
    }
    for (int64_t j = 0; j < n_keys; ++j) {
        const double w = a[j] * (1.0 + ubar - u[j]);
        const double *vj = vmat + j * (int64_t)d;
        for (int c = 0; c < d; ++c) o[c] += w * vj[c];
    }
}

/*
 * Full evaluation on double inputs.
 *   q, r : [B][Hq][Tq][d]      k, v : [B][Hkv][Lk][d]      o : [B][Hq][Tq][d]
 *   causal != 0 requires Tq <= Lk; seq_lens ([B], may be NULL) is ignored when causal.
 *   window: 0 = none; W > 0 keeps the last W allowed keys of every row (causal or Tq == 1 only).
 *   rows: optional list of n_rows triples (b, h, i); when NULL every row is computed.
 *   For a row list, o is [n_rows][d].
 * Returns 0, or -1 on a bad argument.
 */
int plx_oracle_f64(const double *q, const double *r, const double *k, const double *v, double *o,
                   int B, int Hq, int Hkv, int Tq, int Lk, int d, double scale, int causal,
                   const int32_t *seq_lens, const int32_t *rows, int64_t n_rows, int window)
{
    if (!q || !r || !k || !v || !o) return -1;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Tq <= 0 || Lk <= 0 || d <= 0) return -1;
    if (Hq % Hkv != 0) return -1;
    if (causal && Tq > Lk) return -1;
    if (window < 0 || (window > 0 && !causal && Tq != 1)) return -1;
    const int G = Hq / Hkv;
    const int64_t total = rows ? n_rows : (int64_t)B * Hq * Tq;

#pragma omp parallel
    {
        double *a = (double *)malloc(sizeof(double) * (size_t)Lk);
        double *u = (double *)malloc(sizeof(double) * (size_t)Lk);
#pragma omp for schedule(dynamic, 4)
        for (int64_t t = 0; t < total; ++t) {
            int b, h, i;
            if (rows) {
                b = rows[3 * t + 0];
                h = rows[3 * t + 1];
                i = rows[3 * t + 2];
            } else {
                b = (int)(t / ((int64_t)Hq * Tq));
                h = (int)((t / Tq) % Hq);
                i = (int)(t % Tq);
            }
            const int hk = h / G;
            int64_t n_keys;
            if (causal)
                n_keys = (int64_t)i + 1 + (Lk - Tq);
            else
                n_keys = seq_lens ? seq_lens[b] : Lk;
            if (n_keys > Lk) n_keys = Lk;
            const int64_t first = (window > 0 && n_keys > window) ? n_keys - window : 0;
            const double *qi = q + (((int64_t)b * Hq + h) * Tq + i) * d;
            const double *ri = r + (((int64_t)b * Hq + h) * Tq + i) * d;
            const double *kb = k + ((int64_t)b * Hkv + hk) * (int64_t)Lk * d;
            const double *vb = v + ((int64_t)b * Hkv + hk) * (int64_t)Lk * d;
            double *oi = rows ? o + t * d : o + (((int64_t)b * Hq + h) * Tq + i) * d;
            plx_row(qi, ri, kb + first * d, vb + first * d, n_keys - first, d, scale, oi, a, u);
        }
        free(a);
        free(u);
    }
    return 0;
}

/*
 * Same evaluation on float32 containers (bf16 and fp32 inputs are both exactly
 * representable in float32): every element is widened to double before any
 * arithmetic; K and V are widened one (b, kv-head) slab at a time.
 * Output stays double.
 */
int plx_oracle_f32in(const float *q, const float *r, const float *k, const float *v, double *o,
                     int B, int Hq, int Hkv, int Tq, int Lk, int d, double scale, int causal,
                     const int32_t *seq_lens, const int32_t *rows, int64_t n_rows, int window)
{
    if (!q || !r || !k || !v || !o) return -1;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Tq <= 0 || Lk <= 0 || d <= 0) return -1;
    if (Hq % Hkv != 0) return -1;
    if (causal && Tq > Lk) return -1;
    if (window < 0 || (window > 0 && !causal && Tq != 1)) return -1;
    const int G = Hq / Hkv;
    const int64_t slab = (int64_t)Lk * d;
    double *kd = (double *)malloc(sizeof(double) * (size_t)slab);
    double *vd = (double *)malloc(sizeof(double) * (size_t)slab);
    if (!kd || !vd) {
        free(kd);
        free(vd);
        return -1;
    }
    const int64_t total = rows ? n_rows : (int64_t)B * Hq * Tq;

    for (int b = 0; b < B; ++b) {
        for (int hk = 0; hk < Hkv; ++hk) {
            /* does any requested row touch this slab? */
            int needed = rows ? 0 : 1;
            for (int64_t t = 0; rows && t < n_rows; ++t)
                if (rows[3 * t] == b && rows[3 * t + 1] / G == hk) {
                    needed = 1;
                    break;
                }
            if (!needed) continue;
            const float *kb = k + ((int64_t)b * Hkv + hk) * slab;
            const float *vb = v + ((int64_t)b * Hkv + hk) * slab;
#pragma omp parallel for
            for (int64_t e = 0; e < slab; ++e) {
                kd[e] = (double)kb[e];
                vd[e] = (double)vb[e];
            }
#pragma omp parallel
            {
                double *a = (double *)malloc(sizeof(double) * (size_t)Lk);
                double *u = (double *)malloc(sizeof(double) * (size_t)Lk);
                double *qd = (double *)malloc(sizeof(double) * (size_t)d);
                double *rd = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 4)
                for (int64_t t = 0; t < total; ++t) {
                    int bb, h, i;
                    if (rows) {
                        bb = rows[3 * t + 0];
                        h = rows[3 * t + 1];
                        i = rows[3 * t + 2];
                    } else {
                        bb = (int)(t / ((int64_t)Hq * Tq));
                        h = (int)((t / Tq) % Hq);
                        i = (int)(t % Tq);
                    }
                    if (bb != b || h / G != hk) continue;
                    int64_t n_keys;
                    if (causal)
                        n_keys = (int64_t)i + 1 + (Lk - Tq);
                    else
                        n_keys = seq_lens ? seq_lens[b] : Lk;
                    if (n_keys > Lk) n_keys = Lk;
                    const int64_t first = (window > 0 && n_keys > window) ? n_keys - window : 0;
                    const float *qi = q + (((int64_t)b * Hq + h) * Tq + i) * d;
                    const float *ri = r + (((int64_t)b * Hq + h) * Tq + i) * d;
                    for (int c = 0; c < d; ++c) {
                        qd[c] = (double)qi[c];
                        rd[c] = (double)ri[c];
                    }
                    double *oi = rows ? o + t * d : o + (((int64_t)b * Hq + h) * Tq + i) * d;
                    plx_row(qd, rd, kd + first * d, vd + first * d, n_keys - first, d, scale, oi,
                            a, u);
                }
                free(a);
                free(u);
                free(qd);
                free(rd);
            }
        }
    }
    free(kd);
    free(vd);
    return 0;
}

int plx_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
