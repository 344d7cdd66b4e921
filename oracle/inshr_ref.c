/*
 * inshr_ref.c -- CPU oracle (TEST INFRASTRUCTURE ONLY; see inshr_ref.h).
 *
 * Reading of the paper used here (each choice is listed with its reason in the design notes):
 *   - ranking metric: magnitude I_m(w) = |w|                               (Sec. 4.1)
 *   - protection: the F_prot largest magnitudes keep their original value   (Sec. 4.2)
 *   - pruning: the F_prun smallest magnitudes decode to zero                (Sec. 4.2)
 *   - thresholds are exact quantiles of the magnitudes, i.e. the alpha -> 0 limit of the
 *     relative-error quantile bound                                         (Sec. 4.3)
 *   - bins: K = 2^bits equal-frequency bins over the remaining values (frequency-only sample
 *     weights), one centre per bin = mean of its members (a single centre update) (Sec. 4.4)
 *   - search: smallest payload whose relative squared error is <= eps       (Sec. 5)
 *   - delta: D = (C_prev - C_cur) mod B with prune / protect as extra levels,
 *     B = larger level count of the two checkpoints                         (Sec. 6)
 *   - regrouping: deltas split by the previous checkpoint's symbol, groups ascending,
 *     members in ascending index                                            (Algorithm 5)
 *
 * Floats are compared through two integer images so that the order is total and identical
 * on every machine: -0.0 is first replaced by +0.0;
 *   mag(x) = bits(x) & 0x7fffffff              orders |x|
 *   key(x) = bits(x) ^ (sign ? ~0 : 1<<31)     orders x
 */
#include "inshr_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

static uint32_t canon_bits(float x)
{
    uint32_t b;
    memcpy(&b, &x, 4);
    if (b == 0x80000000u) b = 0u; /* -0.0 -> +0.0 */
    return b;
}
static uint32_t mag_of_bits(uint32_t b) { return b & 0x7fffffffu; }
static uint32_t key_of_bits(uint32_t b) { return (b & 0x80000000u) ? ~b : (b | 0x80000000u); }
static uint32_t mag_of_key(uint32_t k) { return (k & 0x80000000u) ? (k & 0x7fffffffu) : (~k & 0x7fffffffu); }
static float float_of_key(uint32_t k)
{
    uint32_t b = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    float f;
    memcpy(&f, &b, 4);
    return f;
}

static int cmp_u32(const void *a, const void *b)
{
    uint32_t x = *(const uint32_t *)a, y = *(const uint32_t *)b;
    return (x > y) - (x < y);
}

/* number of bins of a configuration: the count itself when given (Sec. 5, search space), else 2^bits */
static uint32_t bins_of(const inshr_ref_config *c) { return c->bins ? c->bins : (1u << c->bits); }

uint32_t inshr_ref_symbol_bits(uint32_t K)
{
    uint32_t w = 1;
    while ((1u << w) < K + 2u) w++; /* K bins + the pruned and the protected level (Sec. 6) */
    return w;
}

/* payload of the quantized values: an ideal fixed-length code spends log2 K bits on each; log2 K is
 * taken in units of 2^-16 (exact for powers of two) and the product rounded up */
static uint64_t code_bits(uint64_t n_kept, uint32_t K)
{
    const uint64_t l16 = (uint64_t)floor(log2((double)K) * 65536.0 + 0.5);
    return (n_kept * l16 + 65535ull) >> 16;
}

static int check_config(const inshr_ref_config *c)
{
    if (c->bins) {
        if (c->bins < 2 || c->bins > 256) return INSHR_REF_E_CONFIG;
    } else if (c->bits < 1 || c->bits > 8) {
        return INSHR_REF_E_CONFIG;
    }
    if ((uint64_t)c->prune_ppm + (uint64_t)c->outlier_ppm >= 1000000ull) return INSHR_REF_E_CONFIG;
    return INSHR_REF_OK;
}

/* Sorted magnitude and key images of one tensor; shared by all configurations of a grid
 * because they do not depend on the configuration. */
typedef struct {
    uint32_t *A; /* mag images ascending */
    uint32_t *S; /* key images ascending */
} sorted_images;

static int make_sorted_images(const float *x, uint64_t n, sorted_images *out)
{
    out->A = (uint32_t *)malloc(n * sizeof(uint32_t));
    out->S = (uint32_t *)malloc(n * sizeof(uint32_t));
    if (!out->A || !out->S) return INSHR_REF_E_ARG;
    for (uint64_t i = 0; i < n; i++) {
        uint32_t b = canon_bits(x[i]);
        if ((b & 0x7f800000u) == 0x7f800000u) return INSHR_REF_E_NONFINITE;
        out->A[i] = mag_of_bits(b);
        out->S[i] = key_of_bits(b);
    }
    qsort(out->A, n, sizeof(uint32_t), cmp_u32);
    qsort(out->S, n, sizeof(uint32_t), cmp_u32);
    return INSHR_REF_OK;
}
static void free_sorted_images(sorted_images *s)
{
    free(s->A);
    free(s->S);
    s->A = s->S = NULL;
}

/* number of boundaries t_j (as keys) with t_j <= key: the bin of a quantized value */
static uint32_t bin_of_key(const uint32_t *tkeys, uint32_t n_t, uint32_t key)
{
    uint32_t lo = 0, hi = n_t; /* first index with tkeys[idx] > key */
    while (lo < hi) {
        uint32_t mid = lo + (hi - lo) / 2;
        if (tkeys[mid] <= key)
            lo = mid + 1;
        else
            hi = mid;
    }
    return lo;
}

/* One configuration, from the sorted images.  sym / boundaries / codebook / out_* may be NULL.
 * pool / n_pool: the ascending magnitude images of all tensors of the layer type (Sec. 4.2: the
 * same pruning fraction across all layers of a given type, i.e. thresholds that are quantiles of
 * the type's pooled values); NULL = the tensor alone. */
static int quantize_one(const float *x, uint64_t n, const sorted_images *si, const uint32_t *pool,
                        uint64_t n_pool, const inshr_ref_config *cfg, uint16_t *sym, float *boundaries,
                        float *codebook, uint32_t *out_idx, float *out_val, inshr_ref_qinfo *info)
{
    const uint32_t K = bins_of(cfg);
    const uint32_t *A = pool ? pool : si->A;
    const uint64_t nA = pool ? n_pool : n;
    const uint64_t n_p = nA * (uint64_t)cfg->prune_ppm / 1000000ull;
    const uint64_t n_o = nA * (uint64_t)cfg->outlier_ppm / 1000000ull;

    /* thresholds: exact order statistics of the magnitudes */
    const uint32_t tau_p = A[n_p];          /* pruned    <=> mag <  tau_p */
    const uint32_t tau_o = A[nA - 1 - n_o]; /* protected <=> mag >  tau_o */

    /* Y: quantized ("kept") values in ascending order = the sorted keys with the pruned and
     * protected ones taken out */
    uint32_t *Y = (uint32_t *)malloc(n * sizeof(uint32_t));
    if (!Y) return INSHR_REF_E_ARG;
    uint64_t M = 0;
    for (uint64_t r = 0; r < n; r++) {
        uint32_t k = si->S[r];
        uint32_t m = mag_of_key(k);
        if (m < tau_p || m > tau_o) continue;
        Y[M++] = k;
    }
    /* M >= 1 for a tensor alone, because tau_p <= tau_o and the element of rank n_p is kept; pooled
     * thresholds can leave a tensor without quantized values: no bins can be made for it */
    if (M == 0) {
        free(Y);
        return INSHR_REF_E_EMPTY;
    }

    /* equal-frequency boundaries t_j = Y[floor(j*M/K)] */
    uint32_t tkeys[255];
    for (uint32_t j = 1; j < K; j++) tkeys[j - 1] = Y[(uint64_t)j * M / K];
    const uint32_t y0 = Y[0];
    free(Y);

    /* symbols, per-bin sums in index order */
    double bsum[256];
    uint64_t bcnt[256];
    for (uint32_t k = 0; k < K; k++) {
        bsum[k] = 0.0;
        bcnt[k] = 0;
    }
    uint64_t n_pruned = 0, n_outlier = 0, n_kept = 0;
    for (uint64_t i = 0; i < n; i++) {
        uint32_t b = canon_bits(x[i]);
        uint32_t m = mag_of_bits(b);
        uint16_t s;
        if (m < tau_p) {
            s = 0;
            n_pruned++;
        } else if (m > tau_o) {
            s = 1;
            if (out_idx) out_idx[n_outlier] = (uint32_t)i;
            if (out_val) out_val[n_outlier] = x[i];
            n_outlier++;
        } else {
            uint32_t bin = bin_of_key(tkeys, K - 1, key_of_bits(b));
            s = (uint16_t)(2 + bin);
            bsum[bin] += (double)x[i];
            bcnt[bin]++;
            n_kept++;
        }
        if (sym) sym[i] = s;
    }

    /* centres: mean of the members; an empty bin takes its lower boundary */
    float cb[256];
    for (uint32_t k = 0; k < K; k++) {
        if (bcnt[k])
            cb[k] = (float)(bsum[k] / (double)bcnt[k]);
        else
            cb[k] = (k == 0) ? float_of_key(y0) : float_of_key(tkeys[k - 1]);
    }

    /* error of the decoded tensor */
    double sse = 0.0, sumsq = 0.0;
    for (uint64_t i = 0; i < n; i++) {
        uint32_t b = canon_bits(x[i]);
        uint32_t m = mag_of_bits(b);
        double xd = (double)x[i];
        sumsq += xd * xd;
        if (m < tau_p) {
            sse += xd * xd;
        } else if (m > tau_o) {
            /* exact */
        } else {
            uint32_t bin = bin_of_key(tkeys, K - 1, key_of_bits(b));
            double e = xd - (double)cb[bin];
            sse += e * e;
        }
    }

    if (boundaries)
        for (uint32_t j = 0; j + 1 < K; j++) boundaries[j] = float_of_key(tkeys[j]);
    if (codebook)
        for (uint32_t k = 0; k < K; k++) codebook[k] = cb[k];
    if (info) {
        info->n_pruned = n_pruned;
        info->n_outlier = n_outlier;
        info->n_kept = n_kept;
        info->sym_bits = inshr_ref_symbol_bits(K);
        info->tau_prune_bits = tau_p;
        info->tau_outlier_bits = tau_o;
        info->sse = sse;
        info->sumsq = sumsq;
    }
    return INSHR_REF_OK;
}

float inshr_ref_bf16_round(float x)
{
    uint32_t b;
    memcpy(&b, &x, 4);
    /* round to nearest, ties to the even upper half; finite inputs only (a carry out of the largest
     * finite exponent gives infinity, as the format defines) */
    const uint32_t upper = b >> 16, lower = b & 0xFFFFu;
    uint32_t r = upper;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) r = upper + 1u;
    r <<= 16;
    float f;
    memcpy(&f, &r, 4);
    return f;
}

int inshr_ref_quantize_pooled(const float *x, uint64_t n, const uint32_t *pool, uint64_t n_pool,
                              const inshr_ref_config *cfg, uint16_t *sym, float *boundaries,
                              float *codebook, uint32_t *out_idx, float *out_val, inshr_ref_qinfo *info)
{
    if (!x || !cfg || n == 0 || n >= (1ull << 32)) return INSHR_REF_E_ARG;
    if (pool && n_pool < n) return INSHR_REF_E_ARG;
    int rc = check_config(cfg);
    if (rc) return rc;
    sorted_images si;
    rc = make_sorted_images(x, n, &si);
    if (rc == INSHR_REF_OK)
        rc = quantize_one(x, n, &si, pool, n_pool, cfg, sym, boundaries, codebook, out_idx, out_val, info);
    free_sorted_images(&si);
    return rc;
}

int inshr_ref_quantize(const float *x, uint64_t n, const inshr_ref_config *cfg, uint16_t *sym,
                       float *boundaries, float *codebook, uint32_t *out_idx, float *out_val,
                       inshr_ref_qinfo *info)
{
    return inshr_ref_quantize_pooled(x, n, NULL, 0, cfg, sym, boundaries, codebook, out_idx, out_val, info);
}

int inshr_ref_search(const float *x, uint64_t n, const inshr_ref_config *grid, uint32_t n_cfg,
                     double eps, uint32_t *best, uint8_t *feasible, inshr_ref_score *scores)
{
    return inshr_ref_search_pooled(x, n, NULL, 0, grid, n_cfg, eps, best, feasible, scores);
}

int inshr_ref_search_pooled(const float *x, uint64_t n, const uint32_t *pool, uint64_t n_pool,
                            const inshr_ref_config *grid, uint32_t n_cfg, double eps, uint32_t *best,
                            uint8_t *feasible, inshr_ref_score *scores)
{
    if (!x || !grid || !best || !feasible || n == 0 || n >= (1ull << 32) || n_cfg == 0)
        return INSHR_REF_E_ARG;
    if (pool && n_pool < n) return INSHR_REF_E_ARG;
    for (uint32_t g = 0; g < n_cfg; g++) {
        int rc = check_config(&grid[g]);
        if (rc) return rc;
    }
    sorted_images si;
    int rc = make_sorted_images(x, n, &si);
    if (rc) {
        free_sorted_images(&si);
        return rc;
    }

    int have_feasible = 0, have_any = 0;
    uint32_t best_f = 0, best_a = 0;
    uint64_t best_cost = 0;
    double best_sse = 0.0;
    for (uint32_t g = 0; g < n_cfg; g++) {
        inshr_ref_qinfo qi;
        rc = quantize_one(x, n, &si, pool, n_pool, &grid[g], NULL, NULL, NULL, NULL, NULL, &qi);
        if (rc) break;
        inshr_ref_score sc;
        sc.sse = qi.sse;
        sc.sumsq = qi.sumsq;
        sc.n_pruned = qi.n_pruned;
        sc.n_outlier = qi.n_outlier;
        sc.n_kept = qi.n_kept;
        sc.cost_bits = code_bits(qi.n_kept, bins_of(&grid[g])) + 32ull * qi.n_outlier +
                       32ull * (uint64_t)bins_of(&grid[g]);
        if (scores) scores[g] = sc;

        double rel = (sc.sumsq > 0.0) ? sc.sse / sc.sumsq : 0.0;
        if (rel <= eps) {
            if (!have_feasible || sc.cost_bits < best_cost) {
                have_feasible = 1;
                best_f = g;
                best_cost = sc.cost_bits;
            }
        }
        if (!have_any || sc.sse < best_sse) {
            have_any = 1;
            best_a = g;
            best_sse = sc.sse;
        }
    }
    free_sorted_images(&si);
    if (rc) return rc;
    *best = have_feasible ? best_f : best_a;
    *feasible = (uint8_t)have_feasible;
    return INSHR_REF_OK;
}

int inshr_ref_quantize_sens(const float *x, const float *g, uint64_t n, const inshr_ref_config *cfg,
                            int prune_by_sensitivity, uint16_t *sym, float *boundaries, float *codebook,
                            uint32_t *out_idx, float *out_val, inshr_ref_qinfo *info,
                            uint32_t *tau_outlier_sens_bits)
{
    if (!x || !g || !cfg || n == 0 || n >= (1ull << 32)) return INSHR_REF_E_ARG;
    int rc = check_config(cfg);
    if (rc) return rc;
    const uint32_t K = bins_of(cfg);
    const uint64_t n_p = n * (uint64_t)cfg->prune_ppm / 1000000ull;
    const uint64_t n_o = n * (uint64_t)cfg->outlier_ppm / 1000000ull;
    uint32_t *mag = (uint32_t *)malloc(n * 4), *sc = (uint32_t *)malloc(n * 4);
    uint32_t *A = (uint32_t *)malloc(n * 4), *S = (uint32_t *)malloc(n * 4), *Y = (uint32_t *)malloc(n * 4);
    uint8_t *cls = (uint8_t *)malloc(n);
    rc = (mag && sc && A && S && Y && cls) ? INSHR_REF_OK : INSHR_REF_E_ARG;
    for (uint64_t i = 0; rc == INSHR_REF_OK && i < n; i++) {
        const uint32_t b = canon_bits(x[i]);
        volatile float prod = g[i] * x[i]; /* one fp32 multiplication, rounded to fp32 */
        const uint32_t sb = mag_of_bits(canon_bits(prod));
        if ((b & 0x7f800000u) == 0x7f800000u || (sb & 0x7f800000u) == 0x7f800000u ||
            (canon_bits(g[i]) & 0x7f800000u) == 0x7f800000u)
            rc = INSHR_REF_E_NONFINITE;
        mag[i] = A[i] = mag_of_bits(b);
        sc[i] = S[i] = sb; /* the bit image of a non-negative float orders like the float */
    }
    if (rc == INSHR_REF_OK) {
        qsort(A, n, 4, cmp_u32);
        qsort(S, n, 4, cmp_u32);
        const uint32_t tau_om = A[n - 1 - n_o], tau_os = S[n - 1 - n_o];
        const uint32_t tau_p = prune_by_sensitivity ? S[n_p] : A[n_p];
        uint64_t M = 0, n_pruned = 0, n_outlier = 0;
        for (uint64_t i = 0; i < n; i++) {
            const uint32_t m = prune_by_sensitivity ? sc[i] : mag[i];
            if (mag[i] > tau_om || sc[i] > tau_os) {
                cls[i] = 1;
                if (out_idx) out_idx[n_outlier] = (uint32_t)i;
                if (out_val) out_val[n_outlier] = x[i];
                n_outlier++;
            } else if (m < tau_p) {
                cls[i] = 0;
                n_pruned++;
            } else {
                cls[i] = 2;
                Y[M++] = key_of_bits(canon_bits(x[i]));
            }
        }
        if (M == 0) rc = INSHR_REF_E_EMPTY;
        if (rc == INSHR_REF_OK) {
            qsort(Y, M, 4, cmp_u32);
            uint32_t tkeys[255];
            for (uint32_t j = 1; j < K; j++) tkeys[j - 1] = Y[(uint64_t)j * M / K];
            double bsum[256];
            uint64_t bcnt[256];
            for (uint32_t k = 0; k < K; k++) {
                bsum[k] = 0.0;
                bcnt[k] = 0;
            }
            for (uint64_t i = 0; i < n; i++) {
                uint16_t s = cls[i];
                if (cls[i] == 2) {
                    const uint32_t bin = bin_of_key(tkeys, K - 1, key_of_bits(canon_bits(x[i])));
                    s = (uint16_t)(2 + bin);
                    bsum[bin] += (double)x[i];
                    bcnt[bin]++;
                }
                if (sym) sym[i] = s;
            }
            float cb[256];
            for (uint32_t k = 0; k < K; k++) {
                if (bcnt[k])
                    cb[k] = (float)(bsum[k] / (double)bcnt[k]);
                else
                    cb[k] = (k == 0) ? float_of_key(Y[0]) : float_of_key(tkeys[k - 1]);
            }
            double sse = 0.0, sumsq = 0.0;
            for (uint64_t i = 0; i < n; i++) {
                const double xd = (double)x[i];
                sumsq += xd * xd;
                if (cls[i] == 0) {
                    sse += xd * xd;
                } else if (cls[i] == 2) {
                    const uint32_t bin = bin_of_key(tkeys, K - 1, key_of_bits(canon_bits(x[i])));
                    const double e = xd - (double)cb[bin];
                    sse += e * e;
                }
            }
            if (boundaries)
                for (uint32_t j = 0; j + 1 < K; j++) boundaries[j] = float_of_key(tkeys[j]);
            if (codebook)
                for (uint32_t k = 0; k < K; k++) codebook[k] = cb[k];
            if (info) {
                info->n_pruned = n_pruned;
                info->n_outlier = n_outlier;
                info->n_kept = M;
                info->sym_bits = inshr_ref_symbol_bits(K);
                info->tau_prune_bits = tau_p;
                info->tau_outlier_bits = tau_om;
                info->sse = sse;
                info->sumsq = sumsq;
            }
            if (tau_outlier_sens_bits) *tau_outlier_sens_bits = tau_os;
        }
    }
    free(mag);
    free(sc);
    free(A);
    free(S);
    free(Y);
    free(cls);
    return rc;
}

int inshr_ref_dequantize(const uint16_t *sym, uint64_t n, uint32_t bits, const float *codebook,
                         const uint32_t *out_idx, const float *out_val, uint64_t n_outlier,
                         float *xhat)
{
    if (bits < 1 || bits > 8) return INSHR_REF_E_ARG;
    return inshr_ref_dequantize_k(sym, n, 1u << bits, codebook, out_idx, out_val, n_outlier, xhat);
}

int inshr_ref_dequantize_k(const uint16_t *sym, uint64_t n, uint32_t K, const float *codebook,
                           const uint32_t *out_idx, const float *out_val, uint64_t n_outlier,
                           float *xhat)
{
    if (!sym || !codebook || !xhat || K < 2 || K > 256) return INSHR_REF_E_ARG;
    uint64_t q = 0;
    for (uint64_t i = 0; i < n; i++) {
        uint16_t s = sym[i];
        if (s == 0) {
            xhat[i] = 0.0f;
        } else if (s == 1) {
            if (q >= n_outlier || !out_idx || !out_val || out_idx[q] != i) return INSHR_REF_E_SHAPE;
            xhat[i] = out_val[q++];
        } else {
            if ((uint32_t)s - 2u >= K) return INSHR_REF_E_ARG;
            xhat[i] = codebook[s - 2];
        }
    }
    return (q == n_outlier) ? INSHR_REF_OK : INSHR_REF_E_SHAPE;
}

int inshr_ref_delta(const uint16_t *s_prev, uint32_t bits_prev, const uint16_t *s_cur,
                    uint32_t bits_cur, uint64_t n, uint16_t *delta, uint32_t *perm,
                    uint64_t *group_off, uint16_t *stream)
{
    if (bits_prev < 1 || bits_prev > 8 || bits_cur < 1 || bits_cur > 8) return INSHR_REF_E_CONFIG;
    return inshr_ref_delta_k(s_prev, 1u << bits_prev, s_cur, 1u << bits_cur, n, delta, perm, group_off, stream);
}

int inshr_ref_delta_k(const uint16_t *s_prev, uint32_t K_prev, const uint16_t *s_cur, uint32_t K_cur,
                      uint64_t n, uint16_t *delta, uint32_t *perm, uint64_t *group_off,
                      uint16_t *stream)
{
    if (!s_prev || !s_cur || !group_off || n == 0 || n >= (1ull << 32)) return INSHR_REF_E_ARG;
    if (K_prev < 2 || K_prev > 256 || K_cur < 2 || K_cur > 256) return INSHR_REF_E_CONFIG;
    const uint32_t Sp = K_prev + 2u; /* levels of the previous checkpoint */
    const uint32_t Sc = K_cur + 2u;
    const uint32_t B = (Sp > Sc) ? Sp : Sc;     /* cyclic range */
    for (uint64_t i = 0; i < n; i++)
        if (s_prev[i] >= Sp || s_cur[i] >= Sc) return INSHR_REF_E_ARG;

    /* group_off[g] = #{i : s_prev[i] < g}, g = 0..Sp */
    for (uint32_t g = 0; g <= Sp; g++) group_off[g] = 0;
    for (uint64_t i = 0; i < n; i++) group_off[s_prev[i] + 1u]++;
    for (uint32_t g = 0; g < Sp; g++) group_off[g + 1] += group_off[g];

    /* walk indices in order; each appends its delta to the group of its previous symbol */
    uint64_t *cursor = (uint64_t *)malloc(Sp * sizeof(uint64_t));
    if (!cursor) return INSHR_REF_E_ARG;
    for (uint32_t g = 0; g < Sp; g++) cursor[g] = group_off[g];
    for (uint64_t i = 0; i < n; i++) {
        int32_t diff = (int32_t)s_prev[i] - (int32_t)s_cur[i];
        uint16_t d = (uint16_t)(((diff % (int32_t)B) + (int32_t)B) % (int32_t)B);
        uint64_t r = cursor[s_prev[i]]++;
        if (delta) delta[i] = d;
        if (perm) perm[r] = (uint32_t)i;
        if (stream) stream[r] = d;
    }
    free(cursor);
    return INSHR_REF_OK;
}

int inshr_ref_reconstruct(const uint16_t *s_prev, uint32_t bits_prev, uint32_t bits_cur,
                          uint64_t n, const uint64_t *group_off, const uint16_t *stream,
                          uint16_t *s_cur)
{
    if (bits_prev < 1 || bits_prev > 8 || bits_cur < 1 || bits_cur > 8) return INSHR_REF_E_CONFIG;
    return inshr_ref_reconstruct_k(s_prev, 1u << bits_prev, 1u << bits_cur, n, group_off, stream, s_cur);
}

int inshr_ref_reconstruct_k(const uint16_t *s_prev, uint32_t K_prev, uint32_t K_cur, uint64_t n,
                            const uint64_t *group_off, const uint16_t *stream, uint16_t *s_cur)
{
    if (!s_prev || !group_off || !stream || !s_cur) return INSHR_REF_E_ARG;
    if (K_prev < 2 || K_prev > 256 || K_cur < 2 || K_cur > 256) return INSHR_REF_E_CONFIG;
    const uint32_t Sp = K_prev + 2u;
    const uint32_t Sc = K_cur + 2u;
    const uint32_t B = (Sp > Sc) ? Sp : Sc;
    uint64_t *cursor = (uint64_t *)malloc(Sp * sizeof(uint64_t));
    if (!cursor) return INSHR_REF_E_ARG;
    for (uint32_t g = 0; g < Sp; g++) cursor[g] = group_off[g];
    for (uint64_t j = 0; j < n; j++) {
        uint32_t g = s_prev[j];
        if (g >= Sp || cursor[g] >= group_off[g + 1]) {
            free(cursor);
            return INSHR_REF_E_SHAPE;
        }
        uint32_t e = stream[cursor[g]++]; /* pop the next delta of this group */
        s_cur[j] = (uint16_t)((g + B - e) % B);
    }
    free(cursor);
    return INSHR_REF_OK;
}

int inshr_ref_pack(const uint16_t *v, uint64_t n, uint32_t w, uint64_t *words)
{
    if (!v || !words || w < 1 || w > 16) return INSHR_REF_E_ARG;
    const uint64_t n_words = (n * w + 63) / 64;
    for (uint64_t k = 0; k < n_words; k++) words[k] = 0;
    for (uint64_t i = 0; i < n; i++) {
        if ((uint32_t)v[i] >> w) return INSHR_REF_E_ARG;
        for (uint32_t b = 0; b < w; b++) {
            uint64_t pos = i * w + b;
            if ((v[i] >> b) & 1u) words[pos / 64] |= 1ull << (pos % 64);
        }
    }
    return INSHR_REF_OK;
}

int inshr_ref_unpack(const uint64_t *words, uint64_t n, uint32_t w, uint16_t *v)
{
    if (!v || !words || w < 1 || w > 16) return INSHR_REF_E_ARG;
    for (uint64_t i = 0; i < n; i++) {
        uint16_t s = 0;
        for (uint32_t b = 0; b < w; b++) {
            uint64_t pos = i * w + b;
            if ((words[pos / 64] >> (pos % 64)) & 1ull) s |= (uint16_t)(1u << b);
        }
        v[i] = s;
    }
    return INSHR_REF_OK;
}
