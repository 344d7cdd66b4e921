/*
 * inshr_ref -- CPU oracle for the checkpoint-compressor hot path (TEST INFRASTRUCTURE ONLY).
 *
 * A plain, slow, single-threaded C implementation of what the path computes, written from the
 * paper's definitions: magnitude ranking (Sec. 4.1), prune / protect / quantize partition
 * (Sec. 4.2), non-uniform bins with one centre per bin (Sec. 4.4, frequency-only reading with
 * one centre update), the search for the most compact configuration that meets the error
 * threshold (Sec. 5), cyclic delta of integer codes (Sec. 6, "Calculating Delta") and the
 * regrouping by the previous checkpoint's bucket (Sec. 6, "Parameter Rearrangement",
 * Algorithms 5 and 6).
 *
 * Nothing in the product path may include, link or call this file.  It shares no code with the
 * HIP implementation.  All pointers are HOST pointers.  All order comparisons are made on
 * integer images of the floats (see inshr_ref.c), sums are fp64 in ascending index order.
 *
 * Parity pins live in tests/test_oracle_*.py (closed forms, library sort/searchsorted,
 * pure-Python brute force, invariants).  No function here is "parity unpinned".
 */
#ifndef INSHR_REF_H
#define INSHR_REF_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    INSHR_REF_OK = 0,
    INSHR_REF_E_ARG = -1,       /* null pointer, n == 0, n >= 2^32 */
    INSHR_REF_E_CONFIG = -2,    /* bits outside 1..8 or prune_ppm + outlier_ppm >= 1e6 */
    INSHR_REF_E_NONFINITE = -3, /* NaN or Inf in the input */
    INSHR_REF_E_SHAPE = -5,
    INSHR_REF_E_EMPTY = -7      /* pooled thresholds leave the tensor without quantized values */
};

typedef struct {
    uint8_t bits;         /* K = 1 << bits bins, 1..8, when bins == 0 */
    uint16_t bins;        /* 0, or the number of bins K itself, 2..256: the search space of Sec. 5
                             lists bin counts (4, 6, 8, 12, 16, 32), not bit widths */
    uint32_t prune_ppm;   /* pruning fraction x 1e6   */
    uint32_t outlier_ppm; /* protection fraction x 1e6 */
} inshr_ref_config;

typedef struct {
    double sse;   /* sum over pruned of x^2 + sum over quantized of (x - centre)^2 */
    double sumsq; /* sum over all of x^2 */
    uint64_t n_pruned, n_outlier, n_kept;
    uint64_t cost_bits; /* ceil(n_kept * log2 K) + 32*n_outlier + 32*K, with log2 K in units of 2^-16
                           (n_kept * bits for K = 2^bits) */
} inshr_ref_score;

typedef struct {
    uint64_t n_pruned, n_outlier, n_kept;
    uint32_t sym_bits;          /* ceil(log2(K + 2)); bits + 1 for K = 2^bits */
    uint32_t tau_prune_bits;    /* magnitude image (bits & 0x7fffffff) of the prune threshold   */
    uint32_t tau_outlier_bits;  /* magnitude image of the protection threshold                 */
    double sse, sumsq;
} inshr_ref_qinfo;

/* Quantize one tensor with one configuration.
 *   sym        [n]      out: symbol per element, 0 pruned, 1 protected, 2+bin quantized
 *   boundaries [K-1]    out: interior bin boundaries t_1..t_{K-1} as floats
 *   codebook   [K]      out: one centre per bin
 *   out_idx/out_val [n_outlier_cap] out: protected (index ascending, original value); may be NULL
 *                       when the configuration protects nothing; capacity floor(n*ppm/1e6)
 */
int inshr_ref_quantize(const float *x, uint64_t n, const inshr_ref_config *cfg, uint16_t *sym,
                       float *boundaries, float *codebook, uint32_t *out_idx, float *out_val,
                       inshr_ref_qinfo *info);

/* Sec. 4.2 keeps the protected values in bfloat16: the value rounded to nearest even on the upper
 * 16 bits of its fp32 image (returned as a float whose lower 16 bits are zero). */
float inshr_ref_bf16_round(float x);

/* Score every configuration of a grid independently and choose (Sec. 5): among configurations
 * with sse/sumsq <= eps the least cost_bits, ties to the lowest grid index; if none, the least
 * sse and *feasible = 0.  scores may be NULL. */
int inshr_ref_search(const float *x, uint64_t n, const inshr_ref_config *grid, uint32_t n_cfg,
                     double eps, uint32_t *best, uint8_t *feasible, inshr_ref_score *scores);

/* Per-layer-type partition (Sec. 4.2, "Pruning": the same pruning fraction across all layers of a
 * given type): the thresholds are order statistics of the pooled magnitudes of all tensors of the
 * type, pool[0..n_pool) = their magnitude images in ascending order (this tensor's among them):
 * tau_p = pool[floor(n_pool * prune_ppm / 1e6)], tau_o = pool[n_pool - 1 - floor(n_pool *
 * outlier_ppm / 1e6)]; the tensor is then partitioned by them (pruned <=> mag < tau_p, protected
 * <=> mag > tau_o) and its quantized values are binned as before.  The protected fraction of one
 * tensor is no longer bounded by the configuration: out_idx / out_val need room for n entries.
 * INSHR_REF_E_EMPTY when the thresholds leave the tensor no quantized value.  pool == NULL: the
 * tensor alone. */
int inshr_ref_quantize_pooled(const float *x, uint64_t n, const uint32_t *pool, uint64_t n_pool,
                              const inshr_ref_config *cfg, uint16_t *sym, float *boundaries,
                              float *codebook, uint32_t *out_idx, float *out_val, inshr_ref_qinfo *info);
int inshr_ref_search_pooled(const float *x, uint64_t n, const uint32_t *pool, uint64_t n_pool,
                            const inshr_ref_config *grid, uint32_t n_cfg, double eps, uint32_t *best,
                            uint8_t *feasible, inshr_ref_score *scores);

/* Partition by magnitude and sensitivity (Sec. 4.1, 4.2).  g[i] is the gradient of the loss with
 * respect to x[i]; the sensitivity score is s_i = |g_i * x_i|, one fp32 multiplication.
 *   protected <=> |x_i| > tau_om  or  s_i > tau_os, where tau_om and tau_os are the values of rank
 *                 n - 1 - floor(n * outlier_ppm / 1e6) of the magnitudes and of the scores ("a small
 *                 fraction of both the highest magnitude and sensitivity parameters");
 *   pruned    <=> not protected and m_i < tau_p, where m is the pruning metric (the magnitudes, or
 *                 the scores when prune_by_sensitivity != 0) and tau_p its value of rank
 *                 floor(n * prune_ppm / 1e6);
 *   everything else is quantized: bins, centres, symbols and errors as in inshr_ref_quantize, over
 *   these values.  info->tau_prune_bits is the bit image of tau_p (a magnitude image or a score),
 *   tau_outlier_bits that of tau_om; *tau_outlier_sens_bits receives that of tau_os.
 * out_idx / out_val need room for n entries.  INSHR_REF_E_EMPTY when nothing is left to quantize,
 * INSHR_REF_E_NONFINITE also for a non-finite gradient or score. */
int inshr_ref_quantize_sens(const float *x, const float *g, uint64_t n, const inshr_ref_config *cfg,
                            int prune_by_sensitivity, uint16_t *sym, float *boundaries, float *codebook,
                            uint32_t *out_idx, float *out_val, inshr_ref_qinfo *info,
                            uint32_t *tau_outlier_sens_bits);

/* Decode symbols back to floats: 0 -> +0.0, 1 -> listed original value, 2+b -> codebook[b]. */
int inshr_ref_dequantize(const uint16_t *sym, uint64_t n, uint32_t bits, const float *codebook,
                         const uint32_t *out_idx, const float *out_val, uint64_t n_outlier,
                         float *xhat);

/* Cyclic delta of symbols and regrouping by the previous checkpoint's symbol.
 *   delta     [n]  out: d[i] = (s_prev[i] - s_cur[i]) mod B, B = max(K_prev,K_cur) + 2 (may be NULL)
 *   perm      [n]  out: indices in stable order of s_prev (may be NULL)
 *   group_off [(1<<bits_prev)+3] out: group_off[g] = #{i : s_prev[i] < g}
 *   stream    [n]  out: stream[r] = d[perm[r]]
 */
int inshr_ref_delta(const uint16_t *s_prev, uint32_t bits_prev, const uint16_t *s_cur,
                    uint32_t bits_cur, uint64_t n, uint16_t *delta, uint32_t *perm,
                    uint64_t *group_off, uint16_t *stream);

/* Inverse of the regrouping + delta (Algorithm 6 with the sign of the delta formula):
 * walks positions in index order and pops the next delta of the previous symbol's group. */
int inshr_ref_reconstruct(const uint16_t *s_prev, uint32_t bits_prev, uint32_t bits_cur,
                          uint64_t n, const uint64_t *group_off, const uint16_t *stream,
                          uint16_t *s_cur);

/* The same three with the numbers of bins K (2..256) given directly instead of as 2^bits. */
int inshr_ref_dequantize_k(const uint16_t *sym, uint64_t n, uint32_t K, const float *codebook,
                           const uint32_t *out_idx, const float *out_val, uint64_t n_outlier,
                           float *xhat);
int inshr_ref_delta_k(const uint16_t *s_prev, uint32_t K_prev, const uint16_t *s_cur, uint32_t K_cur,
                      uint64_t n, uint16_t *delta, uint32_t *perm, uint64_t *group_off,
                      uint16_t *stream);
int inshr_ref_reconstruct_k(const uint16_t *s_prev, uint32_t K_prev, uint32_t K_cur, uint64_t n,
                            const uint64_t *group_off, const uint16_t *stream, uint16_t *s_cur);
/* Width of a symbol stream with K bins: the smallest w with 2^w >= K + 2. */
uint32_t inshr_ref_symbol_bits(uint32_t K);

/* Little-endian bit stream: value i occupies bits [i*w, (i+1)*w) of the u64 word array,
 * tail zero-padded.  words must hold ceil(n*w/64) entries. */
int inshr_ref_pack(const uint16_t *v, uint64_t n, uint32_t w, uint64_t *words);
int inshr_ref_unpack(const uint64_t *words, uint64_t n, uint32_t w, uint16_t *v);

#ifdef __cplusplus
}
#endif
#endif
