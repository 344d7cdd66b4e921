/*
 * inshr.h -- C ABI of the MI355X checkpoint-compressor hot path.
 *
 * Three operations on fp32 tensors that live in device memory, following the paper's statement
 * of the problem (System Overview: a configuration goes in; integer codes, bin centres and
 * protected values come out; previous and current codes give delta groups):
 *
 *   inshr_search    Quantization Config Manager (Sec. 5): score every configuration of a grid on
 *                   every tensor in one sweep and pick, per tensor, the most compact one whose
 *                   relative squared error stays within eps.
 *   inshr_quantize  Quantizer (Sec. 4): prune / protect / quantize partition by magnitude
 *                   (Sec. 4.1-4.2) with exact quantile thresholds (Sec. 4.3, alpha -> 0),
 *                   K = 2^bits equal-frequency bins and one centre per bin (Sec. 4.4), emitted as
 *                   bit-packed symbols + codebook + protected-value list.
 *   inshr_delta     Delta Encoder (Sec. 6): cyclic difference of symbols against the previous
 *                   checkpoint, regrouped by the previous checkpoint's symbol (Algorithm 5).
 * and their inverses for the restore side: inshr_reconstruct (Algorithm 6) and inshr_dequantize;
 * inshr_quantize_sketch is the Quantizer with the paper's own bins (log-space sketch, Algorithm 1,
 * and weighted K-Means on its buckets, Algorithms 2 and 3), inshr_search_sketch the search for the
 * fewest such bins that keep the error within eps (Sec. 5, over the number of bins).
 *
 * Conventions
 *   - Every function returns 0 on success or a negative INSHR_E_* code; nothing aborts or throws.
 *     Outputs are undefined after an error.
 *   - "device" pointers are HIP device allocations on the context's GPU, "host" pointers are
 *     ordinary host memory.  The caller allocates and owns every buffer; the library never frees
 *     caller memory and keeps no caller pointer after a call returns.
 *   - All work is enqueued on the context's stream.  inshr_search and inshr_quantize return
 *     after that work has completed (they read small results back); inshr_delta returns after
 *     enqueueing, use inshr_sync before reading its outputs on the host.
 *   - Calls on one context must not overlap in time (the context owns scratch memory).
 *   - Order comparisons use integer images of the floats: -0.0 counts as +0.0, denormals are
 *     ordinary values, NaN / Inf are rejected with INSHR_E_NONFINITE.
 *   - Symbols: 0 = pruned, 1 = protected, 2 + bin = quantized.  A symbol stream is a little-endian
 *     bit stream in u64 words: symbol i occupies bits [i*w, (i+1)*w), tail bits are zero.
 */
#ifndef INSHR_H
#define INSHR_H
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    INSHR_OK = 0,
    INSHR_E_ARG = -1,       /* null / misaligned pointer, n == 0, n >= 2^32, zero counts          */
    INSHR_E_CONFIG = -2,    /* bits outside 1..8, prune_ppm + outlier_ppm >= 1e6, grid too large  */
    INSHR_E_NONFINITE = -3, /* NaN or Inf found in a tensor                                       */
    INSHR_E_CAPACITY = -4,  /* a caller buffer or the context scratch is too small                */
    INSHR_E_SHAPE = -5,     /* prev.n != cur.n, or reuse requested without a matching search      */
    INSHR_E_DEVICE = -6,    /* a HIP call failed; inshr_last_device_error gives its text          */
    INSHR_E_INTERNAL = -7   /* a self-check inside the kernels failed (a bug, never bad input)    */
};

/* Most distinct (prune_ppm, outlier_ppm) pairs, and most distinct values of either, in one grid. */
#define INSHR_MAX_PAIRS 15
#define INSHR_MAX_FRACTIONS 8

typedef struct inshr_ctx inshr_ctx; /* opaque: one device, one stream, scratch memory */

/* device: HIP device ordinal.  hip_stream: a hipStream_t or NULL for the default stream.
 * scratch_bytes: largest single device allocation the context may make for its scratch (0 = no
 * limit).  A search over tensors of N elements in total needs about 8*N bytes plus about 1.5 MB per
 * tensor; a call that needs more than the limit returns INSHR_E_CAPACITY.
 * Environment read here (test and tuning switches; results never depend on them):
 * INSHR_SAMPLE_MIN_N (default 16777216): tensors with at least this many elements read one tile in
 * eight in the first sweep of a search and predict where the thresholds fall (a wrong prediction
 * repeats the exact sweeps for that tensor); INSHR_SAMPLE_FORCE_MISS=1 treats every prediction as
 * wrong; INSHR_SAMPLE_DEBUG=1 prints how many tensors were sampled and repeated;
 * INSHR_NO_LDS_ORDER=1 selects the ballot-ranked paths of the group sort and the delta scatter. */
int inshr_create(inshr_ctx **out, int device, void *hip_stream, uint64_t scratch_bytes);
void inshr_destroy(inshr_ctx *ctx);
const char *inshr_strerror(int code);
const char *inshr_last_device_error(const inshr_ctx *ctx);
int inshr_sync(inshr_ctx *ctx);
/* 1 when the context ranks equal symbols (delta regrouping, group sort of the search) with one
 * returning LDS add per element, which needs same-address LDS atomics to be served in lane order:
 * checked on the device when the context is created and cross-checked against ballot ranks inside
 * the kernels on a quarter of the tiles; 0 when the ballot-ranked kernels are in use
 * (INSHR_NO_LDS_ORDER=1, or the check at creation failed). */
int inshr_lds_ordered(const inshr_ctx *ctx);

typedef struct {
    uint8_t bits;         /* 1..8; K = 1 << bits bins (when bins == 0)               */
    uint16_t bins;        /* 0, or the number of bins K itself (Sec. 5 lists counts: 4, 6, 8, 12, 16,
                             32): a power of two up to 256, or 3, 6, 12; bits is then ignored  */
    uint32_t prune_ppm;   /* pruning fraction x 1e6 (floor(n*ppm/1e6) smallest |x|)  */
    uint32_t outlier_ppm; /* protection fraction x 1e6 (largest |x|); sum < 1e6      */
} inshr_config;
/* Symbols take the smallest w with 2^w >= K + 2 bits (bits + 1 for K = 2^bits). */

typedef struct {
    const float *data; /* device, 4-byte aligned, read-only, caller-owned */
    uint64_t n;        /* 1 <= n < 2^32 */
} inshr_tensor;

typedef struct {
    double sse;   /* sum_pruned x^2 + sum_quantized (x - centre)^2, fp64 */
    double sumsq; /* sum_all x^2 */
    uint64_t n_pruned, n_outlier, n_kept;
    uint64_t cost_bits; /* payload model used to rank configs: ceil(n_kept * log2 K) + 32*n_outlier +
                           32*K, log2 K taken in units of 2^-16 (n_kept * bits for K = 2^bits)       */
} inshr_score;

/* Score all n_cfg configurations on each of n_tensors tensors (Sec. 5).
 *   best     host [n_tensors]: chosen grid index.  Feasible = sse/sumsq <= eps (0/0 counts as 0);
 *            among feasible the least cost_bits, ties to the lowest index; if none is feasible
 *            the least sse (ties lowest index) and feasible = 0.
 *   feasible host [n_tensors]
 *   scores   host [n_tensors * n_cfg] row-major by tensor, or NULL. */
int inshr_search(inshr_ctx *ctx, const inshr_tensor *tensors, uint32_t n_tensors,
                 const inshr_config *grid, uint32_t n_cfg, double eps, uint32_t *best,
                 uint8_t *feasible, inshr_score *scores);

/* inshr_search with thresholds per layer type (Sec. 4.2, "Pruning": the same pruning fraction
 * across all layers of a given type).  group: host array, one number per tensor; tensors with
 * equal numbers form a group, and a group's prune / protect thresholds are the order statistics
 * of its pooled magnitudes: tau_p = the value of rank floor(N * prune_ppm / 1e6) among all N values
 * of the group, tau_o that of rank N - 1 - floor(N * outlier_ppm / 1e6).  Every tensor is then
 * partitioned by its group's thresholds and binned, scored and chosen as in inshr_search (a group of
 * one tensor is inshr_search).  Limits: a group holds fewer than 2^32 values; the first sweep of
 * grouped tensors is never sampled.  A tensor's share of the protected values is no longer bounded
 * by the fraction: size outlier buffers from the scores' n_outlier (inshr_quantize with
 * INSHR_REUSE_SEARCH reports INSHR_E_CAPACITY otherwise).  INSHR_E_CONFIG when the thresholds of
 * some (prune, protect) pair leave a tensor without quantized values (inshr_last_device_error
 * names it).  Stand-alone inshr_quantize knows no groups. */
int inshr_search_pooled(inshr_ctx *ctx, const inshr_tensor *tensors, const uint32_t *group,
                        uint32_t n_tensors, const inshr_config *grid, uint32_t n_cfg, double eps,
                        uint32_t *best, uint8_t *feasible, inshr_score *scores);

typedef struct {
    /* caller-allocated device buffers */
    uint64_t *packed;       /* symbol stream, packed_words words (inshr_quantize_bound)          */
    uint64_t packed_words;
    float *codebook;        /* >= 256 floats; first K are written                                 */
    float *boundaries;      /* >= 255 floats or NULL; first K-1 interior bin boundaries           */
    uint32_t *outlier_idx;  /* protected indices, ascending; capacity outlier_cap (may be NULL    */
    float *outlier_val;     /*   when outlier_cap == 0); original values, bit-exact (or bfloat16, see
                                 INSHR_PROTECT_BF16)                                              */
    uint64_t outlier_cap;
    /* filled by the call (host side) */
    uint64_t n_pruned, n_outlier, n_kept;
    uint32_t sym_bits;      /* width of a symbol: bits + 1 for K = 2^bits */
    float tau_prune;        /* pruned    <=> |x| <  tau_prune   */
    float tau_outlier;      /* protected <=> |x| >  tau_outlier */
    uint32_t n_bins;        /* K */
} inshr_quantized;

/* Sizes of the buffers inshr_quantize needs for a tensor of n elements. */
int inshr_quantize_bound(uint64_t n, const inshr_config *cfg, uint64_t *packed_words,
                         uint64_t *outlier_cap);

#define INSHR_REUSE_SEARCH 1u /* thresholds / boundaries / centres come from the last inshr_search
                                 on this context, which must have covered exactly these tensors
                                 (same pointers, sizes, order) and contained each cfg[i] in its
                                 grid; the data must not have changed since */

#define INSHR_PROTECT_BF16 2u  /* protected values are stored in bfloat16 (Sec. 4.2): out[i].outlier_val
                                 then receives outlier_cap uint16_t values, the fp32 value rounded to
                                 nearest even on its upper 16 bits (a magnitude above the largest
                                 finite bfloat16 becomes infinity, as the format defines).  Scores of
                                 inshr_search count protected values as exact either way. */

/* Quantize tensors[i] with cfg[i] into out[i] (arrays of n_tensors entries, host). */
int inshr_quantize(inshr_ctx *ctx, const inshr_tensor *tensors, const inshr_config *cfg,
                   inshr_quantized *out, uint32_t n_tensors, uint32_t flags);

typedef struct {
    const uint64_t *packed; /* device symbol stream */
    uint32_t sym_bits;      /* width of a symbol: bits + 1, or what n_bins of inshr_quantized implies */
    uint8_t bits;           /* K = 1 << bits when bins == 0 */
    uint16_t bins;          /* 0, or the number of bins K (2 .. 256) */
    uint64_t n;
} inshr_codes;

typedef struct {
    uint64_t *packed;       /* device, packed_words words (inshr_delta_bound): stream e[r]        */
    uint64_t packed_words;
    uint64_t *group_off;    /* device, K_prev + 3 entries: #{i : s_prev[i] < g}                    */
    uint32_t *perm;         /* device [n] or NULL: perm[r] = index of the r-th regrouped element   */
    uint32_t delta_bits;    /* filled: width of a symbol of the side with more bins                */
    uint32_t group_off_entries; /* capacity of group_off in entries, or 0 = not stated; a stated
                                   capacity below (1 << prev.bits) + 3 gives INSHR_E_CAPACITY      */
} inshr_delta_out;

int inshr_delta_bound(const inshr_codes *prev, const inshr_codes *cur, uint64_t *packed_words);

/* d[i] = (s_prev[i] - s_cur[i]) mod B, B = max(K_prev, K_cur) + 2; elements are regrouped in the
 * stable order of s_prev (Algorithm 5): e[r] = d[perm[r]].  Arrays have n_tensors entries (host).
 * prev_perm: NULL, or host array of n_tensors device pointers (entries may be NULL) holding the
 * permutation of a previous call for the same prev codes; when given it is used instead of being
 * recomputed (out[t].perm must then be NULL: INSHR_E_ARG).  The call returns after enqueueing; what
 * its kernels find wrong is reported by the next inshr_sync or inshr_delta on the context:
 * INSHR_E_ARG when a given permutation holds an index outside its tensor (those elements are left
 * out of the stream), INSHR_E_INTERNAL when the device did not rank equal symbols in order (see
 * inshr_lds_ordered). */
int inshr_delta(inshr_ctx *ctx, const inshr_codes *prev, const uint32_t *const *prev_perm,
                const inshr_codes *cur, inshr_delta_out *out, uint32_t n_tensors);

/* inshr_delta for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same operation, arguments and outputs as inshr_delta without
 * prev_perm, but the call allocates nothing on the device or through HIP (no hipMalloc, hipFree,
 * pinned staging or memset node): the descriptors travel as kernel arguments and all scratch (chunk
 * table, per-chunk symbol populations, flag word) is a static device array of about 2.2 MB that every
 * GPU the library runs on holds until the process ends.  Limits: at most INSHR_STATIC_MAX_TENSORS
 * tensors per call and INSHR_STATIC_MAX_ELEMENTS elements in total, each tensor rounded up to whole
 * chunks of 786432 elements; beyond them the call returns INSHR_E_CAPACITY (inshr_last_device_error
 * says which limit).  All calls on one GPU share the array, which keeps the last call's contents:
 * calls that overlap in time on one GPU (two contexts, two streams) race; calls on one stream do
 * not.  Only kernel launches are enqueued on the context's stream and the call returns at once;
 * errors found by the kernels are reported by the next inshr_sync / inshr_delta, as for inshr_delta.
 * Per-kernel timing (inshr_profile) must be off where event creation is not allowed. */
#define INSHR_STATIC_MAX_TENSORS 16
#define INSHR_STATIC_MAX_ELEMENTS (2048ull * 786432ull)
int inshr_delta_static(inshr_ctx *ctx, const inshr_codes *prev, const inshr_codes *cur,
                       inshr_delta_out *out, uint32_t n_tensors);

/* ---- partition by magnitude and sensitivity (Sec. 4.1, 4.2) --------------------------------- */

typedef struct {
    float tau_outlier_sens; /* protect threshold of the sensitivity score                          */
    double sse, sumsq;      /* error of the decoded tensor as inshr_score defines it, sum of x^2   */
} inshr_sens_info;

/* One configuration per tensor, with gradients: grads[t] (device, n floats, 4-byte aligned) is the
 * gradient of the loss with respect to tensors[t].  The sensitivity score of an element is
 * s = |g * x| (one fp32 multiplication).  protected <=> |x| > tau_om or s > tau_os, the values of
 * rank n - 1 - floor(n * outlier_ppm / 1e6) of the magnitudes and of the scores; pruned <=> not
 * protected and m < tau_p, where m is the pruning metric (the magnitude, or the score where
 * prune_by_sensitivity[t] != 0; the array may be NULL) and tau_p its value of rank
 * floor(n * prune_ppm / 1e6); the rest is quantized with equal-frequency bins over exactly these
 * values.  out as for inshr_quantize (tau_prune is the image of tau_p in its metric, tau_outlier is
 * tau_om); up to 2 * floor(n * outlier_ppm / 1e6) values can be protected, and outlier_cap must hold
 * them (INSHR_E_CAPACITY).  info may be NULL.  The call synchronises, runs three searches inside
 * (thresholds of the scores, thresholds of the weights, bins of the quantized values) and leaves no
 * state for INSHR_REUSE_SEARCH.  INSHR_E_NONFINITE also for a non-finite gradient or score,
 * INSHR_E_CONFIG when a tensor is left without quantized values or the call names more distinct
 * fractions than one grid takes. */
int inshr_quantize_sens(inshr_ctx *ctx, const inshr_tensor *tensors, const float *const *grads,
                        const inshr_config *cfg, const uint8_t *prune_by_sensitivity,
                        inshr_quantized *out, inshr_sens_info *info, uint32_t n_tensors);

/* ---- restore side ------------------------------------------------------------------------- */

typedef struct {
    const uint64_t *packed;      /* device symbol stream, (bits + 1)-bit symbols                  */
    const float *codebook;       /* device, 1 << bits bin centres                                 */
    const uint32_t *outlier_idx; /* device, n_outlier ascending indices (may be NULL if 0)        */
    const float *outlier_val;    /* device, their original values                                 */
    uint64_t n_outlier;
    uint64_t n;
    uint8_t bits;                /* K = 1 << bits when bins == 0 */
    uint8_t protected_bf16;      /* nonzero: outlier_val holds uint16_t bfloat16 values (INSHR_PROTECT_BF16) */
    uint16_t bins;               /* 0, or the number of bins K (2 .. 256) */
} inshr_dequant_in;

/* Inverse of the Quantizer (Sec. 4): out[t][i] = +0.0 for symbol 0, the protected value for symbol
 * 1 and codebook[s - 2] for symbol s >= 2.  out: host array of n_tensors device pointers, each to n
 * floats (4-byte aligned).  Returns after the work has completed.  INSHR_E_ARG: a symbol above
 * K + 1; INSHR_E_SHAPE: the elements with symbol 1 are not exactly the listed indices (or these are
 * not ascending). */
int inshr_dequantize(inshr_ctx *ctx, const inshr_dequant_in *in, float *const *out,
                     uint32_t n_tensors);

typedef struct {
    uint64_t *packed;      /* device, receives the symbols of the current checkpoint              */
    uint64_t packed_words; /* >= ceil(n * symbol width / 64)                                        */
    uint8_t bits;          /* bits of the current checkpoint's configuration (when bins == 0)      */
    uint16_t bins;         /* 0, or its number of bins K (2 .. 256)                                */
} inshr_codes_out;

/* Inverse of the Delta Encoder (Sec. 6, Algorithm 6): element i, whose previous symbol is g, takes
 * the next delta e of group g in the stream and becomes (g - e) mod B.  delta[t] is what
 * inshr_delta wrote for the same prev codes: packed, packed_words and delta_bits are read; group_off
 * (may be NULL) is compared with the offsets that prev implies; perm is not used.  Returns after the
 * work has completed.  INSHR_E_SHAPE: group offsets disagree with prev; INSHR_E_ARG: a delta >= B or
 * a result above K_cur + 1 (the stream does not belong to these codes). */
int inshr_reconstruct(inshr_ctx *ctx, const inshr_codes *prev, const inshr_delta_out *delta,
                      inshr_codes_out *cur, uint32_t n_tensors);

/* ---- the paper's own boundary rule: sketch + weighted K-Means --------------------------------- */

typedef struct {
    double alpha;           /* relative error bound of the sketch, 0.01 <= alpha <= 0.5 (Sec. 4.3)  */
    double sigma;           /* weight of the frequency term of the sample weights, 0..1 (Sec. 4.4)  */
    uint32_t max_iter;      /* most Lloyd rounds after the K-Means++ start                          */
    const double *uniforms; /* host [n_tensors * 256]: the random numbers in [0, 1) of the draws;   */
                            /* draw r of tensors[t] uses uniforms[t * 256 + r]                      */
} inshr_sketch_params;

typedef struct {
    uint32_t n_buckets; /* non-empty sketch buckets of the quantized values */
    uint32_t rounds;    /* Lloyd rounds that changed the centres            */
} inshr_sketch_info;

/* inshr_quantize with the bins of Sec. 4.3-4.4 instead of equal-frequency bins: the values that
 * are neither pruned nor protected (same exact thresholds as inshr_quantize) are counted per sketch
 * bucket (sign, ceil(log_gamma |x|)), gamma = (1 + alpha) / (1 - alpha) (Algorithm 1, no bucket
 * merging; exact zeros form a bucket of their own); a bucket stands for 2 gamma^i / (gamma + 1);
 * the buckets are clustered into K = 2^bits clusters by K-Means with sample weights
 * sigma * C / max C + (1 - sigma) * |X| / max |X| (Algorithm 2), started by weighted K-Means++
 * (Algorithm 3: squared distances; a draw with number u takes the first bucket whose running sum
 * of probabilities exceeds u times their total; when all remaining distances are zero the last
 * centre is repeated) and iterated until the memberships repeat or max_iter rounds are done.  The
 * codebook is the centres in fp32, ascending; a value takes the upper of two neighbouring centres
 * when it lies strictly above their midpoint.  out[i].boundaries receives the smallest fp32 number
 * above each midpoint.  All arithmetic of the clustering is fp64.  info (host, n_tensors entries)
 * may be NULL.  flags and everything else as inshr_quantize: with INSHR_REUSE_SEARCH the thresholds
 * come from the last inshr_search on the context, otherwise one single-configuration search per
 * distinct configuration replaces that state. */
int inshr_quantize_sketch(inshr_ctx *ctx, const inshr_tensor *tensors, const inshr_config *cfg,
                          const inshr_sketch_params *params, inshr_quantized *out,
                          inshr_sketch_info *info, uint32_t n_tensors, uint32_t flags);

/* The sketch as the quantile estimator (Sec. 4.3, Algorithm 1): one sweep counts the magnitudes of
 * every tensor per bucket of the law below; the estimate of the magnitude of rank floor(q (n - 1))
 * is the value of the bucket in which the running count (zeros first, then ascending buckets) passes
 * the rank: within a factor 1 +- alpha of the exact order statistic.  q: host array of n_q numbers in
 * [0, 1]; estimates: host array [n_tensors][n_q].  The hot path's thresholds stay exact; this call is
 * the paper's estimator on its own (prune / protect thresholds are q = prune fraction and
 * q = 1 - protect fraction).  0.01 <= alpha <= 0.5.  Synchronises. */
int inshr_sketch_quantiles(inshr_ctx *ctx, const inshr_tensor *tensors, uint32_t n_tensors, const double *q,
                           uint32_t n_q, double alpha, double *estimates);

/* Host only (no GPU work): the bucket law the sketch calls use for alpha.  Bucket index i_lo + b
 * (b = 0 .. n_buckets - 1) holds the magnitudes above tops[b - 1] up to tops[b], the largest fp32
 * number not above gamma^(i_lo + b), and stands for values[b] = 2 gamma^(i_lo + b) / (gamma + 1).
 * tops / values: host arrays of cap entries, or NULL (then only i_lo and n_buckets are returned). */
int inshr_sketch_buckets(double alpha, int32_t *i_lo, uint32_t *n_buckets, float *tops, double *values,
                         uint32_t cap);

typedef struct {
    double sse[7];      /* squared error of the tensor with 2, 3, ..., 8 bits (fp64)          */
    double sumsq;       /* sum_all x^2                                                        */
    uint32_t rounds[7]; /* Lloyd rounds of each width                                         */
    uint32_t best_bits; /* the fewest bits with sse <= eps * sumsq; 8 when there are none ... */
    uint32_t feasible;  /* ... and then 0                                                     */
} inshr_sketch_choice;

/* The search of Sec. 5 restricted to the number of bins, with the bins of inshr_quantize_sketch:
 * for tensors[i] and the prune / protect fractions of cfg[i] (cfg[i].bits is ignored) the sketch
 * is clustered into 2^b clusters for b = 2 .. 8 (draw r of every width uses uniforms[t * 256 + r],
 * so the start of a narrower width is a prefix of the start of a wider one), every width is scored
 * exactly (sse = sum_pruned x^2 + sum_quantized (x - its centre)^2 over the tensor, one more sweep),
 * the fewest bits within eps are chosen and the tensor is quantized with them into out[i] (sized
 * for 8 bits).  choice: host, n_tensors entries.  info: host, n_tensors entries or NULL (n_buckets,
 * and the Lloyd rounds of the 8-bit set).  With INSHR_REUSE_SEARCH the grid of the last
 * inshr_search must hold the tensor's fractions with every width from 2 to 8 bits. */
int inshr_search_sketch(inshr_ctx *ctx, const inshr_tensor *tensors, const inshr_config *cfg,
                        const inshr_sketch_params *params, double eps, inshr_quantized *out,
                        inshr_sketch_choice *choice, inshr_sketch_info *info, uint32_t n_tensors,
                        uint32_t flags);

/* The search of Sec. 5 with the bins of inshr_quantize_sketch over (prune, protect) pairs as well:
 * pairs[q] names the fractions (bits and bins ignored); every pair is searched over 2 .. 8 bits as
 * by inshr_search_sketch, one pair after the other (each costs that call's sweeps), and among all
 * (pair, width) within eps the least payload n_kept * bits + 32 * n_protected + 32 * 2^bits wins
 * (ties: the lower pair; within a pair the fewest feasible bits are the cheapest); when none is
 * within eps, the pair whose 8-bit error is least, with 8 bits.  out[t] (sized for 8 bits and the
 * largest protect fraction) receives the winner's codes, best_pair[t] its index, choice[t] the
 * winner's row; table (host, [n_tensors][n_pairs], may be NULL) all rows.  params->uniforms holds
 * 256 numbers per tensor, used for every pair. */
int inshr_search_sketch_grid(inshr_ctx *ctx, const inshr_tensor *tensors, const inshr_config *pairs,
                             uint32_t n_pairs, const inshr_sketch_params *params, double eps,
                             inshr_quantized *out, uint32_t *best_pair, inshr_sketch_choice *choice,
                             inshr_sketch_choice *table, uint32_t n_tensors);

/* ---- entropy stage of the delta (host memory only, outside the timed path) ------------------- */

typedef struct {
    uint64_t n_tokens;      /* run-length tokens of all groups                                    */
    uint64_t table_bytes;   /* group headers and code tables                                      */
    uint64_t payload_bytes; /* Huffman-coded tokens                                               */
} inshr_entropy_stats;

/* Sec. 6, "Encoding Delta": every group of the delta stream is run-length encoded (a run of r equal
 * values v becomes the token -v, followed by +r when r > 1) and Huffman coded with a code of its
 * own.  Input, all host memory: either `packed` (the stream inshr_delta wrote, copied to the host:
 * delta_bits-bit fields) or `values` (one uint16 per delta value), the other NULL; group_off with
 * n_groups + 1 entries (group g = values [group_off[g], group_off[g+1]); group_off[0] = 0,
 * group_off[n_groups] = n).  One group spanning everything encodes a stream without regrouping.
 * out (host, out_cap bytes) receives the container; *out_bytes its size.  With out == NULL or
 * out_cap too small the call returns INSHR_E_CAPACITY and *out_bytes is the size needed.
 * stats may be NULL. */
int inshr_entropy_encode(const uint64_t *packed, const uint16_t *values, uint64_t n,
                         uint32_t delta_bits, const uint64_t *group_off, uint32_t n_groups,
                         uint8_t *out, uint64_t out_cap, uint64_t *out_bytes,
                         inshr_entropy_stats *stats);

/* Inverse: the container back into `packed` (ceil(n * delta_bits / 64) words) or `values` (n
 * entries), the other NULL, and group_off (n_groups + 1 entries, may be NULL).  n, delta_bits and
 * n_groups must be those of the encoder.  INSHR_E_SHAPE: the container is malformed. */
int inshr_entropy_decode(const uint8_t *in, uint64_t in_bytes, uint64_t n, uint32_t delta_bits,
                         uint32_t n_groups, uint64_t *packed, uint16_t *values, uint64_t *group_off);

/* ---- search-space navigation (host only; Sec. 5) --------------------------------------------- */

/* The configuration cube of Sec. 5: axis 0 = number of bins, ascending; axis 1 = prune fraction,
 * descending; axis 2 = protect fraction, ascending, so that one step up along any axis raises
 * quality and cost.  Cell (i, j, k) holds the configuration whose score is
 * scores[cell_cfg[(i * dims[1] + j) * dims[2] + k]]; scores is one row of inshr_search's score
 * table (or the caller's sum of rows over a group of tensors: sse, sumsq and cost_bits add).
 * A cell is feasible when sse <= eps * sumsq.  All pointers are host memory; nothing runs on the
 * GPU.
 *
 * inshr_guided_search (Sec. 5, Alg. 4, guided exhaustive search): evaluates the diagonal of the
 * cube from its most aggressive corner, takes the cheapest feasible diagonal cell as the incumbent
 * and splits the cube at it; the part that is more conservative along every axis can only cost
 * more, the part more aggressive along every axis is infeasible when quality is monotone, and the
 * remaining parts are searched in the same way.  With scores monotone along every axis the result
 * has the least cost_bits of all feasible cells; on other tables it is the heuristic's answer.
 * *best_cell = i, j, k packed as (i << 16 | j << 8 | k), *feasible = 0 when no evaluated cell was
 * feasible (then *best_cell is the most conservative corner); *trials = distinct cells whose
 * score was read; visited (dims[0] * dims[1] * dims[2] bytes, may be NULL) is set to 1 for them.
 *
 * inshr_neighbourhood_search (Sec. 5, delta-neighbourhood search): the cells at most e steps
 * (sum over the axes) from prev_cell, without those that are at least as aggressive as prev_cell
 * along every axis and more aggressive along one, are read in ascending order of cost_bits (ties:
 * lower configuration index) until one is feasible.  *feasible = 0 when none is: the caller then
 * falls back to inshr_guided_search.  The pruning-metric probe of Sec. 5 is not part of this call
 * (one metric, the magnitude, exists here).
 *
 * Errors: INSHR_E_ARG for NULL pointers, an axis of length 0 or above 255, or prev_cell outside. */
int inshr_guided_search(const inshr_score *scores, const uint32_t *cell_cfg, const uint32_t dims[3],
                        double eps, uint32_t *best_cell, uint32_t *feasible, uint32_t *trials,
                        uint8_t *visited);
int inshr_neighbourhood_search(const inshr_score *scores, const uint32_t *cell_cfg,
                               const uint32_t dims[3], uint32_t prev_cell, uint32_t e, double eps,
                               uint32_t *best_cell, uint32_t *feasible, uint32_t *trials);

/* Per-kernel timing for benchmarks (not part of the method): when enabled, every kernel launch of
 * this process is bracketed by HIP events on its stream.  inshr_profile(ctx, 1) clears the totals
 * and starts recording, inshr_profile(ctx, 0) stops.  inshr_profile_read synchronises the stream
 * and returns the accumulated time and launch count per kernel name (*n = number of names; at most
 * cap entries are written to out, which may be NULL to query the count). */
typedef struct {
    char name[32];
    double total_ms;
    uint64_t launches;
} inshr_kernel_time;
int inshr_profile(inshr_ctx *ctx, int enable);
int inshr_profile_read(inshr_ctx *ctx, inshr_kernel_time *out, uint32_t cap, uint32_t *n);

#ifdef __cplusplus
}
#endif
#endif
