// Descriptors of the sketch-based boundary rule (kernels in inshr_sketch.hip, tables and
// sequencing in inshr_api.hip).
#pragma once
#include "inshr_launch.h"

namespace inshr {

constexpr int SK_CELLS = 16384;            // magnitude >> 17: sign-free exponent and 6 mantissa bits
constexpr int SK_MAX_IDX = 9728;           // most bucket indices per sign (alpha = 0.01 needs 9604)
constexpr int SK_HIST = 2 * SK_MAX_IDX + 1; // positive buckets, negative buckets, zeros
constexpr int SK_LDS = 4096;               // longest bucket list that the clustering keeps in LDS
constexpr int SK_SETS = 7;                 // sets of centres of a search over the bits: 2 .. 8 bits
constexpr int SK_EDGES = 501;              // boundaries of all sets: sum of 2^b - 1
constexpr int SK_SLOTS = 512;              // stride of the per-slot arrays (SK_EDGES + 1 slots)
constexpr int SK_COPIES = 4;               // LDS copies of the slot moments in the scoring sweep (power of two)

struct SketchDesc { // one tensor of the batch
    u32 active;     // part of the call
    u32 cfg;        // its configuration in the grid of the search state (thresholds, bits)
};
struct SketchInfo {
    u32 n_buckets;  // non-empty buckets
    u32 rounds;     // Lloyd rounds that changed the centres
};
struct SketchChoice { // result of the search over the bits, per tensor
    double sse[SK_SETS];   // squared error with 2 .. 8 bits
    double sumsq;
    u32 rounds[SK_SETS];
    u32 best_bits, feasible;
};
struct SketchParams {
    double sigma;
    u32 max_iter;
    u32 n_idx;             // bucket b stands for index i_lo + b
    const u32 *cell;       // [SK_CELLS] first bucket of the cell << 17 | 2^17 - 1 - low bits of that bucket's largest magnitude
    const u32 *tops;       // [n_idx] magnitude image of the largest fp32 number <= gamma^(i_lo + b)
    const double *rep;     // [n_idx] 2 gamma^(i_lo + b) / (gamma + 1)
    const double *uniforms; // [nT][256] the random numbers of the draws
    u32 *hist;             // [nT][SK_HIST], zero on entry
    double *xq, *w, *d;    // [nT][SK_HIST] bucket values, weights, squared distances
    u32 *alt_key;          // [nT][256] boundary keys where the quantizer looks for them
    float *alt_cb;         // [nT][256] codebook
    SketchInfo *info;      // [nT]
    // search over the bits (multi != 0): alt_key / alt_cb hold SK_SETS rows of 256 per tensor
    u32 multi;
    u32 light;             // the search state is a light one: this sweep also takes the protected counts
                           // per tile and their sum of squares, and the choice sums the squares itself
    double eps;            // bound on sse / sumsq
    u32 *set_rounds;       // [nT][SK_SETS]
    u32 *slot_cnt;         // [nT][SK_SLOTS] values per slot between all boundaries, zero on entry
    double *slot_sx;       // [nT][SK_SLOTS] their sums, zero on entry
    u32 *slot_edge;        // [nT][SK_SLOTS] the sorted boundaries
    SketchChoice *choice;  // [nT]
    u32 *final_key;        // [nT][256] the chosen set, where the quantizer looks for it
    float *final_cb;       // [nT][256]
};

hipError_t launch_sketch(const Batch &bt, const SketchDesc *sd, const SketchParams &P, hipStream_t s);
// The sketch as the quantile estimator (Sec. 4.3): histogram of all magnitudes of a tensor by bucket,
// then the bucket that holds a rank.
constexpr int SK_MAG_HIST = SK_MAX_IDX + 1;  // zeros at 0, bucket b at 1 + b
constexpr int SK_MAG_CHUNK = 65536;          // elements per workgroup
struct MagDesc {
    const float *x;
    u64 n;
    u64 chunk0; // first chunk of this tensor in the call-wide numbering
    u32 aligned16, pad;
};
hipError_t launch_sketch_quantiles(const MagDesc *md, int nT, u64 n_chunks, int n_wg, const u32 *cell, const u32 *tops,
                                   const double *rep, u32 n_idx, u32 *hist, u32 *nonfinite,
                                   const u64 *ranks, u32 n_q, double *est, hipStream_t s);


} // namespace inshr
