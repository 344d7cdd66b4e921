// Shared device-side definitions of the hot path: integer images of floats, the two-level
// binning of keys, per-tensor state records and wavefront helpers.  gfx950 only (64-wide waves).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint32_t u32;
typedef uint64_t u64;
typedef uint16_t u16;

// Pointers that reach a kernel through a descriptor in memory are generic to the compiler and
// would be accessed with FLAT instructions, whose completion is tracked together with LDS traffic;
// every such pointer is device memory, so it is cast to the global address space before use.
#define GLOBAL_AS __attribute__((address_space(1)))
#define LDS_AS __attribute__((address_space(3)))

namespace inshr {

template <class T>
__device__ __forceinline__ GLOBAL_AS T *gptr(T *p)
{
    return (GLOBAL_AS T *)p;
}

// ------------------------------------------------------------------------------------------
// sizes
// ------------------------------------------------------------------------------------------
constexpr int TILE = 16384;         // elements per tile: 1024 threads x 4 float4
constexpr int BLOCK = 1024;         // threads per streaming workgroup
constexpr int L1_SHIFT = 17;        // first-level bin = key >> 17 (sign, exponent, 6 mantissa bits)
constexpr int L1_BINS = 32768;
constexpr int L1_MAGBINS = 16384;   // first-level bins of the magnitude (fold of the two signs)
constexpr int COARSE_SHIFT = 20;    // second level: table indexed by key >> 20 ...
constexpr int COARSE = 4096;        // ... gives (base, depth) of a run of 2^depth bins
constexpr int L2_BINS = 32768;      // most second-level bins (LDS-resident counters)
constexpr int MAX_FRAC = 8;         // distinct prune fractions, distinct protect fractions
constexpr int MAX_THR = 2 * MAX_FRAC;
constexpr int MAX_PAIRS = 15;       // distinct (prune, protect) pairs in a grid
constexpr int NB8 = 255;            // interior boundaries at 8 bits; fewer bits use a subset
constexpr int NBT = NB8 + 8;        // ... plus the boundaries of 12 bins that are not among them (the
                                    // search space of Sec. 5 has 6 and 12 bins: 3, 6 and 12 bins nest)
constexpr int MAX_EDGES = 4096;     // merged edge list of all pairs (15 * 267 = 4005 fits)
constexpr int MAX_SUB = 4608;       // sub-slots: slots cut where the exponent changes (4006 + 511 fits)
constexpr int EPP = NBT + 4;        // edge items per pair: boundaries 0 .. NBT - 1, class edges NBT .. NBT + 3
constexpr int EIDX_STRIDE = 268;    // per-pair stride of the edge positions
constexpr int MAX_CFG = 256;
constexpr int GROUP_SHIFT = 12;     // gathered keys per group of active bins: about 2^12
constexpr int MAX_GROUPS = 8192;    // groups per tensor (the shift grows for huge tensors)
constexpr u32 INACTIVE = 0xFFFFFFFFu;
constexpr u32 RESOLVED = 0xFFFFFFFEu;
constexpr u32 ZERO_KEY = 0x80000000u;

// ------------------------------------------------------------------------------------------
// integer images (Sec. 4.1: ranking by magnitude; all order comparisons are made on these)
// ------------------------------------------------------------------------------------------
__host__ __device__ __forceinline__ u32 canon_bits(u32 b) { return b == 0x80000000u ? 0u : b; }
__host__ __device__ __forceinline__ u32 key_of_bits(u32 b)
{
    return b ^ ((u32)((int)b >> 31) | 0x80000000u); // negative: all bits flip; else the sign bit is set
}
// key of a value; -0.0 becomes +0.0 first (x + 0.0f is +0.0 for either zero, x otherwise;
// denormals are kept: the library is built without flush-to-zero)
__device__ __forceinline__ u32 key_of_float(float x) { return key_of_bits(__float_as_uint(x + 0.0f)); }
__host__ __device__ __forceinline__ u32 mag_of_key(u32 k)
{
    return (k & 0x80000000u) ? (k & 0x7fffffffu) : (~k & 0x7fffffffu);
}
__host__ __device__ __forceinline__ u32 bits_of_key(u32 k)
{
    return (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
}
__host__ __device__ __forceinline__ bool key_is_neg(u32 k) { return (k & 0x80000000u) == 0; }
// keys of +m and -m for a magnitude image m (m == 0 maps both to ZERO_KEY's neighbourhood)
__host__ __device__ __forceinline__ u32 key_pos(u32 m) { return 0x80000000u + m; }
__host__ __device__ __forceinline__ u32 key_neg(u32 m) { return 0x7fffffffu - m; }

// The four class edges of a (prune threshold tp, protect threshold to) pair on the key axis:
// 0 first quantized negative key, 1 first pruned key, 2 first quantized positive key,
// 3 first protected positive key.
__host__ __device__ __forceinline__ u32 class_edge_key(u32 which, u32 tp, u32 to)
{
    switch (which) {
    case 0: return key_neg(to);
    case 1: return key_neg(tp) + 1u;
    case 2: return key_pos(tp);
    default: return to >= 0x7fffffffu ? 0xFFFFFFFFu : key_pos(to) + 1u;
    }
}

// second-level bin of a key: table entry = bucket mask << 24 | base << 5 | depth.  Bit 31 - s of
// the entry says that first-level bin s of the 8 under this 12-bit key prefix holds a threshold.
__host__ __device__ __forceinline__ u32 l2_bin(u32 key, u32 entry)
{
#if defined(__HIP_DEVICE_COMPILE__)
    // bit-field extract takes offset and width from the low five bits of its operands
    return ((entry >> 5) & 0x7fffu) + __builtin_amdgcn_ubfe(key, (u32)COARSE_SHIFT - entry, entry);
#else
    const u32 d = entry & 31u;
    return ((entry >> 5) & 0x7fffu) + ((key >> (COARSE_SHIFT - d)) & ((1u << d) - 1u));
#endif
}
// The same table entry for kernels that index 16-bit tables by the bin: base << 6 | depth, so that
// entry >> 5 is the byte offset of the first bin and no mask is needed.
__host__ __device__ __forceinline__ u32 entry_for_u16(u32 entry)
{
    return (((entry >> 5) & 0x7fffu) << 6) | (entry & 31u);
}
__device__ __forceinline__ u32 lookup_u16(const u16 *table, u32 key, u32 entry16)
{
#if defined(__HIP_DEVICE_COMPILE__)
    // bit-field extract takes offset and width from the low five bits of its operands
    const u32 sub = __builtin_amdgcn_ubfe(key, (u32)COARSE_SHIFT - entry16, entry16);
#else
    const u32 d = entry16 & 31u;
    const u32 sub = (key >> (COARSE_SHIFT - d)) & ((1u << d) - 1u);
#endif
    return *reinterpret_cast<const u16 *>(reinterpret_cast<const char *>(table) + (entry16 >> 5) + sub * 2u);
}
// Boundary j (1 .. K - 1) of K equal-frequency bins is the quantized value of rank floor(j M / K)
// (Sec. 4.4, frequency-only reading).  A pair keeps NBT boundaries: index i < 255 is rank fraction
// (i + 1) / 256 — every power of two K up to 256 uses a subset, floor(j M / K) =
// floor(j (256 / K) M / 256) — and indices 255 .. 262 are the twelfths 1, 2, 4, 5, 7, 8, 10, 11 / 12
// for K = 3, 6, 12 (the twelfths 3, 6, 9 are 64, 128, 192 / 256).
__host__ __device__ __forceinline__ bool bins_supported(u32 K)
{
    return K >= 2u && K <= 256u && ((K & (K - 1u)) == 0u || K == 3u || K == 6u || K == 12u);
}
__host__ __device__ __forceinline__ u32 bnd_index(u32 K, u32 j)
{
    if ((K & (K - 1u)) == 0u) return j * (256u / K) - 1u;
    const u32 jj = j * (12u / K);
    if (jj % 3u == 0u) return (jj / 3u) * 64u - 1u;
    return 255u + (jj - jj / 3u - 1u);
}
__host__ __device__ __forceinline__ void bnd_fraction(u32 i, u32 &num, u32 &den)
{
    if (i < (u32)NB8) {
        num = i + 1u;
        den = 256u;
    } else {
        const u32 k = i - (u32)NB8; // 0 .. 7 -> 1, 2, 4, 5, 7, 8, 10, 11
        num = k + k / 2u + 1u;
        den = 12u;
    }
}
// width of a symbol stream with K bins: pruned, protected and K bins need K + 2 levels (Sec. 6)
__host__ __device__ __forceinline__ u32 symbol_bits(u32 K)
{
    u32 w = 1u;
    while ((1u << w) < K + 2u) w++;
    return w;
}

__host__ __device__ __forceinline__ u32 bucket_flag(u32 l1_bin) { return 0x80000000u >> (l1_bin & 7u); }
__host__ __device__ __forceinline__ bool in_threshold_bucket(u32 key, u32 entry)
{
    return (int)(entry << ((key >> L1_SHIFT) & 7u)) < 0;
}

// ------------------------------------------------------------------------------------------
// per-tensor records
// ------------------------------------------------------------------------------------------
struct TDesc {           // one tensor of a batch
    const float *data;
    u64 n;
    u64 tile0;           // first tile of this tensor in the batch-wide tile numbering
    u64 pool_grp;        // where this tensor's keys in bin-group order go in the first pool (u32 units):
                         // the span of the tensor's (workgroup, tensor) units there, ...
    u64 pool_len;        // ... and its length
    u32 aligned16;       // data pointer is 16-byte aligned (float4 loads allowed)
    u32 sampled;         // sweep 1 reads one tile in SAMPLE_RATE (large tensors): its histogram only
                         // shapes the second-level table and predicts where the thresholds lie
    // thresholds per layer type (Sec. 4.2): the tensors of a group share the thresholds, which are
    // order statistics of the group's pooled magnitudes
    u32 leader;          // first tensor of this tensor's group (itself when it stands alone)
    u32 pooled;          // the group has more than one tensor
    u64 n_pool;          // elements of the whole group
};
constexpr int SAMPLE_RATE = 8;

struct GridDesc {        // the configuration grid, decomposed
    u32 n_cfg, n_pairs, n_p, n_o;
    u32 p_ppm[MAX_FRAC], o_ppm[MAX_FRAC];     // distinct fractions
    u32 pair_p[MAX_PAIRS], pair_o[MAX_PAIRS]; // indices into p_ppm / o_ppm
    u32 cfg_pair[MAX_CFG];
    u32 cfg_bits[MAX_CFG];                    // (meaningful for K = 2^bits only)
    u32 cfg_K[MAX_CFG];                       // number of bins
    u32 cfg_l16[MAX_CFG];                     // log2 K in units of 2^-16, rounded (payload model)
    u32 n_bnd;                                // boundaries per pair in use: NB8, or NBT when some K is 3, 6 or 12
    u32 pad;
    double eps;
};

struct TState {
    u32 nonfinite;
    u32 internal_err;
    u32 pool_overflow;                 // a wave's share of a gather pool, or the tensor's span for the keys
                                       // in group order, was too small: the search is repeated with larger pools
    u64 n_neg, n_zero;                 // strictly negative values; exact zeros (after -0 -> +0)
    // thresholds: index t < n_p is the prune threshold of p_ppm[t], t >= n_p the protect
    // threshold of o_ppm[t - n_p]
    u32 n_thr;
    u32 redo;                          // a sampled sweep 1 mispredicted a threshold: the tensor takes
                                       // the exact sweeps again
    u32 thr_jlo[MAX_THR], thr_jhi[MAX_THR]; // first-level magnitude bins gathered for each threshold
    // exact selection inside the buckets (k_thr_setup / k_thr_count / k_thr_pick)
    u32 sel_k[MAX_THR];                // rank still to resolve inside the chosen bins
    u32 sel_want[MAX_THR];             // magnitude >> 8 of the keys that still take part, or ~0: none
    u32 sel_prefix[MAX_THR];           // chosen bits of the low 17
    u32 sel_cn[MAX_THR][4];            // keys of the bucket below (neg, pos) / above (neg, pos) so far
    u32 sel_seen[MAX_THR];             // keys of the bucket that were found
    u32 sel_nmem[MAX_THR];             // thresholds that share bucket b ...
    unsigned char sel_members[MAX_THR][MAX_THR]; // ... and which
    u32 mag_min, mag_max;              // smallest / largest magnitude image (sampled first sweep only:
                                       // the thresholds of rank 0 and n - 1 are these)
    u32 thr_bucket[MAX_THR];
    u64 thr_res[MAX_THR];              // rank inside the bucket, magnitude order, zeros first (for a pooled
                                       // tensor: inside the group's bucket)
    u32 pool_expect[MAX_THR];          // pooled tensor: keys of the whole group in the threshold's bucket
    u64 pool_zero;                     // group leader: exact zeros of the whole group
    u32 thr_mag[MAX_THR];              // result: magnitude image of the threshold
    u64 thr_lt_neg[MAX_THR], thr_lt_pos[MAX_THR]; // #{mag < tau} by sign
    u64 thr_gt_neg[MAX_THR], thr_gt_pos[MAX_THR]; // #{mag > tau} by sign
    // buckets: distinct first-level magnitude bins that hold a threshold
    u32 n_buckets;
    u32 bucket_magbin[MAX_THR];
    u64 bucket_below_neg[MAX_THR], bucket_below_pos[MAX_THR];
    u32 bucket_cnt_neg[MAX_THR], bucket_cnt_pos[MAX_THR];
    u64 bucket_off[MAX_THR];           // offset into this tensor's threshold-candidate region
    u32 bucket_cursor[MAX_THR];
    // second level
    u32 nb2;                           // bins in use
    u32 zbin;                          // bin that holds ZERO_KEY
    u64 cand_total;
    u32 n_groups, gshift;
    // pairs
    u64 pair_An[MAX_PAIRS], pair_Mn[MAX_PAIRS], pair_Pn[MAX_PAIRS], pair_Pp[MAX_PAIRS];
    u64 pair_M[MAX_PAIRS], pair_Ap[MAX_PAIRS];
    // scoring
    u32 n_edges, n_sub;
    double sumsq;                      // sum of x^2
    double thr_sumsq[MAX_THR];         // prune: sum x^2 over mag < tau; protect: over mag > tau
    u32 best, feasible;
};

struct Score {           // mirrors inshr_score
    double sse, sumsq;
    u64 n_pruned, n_outlier, n_kept, cost_bits;
};

// ------------------------------------------------------------------------------------------
// wavefront helpers
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ u32 wave_sum(u32 v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
// Inclusive prefix sum over the 64 lanes with data-parallel-primitive moves (no LDS traffic):
// shifts by 1, 2, 4, 8 inside each row of 16 lanes, then lane 15 of rows 0 and 2 goes to rows 1
// and 3, then lane 31 to rows 2 and 3.
__device__ __forceinline__ u32 wave_incl_scan(u32 x)
{
    x += (u32)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, true);
    x += (u32)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, true);
    x += (u32)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, true);
    x += (u32)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, true);
    x += (u32)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false);
    x += (u32)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false);
    return x;
}
__device__ __forceinline__ u32 wave_or(u32 v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v |= __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ u32 wave_and(u32 v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v &= __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Exclusive scan of in(0) .. in(n - 1) (n <= 32 * BLOCK) into out[0..n], out[n] = total; whole
// workgroup of BLOCK threads; tmp is LDS scratch of BLOCK/64 + 1 words.  in may read out[i] only
// at the index it is asked for.
template <class F> __device__ inline u32 block_excl_scan_fn(F in, u32 *out, int n, u32 *tmp)
{
    const int t = threadIdx.x;
    const int per = (n + BLOCK - 1) / BLOCK;
    const int lo = t * per;
    u32 s = 0;
    for (int i = 0; i < per; i++) {
        int idx = lo + i;
        if (idx < n) s += in(idx);
    }
    // inclusive scan of s across the wave
    u32 inc = s;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        u32 v = __shfl_up(inc, o);
        if ((t & 63) >= o) inc += v;
    }
    if ((t & 63) == 63) tmp[t >> 6] = inc;
    __syncthreads();
    if (t == 0) {
        u32 run = 0;
        for (int w = 0; w < BLOCK / 64; w++) {
            u32 v = tmp[w];
            tmp[w] = run;
            run += v;
        }
        tmp[BLOCK / 64] = run;
    }
    __syncthreads();
    u32 base = tmp[t >> 6] + inc - s;
    for (int i = 0; i < per; i++) {
        int idx = lo + i;
        if (idx < n) {
            u32 v = in(idx);
            out[idx] = base;
            base += v;
        }
    }
    u32 total = tmp[BLOCK / 64];
    if (t == 0) out[n] = total;
    __syncthreads();
    return total;
}
// The same for an array; in and out may alias only if equal.
__device__ inline u32 block_excl_scan(const u32 *in, u32 *out, int n, u32 *tmp)
{
    return block_excl_scan_fn([in](int i) { return in[i]; }, out, n, tmp);
}

} // namespace inshr
