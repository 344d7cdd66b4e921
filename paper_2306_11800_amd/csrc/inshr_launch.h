// Batch description shared by the kernels' translation units and the host API.
#pragma once
#include "inshr_dev.h"

namespace inshr {

constexpr int CURSOR_STRIDE = L2_BINS + 64; // per-tensor stride of the gather cursors
constexpr int TGT_STRIDE = 4096;            // per-tensor stride of boundary targets (15 * NBT fits)
constexpr int SQ_STRIDE = MAX_FRAC + 1;     // partial sums of squares per (workgroup, tensor) unit
constexpr int SEL_WORDS = MAX_THR * 1024;    // a tensor's selection histograms ([slot][sign][512])
constexpr int CB_STRIDE = 256;              // codebook entries per configuration

struct Bufs { // device pointers, indexed by the tensor's position in the batch unless noted
    TState *ts;
    u32 *hist1;     // [nT][32768]
    u32 *pool_h1;   // [nT][32768] row of a group's leader: the first-level histograms of the group, added up
    u32 *pool_sel;  // [nT][2][SEL_WORDS] row of a group's leader: the group's selection histograms, per pass
    u32 *table2;    // [nT][4096]
    const u64 *unit_off; // [units] start of each (workgroup, tensor) unit's share of a gather pool (u32 units)
    const u32 *unit_capw; // [units] one wave's share of it: wave w of the unit owns
                         // [unit_off + w * capw, unit_off + (w + 1) * capw)
    u32 *unit_thr;   // [units][16] threshold-bucket keys each wave of the unit gathered
    u32 *hist2;     // [nT][32768]
    u32 *binfo;     // [nT][32768] offset of an active bin's elements in the gather pool, or INACTIVE
    u32 *cursor2;   // [nT][CURSOR_STRIDE]
    u32 *tgt_bin;   // [nT][TGT_STRIDE] boundary i of pair q at q*NBT + i
    u32 *tgt_res;
    u32 *tgt_key;   // results: boundary keys
    u32 *pool;      // first gather pool: the keys of the threshold windows (sweep 2), wave-private shares;
                    // afterwards every tensor's keys of active bins in bin-group order (TDesc::pool_grp)
    u32 *pool2;     // second gather pool, same layout: the keys of active bins as sweep 3 gathers them
    u32 *unit_cand; // [units][16] active-bin keys each wave of the unit gathered
    u16 *bin_group; // [nT][32768] group of each active bin
    u32 *grp_off;   // [nT][MAX_GROUPS] first / one-past-last position of each group in bin order
    u32 *grp_end;
    u32 *grp_cur;   // [nT][MAX_GROUPS] keys placed so far
    u32 *tgt_rank;  // [nT][TGT_STRIDE] rank of each boundary among all keys of the tensor
    u32 *tgt_klo;   // [nT][TGT_STRIDE] first and last key of each boundary's bin
    u32 *tgt_khi;
    u32 *tile_out;  // [tiles][MAX_FRAC] protected values per tile and protect fraction
    double *sq_part; // [units][SQ_STRIDE]
    // scoring: all boundaries and class edges of all pairs in one list ordered by key ("edges");
    // slot s holds the keys with exactly s edges at or below them
    u32 *edges;     // [nT][MAX_EDGES] edge keys in that order
    u32 *edge_bin;  // [nT][MAX_EDGES] second-level bin of each edge
    u16 *edge_item; // [nT][MAX_EDGES] pair * 259 + (boundary j - 1, or 255 + class edge)
    u16 *sl;        // [nT][32768 + 64] sub-slot of every bin without an edge; 0xFFFF for the others
    u32 *sub_code;  // [nT][MAX_SUB] slot << 9 | sign and exponent (key >> 23) of each sub-slot
    u32 *sub_cnt;   // [nT][MAX_SUB] keys per sub-slot (in bins without an edge)
    u16 *pair_eidx; // [nT][MAX_PAIRS][EIDX_STRIDE] position of each pair's edges in the list
    u32 *grp_elo;   // [nT][MAX_GROUPS] first / one-past-last edge of each group of active bins
    u32 *grp_ehi;
    u32 *seg_cnt;   // [nT][MAX_EDGES] keys per slot that lie in bins without an edge
    u32 *grp_cnt;   // [nT][2][MAX_EDGES] keys per slot from the group of the slot's lower / upper edge
    double *grp_sx; // [nT][2][MAX_EDGES] ... and their sums
    u64 *mom_sx;    // [units][MAX_SUB] per sub-slot: sum of the 23 mantissa bits over the unit's keys in
                    // bins without an edge
    float *codebook; // [nT][n_cfg][CB_STRIDE]
    Score *scores;  // [nT][n_cfg]
    double *bin_term; // [nT][n_cfg][CB_STRIDE] per-bin 2cS - nc^2
    u32 *tile_off;  // [tiles] exclusive prefix of protected values per tensor (quantize)
};

struct Batch {
    const TDesc *td;     // device
    const GridDesc *gd;  // device
    const u64 *wg_tile0; // device [n_wg + 1]
    const u32 *wg_fu0;   // device [n_wg] first (workgroup, tensor) unit of each workgroup
    const u32 *t_fu_off; // device [nT + 1] CSR of the units that touch each tensor ...
    const u32 *t_fu_ids; // device         ... in ascending workgroup order
    const u32 *fu_tensor; // device [units] tensor of each unit
    u32 *grp_list;       // device [nT * MAX_GROUPS] (tensor << 13 | group) of every group
    u32 *n_grp_total;    // device
    int nT;
    int n_wg;
    int n_units;
    int n_bucket_blocks;
    bool lds_ordered;    // same-address LDS atomics return in lane order on this device
    bool light;          // thresholds and class counts only: no boundaries, no scores (the sketch
                         // quantizer brings its own bins)
    bool any_sampled;    // some tensor's sweep 1 is sampled
    bool any_pooled;     // some tensors share their thresholds (TDesc::pooled)
    bool force_miss;     // (tests) every sampled tensor is sent through the exact sweeps again
    u32 n_pairs, n_cfg;
    u64 n_tiles;
    Bufs bufs;
};

struct QDesc { // one tensor of a quantize call (indexed like the batch)
    unsigned long long *packed; // NULL: tensor not part of the call
    float *codebook;
    float *boundaries;
    u32 *out_idx;
    float *out_val;
    u64 out_cap;
    u32 cfg;   // index into the grid of the search state
    u32 val_bf16; // protected values are stored as bfloat16 (u16), rounded to nearest even
    const u32 *alt_key; // NULL, or 256 boundary keys that replace the search's (boundary j of K at
                        // (j << (8 - bits)) - 1) ...
    const float *alt_cb; // ... and the K centres that go with them
};
struct QInfo {
    u64 n_pruned, n_outlier, n_kept;
    u32 tau_p, tau_o, flags, pad;
};

struct SDesc { // one tensor of a call that partitions by magnitude and sensitivity
    const float *w, *g;
    float *S;           // scratch: the sensitivity scores |g * w|
    float *Wm;          // scratch: the quantized values in index order
    u64 n;
    u64 blk0;           // first 1024-element block of this tensor in the call-wide numbering
    u32 tau_p;          // prune threshold: image of the pruning metric (magnitude or score bits)
    u32 tau_om, tau_os; // protect thresholds: magnitude image, score bits
    u32 by_sens;        // the pruning metric is the score
    unsigned long long *packed;
    u32 *out_idx;
    float *out_val;
    u64 out_cap;
    float *codebook, *boundaries;
    const u32 *bkeys;   // the compact tensor's boundary keys (one pair: NBT candidates)
    const float *cb;    // ... and the centres of the chosen number of bins
    u32 K, sym_bits;
};
struct SInfo {
    u64 n_pruned, n_outlier, n_kept;
    double sq_pruned, sq_prot; // sums of squares of the pruned / protected values
};

struct DDesc { // one tensor of a delta call
    const unsigned long long *prev, *cur;
    unsigned long long *out;
    u64 *group_off;
    u32 *perm;
    const u32 *prev_perm;
    u64 n, out_words;
    u64 dtile0, chunk0, n_chunks;
    u32 wp, wc, Kp, B, wB, pad;
};
struct RDesc { // one tensor of a dequantize call
    const unsigned long long *packed;
    const float *codebook;
    const u32 *out_idx;
    const float *out_val;
    float *dst;
    u64 n, n_outlier, tile0;
    u32 w, K;
    u32 val_bf16, pad; // out_val holds bfloat16 values (u16)
};
constexpr int DEQUANT_TILE = 16384; // elements per workgroup of the decoding kernel (RDesc::tile0 counts these)
struct XDesc { // one tensor of a reconstruct call: the delta descriptor plus what is checked
    unsigned long long *cur_out; // receives the current symbols
    const u64 *group_off_in;     // group offsets that came with the stream, or NULL
    u32 Sc, pad;                 // symbols of the current checkpoint
};
// bits of the flag word the restore kernels raise
constexpr u32 RF_SYMBOL = 1u;  // a symbol outside 0 .. K + 1
constexpr u32 RF_LIST = 2u;    // protected list and symbol stream disagree
constexpr u32 RF_GROUPS = 4u;  // group offsets do not match the previous symbols
constexpr u32 RF_DELTA = 8u;   // a delta outside 0 .. B - 1, or a result outside 0 .. K_cur + 1
constexpr u32 RF_ORDER = 16u;  // ranks from returning LDS adds disagree with ranks from ballots
// bits of the flag word of a delta call
constexpr u32 DF_PERM = 1u;    // a given permutation holds an index outside its tensor
constexpr u32 DF_ORDER = 2u;   // ranks from returning LDS adds disagree with ranks from ballots
constexpr int DELTA_TILE = 12288;
constexpr int DELTA_CHUNK = 64;
constexpr int DELTA_SS = 264;
// the delta entry point that allocates nothing: its limits, and its descriptors as kernel arguments
constexpr int DELTA_STATIC_MAX_TENSORS = 16;
constexpr int DELTA_STATIC_MAX_CHUNKS = 2048; // chunks of DELTA_TILE * DELTA_CHUNK elements, all tensors
struct DeltaStaticArgs {
    DDesc dd[DELTA_STATIC_MAX_TENSORS];
    u32 n_tensors, pad;
};

// Optional per-kernel timing with HIP events on the launch stream (off by default).
void prof_begin(const char *name, hipStream_t s);
void prof_end(hipStream_t s);
#define PROF(name, s, ...)                                                                        \
    do {                                                                                          \
        prof_begin(name, s);                                                                      \
        __VA_ARGS__;                                                                              \
        prof_end(s);                                                                              \
    } while (0)

hipError_t launch_select(const Batch &bt, hipStream_t s);
hipError_t launch_edges(const Batch &bt, hipStream_t s); // edge order, bins without edges (inside launch_select)
hipError_t launch_score(const Batch &bt, hipStream_t s);
hipError_t launch_quantize(const Batch &bt, const QDesc *qd, QInfo *qi, hipStream_t s);
hipError_t launch_delta(const DDesc *dd, int nT, u64 n_dtiles, u64 n_chunks,
                        const u32 *chunk_tensor, u32 *chunk_tot, u32 *flags, bool any_scatter,
                        bool any_perm, bool any_gather, bool lds_ordered, hipStream_t s);
hipError_t delta_static_init(int device); // once per device, with that device current
u32 *delta_static_flags(int device);      // the flag word of launch_delta_static on that device
hipError_t launch_delta_static(int device, const DeltaStaticArgs &a, u64 n_dtiles, u64 n_chunks,
                               bool any_scatter, bool any_perm, bool lds_ordered, hipStream_t s);
hipError_t launch_sens_score(const SDesc *sd, int nT, u64 n_blocks, hipStream_t s);
hipError_t launch_sens_partition(const SDesc *sd, int nT, u64 n_blocks, u32 *blk_kept, u32 *blk_prot,
                                 double *blk_sq, SInfo *info, hipStream_t s);
hipError_t launch_sens_quant(const SDesc *sd, int nT, u64 n_blocks, const u32 *blk_prot, u32 *flags,
                             hipStream_t s);
hipError_t launch_lds_order_check(u32 *violations, hipStream_t s);
hipError_t launch_dequantize(const RDesc *rd, int nT, u64 n_tiles, u64 max_outlier, u32 *flags,
                             u32 *ones, int n_cu, hipStream_t s);
hipError_t launch_reconstruct(const DDesc *dd, const XDesc *xd, int nT, u64 n_chunks,
                              const u32 *chunk_tensor, u32 *chunk_tot, u32 *flags, bool lds_ordered,
                              hipStream_t s);

// ------------------------------------------------------------------------------------------
// tile iteration shared by the streaming kernels
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ int find_tensor(const TDesc *td, int nT, u64 tile)
{
    int lo = 0, hi = nT - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (td[mid].tile0 <= tile)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

// v[4*j + c] = element 4*(tid + 1024*j) + c of the tile; returns the mask of valid entries
__device__ __forceinline__ u32 load_tile(const TDesc &d, u64 e0, u32 cnt, float (&v)[16])
{
    const GLOBAL_AS float *p = gptr(d.data) + e0;
    const u32 tid = threadIdx.x;
    if (cnt == (u32)TILE && d.aligned16) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        const GLOBAL_AS f4 *p4 = (const GLOBAL_AS f4 *)p;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const f4 q = p4[tid + 1024u * j];
            v[4 * j + 0] = q.x;
            v[4 * j + 1] = q.y;
            v[4 * j + 2] = q.z;
            v[4 * j + 3] = q.w;
        }
        return 0xFFFFu;
    }
    u32 mask = 0u;
#pragma unroll
    for (int j = 0; j < 4; j++) {
#pragma unroll
        for (int c = 0; c < 4; c++) {
            u32 idx = 4u * (tid + 1024u * j) + c;
            float x = 0.0f;
            if (idx < cnt) {
                x = p[idx];
                mask |= 1u << (4 * j + c);
            }
            v[4 * j + c] = x;
        }
    }
    return mask;
}

// A whole tile at a 16-byte aligned address, asked for without any branch: the values may stay in
// flight until their first use (a tile fetched ahead).
__device__ __forceinline__ void load_tile_ahead(const TDesc &d, u64 e0, float (&v)[16])
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    const GLOBAL_AS f4 *p4 = (const GLOBAL_AS f4 *)(gptr(d.data) + e0);
#pragma unroll
    for (int j = 0; j < 4; j++) {
        const f4 q = p4[threadIdx.x + 1024u * j];
        v[4 * j + 0] = q.x;
        v[4 * j + 1] = q.y;
        v[4 * j + 2] = q.z;
        v[4 * j + 3] = q.w;
    }
}

} // namespace inshr
