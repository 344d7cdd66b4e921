// Exact thresholds and bin boundaries (Sec. 4.2-4.4) by two counting sweeps and one gathering
// sweep over the tensors; every launch covers all tensors of a batch.
//
//   sweep 1  k_hist<1>     LDS histogram of key >> 17 (32768 bins), sum of squares, exact zeros
//                          (negative and non-finite counts follow from the histogram).  Tensors of
//                          16 Mi elements or more read only one tile in eight here ("sampled").
//   k_plan1                per tensor: first-level magnitude bin ("bucket") of every prune /
//                          protect threshold rank; a key -> bin table whose bins hold about
//                          n / 32768 elements each.  From a sampled histogram the bucket is only
//                          predicted: a window of bins around it is gathered (8 standard deviations
//                          of the rank estimate wide), and the table gives the key prefixes of the
//                          window at least 8 bins, so that sweep 2 resolves first-level bins there.
//   sweep 2  k_hist<2>     LDS histogram over the table's bins; elements of threshold buckets are
//                          gathered into wave-private regions.  For sampled tensors also what
//                          sweep 1 gives otherwise (sum of squares, zeros).  The thresholds of rank
//                          0 and n - 1 (the smallest and the largest magnitude) cannot be predicted
//                          to a bin from a sample, but the sample's extreme bins bound them: all
//                          bins beyond those are gathered (a handful of keys) and the select takes
//                          the extremes of the gathered keys.
//   k_plan1b               sampled tensors: exact size checks and the exact bucket of every
//                          threshold from the second histogram; a bucket outside its window marks
//                          the tensor, and k_hist<1>, k_plan1, k_hist<2> run once more for the
//                          marked tensors alone, unsampled (the results never depend on sampling).
//   k_thr_setup/count/pick exact thresholds and class counts from the gathered buckets: all
//                          thresholds of a tensor in two counting passes over its gathered keys
//   k_plan2                exact rank of every boundary of every (prune, protect) pair -> its bin;
//                          only those bins (and the bins of the class edges) are "active";
//                          groups of consecutive active bins
//   (k_edges, in the scoring file: order of all boundaries and class edges, slot of every bin
//   without an edge)
//   sweep 3  k_gather      keys of bins without an edge add to their slot's sum; keys of active
//                          bins are gathered; protected counts per tile and their squares
//   k_split                gathered keys -> groups of consecutive active bins
//   k_bucket               one group per step: sort in LDS, every boundary read at its rank, counts
//                          and sums per slot
#include "inshr_launch.h"

namespace inshr {

// ------------------------------------------------------------------------------------------
// sweeps 1 and 2: histograms
// ------------------------------------------------------------------------------------------
// One tile of sweep 1: first-level histogram, sum of squares, exact zeros (the numbers of negative
// and of non-finite values follow from the histogram).
template <bool FULL>
__device__ __forceinline__ void hist1_tile(const float (&v)[16], u32 mask, u32 *h, double &q_tot,
                                           u32 &c_zero)
{
#pragma unroll
    for (int i = 0; i < 16; i++) {
        const bool valid = FULL || ((mask >> i) & 1u);
        const u32 key = key_of_float(v[i]);
        const double xd = (double)v[i];
        q_tot = fma(xd, xd, q_tot); // invalid entries are 0.0
        c_zero += (u32)__popcll(__ballot(valid && key == ZERO_KEY)); // wave-uniform
        if (valid) atomicAdd(&h[key >> L1_SHIFT], 1u);
    }
}

// One tile of sweep 2: exact second-level histogram; the elements of a threshold's first-level
// magnitude bin are appended to the wave's gather region.
// STATS: also the sum of squares and the exact zeros (tensors whose sweep 1 was sampled).
template <bool FULL, bool STATS>
__device__ __forceinline__ void hist2_tile(const float (&v)[16], u32 mask, u32 *h, const u32 *T,
                                           GLOBAL_AS u32 *gdst, u32 &gathered, double &q_tot,
                                           u32 &c_zero)
{
    u32 key[16], ent[16];
#pragma unroll
    for (int i = 0; i < 16; i++) { // all table reads are in flight together
        key[i] = key_of_float(v[i]);
        ent[i] = T[key[i] >> COARSE_SHIFT];
        if (STATS) {
            const double xd = (double)v[i];
            q_tot = fma(xd, xd, q_tot); // invalid entries are 0.0
            const bool valid = FULL || ((mask >> i) & 1u);
            c_zero += (u32)__popcll(__ballot(valid && key[i] == ZERO_KEY)); // wave-uniform
        }
    }
#pragma unroll
    for (int i = 0; i < 16; i++) {
        const bool valid = FULL || ((mask >> i) & 1u);
        if (valid) atomicAdd(&h[l2_bin(key[i], ent[i])], 1u);
        const bool cand = valid && in_threshold_bucket(key[i], ent[i]) && key[i] != ZERO_KEY;
        u64 cm = __ballot(in_threshold_bucket(key[i], ent[i])) & __ballot(key[i] != ZERO_KEY);
        if (!FULL) cm &= __ballot(valid);
        if (cand)
            gdst[__builtin_amdgcn_mbcnt_hi((u32)(cm >> 32), __builtin_amdgcn_mbcnt_lo((u32)cm, gathered))] = key[i];
        gathered += (u32)__popcll(cm);
    }
}

// REDO: the pass over the tensors whose sampled sweep 1 mispredicted a threshold (TState::redo);
// they are treated as not sampled, all other tensors are skipped.
template <int LEVEL, bool REDO>
__global__ __launch_bounds__(BLOCK) void k_hist(const TDesc *__restrict__ td, int nT,
                                                const u64 *__restrict__ wg_tile0,
                                                const u32 *__restrict__ wg_fu0, Bufs B)
{
    // one static array (it starts at LDS address 0, so offsets fold into the LDS instructions)
    __shared__ __attribute__((aligned(16))) u32 smem[L2_BINS + (LEVEL == 2 ? COARSE : 0) + 2 * (BLOCK / 64)];
    u32 *h = smem;                 // 32768 counters
    u32 *T = smem + L2_BINS;       // LEVEL 2: 4096 table entries
    double *s_red = reinterpret_cast<double *>(smem + L2_BINS + (LEVEL == 2 ? COARSE : 0));

    const u32 tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int i = tid; i < L2_BINS; i += BLOCK) h[i] = 0u;
    const u64 tile_lo = wg_tile0[blockIdx.x], tile_hi = wg_tile0[blockIdx.x + 1];
    if (tile_lo >= tile_hi) return;
    int t = find_tensor(td, nT, tile_lo);
    const int t_first = t;
    u64 tile = tile_lo;
    while (tile < tile_hi) {
        const TDesc d = td[t];
        const u64 n_tiles_t = (d.n + TILE - 1) / TILE;
        const u64 t_end = d.tile0 + n_tiles_t;
        const u64 stop = t_end < tile_hi ? t_end : tile_hi;
        TState *st = B.ts + t;
        const u32 fu = wg_fu0[blockIdx.x] + (u32)(t - t_first);
        if (REDO && !st->redo) { // (the same for the whole workgroup)
            tile = stop;
            t++;
            continue;
        }
        const bool sampled = !REDO && d.sampled != 0u;
        // Elements of the thresholds' first-level magnitude bins are gathered into a region of the
        // pool that belongs to this wave alone: the workgroup's region starts at its first element
        // of the tensor, and a wave's share of it is as large as the wave's share of the elements
        // (1024 per tile), so no counter is shared.
        const u32 capw = B.unit_capw[fu];
        GLOBAL_AS u32 *gdst = gptr(B.pool) + B.unit_off[fu] + (u64)wave * capw;
        u32 gathered = 0u; // wave-uniform
        bool overflow = false;
        if (LEVEL == 2) {
            for (int i = tid; i < COARSE; i += BLOCK) T[i] = B.table2[(size_t)t * COARSE + i];
        }
        __syncthreads();
        u32 c_zero = 0u;    // exact zeros seen by this wave (LEVEL 1; LEVEL 2 of a sampled tensor)
        double q_tot = 0.0; // sum of squares (the same)
        for (; tile < stop; tile++) {
            // a sampled sweep 1 takes one tile in SAMPLE_RATE
            if (LEVEL == 1 && sampled && (tile - d.tile0) % (u64)SAMPLE_RATE != 0u) continue;
            const u64 e0 = (tile - d.tile0) * (u64)TILE;
            const u64 rem = d.n - e0;
            const u32 cnt = rem < (u64)TILE ? (u32)rem : (u32)TILE;
            float v[16];
            const u32 mask = load_tile(d, e0, cnt, v);
            if (LEVEL == 1) {
                if (cnt == (u32)TILE) // the same for every lane: the tile code uses ballots
                    hist1_tile<true>(v, mask, h, q_tot, c_zero);
                else
                    hist1_tile<false>(v, mask, h, q_tot, c_zero);
            } else {
                // A share that cannot take a whole tile any more is too small: the tile's keys go over
                // the last ones (every share holds at least one tile), and the overflow is reported;
                // the host then repeats the search with larger pools.
                if (gathered + (u32)(TILE / (BLOCK / 64)) > capw) {
                    overflow = true;
                    gathered = capw - (u32)(TILE / (BLOCK / 64));
                }
                if (sampled) {
                    if (cnt == (u32)TILE) // the same for every lane: the tile code uses ballots
                        hist2_tile<true, true>(v, mask, h, T, gdst, gathered, q_tot, c_zero);
                    else
                        hist2_tile<false, true>(v, mask, h, T, gdst, gathered, q_tot, c_zero);
                } else {
                    if (cnt == (u32)TILE)
                        hist2_tile<true, false>(v, mask, h, T, gdst, gathered, q_tot, c_zero);
                    else
                        hist2_tile<false, false>(v, mask, h, T, gdst, gathered, q_tot, c_zero);
                }
            }
        }
        __syncthreads();
        // flush this tensor's counts
        u32 *gh = (LEVEL == 1 ? B.hist1 : B.hist2) + (size_t)t * L2_BINS;
        for (int i = tid; i < L2_BINS; i += BLOCK) {
            u32 c = h[i];
            if (c) {
                atomicAdd(&gh[i], c);
                h[i] = 0u;
            }
        }
        if (LEVEL == 2) {
            if (lane == 0u) {
                B.unit_thr[(size_t)fu * 16 + wave] = gathered;
                if (overflow) atomicOr(&st->pool_overflow, 1u);
            }
        }
        // sum of squares and zeros: from sweep 1, or from sweep 2 when sweep 1 was sampled (the
        // sampled sweep's own zeros, scaled, are an estimate that shapes the table; k_plan1 clears it)
        if (LEVEL == 1 || sampled) {
            if (LEVEL == 1 && sampled) c_zero *= (u32)SAMPLE_RATE;
            q_tot = wave_sum_f64(q_tot);
            if (lane == 0u) {
                if (c_zero) atomicAdd((unsigned long long *)&st->n_zero, (unsigned long long)c_zero);
                s_red[wave] = q_tot;
            }
            __syncthreads();
            if (tid == 0) { // partial sum of squares of this (workgroup, tensor) unit, fixed order
                double sum = 0.0;
                for (int w = 0; w < BLOCK / 64; w++) sum += s_red[w];
                B.sq_part[(size_t)fu * SQ_STRIDE] = sum;
            }
        }
        __syncthreads();
        t++;
    }
}

// ------------------------------------------------------------------------------------------
// plan 1: threshold buckets and the second-level table
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ u32 depth_for(u32 nc, u64 target)
{
    u32 d = 0;
    while (d < 20u && (u64)nc > (target << d)) d++;
    return d;
}

// rank of threshold q: the floor(n * ppm / 1e6) smallest magnitudes are pruned, as many of the
// largest are protected
__device__ __forceinline__ u64 threshold_rank(const GridDesc *gd, u32 q, u64 n)
{
    if (q < gd->n_p) return n * (u64)gd->p_ppm[q] / 1000000ull;
    return n - 1ull - n * (u64)gd->o_ppm[q - gd->n_p] / 1000000ull;
}

// which of the 8 first-level bins under key prefix c are gathered for some threshold
// (thresholds whose bit is set in skip are left out)
__device__ __forceinline__ u32 cell_flags(u32 c, const u32 *jlo, const u32 *jhi, u32 n_thr, u32 skip = 0u)
{
    u32 flag = 0u;
    for (u32 q = 0; q < n_thr; q++) {
        if ((skip >> q) & 1u) continue;
        // magnitude bin j is first-level key bin 16384 + j for positive, 16383 - j for negative
        const u32 p0 = (u32)L1_MAGBINS + jlo[q], p1 = (u32)L1_MAGBINS + jhi[q];
        const u32 n0 = (u32)L1_MAGBINS - 1u - jhi[q], n1 = (u32)L1_MAGBINS - 1u - jlo[q];
        for (u32 i = 0; i < 8u; i++) {
            const u32 k = 8u * c + i;
            if ((k >= p0 && k <= p1) || (k >= n0 && k <= n1)) flag |= bucket_flag(k);
        }
    }
    return flag;
}

constexpr u32 NO_BUCKET = 0xFFFFFFFFu;

// The buckets of a tensor from the exact figures of its thresholds (one thread): thresholds that
// fall into the same first-level magnitude bin share a bucket.
__device__ inline void make_buckets(TState *st, u32 n_thr, const u32 *s_j, const u64 *s_res,
                                    const u64 *s_bn, const u64 *s_bp, const u32 *s_cn, const u32 *s_cp)
{
    u32 nb = 0;
    u64 off = 0;
    st->n_thr = n_thr;
    for (u32 q = 0; q < n_thr; q++) {
        const u32 j = s_j[q];
        if (j == NO_BUCKET) { // rank 0 or n - 1 of a sampled tensor: the extreme magnitude itself
            st->thr_bucket[q] = NO_BUCKET;
            st->thr_res[q] = s_res[q]; // 0: the smallest magnitude, 1: the largest
            continue;
        }
        u32 found = nb;
        for (u32 k = 0; k < nb; k++)
            if (st->bucket_magbin[k] == j) found = k;
        if (found == nb) {
            st->bucket_magbin[nb] = j;
            st->bucket_below_neg[nb] = s_bn[q];
            st->bucket_below_pos[nb] = s_bp[q];
            st->bucket_cnt_neg[nb] = s_cn[q];
            st->bucket_cnt_pos[nb] = s_cp[q];
            st->bucket_off[nb] = off;
            st->bucket_cursor[nb] = 0u;
            off += (u64)s_cn[q] + s_cp[q];
            nb++;
        }
        st->thr_bucket[q] = found;
        st->thr_res[q] = s_res[q];
    }
    st->n_buckets = nb;
}

// Thresholds per layer type (Sec. 4.2): the first-level histograms and the zero counts of a group's
// tensors, added up in the row of the group's leader (cleared beforehand).
__global__ __launch_bounds__(BLOCK) void k_pool_sum(const TDesc *__restrict__ td, Bufs B)
{
    const int t = blockIdx.x;
    const TDesc d = td[t];
    if (!d.pooled) return;
    const u32 *h1 = B.hist1 + (size_t)t * L1_BINS;
    u32 *ph = B.pool_h1 + (size_t)d.leader * L1_BINS;
    for (u32 i = threadIdx.x; i < (u32)L1_BINS; i += BLOCK) {
        const u32 c = h1[i];
        if (c) atomicAdd(&ph[i], c);
    }
    if (threadIdx.x == 0)
        atomicAdd((unsigned long long *)&B.ts[d.leader].pool_zero, (unsigned long long)B.ts[t].n_zero);
}

// magnitude bin of a rank: last j in [0, 16384) with A[j] <= rank (A: exclusive prefix of the counts)
__device__ __forceinline__ u32 magbin_of_rank(const u32 *A, u64 rank)
{
    int lo = 0, hi = L1_MAGBINS;
    while (lo < hi) {
        int mid = (lo + hi) >> 1;
        if ((u64)A[mid] > rank)
            hi = mid;
        else
            lo = mid + 1;
    }
    return (u32)(lo > 0 ? lo - 1 : 0);
}

// REDO: only the tensors whose sampled sweep 1 mispredicted (their histogram is exact now).
template <bool REDO>
__global__ __launch_bounds__(BLOCK) void k_plan1(const TDesc *__restrict__ td,
                                                 const GridDesc *__restrict__ gd, Bufs B)
{
    extern __shared__ u32 smem[];
    u32 *A = smem;                    // [16385] magnitude-bin counts -> exclusive prefix
    u32 *Bn = smem + (L1_MAGBINS + 4); // [16385] negative counts -> exclusive prefix
    u32 *nc = Bn + (L1_MAGBINS + 4);  // [4097] per coarse prefix
    __shared__ u32 tmp[BLOCK / 64 + 1];
    __shared__ u32 s_j[MAX_THR], s_jlo[MAX_THR], s_jhi[MAX_THR], s_cn[MAX_THR], s_cp[MAX_THR];
    __shared__ u64 s_res[MAX_THR], s_bn[MAX_THR], s_bp[MAX_THR];

    const int t = blockIdx.x;
    const u32 tid = threadIdx.x;
    const u64 n = td[t].n;
    TState *st = B.ts + t;
    if (REDO && !st->redo) return;
    const bool sampled = !REDO && td[t].sampled != 0u;
    const u32 scale = sampled ? (u32)SAMPLE_RATE : 1u; // a sampled histogram stands for the whole
    const u32 *h1 = B.hist1 + (size_t)t * L1_BINS;
    const bool pooled = td[t].pooled != 0u; // (never sampled)
    if (pooled) {
        // the thresholds are order statistics of the group: their bins and the ranks inside them
        // come from the group's histogram; everything else below is the tensor's own
        const u32 *ph = B.pool_h1 + (size_t)td[t].leader * L1_BINS;
        for (int j = tid; j < L1_MAGBINS; j += BLOCK) A[j] = ph[L1_MAGBINS - 1 - j] + ph[L1_MAGBINS + j];
        __syncthreads();
        const u32 gtotal = block_excl_scan(A, A, L1_MAGBINS, tmp);
        if (tid == 0 && (u64)gtotal != td[t].n_pool) atomicOr(&st->internal_err, 1u);
        if (tid < gd->n_p + gd->n_o) {
            const u64 R = threshold_rank(gd, tid, td[t].n_pool);
            const u32 j = magbin_of_rank(A, R);
            s_j[tid] = j;
            s_res[tid] = R - (u64)A[j];
            st->pool_expect[tid] = A[j + 1] - A[j];
        }
        __syncthreads();
    }
    for (int j = tid; j < L1_MAGBINS; j += BLOCK) {
        u32 cn = h1[L1_MAGBINS - 1 - j] * scale, cp = h1[L1_MAGBINS + j] * scale;
        A[j] = cn + cp;
        Bn[j] = cn;
    }
    for (int c = tid; c < COARSE; c += BLOCK) {
        u32 s = 0;
        for (int i = 0; i < 8; i++) s += h1[8 * c + i];
        nc[c] = s * scale;
    }
    __syncthreads();
    u32 total = block_excl_scan(A, A, L1_MAGBINS, tmp);
    const u32 total_neg = block_excl_scan(Bn, Bn, L1_MAGBINS, tmp);
    if (tid == 0 && !sampled) { // (a sampled tensor gets these from the exact second histogram)
        if ((u64)total != n) atomicOr(&st->internal_err, 1u);
        st->n_neg = total_neg;
        // magnitude bins from 0x7f800000 >> 17 on hold Inf and NaN only
        if (total - A[0x7f800000u >> L1_SHIFT] != 0u) st->nonfinite = 1u;
    }

    const u32 n_p = gd->n_p, n_o = gd->n_o, n_thr = n_p + n_o;
    if (tid < n_thr) {
        const u64 R = threshold_rank(gd, tid, n);
        // bin of a rank: last j in [0, 16384) with A[j] <= rank
        auto bin_of = [&](u64 rank) -> u32 {
            int lo = 0, hi = L1_MAGBINS;
            while (lo < hi) {
                int mid = (lo + hi) >> 1;
                if ((u64)A[mid] > rank)
                    hi = mid;
                else
                    lo = mid + 1;
            }
            return (u32)(lo > 0 ? lo - 1 : 0);
        };
        if (!sampled) {
            const u32 j = pooled ? s_j[tid] : bin_of(R);
            s_j[tid] = s_jlo[tid] = s_jhi[tid] = j;
            if (!pooled) s_res[tid] = R - (u64)A[j];
            s_bn[tid] = Bn[j];
            s_bp[tid] = A[j] - Bn[j];
            s_cn[tid] = h1[L1_MAGBINS - 1 - j];
            s_cp[tid] = h1[L1_MAGBINS + j];
        } else {
            // The rank's bin is only predicted: all bins that may hold it are gathered.  The
            // estimate of a cumulative count c from one tile in SAMPLE_RATE has a standard
            // deviation of about sqrt(SAMPLE_RATE * c) for independent elements; tiles are not
            // independent draws, so the margin is generous, and a miss is caught afterwards.
            const u64 tail = R < n - R ? R + 1ull : n - R;
            const u64 margin = (u64)(8.0 * sqrt((double)SAMPLE_RATE * (double)tail)) + 8ull * SAMPLE_RATE;
            // The scaled total is not n.  A rank of the upper half is counted from the top of the
            // scaled histogram, so that an error in the estimate of a large population below it
            // (exact zeros that come in whole rows, say) does not shift it.
            const u64 last = total ? (u64)total - 1ull : 0ull;
            const bool from_top = R > n - 1ull - R;
            const u64 Rs = !from_top ? R : (last > n - 1ull - R ? last - (n - 1ull - R) : 0ull);
            const u64 r_lo = Rs > margin ? Rs - margin : 0ull;
            const u64 r_hi = Rs + margin;
            s_jlo[tid] = bin_of(r_lo < last ? r_lo : last);
            u32 jh = bin_of(r_hi < last ? r_hi : last);
            if (r_hi >= last && jh + 1u < (u32)L1_MAGBINS) jh++; // the sample may have missed the top
            s_jhi[tid] = jh;
            s_j[tid] = 0u;
            // Ranks 0 and n - 1 are the smallest and the largest magnitude themselves.  The sample's
            // extreme bins bound them: every bin up to the sample's lowest occupied one (from its
            // highest occupied one on) is gathered — a handful of keys — and the threshold select
            // takes the smallest (largest) magnitude of all gathered keys.
            if (R == 0ull) {
                s_jlo[tid] = 0u;
                s_jhi[tid] = bin_of(0ull);
            } else if (R == n - 1ull) {
                s_jlo[tid] = bin_of(last);
                s_jhi[tid] = (u32)L1_MAGBINS - 1u;
            }
        }
        st->thr_jlo[tid] = s_jlo[tid];
        st->thr_jhi[tid] = s_jhi[tid];
    }
    __syncthreads();
    if (tid == 0) {
        if (!sampled) make_buckets(st, n_thr, s_j, s_res, s_bn, s_bp, s_cn, s_cp);
        st->n_thr = n_thr;
    }
    __syncthreads();

    // second-level table: smallest target population whose bin total fits
    // (exact zeros are counted, never gathered or sorted: they do not ask for bins; a prefix with
    // gathered first-level bins gets at least 8 bins, so that the second histogram resolves them)
    if (tid == 0) {
        const u32 zc = ZERO_KEY >> COARSE_SHIFT;
        const u64 nz = st->n_zero;
        nc[zc] = (u64)nc[zc] > nz ? (u32)(nc[zc] - nz) : 1u;
        if (sampled) {
            st->n_zero = 0ull; // (an estimate: the second sweep counts the zeros exactly)
            st->mag_min = 0xFFFFFFFFu;
            st->mag_max = 0u;
        }
    }
    __syncthreads();
    // gathered first-level bins of this thread's key prefixes (prefix c = tid + BLOCK * k)
    // (the windows of the ranks 0 and n - 1 of a sampled tensor are gathered, but nothing has to be
    // resolved inside them: they ask for no bins)
    u32 extreme = 0u;
    if (sampled)
        for (u32 q = 0; q < n_thr; q++) {
            const u64 R = threshold_rank(gd, q, n);
            if (R == 0ull || R == n - 1ull) extreme |= 1u << q;
        }
    u32 my_flags[COARSE / BLOCK], my_force[COARSE / BLOCK];
#pragma unroll
    for (int k = 0; k < COARSE / BLOCK; k++) {
        my_flags[k] = cell_flags(tid + (u32)BLOCK * k, s_jlo, s_jhi, n_thr);
        my_force[k] = extreme ? cell_flags(tid + (u32)BLOCK * k, s_jlo, s_jhi, n_thr, extreme) : my_flags[k];
    }
    auto depth_of = [&](int c, u64 target, int k) -> u32 {
        u32 d = nc[c] ? depth_for(nc[c], target) : 0u;
        if (sampled && d < 3u && my_force[k]) d = 3u;
        return d;
    };
    u64 lo = 1, hi = n;
    while (lo < hi) {
        u64 mid = lo + ((hi - lo) >> 1);
        u32 s = 0;
#pragma unroll
        for (int k = 0; k < COARSE / BLOCK; k++) s += 1u << depth_of(tid + BLOCK * k, mid, k);
        s = wave_sum(s);
        __syncthreads();
        if ((tid & 63u) == 0u) tmp[tid >> 6] = s;
        __syncthreads();
        u32 tot = 0;
        for (int w = 0; w < BLOCK / 64; w++) tot += tmp[w];
        if (tot <= (u32)L2_BINS)
            hi = mid;
        else
            lo = mid + 1;
    }
    __syncthreads();
    u32 *cnt = A; // reuse: bins per coarse prefix
#pragma unroll
    for (int k = 0; k < COARSE / BLOCK; k++) cnt[tid + BLOCK * k] = 1u << depth_of(tid + BLOCK * k, lo, k);
    __syncthreads();
    u32 nb2 = block_excl_scan(cnt, Bn, COARSE, tmp); // Bn[c] = base
    u32 *tab = B.table2 + (size_t)t * COARSE;
#pragma unroll
    for (int k = 0; k < COARSE / BLOCK; k++) {
        const int c = tid + BLOCK * k;
        const u32 d = depth_of(c, lo, k);
        // top byte: which of the 8 first-level bins under this key prefix are gathered
        tab[c] = my_flags[k] | (Bn[c] << 5) | d;
    }
    if (tid == 0) {
        st->nb2 = nb2;
        st->zbin = Bn[ZERO_KEY >> COARSE_SHIFT];
        if (nb2 > (u32)L2_BINS) atomicOr(&st->internal_err, 2u);
    }
}

// After the second histogram of a tensor whose sweep 1 was sampled: the exact figures that sweep 1
// gives otherwise (size, negative count, non-finite values) and, for every threshold, the
// first-level magnitude bin that holds its rank, with the exact counts below and inside it by sign.
// The bins resolve only where the table has at least 8 bins under a key prefix, which k_plan1
// arranged for the bins it had gathered; a rank outside them sends the tensor through the exact
// sweeps again (TState::redo).
__global__ __launch_bounds__(BLOCK) void k_plan1b(const TDesc *__restrict__ td,
                                                  const GridDesc *__restrict__ gd, Bufs B, u32 force_miss)
{
    __shared__ u32 Am[COARSE / 2 + 1];     // per magnitude prefix, both signs -> exclusive prefix
    __shared__ u32 Nm[COARSE / 2 + 1];     // negative ones -> exclusive prefix
    __shared__ u32 tmp[BLOCK / 64 + 1];
    __shared__ u32 s_j[MAX_THR], s_cn[MAX_THR], s_cp[MAX_THR], s_miss;
    __shared__ u64 s_res[MAX_THR], s_bn[MAX_THR], s_bp[MAX_THR];
    const int t = blockIdx.x;
    const u32 tid = threadIdx.x;
    if (!td[t].sampled) return;
    const u64 n = td[t].n;
    TState *st = B.ts + t;
    const u32 *tab = B.table2 + (size_t)t * COARSE;
    u32 *h2 = B.hist2 + (size_t)t * L2_BINS;
    constexpr int HALF = COARSE / 2;
    if (tid == 0) s_miss = force_miss;
    extern __shared__ u32 pre2[]; // [L2_BINS + 1] exclusive prefix of the second histogram
    block_excl_scan(h2, pre2, L2_BINS, tmp);
    auto cc = [&](u32 c) -> u32 { // exact count under key prefix c
        const u32 e = tab[c], base = (e >> 5) & 0x7fffu, nb = 1u << (e & 31u);
        return pre2[base + nb] - pre2[base];
    };
    for (int m = tid; m < HALF; m += BLOCK) {
        Am[m] = cc(HALF + m) + cc(HALF - 1 - m);
        Nm[m] = cc(HALF - 1 - m);
    }
    __syncthreads();
    const u32 total = block_excl_scan(Am, Am, HALF, tmp);
    const u32 total_neg = block_excl_scan(Nm, Nm, HALF, tmp);
    if (tid == 0) {
        if ((u64)total != n) atomicOr(&st->internal_err, 1u);
        st->n_neg = total_neg;
        if (total - Am[0x7f800000u >> COARSE_SHIFT] != 0u) st->nonfinite = 1u;
    }
    const u32 n_thr = gd->n_p + gd->n_o;
    if (tid < n_thr && (threshold_rank(gd, tid, n) == 0ull || threshold_rank(gd, tid, n) == n - 1ull)) {
        s_j[tid] = NO_BUCKET; // the smallest / largest magnitude, taken by the second sweep
        s_res[tid] = threshold_rank(gd, tid, n) == 0ull ? 0ull : 1ull;
    } else if (tid < n_thr) {
        const u64 R = threshold_rank(gd, tid, n);
        int lo = 0, hi = HALF; // last magnitude prefix m with Am[m] <= R
        while (lo < hi) {
            int mid = (lo + hi) >> 1;
            if ((u64)Am[mid] > R)
                hi = mid;
            else
                lo = mid + 1;
        }
        const u32 m = (u32)(lo > 0 ? lo - 1 : 0);
        const u32 ep = tab[HALF + m], en = tab[HALF - 1 - m];
        const u32 dp = ep & 31u, dn = en & 31u;
        bool ok = (dp >= 3u || cc(HALF + m) == 0u) && (dn >= 3u || cc(HALF - 1 - m) == 0u);
        if (ok) {
            u64 cum = Am[m], cum_neg = Nm[m];
            u32 found = 8u, fcn = 0u, fcp = 0u;
            for (u32 i = 0; i < 8u; i++) { // the 8 first-level magnitude bins of the prefix, ascending
                u32 cp = 0u, cn = 0u;
                if (dp >= 3u) {
                    const u32 per = 1u << (dp - 3u), b0 = ((ep >> 5) & 0x7fffu) + i * per;
                    cp = pre2[b0 + per] - pre2[b0];
                }
                if (dn >= 3u) { // negative keys ascend as the magnitude descends
                    const u32 per = 1u << (dn - 3u), b0 = ((en >> 5) & 0x7fffu) + (7u - i) * per;
                    cn = pre2[b0 + per] - pre2[b0];
                }
                if (R < cum + cp + cn) {
                    found = i;
                    fcn = cn;
                    fcp = cp;
                    break;
                }
                cum += (u64)cp + cn;
                cum_neg += cn;
            }
            const u32 j = m * 8u + found;
            ok = found < 8u && j >= st->thr_jlo[tid] && j <= st->thr_jhi[tid];
            if (ok) {
                s_j[tid] = j;
                s_res[tid] = R - cum;
                s_bn[tid] = cum_neg;
                s_bp[tid] = cum - cum_neg;
                s_cn[tid] = fcn;
                s_cp[tid] = fcp;
            }
        }
        if (!ok) atomicOr(&s_miss, 2u << tid); // (bit 0: forced)
    }
    __syncthreads();
    if (s_miss) { // the exact sweeps start from cleared histograms and zero count
        u32 *h1 = B.hist1 + (size_t)t * L1_BINS;
        for (int i = tid; i < L2_BINS; i += BLOCK) {
            h1[i] = 0u;
            h2[i] = 0u;
        }
        if (tid == 0) {
            st->redo = s_miss; // which thresholds missed (bit q + 1), for diagnosis
            st->n_zero = 0ull;
            st->nonfinite = 0u;
        }
        return;
    }
    if (tid == 0) make_buckets(st, n_thr, s_j, s_res, s_bn, s_bp, s_cn, s_cp);
}

// ------------------------------------------------------------------------------------------
// exact thresholds from the gathered buckets
// ------------------------------------------------------------------------------------------
constexpr int TSEL = 1024;
constexpr int SEL_HIST = SEL_WORDS; // words of a tensor's selection histograms ([slot][sign][512])

// The gathered keys of a tensor lie in 16 fragments (one per wave) per (workgroup, tensor) unit,
// all buckets mixed.  Every threshold wants the k-th smallest magnitude among the keys of its
// bucket (one first-level magnitude bin: all keys share the bits above bit 16) and the numbers of
// the bucket's keys below and above it by sign.  Two counting passes over the fragments, one
// workgroup per unit, all thresholds of the tensor together: 9 bits per bucket in the first, the
// remaining 8 bits per threshold (inside the bin its first pass chose) in the second.  A byte table
// over the magnitude bins names the bucket of a key, so a key costs one table read and one or two
// LDS atomics however many thresholds the grid has; the unit's counts are added to the tensor's
// histograms in global memory (the first half of its first-level histogram, which is no longer
// needed).  After each pass one workgroup per tensor picks the bins (wave q scans threshold q); the
// histograms are kept per sign, so the counts of the classes fall out of them: keys below = bins
// below the chosen one in pass 1 + digits below the chosen one in pass 2.
__global__ __launch_bounds__(TSEL) void k_thr_setup(const TDesc *__restrict__ td, Bufs B)
{
    const int t = blockIdx.x;
    TState *st = B.ts + t;
    u32 *gh = B.hist1 + (size_t)t * L1_BINS;
    for (u32 i = threadIdx.x; i < (u32)SEL_HIST; i += TSEL) gh[i] = 0u;
    const bool pooled = td[t].pooled != 0u;
    if (pooled && td[t].leader == (u32)t) { // the group's histograms of both passes
        u32 *ps = B.pool_sel + (size_t)t * 2 * SEL_HIST;
        for (u32 i = threadIdx.x; i < 2u * (u32)SEL_HIST; i += TSEL) ps[i] = 0u;
    }
    if (threadIdx.x != 0) return;
    const u32 n_thr = st->n_thr;
    for (u32 b = 0; b < (u32)MAX_THR; b++) st->sel_nmem[b] = 0u;
    for (u32 q = 0; q < n_thr; q++) { // which thresholds take part, and their ranks
        st->sel_want[q] = 0xFFFFFFFFu;
        st->sel_prefix[q] = 0u;
        st->sel_seen[q] = 0u;
        st->sel_cn[q][0] = st->sel_cn[q][1] = st->sel_cn[q][2] = st->sel_cn[q][3] = 0u;
        const u32 bq = st->thr_bucket[q];
        if (bq == NO_BUCKET) continue; // rank 0 or n - 1 of a tensor whose first sweep was sampled
        const u32 mb = st->bucket_magbin[bq];
        // (a pooled tensor: rank, zeros and bucket population of the whole group)
        const u64 zeros = (mb == 0u) ? (pooled ? B.ts[td[t].leader].pool_zero : st->n_zero) : 0ull;
        const u64 expect = (pooled ? (u64)st->pool_expect[q] : (u64)st->bucket_cnt_neg[bq] + st->bucket_cnt_pos[bq]) - zeros;
        const u64 res = st->thr_res[q];
        if (res < zeros) continue; // the threshold is 0
        if (res - zeros >= expect) {
            atomicOr(&st->internal_err, 8u);
            continue;
        }
        st->sel_k[q] = (u32)(res - zeros);
        st->sel_want[q] = mb << 9; // (completed by the chosen 9-bit prefix after the first pass)
        st->sel_members[bq][st->sel_nmem[bq]++] = (unsigned char)q;
    }
}

template <int ROUND>
__global__ __launch_bounds__(TSEL) void k_thr_count(const TDesc *__restrict__ td,
                                                    const u32 *__restrict__ fu_tensor, Bufs B)
{
    __shared__ u32 hist[SEL_HIST];
    __shared__ unsigned char which[L1_MAGBINS]; // bucket of a magnitude bin + 1, or 0
    __shared__ u32 s_want[MAX_THR], s_nmem[MAX_THR];
    __shared__ unsigned char s_members[MAX_THR][MAX_THR];
    const u32 fu = blockIdx.x;
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 c = B.unit_thr[(size_t)fu * 16 + wave]; // keys in this wave's fragment
    if (__syncthreads_or(c != 0u) == 0) return;
    const int t = (int)fu_tensor[fu];
    const TState *st = B.ts + t;
    const u32 n_thr = st->n_thr, nb = st->n_buckets;
    const u32 n_slots = (ROUND == 0 ? nb : n_thr) * 1024u;
    for (u32 i = tid; i < (u32)L1_MAGBINS / 4u; i += TSEL) reinterpret_cast<u32 *>(which)[i] = 0u;
    for (u32 i = tid; i < n_slots; i += TSEL) hist[i] = 0u;
    if (tid < (u32)MAX_THR) {
        s_want[tid] = tid < n_thr ? st->sel_want[tid] : 0xFFFFFFFFu;
        s_nmem[tid] = st->sel_nmem[tid];
        for (u32 e = 0; e < (u32)MAX_THR; e++) s_members[tid][e] = st->sel_members[tid][e];
    }
    __syncthreads();
    if (tid < nb) which[st->bucket_magbin[tid]] = (unsigned char)(tid + 1u);
    __syncthreads();
    const u32 *list = B.pool + B.unit_off[fu] + (u64)wave * B.unit_capw[fu];
    // smallest / largest magnitude among the gathered keys (first pass): for a tensor whose first
    // sweep was sampled the windows of the ranks 0 and n - 1 were gathered, so these are the
    // tensor's own extremes (exact zeros are never gathered: TState::n_zero tells of them)
    u32 mn = 0xFFFFFFFFu, mx = 0u;
    for (u32 i0 = lane; i0 < c; i0 += 256u) {
        u32 kk[4];
#pragma unroll
        for (int j = 0; j < 4; j++) kk[j] = (i0 + j * 64u < c) ? list[i0 + j * 64u] : 0u;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            if (i0 + j * 64u >= c) continue;
            const u32 mag = mag_of_key(kk[j]);
            if (ROUND == 0) {
                mn = mag < mn ? mag : mn;
                mx = mag > mx ? mag : mx;
            }
            const u32 bk = which[mag >> L1_SHIFT];
            if (bk == 0u) continue; // (gathered for a window of bins, not in a bucket)
            const u32 sgn = key_is_neg(kk[j]) ? 0u : 512u;
            if (ROUND == 0) {
                atomicAdd(&hist[(bk - 1u) * 1024u + sgn + ((mag >> 8) & 511u)], 1u);
            } else {
                const u32 nm = s_nmem[bk - 1u];
                for (u32 e = 0; e < nm; e++) {
                    const u32 q = s_members[bk - 1u][e];
                    if ((mag >> 8) == s_want[q]) atomicAdd(&hist[q * 1024u + sgn + (mag & 255u)], 1u);
                }
            }
        }
    }
    if (ROUND == 0 && td[t].sampled) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const u32 a = __shfl_xor(mn, o), b = __shfl_xor(mx, o);
            mn = a < mn ? a : mn;
            mx = b > mx ? b : mx;
        }
        if (lane == 0u && mx) {
            atomicMin(&B.ts[t].mag_min, mn);
            atomicMax(&B.ts[t].mag_max, mx);
        }
    }
    __syncthreads();
    u32 *gh = B.hist1 + (size_t)t * L1_BINS;
    u32 *ps = td[t].pooled ? B.pool_sel + ((size_t)td[t].leader * 2 + ROUND) * SEL_HIST : nullptr;
    for (u32 i = tid; i < n_slots; i += TSEL) {
        const u32 v = hist[i];
        if (v) {
            atomicAdd(&gh[i], v);
            if (ps) atomicAdd(&ps[i], v); // the group's histogram chooses, the tensor's own counts
        }
    }
}

template <int ROUND>
__global__ __launch_bounds__(TSEL) void k_thr_pick(const TDesc *__restrict__ td, Bufs B)
{
    const int t = blockIdx.x;
    TState *st = B.ts + t;
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u32 n_thr = st->n_thr;
    u32 *gh = B.hist1 + (size_t)t * L1_BINS;
    const bool pooled = td[t].pooled != 0u;
    const u32 *ps = pooled ? B.pool_sel + ((size_t)td[t].leader * 2 + ROUND) * SEL_HIST : gh;
    if (wave < n_thr && st->sel_want[wave] != 0xFFFFFFFFu) { // wave q scans the histogram of threshold q
        const u32 q = wave;
        const u32 slot = ROUND == 0 ? st->thr_bucket[q] : q;
        const u32 *hq = gh + slot * 1024u;  // the tensor's own keys: they are counted
        const u32 *hs = ps + slot * 1024u;  // the keys the rank refers to (the group's when pooled): they choose
        const u32 k = st->sel_k[q];
        u32 ln[8], lp[8], gs[8], sn = 0, sp = 0, sg = 0; // 8 bins per lane
#pragma unroll
        for (int j = 0; j < 8; j++) {
            ln[j] = hq[lane * 8u + j];
            lp[j] = hq[512u + lane * 8u + j];
            gs[j] = pooled ? hs[lane * 8u + j] + hs[512u + lane * 8u + j] : ln[j] + lp[j];
            sn += ln[j];
            sp += lp[j];
            sg += gs[j];
        }
        const u32 incn = wave_incl_scan(sn), incp = wave_incl_scan(sp), incg = wave_incl_scan(sg);
        const u32 totn = __builtin_amdgcn_readlane(incn, 63), totp = __builtin_amdgcn_readlane(incp, 63);
        u32 bn = incn - sn, bp = incp - sp, bg = incg - sg; // keys in the bins before this lane's
        if (ROUND == 0 && lane == 63u) st->sel_seen[q] = incn + incp;
        if (k >= bg && k < incg) {
#pragma unroll
            for (int j = 0; j < 8; j++) {
                if (k >= bg && k < bg + gs[j]) {
                    const u32 digit = lane * 8u + j;
                    st->sel_k[q] = k - bg;
                    st->sel_cn[q][0] += bn;                   // below the chosen bin, by sign
                    st->sel_cn[q][1] += bp;
                    st->sel_cn[q][2] += totn - bn - ln[j];    // above it
                    st->sel_cn[q][3] += totp - bp - lp[j];
                    if (ROUND == 0) {
                        st->sel_prefix[q] = digit;
                        st->sel_want[q] |= digit;
                    } else {
                        st->sel_prefix[q] = (st->sel_prefix[q] << 8) | digit;
                    }
                }
                bn += ln[j];
                bp += lp[j];
                bg += gs[j];
            }
        }
    }
    __syncthreads();
    if (ROUND == 0) { // the second pass starts from cleared histograms
        for (u32 i = tid; i < (u32)SEL_HIST; i += TSEL) gh[i] = 0u;
        return;
    }
    if (tid < n_thr) {
        const u32 q = tid;
        const u32 bq = st->thr_bucket[q];
        if (bq == NO_BUCKET) {
            // (the smallest magnitude is 0 when the tensor holds exact zeros; a tensor of zeros
            // only has gathered nothing, and both extremes are 0)
            const u32 lowest = (st->n_zero || st->mag_min == 0xFFFFFFFFu) ? 0u : st->mag_min;
            st->thr_mag[q] = st->thr_res[q] == 0ull ? lowest : st->mag_max;
            st->thr_lt_neg[q] = st->thr_lt_pos[q] = 0ull; // (used for a prune threshold: nothing below the minimum)
            st->thr_gt_neg[q] = st->thr_gt_pos[q] = 0ull; // (used for a protect threshold: nothing above the maximum)
            return;
        }
        const u32 mb = st->bucket_magbin[bq];
        const u64 zeros = (mb == 0u) ? st->n_zero : 0ull;
        const u64 zeros_ranked = (mb == 0u && pooled) ? B.ts[td[t].leader].pool_zero : zeros;
        u32 tau = 0u;
        // keys of the bucket below / above the threshold, by sign (the zeros were not gathered)
        u32 cn[4] = {0u, 0u, st->bucket_cnt_neg[bq], (u32)(st->bucket_cnt_pos[bq] - zeros)};
        if (st->sel_want[q] != 0xFFFFFFFFu) {
            tau = (mb << L1_SHIFT) | st->sel_prefix[q];
            for (int i = 0; i < 4; i++) cn[i] = st->sel_cn[q][i];
            const u64 expect = (u64)st->bucket_cnt_neg[bq] + st->bucket_cnt_pos[bq] - zeros;
            if ((u64)st->sel_seen[q] != expect) atomicOr(&st->internal_err, 4u);
        } else if (st->thr_res[q] >= zeros_ranked) {
            return; // (rank beyond the bucket: the error bit is set)
        }
        const u64 n = td[t].n, n_neg = st->n_neg, n_pos = n - n_neg;
        st->thr_mag[q] = tau;
        st->thr_lt_neg[q] = st->bucket_below_neg[bq] + cn[0];
        st->thr_lt_pos[q] = st->bucket_below_pos[bq] + cn[1] + ((mb == 0u && tau > 0u) ? zeros : 0ull);
        st->thr_gt_neg[q] = n_neg - st->bucket_below_neg[bq] - st->bucket_cnt_neg[bq] + cn[2];
        st->thr_gt_pos[q] = n_pos - st->bucket_below_pos[bq] - st->bucket_cnt_pos[bq] + cn[3];
    }
}

// ------------------------------------------------------------------------------------------
// plan 2: boundary ranks -> active bins -> groups of active bins
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_plan2(const TDesc *__restrict__ td,
                                                 const GridDesc *__restrict__ gd, Bufs B)
{
    extern __shared__ u32 smem[];
    u32 *cum = smem; // [nb2 + 1]
    __shared__ u32 tmp[BLOCK / 64 + 1];
    __shared__ u64 sAn[MAX_PAIRS], sMn[MAX_PAIRS], sPP[MAX_PAIRS], sM[MAX_PAIRS];

    const int t = blockIdx.x;
    const u32 tid = threadIdx.x;
    const TDesc d = td[t];
    const u64 n = d.n;
    TState *st = B.ts + t;
    const u32 nb2 = st->nb2;
    const u32 zbin = st->zbin;
    const u64 n_zero = st->n_zero;
    const u32 *h2 = B.hist2 + (size_t)t * L2_BINS;
    const u32 *tab = B.table2 + (size_t)t * COARSE;
    u32 *binfo = B.binfo + (size_t)t * L2_BINS;
    u32 *cur = B.cursor2 + (size_t)t * CURSOR_STRIDE;
    const u32 n_pairs = gd->n_pairs, n_p = gd->n_p;

    u32 total = block_excl_scan(h2, cum, (int)nb2, tmp);
    if (tid == 0 && (u64)total != n) atomicOr(&st->internal_err, 16u);
    if (tid < n_pairs) {
        const u32 tp = gd->pair_p[tid], to = n_p + gd->pair_o[tid];
        const u64 n_neg = st->n_neg, n_pos = n - n_neg;
        const u64 Pn = st->thr_lt_neg[tp], Pp = st->thr_lt_pos[tp];
        const u64 An = st->thr_gt_neg[to], Ap = st->thr_gt_pos[to];
        const u64 Mn = n_neg - An - Pn, Mp = n_pos - Ap - Pp;
        st->pair_An[tid] = An;
        st->pair_Ap[tid] = Ap;
        st->pair_Pn[tid] = Pn;
        st->pair_Pp[tid] = Pp;
        st->pair_Mn[tid] = Mn;
        st->pair_M[tid] = Mn + Mp;
        sAn[tid] = An;
        sMn[tid] = Mn;
        sPP[tid] = Pn + Pp;
        sM[tid] = Mn + Mp;
        if (Mn + Mp == 0ull || Mn > n || Mp > n) {
            // (shared thresholds can leave a tensor without quantized values: reported, and the
            // tensor's gathered keys are not processed)
            atomicOr(&st->internal_err, 32u);
            atomicOr(&st->pool_overflow, 8u);
        }
    }
    for (u32 i = tid; i < nb2; i += BLOCK) binfo[i] = 0u;
    __syncthreads();
    const u32 n_bnd = gd->n_bnd;
    const u32 TG = n_pairs * n_bnd;
    u32 *tb = B.tgt_bin + (size_t)t * TGT_STRIDE;
    u32 *tr = B.tgt_res + (size_t)t * TGT_STRIDE;
    u32 *tk = B.tgt_key + (size_t)t * TGT_STRIDE;
    u32 *trank = B.tgt_rank + (size_t)t * TGT_STRIDE;
    for (u32 w = tid; w < TG; w += BLOCK) {
        const u32 q = w / n_bnd, i = q * (u32)NBT + w % n_bnd; // boundary w % n_bnd of pair q
        u32 num, den;
        bnd_fraction(w % n_bnd, num, den);
        const u64 M = sM[q];
        const u64 k = (u64)num * M / (u64)den;
        const u64 r = (k < sMn[q]) ? sAn[q] + k : sAn[q] + sPP[q] + k;
        trank[i] = (u32)r;
        // first index in [0, nb2] with cum[idx] > r
        u32 lo = 0, hi = nb2;
        while (lo < hi) {
            u32 mid = (lo + hi) >> 1;
            if ((u64)cum[mid] > r)
                hi = mid;
            else
                lo = mid + 1;
        }
        if (r >= n || lo == 0u) {
            atomicOr(&st->internal_err, 64u);
            tb[i] = RESOLVED;
            tk[i] = 0u;
            continue;
        }
        u32 bin = lo - 1u;
        u64 res = r - (u64)cum[bin];
        if (bin == zbin && res < n_zero) {
            tb[i] = RESOLVED;
            tr[i] = 0u;
            tk[i] = ZERO_KEY;
            binfo[bin] = 1u; // the bin holds an edge: its other keys are classified one by one
        } else {
            if (bin == zbin) res -= n_zero;
            tb[i] = bin;
            tr[i] = (u32)res;
            binfo[bin] = 1u;
        }
    }
    // the bins of the class edges (first quantized / pruned / protected key of either sign) are
    // active too, so that every bin without an edge lies inside one slot
    for (u32 i = tid; i < n_pairs * 4u; i += BLOCK) {
        const u32 q = i >> 2;
        const u32 key = class_edge_key(i & 3u, st->thr_mag[gd->pair_p[q]], st->thr_mag[n_p + gd->pair_o[q]]);
        binfo[l2_bin(key, tab[key >> COARSE_SHIFT])] = 1u;
    }
    __syncthreads();
    // gathered population of every bin in bin order -> offset of the bin in that order
    for (u32 i = tid; i < nb2; i += BLOCK)
        cur[i] = binfo[i] ? (h2[i] - ((i == zbin) ? (u32)n_zero : 0u)) : 0u;
    __syncthreads();
    const u32 ctot = block_excl_scan(cur, cur, (int)nb2, tmp);
    if (tid == 0 && (u64)ctot > d.pool_len) atomicOr(&st->pool_overflow, 2u); // no room for the keys in group order
    // groups: runs of active bins of about 2^gshift gathered keys; at most MAX_GROUPS per tensor
    u32 gshift = GROUP_SHIFT;
    while ((ctot >> gshift) >= (u32)MAX_GROUPS) gshift++;
    const u32 n_groups = ctot ? ((ctot - 1u) >> gshift) + 1u : 1u; // edges exist even without keys
    u32 *goff = B.grp_off + d.tile0 * 0 + (size_t)t * MAX_GROUPS;
    u32 *gend = B.grp_end + (size_t)t * MAX_GROUPS;
    u32 *gcur = B.grp_cur + (size_t)t * MAX_GROUPS;
    for (u32 g = tid; g < (u32)MAX_GROUPS; g += BLOCK) {
        goff[g] = 0xFFFFFFFFu;
        gend[g] = 0u;
        gcur[g] = 0u;
    }
    __syncthreads();
    u16 *gtab = B.bin_group + (size_t)t * L2_BINS;
    for (u32 i = tid; i < nb2; i += BLOCK) {
        if (binfo[i]) {
            const u32 c = h2[i] - ((i == zbin) ? (u32)n_zero : 0u);
            const u32 g = min(cur[i] >> gshift, n_groups - 1u); // an empty bin at the very end
            atomicMin(&goff[g], cur[i]);
            atomicMax(&gend[g], cur[i] + c);
            gtab[i] = (u16)g;
            binfo[i] = cur[i]; // offset of the bin's keys once they are in bin order
        } else {
            binfo[i] = INACTIVE;
            gtab[i] = 0xFFFFu;
        }
    }
    __syncthreads();
    // per target: the key range of its bin
    u32 *tlo = B.tgt_klo + (size_t)t * TGT_STRIDE;
    u32 *thi = B.tgt_khi + (size_t)t * TGT_STRIDE;
    for (u32 w = tid; w < TG; w += BLOCK) {
        const u32 i = (w / n_bnd) * (u32)NBT + w % n_bnd;
        const u32 bin = tb[i];
        if (bin == RESOLVED) continue;
        // last 12-bit prefix whose first bin is <= bin
        u32 lo = 0, hi = COARSE - 1;
        while (lo < hi) {
            u32 mid = (lo + hi + 1) >> 1;
            if (((tab[mid] >> 5) & 0x7fffu) <= bin)
                lo = mid;
            else
                hi = mid - 1;
        }
        const u32 e = tab[lo], dd = e & 31u, sub = bin - ((e >> 5) & 0x7fffu);
        const u32 klo = (lo << COARSE_SHIFT) | (sub << (COARSE_SHIFT - dd));
        tlo[i] = klo;
        thi[i] = klo + ((1u << (COARSE_SHIFT - dd)) - 1u);
    }
    if (tid == 0) {
        st->cand_total = ctot;
        st->n_groups = n_groups;
        st->gshift = gshift;
    }
    // (the pairs' boundaries lie NBT apart; those a grid does not use are never read)
}

// ------------------------------------------------------------------------------------------
// sweep 3: every key either lies in a bin without an edge, and then its slot is known from the bin
// alone (its value is added to the slot's sum), or it is gathered for the exact boundaries.  Also:
// sums of squares, protected counts per tile.
// ------------------------------------------------------------------------------------------
template <bool FULL>
__device__ __forceinline__ void gather_tile(const float (&v)[16], u32 mask, const u32 *T, const u16 *SEG,
                                            u64 *sx, GLOBAL_AS u32 *gdst, u32 &gathered,
                                            u32 tau_o_min, const u32 *s_tau_o, u32 n_o,
                                            double (&q_out)[MAX_FRAC], u32 (&oc)[MAX_FRAC])
{
    u32 key[16], slot[16];
    float amax = 0.0f; // largest magnitude of the lane's values (entries past the end are 0.0)
#pragma unroll
    for (int i = 0; i < 16; i++) {
        const float xc = v[i] + 0.0f; // -0.0 becomes +0.0
        key[i] = key_of_bits(__float_as_uint(xc));
        slot[i] = T[key[i] >> COARSE_SHIFT];
        amax = fmaxf(amax, fabsf(xc));
    }
#pragma unroll
    for (int i = 0; i < 16; i++) slot[i] = lookup_u16(SEG, key[i], slot[i]);
#pragma unroll
    for (int i = 0; i < 16; i++) {
        const bool valid = FULL || ((mask >> i) & 1u);
        const bool cand = valid && key[i] != ZERO_KEY && slot[i] == 0xFFFFu;
        // (a ballot of each comparison, taken next to it and combined as scalars: the ballot of a
        // combined or an earlier condition would be rebuilt from a vector register)
        u64 cm = __ballot(key[i] != ZERO_KEY) & __ballot(slot[i] == 0xFFFFu);
        if (!FULL) cm &= __ballot(valid);
        // (the keys of a sub-slot share sign and exponent: their values add up as count and sum of
        // mantissas, exactly and in any order; a 64-bit integer add costs the LDS half of what a
        // double add does)
        if (valid && slot[i] != 0xFFFFu) atomicAdd(&sx[slot[i]], (u64)(__float_as_uint(v[i]) & 0x7fffffu));
        if (cand) // (the wave's cursor is a scalar: it goes into the address, not into the rank)
            (gdst + gathered)[__builtin_amdgcn_mbcnt_hi((u32)(cm >> 32), __builtin_amdgcn_mbcnt_lo((u32)cm, 0u))] = key[i];
        gathered += (u32)__popcll(cm);
    }
    // the bits of a non-negative float order like its magnitude image
    if (__ballot(__float_as_uint(amax) > tau_o_min)) { // rare: some value of the wave's 1024 is protected
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const bool valid = FULL || ((mask >> i) & 1u);
            const u32 m = mag_of_key(key[i]);
            if (__ballot(valid && m > tau_o_min)) {
                const double xd = (double)v[i];
#pragma unroll
                for (int o = 0; o < MAX_FRAC; o++) {
                    const bool out = o < (int)n_o && valid && m > s_tau_o[o];
                    if (out) q_out[o] = fma(xd, xd, q_out[o]);
                    oc[o] += (u32)__popcll(__ballot(out));
                }
            }
        }
    }
}


constexpr int SM_GATHER = MAX_SUB * 8 + COARSE * 4 + L2_BINS * 2 + (BLOCK / 64) * 8 + MAX_FRAC * 4;

__global__ __launch_bounds__(BLOCK) void k_gather(const TDesc *__restrict__ td, int nT,
                                                  const u64 *__restrict__ wg_tile0,
                                                  const u32 *__restrict__ wg_fu0,
                                                  const GridDesc *__restrict__ gd, Bufs B)
{
    // one static array (the only one, so it starts at LDS address 0): table offsets then fold into
    // the LDS instructions, which the base of a dynamic array does not allow
    __shared__ __attribute__((aligned(16))) u32 smem[SM_GATHER / 4];
    u64 *sx = reinterpret_cast<u64 *>(smem);                   // [MAX_SUB] sum of mantissas per sub-slot
    u32 *T = smem + 2 * MAX_SUB;                               // [COARSE]
    u16 *SEG = reinterpret_cast<u16 *>(T + COARSE);            // [L2_BINS] sub-slot of the bin, or 0xFFFF
    // (no static LDS arrays: the tables then start at LDS address 0 and their offsets fold into
    // the instructions)
    double *s_red = reinterpret_cast<double *>(SEG + L2_BINS); // [BLOCK / 64]
    u32 *s_tau_o = reinterpret_cast<u32 *>(s_red + BLOCK / 64); // [MAX_FRAC]

    const u32 tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const u64 tile_lo = wg_tile0[blockIdx.x], tile_hi = wg_tile0[blockIdx.x + 1];
    if (tile_lo >= tile_hi) return;
    const u32 n_p = gd->n_p, n_o = gd->n_o;
    int t = find_tensor(td, nT, tile_lo);
    const int t_first = t;
    u64 tile = tile_lo;
    while (tile < tile_hi) {
        const TDesc d = td[t];
        const u64 n_tiles_t = (d.n + TILE - 1) / TILE;
        const u64 t_end = d.tile0 + n_tiles_t;
        const u64 stop = t_end < tile_hi ? t_end : tile_hi;
        TState *st = B.ts + t;
        const u32 n_slots = st->n_sub;
        {
            const u32 *gseg = reinterpret_cast<const u32 *>(B.sl + (size_t)t * (L2_BINS + 64));
            u32 *seg32 = reinterpret_cast<u32 *>(SEG);
            for (u32 i = tid; i < (u32)L2_BINS / 2; i += BLOCK) seg32[i] = gseg[i];
        }
        for (int i = tid; i < COARSE; i += BLOCK) T[i] = entry_for_u16(B.table2[(size_t)t * COARSE + i]);
        for (u32 i = tid; i < n_slots; i += BLOCK) sx[i] = 0ull;
        if (tid < MAX_FRAC) s_tau_o[tid] = (tid < n_o) ? st->thr_mag[n_p + tid] : 0x7fffffffu;
        __syncthreads();
        u32 tau_o_min = 0x7fffffffu;
        for (u32 o = 0; o < n_o; o++) tau_o_min = min(tau_o_min, s_tau_o[o]);
        // keys of active bins go, in arrival order, to a region of the pool that belongs to this
        // wave alone (the workgroup's region starts at its first element of the tensor; a wave's
        // share of it is as large as its share of the elements)
        const u32 fu = wg_fu0[blockIdx.x] + (u32)(t - t_first);
        const u32 capw = B.unit_capw[fu];
        GLOBAL_AS u32 *gdst = gptr(B.pool2) + B.unit_off[fu] + (u64)wave * capw;
        u32 gathered = 0u; // wave-uniform
        bool overflow = false;
        double q_out[MAX_FRAC];
#pragma unroll
        for (int o = 0; o < MAX_FRAC; o++) q_out[o] = 0.0;
        for (; tile < stop; tile++) { // no barrier inside: the waves drift apart freely
            const u64 e0 = (tile - d.tile0) * (u64)TILE;
            const u64 rem = d.n - e0;
            const u32 cnt = rem < (u64)TILE ? (u32)rem : (u32)TILE;
            float v[16];
            const u32 mask = load_tile(d, e0, cnt, v);
            u32 oc[MAX_FRAC]; // protected values of this wave in this tile (wave-uniform)
#pragma unroll
            for (int o = 0; o < MAX_FRAC; o++) oc[o] = 0u;
            if (gathered + (u32)(TILE / (BLOCK / 64)) > capw) { // (as in sweep 2: share too small)
                overflow = true;
                gathered = capw - (u32)(TILE / (BLOCK / 64));
            }
            if (cnt == (u32)TILE) // the same for every lane: the tile code uses ballots
                gather_tile<true>(v, mask, T, SEG, sx, gdst, gathered, tau_o_min, s_tau_o, n_o, q_out, oc);
            else
                gather_tile<false>(v, mask, T, SEG, sx, gdst, gathered, tau_o_min, s_tau_o, n_o, q_out, oc);
            if (lane == 0u) {
#pragma unroll
                for (int o = 0; o < MAX_FRAC; o++)
                    if (oc[o]) atomicAdd(&B.tile_out[tile * MAX_FRAC + o], oc[o]); // cleared beforehand
            }
        }
        __syncthreads();
        // flush partial sums of this (workgroup, tensor) unit in a fixed order
        if (lane == 0u) {
            B.unit_cand[(size_t)fu * 16 + wave] = gathered;
            if (overflow) atomicOr(&st->pool_overflow, 4u);
        }
        u64 *gs = B.mom_sx + (size_t)fu * MAX_SUB;
        for (u32 i = tid; i < n_slots; i += BLOCK) gs[i] = sx[i];
        double *part = B.sq_part + (size_t)fu * SQ_STRIDE;
#pragma unroll
        for (int o = 1; o <= MAX_FRAC; o++) {
            if (o > (int)n_o) break;
            double x = wave_sum_f64(q_out[o - 1]);
            if (lane == 0u) s_red[wave] = x;
            __syncthreads();
            if (tid == 0) {
                double s = 0.0;
                for (int w = 0; w < BLOCK / 64; w++) s += s_red[w];
                part[o] = s;
            }
            __syncthreads();
        }
        t++;
    }
}

// ------------------------------------------------------------------------------------------
// gathered keys -> groups of consecutive active bins (one workgroup per (workgroup, tensor) unit)
// ------------------------------------------------------------------------------------------
constexpr int SPLIT_PER = 8; // keys per thread per step
constexpr int SPLIT_PARTS = 4; // workgroups that share one unit (they take its steps in turn)
constexpr int STAGE_G = 1536;   // most groups of a tensor for the staged stores of the split

__global__ __launch_bounds__(BLOCK) void k_split(const TDesc *__restrict__ td,
                                                 const u32 *__restrict__ fu_tensor, Bufs B)
{
    extern __shared__ u32 smem[];
    u32 *T = smem;                                   // [4096]
    u32 *gcount = T + COARSE;                        // [MAX_GROUPS]
    u32 *gbase = gcount + MAX_GROUPS;                // [MAX_GROUPS]
    u16 *gtab = reinterpret_cast<u16 *>(gbase + MAX_GROUPS); // [32768]

    const u32 fu = blockIdx.x;
    const int t = (int)fu_tensor[fu];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const TDesc d = td[t];
    const TState *st = B.ts + t;
    // every wave splits the fragment that the same wave of the gathering sweep wrote
    const u32 c = B.unit_cand[(size_t)fu * 16 + wave];
    u32 cmax = 0u;
    for (int w = 0; w < BLOCK / 64; w++) cmax = max(cmax, B.unit_cand[(size_t)fu * 16 + w]);
    if (cmax == 0u || st->pool_overflow) return; // (an overflow: the search is repeated with larger pools)
    const u32 nb2 = st->nb2, G = st->n_groups;
    const u32 *src = B.pool2 + B.unit_off[fu] + (u64)wave * B.unit_capw[fu];
    u32 *dst = B.pool + d.pool_grp; // the tensor's span of the first pool, one key per slot in bin-group order
    const u32 *goff = B.grp_off + (size_t)t * MAX_GROUPS;
    u32 *gcur = B.grp_cur + (size_t)t * MAX_GROUPS;
    for (int i = tid; i < COARSE; i += BLOCK) T[i] = B.table2[(size_t)t * COARSE + i];
    for (u32 i = tid; i < nb2; i += BLOCK) gtab[i] = B.bin_group[(size_t)t * L2_BINS + i];
    for (u32 g = tid; g < G; g += BLOCK) gcount[g] = 0u;
    __syncthreads();
    // With at most STAGE_G groups the keys of a step are first put in group order in LDS and stored
    // from there: a wave's 64 stores then go to a few runs of consecutive addresses instead of 64
    // places (the stores of a step were what the kernel waited for).
    const bool staged = G <= (u32)STAGE_G;
    // (then counters and starts take STAGE_G entries each of the two MAX_GROUPS arrays, and the
    // stage what is left of them)
    constexpr int STEP_KEYS = 64 * SPLIT_PER * (BLOCK / 64);
    u16 *glp = reinterpret_cast<u16 *>(gcount + 2 * STAGE_G);    // [STAGE_G] first staged place of each group
    u32 *stage_key = gcount + 2 * STAGE_G + STAGE_G / 2;         // [STEP_KEYS]
    u16 *stage_g = reinterpret_cast<u16 *>(stage_key + STEP_KEYS); // [STEP_KEYS] group of each staged key
    static_assert(2 * STAGE_G + STAGE_G / 2 + STEP_KEYS + STEP_KEYS / 2 <= 2 * MAX_GROUPS, "the stage fits the group arrays");
    __shared__ u32 s_part[BLOCK / 64 + 1];
    if (staged) gbase = gcount + STAGE_G;
    for (u32 base = blockIdx.y * 64u * SPLIT_PER; base < cmax; base += SPLIT_PARTS * 64u * SPLIT_PER) {
        u32 key[SPLIT_PER], gr[SPLIT_PER]; // group << 16 | rank inside (step, group)
#pragma unroll
        for (int j = 0; j < SPLIT_PER; j++) {
            const u32 i = base + lane + j * 64u;
            key[j] = (i < c) ? src[i] : 0u;
        }
#pragma unroll
        for (int j = 0; j < SPLIT_PER; j++) {
            const u32 i = base + lane + j * 64u;
            gr[j] = 0xFFFFFFFFu;
            if (i < c) {
                const u32 g = gtab[l2_bin(key[j], T[key[j] >> COARSE_SHIFT])];
                if (g < G) gr[j] = (g << 16) | atomicAdd(&gcount[g], 1u); // at most 8192 keys per step
            }
        }
        __syncthreads();
        if (!staged) {
            for (u32 g = tid; g < G; g += BLOCK) {
                const u32 k = gcount[g];
                if (k) {
                    gbase[g] = goff[g] + atomicAdd(&gcur[g], k);
                    gcount[g] = 0u;
                }
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < SPLIT_PER; j++) {
                const u32 i = base + lane + j * 64u;
                if (i < c && gr[j] != 0xFFFFFFFFu) dst[gbase[gr[j] >> 16] + (gr[j] & 0xFFFFu)] = key[j];
            }
            __syncthreads();
            continue;
        }
        // two groups per thread: where their keys go in the tensor's group order, and in the stage
        u32 k2[2], tot2 = 0u;
#pragma unroll
        for (u32 h = 0; h < 2u; h++) {
            const u32 g = 2u * tid + h;
            k2[h] = g < G ? gcount[g] : 0u;
            if (k2[h]) {
                gbase[g] = goff[g] + atomicAdd(&gcur[g], k2[h]);
                gcount[g] = 0u;
            }
            tot2 += k2[h];
        }
        const u32 inc = wave_incl_scan(tot2);
        if (lane == 63u) s_part[wave] = inc;
        __syncthreads();
        u32 before = inc - tot2;
        for (u32 w = 0; w < wave; w++) before += s_part[w];
        u32 staged_total = 0u;
        for (u32 w = 0; w < (u32)(BLOCK / 64); w++) staged_total += s_part[w];
        if (2u * tid < G) glp[2u * tid] = (u16)before;
        if (2u * tid + 1u < G) glp[2u * tid + 1u] = (u16)(before + k2[0]);
        __syncthreads();
#pragma unroll
        for (int j = 0; j < SPLIT_PER; j++) {
            const u32 i = base + lane + j * 64u;
            if (i < c && gr[j] != 0xFFFFFFFFu) {
                const u32 g = gr[j] >> 16, at = (u32)glp[g] + (gr[j] & 0xFFFFu);
                stage_key[at] = key[j];
                stage_g[at] = (u16)g;
            }
        }
        __syncthreads();
        for (u32 at = tid; at < staged_total; at += BLOCK) {
            const u32 g = stage_g[at];
            dst[gbase[g] + (at - (u32)glp[g])] = stage_key[at];
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------
// exact boundaries: residual-rank element of the boundary's bin, searched in the bin's group
// ------------------------------------------------------------------------------------------
constexpr int BB = 512;            // threads of a group-sort workgroup: two workgroups share a CU
constexpr int BUCKET_CAP = 8192;   // keys of a group sorted in LDS
constexpr int SORT_ROWS = BUCKET_CAP / BB; // keys per thread
constexpr int EDGE_CAP = MAX_PAIRS * EPP + 11; // edges of a group (all of a tensor's at most) + 1, even
constexpr int SLOT_WIN = 1024;     // slots summed per round (a group rarely has more than a few dozen)
static_assert(2 * EDGE_CAP <= BUCKET_CAP && 2 * SLOT_WIN <= (BB / 64) * 256, "edge scratch fits");

// k-th smallest of the keys in [klo, khi] (khi - klo + 1 a power of two) among a[0..n), by the whole
// workgroup of BB threads: radix select, 8 bits per round, LDS histogram.  *found = keys in the
// range (in sh[2]).
template <class Ptr>
__device__ inline u32 block_select_range(Ptr a, u32 n, u32 klo, u32 khi, u32 k, bool skip_zero,
                                         u32 *hist /*[256]*/, u32 *sh /*[3]*/)
{
    const u32 tid = threadIdx.x;
    int R = __popc(khi - klo); // bits that vary inside the range
    u32 P = 0u;                // chosen high part of (key - klo)
    bool first = true;
    while (R > 0) {
        const int w = R < 8 ? R : 8;
        for (u32 i = tid; i < 256u; i += BB) hist[i] = 0u;
        __syncthreads();
        for (u32 i0 = 0; i0 < n; i0 += 4u * BB) {
            u32 v[4];
#pragma unroll
            for (int j = 0; j < 4; j++) v[j] = (i0 + tid + j * BB < n) ? a[i0 + tid + j * BB] : 0u;
#pragma unroll
            for (int j = 0; j < 4; j++) {
                if (i0 + tid + j * BB >= n || v[j] < klo || v[j] > khi) continue;
                if (skip_zero && v[j] == ZERO_KEY) continue;
                const u32 rel = v[j] - klo;
                if (!first && (rel >> R) != P) continue;
                atomicAdd(&hist[(rel >> (R - w)) & ((1u << w) - 1u)], 1u);
            }
        }
        __syncthreads();
        if (tid < 64u) { // 4 bins per lane
            u32 loc[4], s = 0;
#pragma unroll
            for (int j = 0; j < 4; j++) {
                loc[j] = hist[tid * 4u + j];
                s += loc[j];
            }
            u32 inc = s;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                u32 v = __shfl_up(inc, o);
                if ((int)tid >= o) inc += v;
            }
            u32 run = inc - s;
            if (first && tid == 63u) sh[2] = inc;
            if (k >= run && k < inc) {
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    if (k >= run && k < run + loc[j]) {
                        sh[0] = tid * 4u + j;
                        sh[1] = k - run;
                    }
                    run += loc[j];
                }
            }
        }
        __syncthreads();
        P = first ? sh[0] : ((P << w) | sh[0]);
        k = sh[1];
        R -= w;
        first = false;
        __syncthreads();
    }
    return klo + P;
}

// Stable rank of a key's digit among the keys its wave has seen in this pass.  ORDERED: one
// returning LDS add (same-address LDS atomics are served in ascending lane order, verified when the
// context is created).  Otherwise lanes with equal digits find each other with eight ballots.
template <bool ORDERED>
__device__ __forceinline__ u32 digit_rank(u32 *wcnt, u32 digit, bool valid)
{
    if (ORDERED) {
        u32 r = 0u;
        if (valid) r = atomicAdd(&wcnt[digit], 1u);
        return r;
    }
    const u32 lane = threadIdx.x & 63u;
    u64 peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; b++) {
        const bool bit = (digit >> b) & 1u;
        const u64 m = __ballot(bit);
        peers &= bit ? m : ~m;
    }
    const u32 rank = __popcll(peers & ((1ull << lane) - 1ull));
    u32 old = 0u;
    if (valid) old = wcnt[digit];
    if (valid && rank == 0u) wcnt[digit] = old + (u32)__popcll(peers);
    return old + rank;
}

struct GroupHead { // one (tensor, group) of the work list
    int t;
    u32 g, elo, ehi, goff, n;
};
__device__ __forceinline__ GroupHead group_head(const Bufs &B, const u32 *grp_list, u32 idx)
{
    GroupHead h;
    const u32 packed = grp_list[idx];
    h.t = (int)(packed >> 13);
    h.g = packed & 0x1FFFu;
    h.elo = B.grp_elo[(size_t)h.t * MAX_GROUPS + h.g];
    h.ehi = B.grp_ehi[(size_t)h.t * MAX_GROUPS + h.g];
    h.goff = B.grp_off[(size_t)h.t * MAX_GROUPS + h.g];
    const u32 gend = B.grp_end[(size_t)h.t * MAX_GROUPS + h.g];
    h.n = (h.elo < h.ehi && gend > h.goff) ? gend - h.goff : 0u;
    return h;
}

// One group of active bins per step: its keys are sorted in LDS (least significant digit first,
// digits of equal width of at most 8 bits over the bits in which the keys differ).  Every boundary of the group is read
// at its rank (offset of its bin inside the group + residual rank inside the bin); then all edges
// of the group are known, and the group's keys are counted and summed per slot.  The slot below
// the group's first edge is shared with the group before it: its figures go to the "upper" half
// of the per-slot arrays, all others to the "lower" half, so that every entry has one writer.
// The keys of the next group travel from device memory while this one is worked on.
template <bool ORDERED>
__global__ __launch_bounds__(BB) void k_bucket(const TDesc *__restrict__ td, int nT,
                                               const u32 *__restrict__ grp_list,
                                               const u32 *__restrict__ n_grp_total, Bufs B)
{
    extern __shared__ u32 smem[];
    u32 *bufA = smem;                      // [BUCKET_CAP]
    u32 *bufB = smem + BUCKET_CAP;         // [BUCKET_CAP]
    u32 *wcount = smem + 2 * BUCKET_CAP;   // [8 waves][256 digits]; later the sums of a slot window
    __shared__ u32 hist[256];
    __shared__ u32 sh[3];
    __shared__ u32 s_or, s_and, s_lz;
    __shared__ u32 wsum[4];

    const u32 tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const u32 total = *n_grp_total;
    u32 kpre[SORT_ROWS];
    GroupHead nxt;
    auto prefetch = [&](u32 idx2) {
        nxt = group_head(B, grp_list, idx2);
        if (nxt.n && nxt.n <= (u32)BUCKET_CAP) {
            const GLOBAL_AS u32 *src2 = gptr(B.pool) + td[nxt.t].pool_grp + nxt.goff;
#pragma unroll
            for (int r = 0; r < SORT_ROWS; r++) {
                const u32 i = tid + r * BB;
                kpre[r] = (i < nxt.n) ? src2[i] : 0u;
            }
        }
    };
    if (blockIdx.x < total) prefetch(blockIdx.x);
    for (u32 idx = blockIdx.x; idx < total; idx += gridDim.x) {
        const GroupHead hd = nxt;
        const int t = hd.t;
        const u32 g = hd.g, elo = hd.elo, ehi = hd.ehi, goff = hd.goff, n = hd.n;
        TState *st = B.ts + t;
        __syncthreads();
        if (tid == 0) {
            s_or = 0u;
            s_and = 0xFFFFFFFFu;
            s_lz = 0xFFFFFFFFu;
        }
        __syncthreads();
        const bool sorted = n <= (u32)BUCKET_CAP;
        if (sorted && n) { // keys that were fetched ahead -> LDS
            u32 vo = 0u, va = 0xFFFFFFFFu;
#pragma unroll
            for (int r = 0; r < SORT_ROWS; r++) {
                const u32 i = tid + r * BB;
                if (i < n) {
                    bufA[i] = kpre[r];
                    vo |= kpre[r];
                    va &= kpre[r];
                }
            }
            vo = wave_or(vo);
            va = wave_and(va);
            if (lane == 0u) {
                atomicOr(&s_or, vo);
                atomicAnd(&s_and, va);
            }
        }
        if (idx + gridDim.x < total) prefetch(idx + gridDim.x);
        if (elo >= ehi) continue; // no bin falls into this window of the order
        const u32 n_e = ehi - elo;
        const u32 *src = B.pool + td[t].pool_grp + goff;
        const u32 *tb = B.tgt_bin + (size_t)t * TGT_STRIDE;
        const u32 *tr = B.tgt_res + (size_t)t * TGT_STRIDE;
        const u32 *tlo = B.tgt_klo + (size_t)t * TGT_STRIDE;
        const u32 *thi = B.tgt_khi + (size_t)t * TGT_STRIDE;
        u32 *tk = B.tgt_key + (size_t)t * TGT_STRIDE;
        const u32 *h2 = B.hist2 + (size_t)t * L2_BINS;
        const u32 *binfo = B.binfo + (size_t)t * L2_BINS;
        const u16 *eitem = B.edge_item + (size_t)t * MAX_EDGES;
        u32 *ekey = B.edges + (size_t)t * MAX_EDGES;
        const u32 zbin = st->zbin, nz = (u32)st->n_zero;
        u32 *from = bufA, *to = bufB;
        if (sorted && n) {
            __syncthreads();
            if (ORDERED && (idx & 15u) == 0u) {
                // Cross-check of the ordered ranking, one group in sixteen: every wave ranks the low
                // digit of its first 64 keys with returning adds into its (cleared) counters and from
                // ballots, and leaves the counters cleared.
                u32 *wc0 = wcount + wave * 256u;
                for (u32 i = lane; i < 256u; i += 64u) wc0[i] = 0u;
                const u32 i = wave * 64u + lane;
                const bool valid = i < n;
                const u32 digit = valid ? (bufA[i] & 255u) : 0u;
                u32 got = 0u;
                if (valid) got = atomicAdd(&wc0[digit], 1u);
                u64 peers = __ballot(valid);
#pragma unroll
                for (int b = 0; b < 8; b++) {
                    const bool bit = (digit >> b) & 1u;
                    const u64 m = __ballot(bit);
                    peers &= bit ? m : ~m;
                }
                if (valid && got != (u32)__popcll(peers & ((1ull << lane) - 1ull)))
                    atomicOr(&st->internal_err, 1024u);
                __syncthreads(); // (the passes below clear all counters: not before every wave is done here)
            }
            const u32 dbits = s_or ^ s_and; // bits in which the keys differ
            const u32 rows = (n + BB - 1u) / BB; // rows of 64 keys per wave
            const u32 chunk = rows * 64u;
            u32 *wcnt = wcount + wave * 256u;
            // The keys differ in the bits b_lo .. b_hi only.  These are cut into digits of equal
            // width, at most 8 bits: with fixed 8-bit digits the last one is often two or three bits
            // wide, a wave's 64 keys then share a handful of digit values, and the returning adds on
            // one counter serialise (the top pass took as long as the other two together).
            const u32 b_lo = dbits ? (u32)__ffs((int)dbits) - 1u : 0u;
            const u32 n_bits = dbits ? 32u - (u32)__clz((int)dbits) - b_lo : 0u;
            const u32 n_pass = (n_bits + 7u) >> 3;
            const u32 dwidth = n_pass ? (n_bits + n_pass - 1u) / n_pass : 0u;
            const u32 dmask = (1u << dwidth) - 1u;
            for (u32 pass = 0; pass < n_pass; pass++) {
                const u32 shift = b_lo + pass * dwidth;
                for (u32 i = tid; i < (BB / 64) * 256u; i += BB) wcount[i] = 0u;
                __syncthreads();
                u32 kreg[SORT_ROWS], rreg[SORT_ROWS];
#pragma unroll
                for (u32 r = 0; r < (u32)SORT_ROWS; r++) {
                    kreg[r] = 0u;
                    rreg[r] = 0u;
                    if (r < rows) {
                        const u32 i = wave * chunk + r * 64u + lane;
                        const bool valid = i < n;
                        const u32 k = valid ? from[i] : 0u;
                        kreg[r] = k;
                        rreg[r] = digit_rank<ORDERED>(wcnt, (k >> shift) & dmask, valid);
                    }
                }
                __syncthreads();
                // start of every (digit, wave) run: digits in order, waves in order inside a digit
                u32 tot = 0u, excl = 0u;
                u32 cw[BB / 64]; // this digit's count in every wave
                if (tid < 256u) {
#pragma unroll
                    for (int w = 0; w < BB / 64; w++) cw[w] = wcount[w * 256 + tid];
#pragma unroll
                    for (int w = 0; w < BB / 64; w++) tot += cw[w];
                    const u32 inc = wave_incl_scan(tot);
                    excl = inc - tot;
                    if (lane == 63u) wsum[wave] = inc;
                }
                __syncthreads();
                if (tid < 256u) {
                    u32 run = excl;
#pragma unroll
                    for (u32 w = 0; w < 3u; w++) run += w < wave ? wsum[w] : 0u; // (waves 0..3 scan)
#pragma unroll
                    for (int w = 0; w < BB / 64; w++) {
                        wcount[w * 256 + tid] = run;
                        run += cw[w];
                    }
                }
                __syncthreads();
#pragma unroll
                for (u32 r = 0; r < (u32)SORT_ROWS; r++) {
                    if (r < rows) {
                        const u32 i = wave * chunk + r * 64u + lane;
                        if (i < n) to[wcnt[(kreg[r] >> shift) & dmask] + rreg[r]] = kreg[r];
                    }
                }
                __syncthreads();
                u32 *x = from;
                from = to;
                to = x;
            }
        }
        // the buffer that does not hold the sorted keys, and the digit counters, are free now
        u32 *ek = to;                                   // [n_e] edge keys
        u32 *pp = to + EDGE_CAP;                        // [n_e + 1] keys below each edge (sorted)
        u32 *lcnt = from;                               // [n_e + 1] keys per slot (not sorted)
        double *lsx = reinterpret_cast<double *>(wcount); // [SLOT_WIN] sums of the current window
        __syncthreads();
        if (sorted) {
            for (u32 j = tid; j < n_e; j += BB) {
                const u32 item = eitem[elo + j];
                const u32 q = item / EPP, w = item % EPP;
                u32 key = ekey[elo + j]; // class edges are known beforehand
                if (w < (u32)NBT) {
                    const u32 i = q * NBT + w;
                    const u32 bin = tb[i];
                    if (bin == RESOLVED) {
                        key = ZERO_KEY;
                    } else {
                        const u32 pop = h2[bin] - (bin == zbin ? nz : 0u);
                        const u32 res = tr[i];
                        const u32 pos = binfo[bin] - goff + res;
                        bool ok = res < pop && pos < n;
                        if (ok) {
                            key = from[pos];
                            ok = key >= tlo[i] && key <= thi[i];
                        }
                        if (ok)
                            tk[i] = key;
                        else
                            atomicOr(&st->internal_err, 128u);
                    }
                    ekey[elo + j] = key;
                }
                ek[j] = key;
                u32 lo = 0u, hi = n; // keys of the group below the edge
                while (lo < hi) {
                    const u32 mid = (lo + hi) >> 1;
                    if (from[mid] < key)
                        lo = mid + 1u;
                    else
                        hi = mid;
                }
                pp[j] = lo;
            }
            if (tid == 0u) pp[n_e] = n;
        } else {
            // a group too large for LDS (one bin of very many keys): every boundary is selected
            // from the group's keys in device memory by the whole workgroup
            for (u32 j = tid; j <= n_e; j += BB) lcnt[j] = 0u;
            for (u32 j = 0; j < n_e; j++) {
                const u32 item = eitem[elo + j];
                const u32 q = item / EPP, w = item % EPP;
                u32 key = ekey[elo + j];
                if (w < (u32)NBT) {
                    const u32 i = q * NBT + w;
                    const u32 bin = tb[i];
                    if (bin == RESOLVED) {
                        key = ZERO_KEY;
                    } else {
                        __syncthreads();
                        const u32 res = tr[i];
                        const u32 klo = tlo[i], khi = thi[i];
                        const u32 expect = h2[bin] - ((bin == zbin) ? nz : 0u);
                        key = block_select_range((const GLOBAL_AS u32 *)src, n, klo, khi, res,
                                                 klo == ZERO_KEY, hist, sh);
                        if (tid == 0u) {
                            if (sh[2] != expect || res >= expect)
                                atomicOr(&st->internal_err, 128u);
                            else
                                tk[i] = key;
                        }
                    }
                    if (tid == 0u) ekey[elo + j] = key;
                }
                if (tid == 0u) ek[j] = key;
            }
        }
        __syncthreads();
        // exact zeros are counted, never gathered: they join the slot of the zero key
        if (tid == 0u && nz && binfo[zbin] != INACTIVE && B.bin_group[(size_t)t * L2_BINS + zbin] == g) {
            u32 l = 0u, hi = n_e; // edges at or below the zero key (the edges are in key order)
            while (l < hi) {
                const u32 mid = (l + hi) >> 1;
                if (ek[mid] <= ZERO_KEY)
                    l = mid + 1u;
                else
                    hi = mid;
            }
            s_lz = l;
        }
        if (sorted)
            for (u32 j = tid + 1u; j <= n_e; j += BB)
                if (pp[j] < pp[j - 1u]) atomicOr(&st->internal_err, 512u);
        u32 *gc = B.grp_cnt + (size_t)t * 2 * MAX_EDGES;
        double *gs = B.grp_sx + (size_t)t * 2 * MAX_EDGES;
        // counts and sums per slot, a window of slots at a time
        for (u32 w0 = 0; w0 <= n_e; w0 += SLOT_WIN) {
            for (u32 j = tid; j < (u32)SLOT_WIN; j += BB) lsx[j] = 0.0;
            __syncthreads();
            if (sorted) {
                // every thread walks a run of consecutive sorted keys (odd length: no LDS bank is
                // hit twice by a wave) and adds each slot's part once
                const u32 per = ((n + BB - 1u) / BB) | 1u;
                const u32 i0 = tid * per;
                if (i0 < n) {
                    const u32 i1 = min(n, i0 + per);
                    u32 l = 0u, hi = n_e; // slot of key i0 = edges with pp <= i0
                    while (l < hi) {
                        const u32 mid = (l + hi) >> 1;
                        if (pp[mid] <= i0)
                            l = mid + 1u;
                        else
                            hi = mid;
                    }
                    double acc = 0.0;
                    for (u32 i = i0; i < i1; i++) {
                        if (l < n_e && pp[l] <= i) { // key i lies above edge l: slot l is complete
                            if (acc != 0.0 && l - w0 < (u32)SLOT_WIN) atomicAdd(&lsx[l - w0], acc);
                            acc = 0.0;
                            l++;
                            if (l < n_e && pp[l] <= i) { // more edges at the same place (thousands,
                                u32 b = n_e;             // when most boundaries are the zero key)
                                while (l < b) {
                                    const u32 mid = (l + b) >> 1;
                                    if (pp[mid] <= i)
                                        l = mid + 1u;
                                    else
                                        b = mid;
                                }
                            }
                        }
                        acc += (double)__uint_as_float(bits_of_key(from[i]));
                    }
                    if (acc != 0.0 && l - w0 < (u32)SLOT_WIN) atomicAdd(&lsx[l - w0], acc);
                }
            } else {
                for (u32 i = tid; i < n; i += BB) {
                    const u32 key = gptr(src)[i];
                    u32 l = 0u, hi = n_e; // edges at or below the key
                    while (l < hi) {
                        const u32 mid = (l + hi) >> 1;
                        if (ek[mid] <= key)
                            l = mid + 1u;
                        else
                            hi = mid;
                    }
                    if (l - w0 < (u32)SLOT_WIN) {
                        atomicAdd(&lcnt[l], 1u);
                        atomicAdd(&lsx[l - w0], (double)__uint_as_float(bits_of_key(key)));
                    }
                }
            }
            __syncthreads();
            for (u32 j = w0 + tid; j <= n_e && j < w0 + (u32)SLOT_WIN; j += BB) {
                u32 c = sorted ? pp[j] - (j ? pp[j - 1u] : 0u) : lcnt[j];
                if (j == s_lz) c += nz;
                const u32 half = j ? 0u : (u32)MAX_EDGES; // slot elo: this group holds its upper edge
                gc[half + elo + j] = c;
                gs[half + elo + j] = lsx[j - w0];
            }
            __syncthreads();
        }
    }
}

// list of all (tensor, group) pairs of the batch (one workgroup per tensor; the order of the list
// is the order in which the group sort takes them and does not matter)
__global__ __launch_bounds__(256) void k_group_list(int nT, Bufs B, u32 *grp_list, u32 *n_grp_total)
{
    __shared__ u32 s_at;
    const int t = blockIdx.x;
    const u32 G = B.ts[t].pool_overflow ? 0u : B.ts[t].n_groups; // (overflow: nothing valid to sort)
    if (G == 0u) return;
    if (threadIdx.x == 0) s_at = atomicAdd(n_grp_total, G);
    __syncthreads();
    const u32 at = s_at;
    for (u32 g = threadIdx.x; g < G; g += 256u) grp_list[at + g] = ((u32)t << 13) | g;
}

// ------------------------------------------------------------------------------------------
// launch wrappers
// ------------------------------------------------------------------------------------------
constexpr int SM_PLAN1 = (2 * (L1_MAGBINS + 4) + COARSE + 4) * 4;
constexpr int SM_PLAN2 = (L2_BINS + 4) * 4;
constexpr int SM_SPLIT = (COARSE + 2 * MAX_GROUPS) * 4 + L2_BINS * 2;
constexpr int SM_BUCKET = (2 * BUCKET_CAP + (BB / 64) * 256) * 4;

static bool g_attr_done = false;
static hipError_t set_attrs()
{
    if (g_attr_done) return hipSuccess;
    hipError_t e;
    if ((e = hipFuncSetAttribute((const void *)k_plan1<false>, hipFuncAttributeMaxDynamicSharedMemorySize, SM_PLAN1))) return e;
    if ((e = hipFuncSetAttribute((const void *)k_plan1<true>, hipFuncAttributeMaxDynamicSharedMemorySize, SM_PLAN1))) return e;
    if ((e = hipFuncSetAttribute((const void *)k_plan2, hipFuncAttributeMaxDynamicSharedMemorySize, SM_PLAN2))) return e;
    if ((e = hipFuncSetAttribute((const void *)k_plan1b, hipFuncAttributeMaxDynamicSharedMemorySize, SM_PLAN2))) return e;
    if ((e = hipFuncSetAttribute((const void *)k_split, hipFuncAttributeMaxDynamicSharedMemorySize, SM_SPLIT))) return e;
    if ((e = hipFuncSetAttribute((const void *)k_bucket<true>, hipFuncAttributeMaxDynamicSharedMemorySize, SM_BUCKET))) return e;
    if ((e = hipFuncSetAttribute((const void *)k_bucket<false>, hipFuncAttributeMaxDynamicSharedMemorySize, SM_BUCKET))) return e;
    g_attr_done = true;
    return hipSuccess;
}

hipError_t launch_select(const Batch &bt, hipStream_t s)
{
    hipError_t e = set_attrs();
    if (e) return e;
    const Bufs &B = bt.bufs;
    PROF("k_hist1", s, (k_hist<1, false><<<bt.n_wg, BLOCK, 0, s>>>(bt.td, bt.nT, bt.wg_tile0, bt.wg_fu0, B)));
    if (bt.any_pooled) PROF("k_pool_sum", s, k_pool_sum<<<bt.nT, BLOCK, 0, s>>>(bt.td, B));
    PROF("k_plan1", s, k_plan1<false><<<bt.nT, BLOCK, SM_PLAN1, s>>>(bt.td, bt.gd, B));
    PROF("k_hist2", s, (k_hist<2, false><<<bt.n_wg, BLOCK, 0, s>>>(bt.td, bt.nT, bt.wg_tile0, bt.wg_fu0, B)));
    if (bt.any_sampled) {
        // tensors whose sweep 1 was sampled: exact figures from the second histogram; those whose
        // thresholds were mispredicted take the exact sweeps (the kernels skip all other tensors)
        PROF("k_plan1b", s, k_plan1b<<<bt.nT, BLOCK, SM_PLAN2, s>>>(bt.td, bt.gd, B, bt.force_miss ? 1u : 0u));
        PROF("k_hist1_redo", s, (k_hist<1, true><<<bt.n_wg, BLOCK, 0, s>>>(bt.td, bt.nT, bt.wg_tile0, bt.wg_fu0, B)));
        PROF("k_plan1_redo", s, k_plan1<true><<<bt.nT, BLOCK, SM_PLAN1, s>>>(bt.td, bt.gd, B));
        PROF("k_hist2_redo", s, (k_hist<2, true><<<bt.n_wg, BLOCK, 0, s>>>(bt.td, bt.nT, bt.wg_tile0, bt.wg_fu0, B)));
    }
    PROF("k_thr_setup", s, k_thr_setup<<<bt.nT, TSEL, 0, s>>>(bt.td, B));
    PROF("k_thr_count", s, k_thr_count<0><<<bt.n_units, TSEL, 0, s>>>(bt.td, bt.fu_tensor, B));
    PROF("k_thr_pick", s, k_thr_pick<0><<<bt.nT, TSEL, 0, s>>>(bt.td, B));
    PROF("k_thr_count", s, k_thr_count<1><<<bt.n_units, TSEL, 0, s>>>(bt.td, bt.fu_tensor, B));
    PROF("k_thr_pick", s, k_thr_pick<1><<<bt.nT, TSEL, 0, s>>>(bt.td, B));
    PROF("k_plan2", s, k_plan2<<<bt.nT, BLOCK, SM_PLAN2, s>>>(bt.td, bt.gd, B));
    if (bt.light) return hipGetLastError();
    if ((e = launch_edges(bt, s))) return e;
    PROF("k_gather", s, k_gather<<<bt.n_wg, BLOCK, 0, s>>>(bt.td, bt.nT, bt.wg_tile0, bt.wg_fu0, bt.gd, B));
    PROF("k_group_list", s, k_group_list<<<bt.nT, 256, 0, s>>>(bt.nT, B, bt.grp_list, bt.n_grp_total));
    PROF("k_split", s, k_split<<<dim3(bt.n_units, SPLIT_PARTS), BLOCK, SM_SPLIT, s>>>(bt.td, bt.fu_tensor, B));
    if (bt.lds_ordered)
        PROF("k_bucket", s, k_bucket<true><<<bt.n_bucket_blocks, BB, SM_BUCKET, s>>>(bt.td, bt.nT, bt.grp_list, bt.n_grp_total, B));
    else
        PROF("k_bucket_ballots", s, k_bucket<false><<<bt.n_bucket_blocks, BB, SM_BUCKET, s>>>(bt.td, bt.nT, bt.grp_list, bt.n_grp_total, B));
    return hipGetLastError();
}

} // namespace inshr
