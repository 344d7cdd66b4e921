// Boundaries from the log-space sketch and weighted K-Means on its buckets (Sec. 4.3 / Algorithm 1,
// Sec. 4.4 / Algorithms 2 and 3), as an alternative to the equal-population bins of the search: the
// values between the two thresholds are counted per bucket (sign, ceil(log_gamma |x|)), the
// buckets are clustered with sample weights sigma * frequency + (1 - sigma) * magnitude (both
// divided by their largest entry), and the cluster centres become the codebook; the quantizer then
// runs with the midpoints of neighbouring centres as boundaries.
//
//   k_sketch_hist    one more sweep over the tensors (4 bytes per element, like the search's
//                    sweeps): a table in LDS maps the magnitude's top 14 bits to the first bucket
//                    that its 2^17 magnitudes touch and the largest magnitude of that bucket (a
//                    range of 2^(1/64) never touches more than two buckets for alpha >= 0.01), so
//                    the bucket is one LDS read, an add and a shift; the counts go to an LDS
//                    histogram (positive buckets, negative buckets, zeros).  Zeros and denormals,
//                    whose ranges are wider, are set aside and search the bucket list.
//   k_sketch_kmeans  one workgroup per tensor: compacts the non-empty buckets, draws the K
//                    starting centres (running sums by a block scan, the draw itself by the one
//                    thread whose share holds it), then Lloyd rounds on the sorted list — a
//                    cluster is a contiguous run of buckets, found by bisection on the midpoints
//                    and summed in index order by one thread — until the runs repeat.
//                    All arithmetic is fp64 without contraction (products and sums rounded
//                    separately).  For the search over the bit width (Sec. 5 restricted to the
//                    number of bins) the draws are made once for 256 clusters and the rounds run
//                    for 4, 8, ..., 256 clusters from the first 4, 8, ... draws.
//   k_sketch_score   the search's sweep: all boundaries of the seven sets, sorted, cut the key axis
//                    into at most 502 slots; the slot of a key comes from the equal-population
//                    bins of the threshold search (a table gives the slot of every bin without a
//                    boundary; in the few bins with one the key is compared with the boundaries
//                    from the bin's first one on); count and sum per slot in LDS, added to the
//                    tensor's arrays in global memory.
//   k_sketch_choose  per tensor: the error of every set from the slot moments, the fewest bits
//                    within the bound, and that set's keys and centres for the quantizer.
#include "inshr_sketch.h"

// The clustering follows its definition operation by operation: no product may be fused into the
// sum that takes it.  The __dmul_rn / __dadd_rn of the HIP headers are plain operators compiled with
// the headers' own contraction setting, so the operations are written here, with contraction off.
#pragma clang fp contract(off)

namespace inshr {

__device__ __forceinline__ double mul_rn(double a, double b) { return a * b; }
__device__ __forceinline__ double add_rn(double a, double b) { return a + b; }
__device__ __forceinline__ double sub_rn(double a, double b) { return a - b; }
__device__ __forceinline__ double div_rn(double a, double b) { return a / b; }

// Histogram layout: positive bucket b at b, negative bucket b at SK_MAX_IDX + b, zeros at
// 2 * SK_MAX_IDX.  Bucket of a denormal or zero magnitude (rare): search of the bucket list.
__device__ __noinline__ u32 sketch_slot_small(u32 bits, const SketchParams &P)
{
    const u32 mag = bits & 0x7fffffffu;
    if (mag == 0u) return 2u * (u32)SK_MAX_IDX;
    u32 lo = 0u, hi = P.n_idx - 1u;
    while (lo < hi) { // first bucket whose largest magnitude reaches mag
        const u32 mid = (lo + hi) >> 1;
        if (P.tops[mid] >= mag)
            hi = mid;
        else
            lo = mid + 1u;
    }
    return lo + (bits >> 31) * (u32)SK_MAX_IDX;
}

// LIGHT: also the protected values of the tile (wave-uniform count) and their squares.
template <bool FULL, bool LIGHT>
__device__ __forceinline__ void sketch_tile(const float (&v)[16], u32 mask, u32 tau_p, u32 tau_o,
                                            const u32 *cell, u32 *h, const SketchParams &P, u32 &n_prot,
                                            double &q_prot)
{
    u32 small = 0u; // elements between the thresholds whose magnitude is zero or denormal
#pragma unroll
    for (int i = 0; i < 16; i++) {
        const u32 bits = __float_as_uint(v[i]);
        const u32 mag = bits & 0x7fffffffu;
        bool take = mag >= tau_p && mag <= tau_o;
        if (!FULL) take = take && ((mask >> i) & 1u);
        if (LIGHT) {
            const bool prot = mag > tau_o && (FULL || ((mask >> i) & 1u));
            const u64 pm = __ballot(prot);
            if (pm) {
                n_prot += (u32)__popcll(pm);
                if (prot) q_prot = fma((double)v[i], (double)v[i], q_prot);
            }
        }
        if (take && mag < 0x00800000u) small |= 1u << i;
        if (take && mag >= 0x00800000u) {
            // entry = first bucket of the cell << 17 | (2^17 - 1 - low bits of that bucket's largest
            // magnitude): the sum carries into the bucket field when the magnitude lies above it
            const u32 b = (cell[mag >> 17] + (mag & 0x1FFFFu)) >> 17;
            atomicAdd(&h[b + (bits >> 31) * (u32)SK_MAX_IDX], 1u);
        }
    }
    if (__ballot(small != 0u)) {
#pragma unroll 1
        for (int i = 0; i < 16; i++)
            if ((small >> i) & 1u) atomicAdd(&h[sketch_slot_small(__float_as_uint(v[i]), P)], 1u);
    }
}

template <bool LIGHT>
__global__ __launch_bounds__(BLOCK) void k_sketch_hist(const TDesc *__restrict__ td, int nT,
                                                       const u64 *__restrict__ wg_tile0,
                                                       const u32 *__restrict__ wg_fu0,
                                                       const GridDesc *__restrict__ gd,
                                                       const SketchDesc *__restrict__ sd,
                                                       SketchParams P, Bufs B)
{
    // one static array (it starts at LDS address 0, so offsets fold into the LDS instructions)
    __shared__ u32 smem[SK_CELLS + SK_HIST];
    u32 *cell = smem;
    u32 *h = smem + SK_CELLS;
    __shared__ double s_q[BLOCK / 64];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u64 tile_lo = wg_tile0[blockIdx.x], tile_hi = wg_tile0[blockIdx.x + 1];
    if (tile_lo >= tile_hi) return;
    for (int i = tid; i < SK_CELLS; i += BLOCK) cell[i] = P.cell[i];
    for (int i = tid; i < SK_HIST; i += BLOCK) h[i] = 0u;
    int t = find_tensor(td, nT, tile_lo);
    const int t_first = t;
    u64 tile = tile_lo;
    while (tile < tile_hi) {
        const TDesc d = td[t];
        const u64 n_tiles_t = (d.n + TILE - 1) / TILE;
        const u64 t_end = d.tile0 + n_tiles_t;
        const u64 stop = t_end < tile_hi ? t_end : tile_hi;
        const SketchDesc s = sd[t];
        if (!s.active) {
            tile = stop;
            t++;
            continue;
        }
        const TState *st = B.ts + t;
        const u32 pair = gd->cfg_pair[s.cfg];
        const u32 o = gd->pair_o[pair];
        const u32 tau_p = st->thr_mag[gd->pair_p[pair]], tau_o = st->thr_mag[gd->n_p + o];
        double q_prot = 0.0; // squares of this thread's protected values
        __syncthreads();
        for (; tile < stop; tile++) {
            const u64 e0 = (tile - d.tile0) * (u64)TILE;
            const u64 rem = d.n - e0;
            const u32 cnt = rem < (u64)TILE ? (u32)rem : (u32)TILE;
            float v[16];
            const u32 mask = load_tile(d, e0, cnt, v);
            u32 n_prot = 0u; // protected values of this wave in the tile (wave-uniform)
            if (cnt == (u32)TILE)
                sketch_tile<true, LIGHT>(v, mask, tau_p, tau_o, cell, h, P, n_prot, q_prot);
            else
                sketch_tile<false, LIGHT>(v, mask, tau_p, tau_o, cell, h, P, n_prot, q_prot);
            if (LIGHT && lane == 0u && n_prot) atomicAdd(&B.tile_out[tile * MAX_FRAC + o], n_prot);
        }
        if (LIGHT) { // this unit's sum of squares of the protected values, in a fixed order
            q_prot = wave_sum_f64(q_prot);
            if (lane == 0u) s_q[wave] = q_prot;
        }
        __syncthreads();
        if (LIGHT && tid == 0) {
            double sum = 0.0;
            for (int w = 0; w < BLOCK / 64; w++) sum += s_q[w];
            B.sq_part[(size_t)(wg_fu0[blockIdx.x] + (u32)(t - t_first)) * SQ_STRIDE + 1u + o] = sum;
        }
        u32 *gh = P.hist + (size_t)t * SK_HIST;
        for (int i = tid; i < SK_HIST; i += BLOCK) {
            const u32 c = h[i];
            if (c) {
                atomicAdd(&gh[i], c);
                h[i] = 0u;
            }
        }
        t++;
    }
}

// histogram slot of position v in value order: negative buckets descending, zeros, positive ascending
__device__ __forceinline__ u32 slot_in_value_order(u32 v)
{
    if (v < (u32)SK_MAX_IDX) return 2u * (u32)SK_MAX_IDX - 1u - v;
    if (v == (u32)SK_MAX_IDX) return 2u * (u32)SK_MAX_IDX;
    return v - (u32)SK_MAX_IDX - 1u;
}
// value of the bucket at position slot of the histogram
__device__ __forceinline__ double slot_value(u32 slot, const SketchParams &P)
{
    if (slot == 2u * (u32)SK_MAX_IDX) return 0.0;
    if (slot < (u32)SK_MAX_IDX) return P.rep[slot];
    return -P.rep[slot - (u32)SK_MAX_IDX];
}

__global__ __launch_bounds__(BLOCK) void k_sketch_kmeans(const GridDesc *__restrict__ gd,
                                                         const SketchDesc *__restrict__ sd,
                                                         SketchParams P)
{
    __shared__ u32 s_u32[BLOCK / 64 + 2];
    __shared__ double s_red[2 * (BLOCK / 64)];
    __shared__ double cen[256], craw[256];
    __shared__ u32 seg[257], seg_prev[257];
    __shared__ u32 s_pick[2], s_last[2], s_changed, s_chosen;
    const int t = blockIdx.x;
    const SketchDesc s = sd[t];
    if (!s.active) return;
    const u32 tid = threadIdx.x, lane = tid & 63u;
    // one set of centres for the configuration's bits, or (P.multi) one for each of 2 .. 8 bits: the
    // draws of a narrower set are the first draws of the widest
    const u32 K = P.multi ? 256u : 1u << gd->cfg_bits[s.cfg];
    const u32 n_sets = P.multi ? (u32)SK_SETS : 1u;
    const u32 *h = P.hist + (size_t)t * SK_HIST;
    // bucket values, weights and squared distances: in LDS when the list is short enough (a few
    // hundred to a few thousand buckets is the rule), else in the tensor's scratch rows
    __shared__ double l_x[SK_LDS], l_w[SK_LDS], l_d[SK_LDS];

    // ---- the non-empty buckets in value order (Algorithm 1: unique with counts) ----
    constexpr u32 PER = (SK_HIST + BLOCK - 1) / BLOCK;
    u32 mine = 0u, cmax = 0u;
    for (u32 i = 0; i < PER; i++) {
        const u32 v = tid * PER + i;
        const u32 c = v < (u32)SK_HIST ? h[slot_in_value_order(v)] : 0u;
        mine += c ? 1u : 0u;
        cmax = c > cmax ? c : cmax;
    }
    u32 inc = wave_incl_scan(mine);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const u32 y = __shfl_xor(cmax, o);
        cmax = y > cmax ? y : cmax;
    }
    if (lane == 63u) s_u32[tid >> 6] = inc;
    if (lane == 0u) seg_prev[tid >> 6] = cmax; // (scratch until the Lloyd rounds)
    __syncthreads();
    u32 base = 0u, m = 0u, maxc = 0u;
    for (u32 wv = 0; wv < BLOCK / 64; wv++) {
        const u32 y = s_u32[wv];
        if (wv < (tid >> 6)) base += y;
        m += y;
        maxc = seg_prev[wv] > maxc ? seg_prev[wv] : maxc;
    }
    const bool fits = m <= (u32)SK_LDS;
    double *xq = fits ? l_x : P.xq + (size_t)t * SK_HIST;
    double *w = fits ? l_w : P.w + (size_t)t * SK_HIST;
    double *dist = fits ? l_d : P.d + (size_t)t * SK_HIST;
    u32 pos = base + inc - mine;
    for (u32 i = 0; i < PER; i++) {
        const u32 v = tid * PER + i;
        const u32 slot = slot_in_value_order(v < (u32)SK_HIST ? v : 0u);
        const u32 c = v < (u32)SK_HIST ? h[slot] : 0u;
        if (c) {
            xq[pos] = slot_value(slot, P);
            w[pos] = (double)c; // the count, replaced by the weight below
            pos++;
        }
    }
    __syncthreads();
    if (m == 0u) { // (cannot happen: at least one value lies between the thresholds)
        if (tid == 0) {
            P.info[t].n_buckets = 0u;
            P.info[t].rounds = 0u;
        }
        return;
    }
    // ---- sample weights (Algorithm 2): sigma * C / max C + (1 - sigma) * |X| / max |X| ----
    const double x_first = fabs(xq[0]), x_last = fabs(xq[m - 1u]);
    const double mx = x_first > x_last ? x_first : x_last;
    const double one_minus = sub_rn(1.0, P.sigma);
    __syncthreads();
    for (u32 i = tid; i < m; i += BLOCK) {
        const double c_hat = div_rn(w[i], (double)maxc);
        const double x_hat = mx > 0.0 ? div_rn(fabs(xq[i]), mx) : 0.0;
        w[i] = add_rn(mul_rn(P.sigma, c_hat), mul_rn(one_minus, x_hat));
    }
    __syncthreads();

    // ---- weighted K-Means++ draws (Algorithm 3) ----
    const u32 per = (m + BLOCK - 1u) / BLOCK;
    const u32 lo = tid * per < m ? tid * per : m, hi = lo + per < m ? lo + per : m;
    double *uni = cen; // the draws' random numbers (the sorted centres take this array afterwards)
    if (tid < 256u) uni[tid] = P.uniforms[(size_t)t * 256 + tid];
    if (tid < 2u) {
        s_pick[tid] = 0xFFFFFFFFu;
        s_last[tid] = 0u;
    }
    __syncthreads();
    // Per draw: (1) every thread sums the probabilities of its share, a wave scan gives the running
    // sums inside the wave, the wave totals go to LDS; (2) every thread adds the totals of the
    // waves before its own (in wave order) and the first thread whose running sum exceeds the
    // target announces itself; (3) that thread walks its share.  With at most one bucket per
    // thread (the rule) step 3 is empty.  The LDS cells alternate between two copies from draw to
    // draw, so that a draw never waits for the cells of the one before to be read.
    for (u32 r = 0; r < K; r++) {
        const u32 cp = r & 1u;
        double sum = 0.0;
        u32 last_pos = 0u; // last bucket of the share that could be drawn, + 1
        for (u32 i = lo; i < hi; i++) {
            const double p = r ? mul_rn(dist[i], w[i]) : w[i];
            sum = add_rn(sum, p);
            if (p > 0.0) last_pos = i + 1u;
        }
        double inc = sum;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const double y = __shfl_up(inc, o);
            if ((int)lane >= o) inc = add_rn(inc, y);
        }
        const double before = __shfl_up(inc, 1); // inclusive value of the lane below
        if (lane == 63u) s_red[cp * (BLOCK / 64) + (tid >> 6)] = inc;
        __syncthreads();
        double wbase = 0.0, total = 0.0;
        for (u32 wv = 0; wv < BLOCK / 64; wv++) {
            if (wv == (tid >> 6)) wbase = total;
            total = add_rn(total, s_red[cp * (BLOCK / 64) + wv]);
        }
        if (r > 0u && !(total > 0.0)) { // every bucket is a centre already: repeat the last one
            if (tid == 0) craw[r] = craw[r - 1u];
            continue; // (nothing of this draw's cells is used again before two more barriers)
        }
        const double target = mul_rn(uni[r], total);
        const double excl = lane ? add_rn(wbase, before) : wbase;
        const double incl = add_rn(wbase, inc);
        // one atomic per wave: its first lane above the target, its last lane with a drawable bucket
        const u64 above = __ballot(incl > target), drawable = __ballot(last_pos != 0u);
        if (above && lane == (u32)__builtin_ctzll(above)) atomicMin(&s_pick[cp], tid);
        if (drawable && lane == 63u - (u32)__builtin_clzll(drawable)) atomicMax(&s_last[cp], last_pos);
        __syncthreads();
        const u32 pick = s_pick[cp];
        u32 j;
        if (per == 1u) {
            // no running sum exceeds the target (rounding): the last bucket that could be drawn
            j = pick != 0xFFFFFFFFu ? pick : (s_last[cp] ? s_last[cp] - 1u : 0u);
            if (tid == 0) {
                craw[r] = xq[j];
                s_pick[cp ^ 1u] = 0xFFFFFFFFu;
                s_last[cp ^ 1u] = 0u;
            }
        } else {
            if (tid == (pick == 0xFFFFFFFFu ? 0u : pick)) {
                u32 jj = s_last[cp] ? s_last[cp] - 1u : 0u;
                if (pick != 0xFFFFFFFFu) {
                    double run = excl; // the running sum at the start of this thread's share
                    jj = last_pos ? last_pos - 1u : lo;
                    for (u32 i = lo; i < hi; i++) {
                        run = add_rn(run, r ? mul_rn(dist[i], w[i]) : w[i]);
                        if (run > target) {
                            jj = i;
                            break;
                        }
                    }
                }
                s_chosen = jj;
                craw[r] = xq[jj];
                s_pick[cp ^ 1u] = 0xFFFFFFFFu;
                s_last[cp ^ 1u] = 0u;
            }
            __syncthreads();
            j = s_chosen;
        }
        const double cj = xq[j];
        for (u32 i = lo; i < hi; i++) {
            const double df = sub_rn(xq[i], cj);
            const double d2 = mul_rn(df, df);
            dist[i] = (r == 0u || d2 < dist[i]) ? d2 : dist[i];
        }
    }
    __syncthreads();
    u32 rounds = 0u;
    for (u32 set = 0; set < n_sets; set++) {
        const u32 bits = P.multi ? 2u + set : gd->cfg_bits[s.cfg];
        const u32 Kb = 1u << bits;
        // ---- sort the centres ----
        __syncthreads();
        if (tid < Kb) {
            const double x = craw[tid];
            u32 rank = 0u;
            for (u32 i = 0; i < Kb; i++) {
                const double y = craw[i];
                rank += (y < x || (y == x && i < tid)) ? 1u : 0u;
            }
            cen[rank] = x;
        }
        __syncthreads();
        // ---- weighted Lloyd rounds: cluster j = buckets (mid[j-1], mid[j]] ----
        rounds = 0u;
        for (u32 it = 0; it < P.max_iter; it++) {
            if (tid == 0) s_changed = (it == 0u) ? 1u : 0u;
            __syncthreads();
            if (tid <= Kb) {
                u32 first = 0u;
                if (tid == Kb) {
                    first = m;
                } else if (tid > 0u) {
                    const double mid = mul_rn(add_rn(cen[tid - 1u], cen[tid]), 0.5);
                    u32 a = 0u, b = m; // first bucket above the midpoint
                    while (a < b) {
                        const u32 c = (a + b) >> 1;
                        if (xq[c] > mid)
                            b = c;
                        else
                            a = c + 1u;
                    }
                    first = a;
                }
                seg[tid] = first;
                if (it > 0u && seg_prev[tid] != first) s_changed = 1u;
            }
            __syncthreads();
            if (!s_changed) break;
            if (tid < Kb) {
                double sw = 0.0, swx = 0.0;
                for (u32 i = seg[tid]; i < seg[tid + 1u]; i++) {
                    sw = add_rn(sw, w[i]);
                    swx = add_rn(swx, mul_rn(w[i], xq[i]));
                }
                if (sw > 0.0) cen[tid] = div_rn(swx, sw);
            }
            if (tid <= Kb) seg_prev[tid] = seg[tid];
            rounds++;
            __syncthreads();
        }
        __syncthreads();
        // ---- codebook and boundaries ----
        const u32 sh = 8u - bits;
        u32 *ak = P.alt_key + ((size_t)t * n_sets + set) * 256;
        float *acb = P.alt_cb + ((size_t)t * n_sets + set) * 256;
        if (tid < 256u) ak[tid] = 0u;
        __syncthreads();
        if (tid < Kb) {
            acb[tid] = __double2float_rn(cen[tid]);
            if (tid + 1u < Kb) {
                const double a = (double)__double2float_rn(cen[tid]), b = (double)__double2float_rn(cen[tid + 1u]);
                const double mid = mul_rn(add_rn(a, b), 0.5);
                // a value goes to the upper centre when it lies strictly above the midpoint: the
                // boundary is the smallest fp32 number above it
                ak[((tid + 1u) << sh) - 1u] = key_of_float(__double2float_rd(mid)) + 1u;
            }
        } else if (tid < 256u) {
            acb[tid] = 0.0f;
        }
        if (tid == 0 && P.multi) P.set_rounds[(size_t)t * SK_SETS + set] = rounds;
    }
    if (tid == 0) {
        P.info[t].n_buckets = m;
        P.info[t].rounds = rounds;
    }
}

// ------------------------------------------------------------------------------------------
// exact error of every set of centres (Sec. 5 restricted to the number of bins)
// ------------------------------------------------------------------------------------------
// All boundaries of a tensor's SK_SETS sets, sorted, cut the key axis into at most SK_EDGES + 1
// slots; a slot lies inside one cluster of every set, so count and sum per slot give the error of
// every set: (sum_all - sum_protected) x^2 - sum over slots of (2 c sx - n c^2), c the slot's centre.
__device__ __forceinline__ u32 n_boundaries_before(u32 set) { return (4u << set) - 4u - set; } // sum of 2^b - 1, b = 2 .. set + 1

__global__ __launch_bounds__(BLOCK) void k_sketch_score(const TDesc *__restrict__ td, int nT,
                                                        const u64 *__restrict__ wg_tile0,
                                                        const GridDesc *__restrict__ gd,
                                                        const SketchDesc *__restrict__ sd,
                                                        SketchParams P, Bufs B)
{
    // The slot of a key = the boundaries at or below it.  The search's equal-population bins (up to
    // 32768 per tensor, found through the key-prefix table) are far finer than the 502 slots: a table
    // gives the slot of every bin that holds no boundary, and for the few bins that do, the first
    // boundary to compare the key with.
    struct ScoreShared {
        u32 T[COARSE];                        // key prefix -> bins
        u16 stab[L2_BINS];                    // slot, or 0x8000 | boundaries below the bin
        u32 raw[SK_EDGES], edge[SK_EDGES + 1];
        // (four copies of the slot moments, one per lane modulo 4: the slots are few and the lanes
        // of a wave that hit the same address are served one after the other)
        u32 cnt[SK_COPIES * SK_SLOTS];
        double sx[SK_COPIES * SK_SLOTS];
    };
    __shared__ ScoreShared sh;
    const u32 tid = threadIdx.x, copy = (tid & (u32)(SK_COPIES - 1)) * (u32)SK_SLOTS;
    const u64 tile_lo = wg_tile0[blockIdx.x], tile_hi = wg_tile0[blockIdx.x + 1];
    if (tile_lo >= tile_hi) return;
    int t = find_tensor(td, nT, tile_lo);
    u64 tile = tile_lo;
    while (tile < tile_hi) {
        const TDesc d = td[t];
        const u64 n_tiles_t = (d.n + TILE - 1) / TILE;
        const u64 t_end = d.tile0 + n_tiles_t;
        const u64 stop = t_end < tile_hi ? t_end : tile_hi;
        const SketchDesc s = sd[t];
        if (!s.active) {
            tile = stop;
            t++;
            continue;
        }
        const TState *st = B.ts + t;
        const u32 pair = gd->cfg_pair[s.cfg];
        const u32 tau_p = st->thr_mag[gd->pair_p[pair]], tau_o = st->thr_mag[gd->n_p + gd->pair_o[pair]];
        const u32 nb2 = st->nb2;
        __syncthreads();
        for (u32 i = tid; i < (u32)COARSE; i += BLOCK) sh.T[i] = entry_for_u16(B.table2[(size_t)t * COARSE + i]);
        if (tid < (u32)SK_EDGES) { // boundary j of set b sits at ((j + 1) << (8 - bits)) - 1 of its row
            u32 set = 0u;
            while (set + 1u < (u32)SK_SETS && tid >= n_boundaries_before(set + 1u)) set++;
            const u32 j = tid - n_boundaries_before(set), bits = 2u + set;
            sh.raw[tid] = P.alt_key[((size_t)t * SK_SETS + set) * 256 + (((j + 1u) << (8u - bits)) - 1u)];
        }
        for (u32 i = tid; i < (u32)(SK_COPIES * SK_SLOTS); i += BLOCK) {
            sh.cnt[i] = 0u;
            sh.sx[i] = 0.0;
        }
        __syncthreads();
        if (tid < (u32)SK_EDGES) { // sort by counting the smaller ones
            const u32 x = sh.raw[tid];
            u32 r = 0u;
            for (u32 i = 0; i < (u32)SK_EDGES; i++) {
                const u32 y = sh.raw[i];
                r += (y < x || (y == x && i < tid)) ? 1u : 0u;
            }
            sh.edge[r] = x;
        }
        if (tid == 0) sh.edge[SK_EDGES] = 0xFFFFFFFFu;
        __syncthreads();
        for (u32 b = tid; b < nb2; b += BLOCK) { // slot of every bin, or its first boundary
            u32 lo = 0u, hi = COARSE - 1u; // key prefix of the bin: last one that starts at or below it
            while (lo < hi) {
                const u32 mid = (lo + hi + 1u) >> 1;
                if ((sh.T[mid] >> 6) <= b)
                    lo = mid;
                else
                    hi = mid - 1u;
            }
            const u32 e = sh.T[lo], dd = e & 31u, sub = b - (e >> 6);
            const u32 first = (lo << COARSE_SHIFT) | (sub << (COARSE_SHIFT - dd));
            const u32 last = first + ((1u << (COARSE_SHIFT - dd)) - 1u);
            u32 below = 0u, upto = 0u; // boundaries < first, boundaries <= last
#pragma unroll
            for (u32 step = 256u; step > 0u; step >>= 1) {
                if (below + step <= (u32)SK_EDGES && sh.edge[below + step - 1u] < first) below += step;
                if (upto + step <= (u32)SK_EDGES && sh.edge[upto + step - 1u] <= last) upto += step;
            }
            sh.stab[b] = (u16)((below == upto) ? below : (0x8000u | below));
        }
        __syncthreads();
        for (; tile < stop; tile++) {
            const u64 e0 = (tile - d.tile0) * (u64)TILE;
            const u64 rem = d.n - e0;
            const u32 c = rem < (u64)TILE ? (u32)rem : (u32)TILE;
            float v[16];
            const u32 mask = load_tile(d, e0, c, v);
#pragma unroll 4
            for (int i = 0; i < 16; i++) {
                const u32 key = key_of_float(v[i]);
                const u32 mag = mag_of_key(key);
                if (!((mask >> i) & 1u) || mag < tau_p || mag > tau_o) continue;
                u32 slot = lookup_u16(sh.stab, key, sh.T[key >> COARSE_SHIFT]);
                if (slot & 0x8000u) {
                    slot &= 0x7fffu;
                    while (sh.edge[slot] <= key) slot++; // (the list ends with 0xFFFFFFFF, above every finite key)
                }
                atomicAdd(&sh.cnt[copy + slot], 1u);
                atomicAdd(&sh.sx[copy + slot], (double)v[i]);
            }
        }
        __syncthreads();
        // this unit's part of the tensor's slot moments
        u32 *gc = P.slot_cnt + (size_t)t * SK_SLOTS;
        double *gx = P.slot_sx + (size_t)t * SK_SLOTS;
        for (u32 i = tid; i <= (u32)SK_EDGES; i += BLOCK) {
            u32 n = 0u;
            double sum = 0.0;
            for (u32 k = 0; k < (u32)SK_COPIES; k++) {
                n += sh.cnt[k * SK_SLOTS + i];
                sum += sh.sx[k * SK_SLOTS + i];
            }
            if (n) {
                atomicAdd(&gc[i], n);
                atomicAdd(&gx[i], sum);
            }
        }
        if (tid < (u32)SK_EDGES) P.slot_edge[(size_t)t * SK_SLOTS + tid] = sh.edge[tid]; // (the same from every unit)
        t++;
    }
}

// per tensor: error of every set, the fewest bits within eps, and that set's keys and centres
// where the quantizer looks for them
__global__ __launch_bounds__(256) void k_sketch_choose(const TDesc *__restrict__ td,
                                                       const u32 *__restrict__ t_fu_off,
                                                       const u32 *__restrict__ t_fu_ids,
                                                       const GridDesc *__restrict__ gd,
                                                       const SketchDesc *__restrict__ sd,
                                                       SketchParams P, Bufs B)
{
    __shared__ double s_sse[SK_SETS];
    __shared__ u32 s_best;
    const int t = blockIdx.x;
    const SketchDesc s = sd[t];
    if (!s.active) return;
    const u32 tid = threadIdx.x;
    const TState *st = B.ts + t;
    const u32 pair = gd->cfg_pair[s.cfg];
    // sum_pruned x^2 + sum_quantized (x - c)^2 = (sum_all - sum_protected) x^2 - sum_quantized (2 c x - c^2)
    double sumsq = st->sumsq, protsq = st->thr_sumsq[gd->n_p + gd->pair_o[pair]];
    if (P.light) { // no scoring kernel has added the units' parts up
        sumsq = 0.0;
        protsq = 0.0;
        for (u32 u = t_fu_off[t]; u < t_fu_off[t + 1]; u++) {
            sumsq += B.sq_part[(size_t)t_fu_ids[u] * SQ_STRIDE];
            protsq += B.sq_part[(size_t)t_fu_ids[u] * SQ_STRIDE + 1u + gd->pair_o[pair]];
        }
    }
    const double not_protected = sumsq - protsq;
    const u32 *gc = P.slot_cnt + (size_t)t * SK_SLOTS;
    const double *gx = P.slot_sx + (size_t)t * SK_SLOTS;
    const u32 *edge = P.slot_edge + (size_t)t * SK_SLOTS;
    if (tid < (u32)SK_SETS) {
        const u32 set = tid, bits = 2u + set, Kb = 1u << bits, sh = 8u - bits;
        const u32 *ak = P.alt_key + ((size_t)t * SK_SETS + set) * 256;
        const float *acb = P.alt_cb + ((size_t)t * SK_SETS + set) * 256;
        double gain = 0.0;
        u32 cluster = 0u; // of the current slot: boundaries of this set at or below the slot's keys
        for (u32 slot = 0; slot <= (u32)SK_EDGES; slot++) {
            if (slot > 0u) { // the slot starts at edge[slot - 1]
                const u32 first = edge[slot - 1u];
                while (cluster + 1u < Kb && ak[((cluster + 1u) << sh) - 1u] <= first) cluster++;
            }
            const u32 n = gc[slot];
            if (n) {
                const double c = (double)acb[cluster];
                gain += 2.0 * c * gx[slot] - (double)n * c * c;
            }
        }
        const double sse = not_protected - gain;
        s_sse[set] = sse > 0.0 ? sse : 0.0;
    }
    __syncthreads();
    if (tid == 0) {
        const double bound = P.eps * sumsq;
        u32 best = SK_SETS - 1u, feasible = 0u;
        for (u32 set = 0; set < (u32)SK_SETS; set++)
            if (s_sse[set] <= bound) {
                best = set;
                feasible = 1u;
                break;
            }
        s_best = best;
        SketchChoice r;
        for (u32 set = 0; set < (u32)SK_SETS; set++) {
            r.sse[set] = s_sse[set];
            r.rounds[set] = P.set_rounds[(size_t)t * SK_SETS + set];
        }
        r.sumsq = sumsq;
        r.best_bits = 2u + best;
        r.feasible = feasible;
        P.choice[t] = r;
    }
    __syncthreads();
    const u32 best = s_best;
    P.final_key[(size_t)t * 256 + tid] = P.alt_key[((size_t)t * SK_SETS + best) * 256 + tid];
    P.final_cb[(size_t)t * 256 + tid] = P.alt_cb[((size_t)t * SK_SETS + best) * 256 + tid];
}

// ------------------------------------------------------------------------------------------
// The sketch as the quantile estimator (Sec. 4.3, Algorithm 1): one sweep counts the magnitudes of
// a tensor per bucket; the estimate of the magnitude of a rank is the value of the bucket in which
// the running count passes the rank (relative error alpha).
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_sketch_maghist(const MagDesc *__restrict__ md, int nT, u64 n_chunks,
                                                          const u32 *__restrict__ gcell,
                                                          const u32 *__restrict__ tops, u32 n_idx,
                                                          u32 *__restrict__ hist, u32 *__restrict__ nonfinite)
{
    __shared__ u32 smem[SK_CELLS + SK_MAG_HIST];
    u32 *cell = smem, *h = smem + SK_CELLS;
    const u32 tid = threadIdx.x;
    // every workgroup takes an equal share of the chunks, in order; its counts go to a tensor's
    // histogram when the share moves on to the next tensor
    const u64 c_lo = n_chunks * (u64)blockIdx.x / gridDim.x, c_hi = n_chunks * ((u64)blockIdx.x + 1u) / gridDim.x;
    if (c_lo >= c_hi) return;
    int t = 0, hi = nT - 1; // last tensor whose first chunk is <= c_lo
    while (t < hi) {
        const int mid = (t + hi + 1) >> 1;
        if (md[mid].chunk0 <= c_lo)
            t = mid;
        else
            hi = mid - 1;
    }
    for (int i = tid; i < SK_CELLS; i += BLOCK) cell[i] = gcell[i];
    for (int i = tid; i < SK_MAG_HIST; i += BLOCK) h[i] = 0u;
    __syncthreads();
    bool bad = false;
    u64 c = c_lo;
    while (c < c_hi) {
        const MagDesc d = md[t];
        const u64 t_end = d.chunk0 + (d.n + SK_MAG_CHUNK - 1) / SK_MAG_CHUNK;
        const u64 stop = t_end < c_hi ? t_end : c_hi;
        for (; c < stop; c++) {
            TDesc td1; // (the tile loader of the sweeps: 16-byte loads where the address allows)
            td1.data = d.x;
            td1.n = d.n;
            td1.aligned16 = d.aligned16;
#pragma unroll 1
            for (u32 tl = 0; tl < (u32)SK_MAG_CHUNK / TILE; tl++) {
                const u64 e0 = (c - d.chunk0) * (u64)SK_MAG_CHUNK + (u64)tl * TILE;
                if (e0 >= d.n) break;
                const u64 rem = d.n - e0;
                const u32 cnt = rem < (u64)TILE ? (u32)rem : (u32)TILE;
                float v[16];
                const u32 mask = load_tile(td1, e0, cnt, v);
#pragma unroll
                for (int j = 0; j < 16; j++) {
                    if (!((mask >> j) & 1u)) continue; // past the end
                    const u32 mag = __float_as_uint(v[j]) & 0x7fffffffu;
                    if (mag >= 0x7f800000u) {
                        bad = true;
                    } else if (mag >= 0x00800000u) {
                        // entry = first bucket of the cell << 17 | (2^17 - 1 - low bits of that bucket's
                        // largest magnitude): the sum carries into the bucket field when the magnitude
                        // lies above it
                        atomicAdd(&h[1u + ((cell[mag >> 17] + (mag & 0x1FFFFu)) >> 17)], 1u);
                    } else if (mag == 0u) {
                        atomicAdd(&h[0], 1u);
                    } else { // a denormal: first bucket whose largest magnitude reaches it
                        u32 a = 0u, b = n_idx - 1u;
                        while (a < b) {
                            const u32 mid = (a + b) >> 1;
                            if (tops[mid] >= mag)
                                b = mid;
                            else
                                a = mid + 1u;
                        }
                        atomicAdd(&h[1u + a], 1u);
                    }
                }
            }
        }
        __syncthreads();
        u32 *gh = hist + (size_t)t * SK_MAG_HIST;
        for (int i = tid; i < SK_MAG_HIST; i += BLOCK) {
            const u32 v = h[i];
            if (v) {
                atomicAdd(&gh[i], v);
                h[i] = 0u;
            }
        }
        __syncthreads();
        t++;
    }
    if (bad) atomicOr(nonfinite, 1u);
}

__global__ __launch_bounds__(256) void k_sketch_quantile_pick(const MagDesc *__restrict__ md,
                                                              const u32 *__restrict__ hist,
                                                              const double *__restrict__ rep, u32 n_idx,
                                                              const u64 *__restrict__ ranks, u32 n_q,
                                                              double *__restrict__ est)
{
    __shared__ u32 cum[SK_MAG_HIST + 1]; // keys in the buckets before each one (n < 2^32)
    const int t = blockIdx.x;
    const u32 *gh = hist + (size_t)t * SK_MAG_HIST;
    if (threadIdx.x == 0) {
        u32 run = 0u;
        for (u32 i = 0; i <= n_idx; i++) {
            cum[i] = run;
            run += gh[i];
        }
        cum[n_idx + 1u] = run;
    }
    __syncthreads();
    for (u32 k = threadIdx.x; k < n_q; k += 256u) {
        const u64 rank = ranks[(size_t)t * n_q + k];
        u32 lo = 0u, hi = n_idx; // first bucket (in magnitude order, zeros first) whose running count passes the rank
        while (lo < hi) {
            const u32 mid = (lo + hi) >> 1;
            if ((u64)cum[mid + 1u] > rank)
                hi = mid;
            else
                lo = mid + 1u;
        }
        est[(size_t)t * n_q + k] = lo == 0u ? 0.0 : rep[lo - 1u];
    }
    (void)md;
}

hipError_t launch_sketch_quantiles(const MagDesc *md, int nT, u64 n_chunks, int n_wg, const u32 *cell, const u32 *tops,
                                   const double *rep, u32 n_idx, u32 *hist, u32 *nonfinite,
                                   const u64 *ranks, u32 n_q, double *est, hipStream_t s)
{
    const unsigned grid = (unsigned)(n_chunks < (u64)n_wg ? n_chunks : (u64)n_wg);
    PROF("k_sketch_maghist", s, k_sketch_maghist<<<grid, BLOCK, 0, s>>>(md, nT, n_chunks, cell, tops, n_idx, hist, nonfinite));
    PROF("k_sketch_quantile_pick", s, k_sketch_quantile_pick<<<nT, 256, 0, s>>>(md, hist, rep, n_idx, ranks, n_q, est));
    return hipGetLastError();
}

hipError_t launch_sketch(const Batch &bt, const SketchDesc *sd, const SketchParams &P, hipStream_t s)
{
    if (P.light)
        PROF("k_sketch_hist", s, k_sketch_hist<true><<<bt.n_wg, BLOCK, 0, s>>>(bt.td, bt.nT, bt.wg_tile0, bt.wg_fu0,
                                                                              bt.gd, sd, P, bt.bufs));
    else
        PROF("k_sketch_hist", s, k_sketch_hist<false><<<bt.n_wg, BLOCK, 0, s>>>(bt.td, bt.nT, bt.wg_tile0, bt.wg_fu0,
                                                                               bt.gd, sd, P, bt.bufs));
    PROF("k_sketch_kmeans", s, k_sketch_kmeans<<<bt.nT, BLOCK, 0, s>>>(bt.gd, sd, P));
    if (P.multi) {
        PROF("k_sketch_score", s,
             k_sketch_score<<<bt.n_wg, BLOCK, 0, s>>>(bt.td, bt.nT, bt.wg_tile0, bt.gd, sd, P, bt.bufs));
        PROF("k_sketch_choose", s,
             k_sketch_choose<<<bt.nT, 256, 0, s>>>(bt.td, bt.t_fu_off, bt.t_fu_ids, bt.gd, sd, P, bt.bufs));
    }
    return hipGetLastError();
}

} // namespace inshr
