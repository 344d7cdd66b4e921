// Scoring of every grid configuration from one pass over the data (Sec. 5: the search evaluates a
// grid of configurations; here all of them share the sweeps).
//
// All boundaries and class edges of all (prune, protect) pairs form one list of "edges" ordered by
// key; slot s holds the keys with exactly s edges at or below them, and a slot fixes class and bin
// under every configuration, because the boundaries for fewer bits are a subset of those for
// 8 bits (floor(j*M/2^b) = floor(j*2^(8-b)*M/2^8)).  The order of the list is known before any
// boundary key is: a boundary is the key of a given rank, a class edge has a known number of keys
// below it, and rank order is key order (a class edge goes before a boundary of equal rank).
// Per slot the sweeps provide (count, sum x); a small kernel turns slots into per-bin centres
// (Sec. 4.4, one centre update) and errors:
//   sse = sum_all x^2 - sum_protected x^2 - sum_bins (2 c S - n c^2)        (c rounded to fp32)
// (a pruned element's error x^2 is its own share of sum_all x^2).
#include "inshr_launch.h"

namespace inshr {

// ------------------------------------------------------------------------------------------
// edge order; for every bin without an edge its slot, and the keys per slot in such bins
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_edges(const TDesc *__restrict__ td,
                                                 const GridDesc *__restrict__ gd, Bufs B)
{
    extern __shared__ u32 smem[];
    u64 *srt = reinterpret_cast<u64 *>(smem); // [4096] sort word, see below
    u32 *ebin = smem + 2 * MAX_EDGES;         // [4096] bin of each edge, in order
    u32 *segc = ebin + MAX_EDGES;             // [4096] keys per slot in bins without an edge

    const int t = blockIdx.x;
    const u32 tid = threadIdx.x;
    TState *st = B.ts + t;
    const u64 n = td[t].n, n_neg = st->n_neg;
    const u32 n_pairs = gd->n_pairs, n_p = gd->n_p;
    // edge items: pair q has the boundaries q * EPP + 0 .. n_bnd - 1 and the class edges
    // q * EPP + NBT .. NBT + 3; the list holds n_e = n_pairs * (n_bnd + 4) of them
    const u32 n_bnd = gd->n_bnd, epp = n_bnd + 4u;
    const u32 n_e = n_pairs * epp;
    const u32 nb2 = st->nb2, zbin = st->zbin;
    const u32 *tb = B.tgt_bin + (size_t)t * TGT_STRIDE;
    const u32 *trank = B.tgt_rank + (size_t)t * TGT_STRIDE;
    const u32 *tab = B.table2 + (size_t)t * COARSE;
    const u32 *binfo = B.binfo + (size_t)t * L2_BINS;
    const u32 *h2 = B.hist2 + (size_t)t * L2_BINS;
    const u16 *gtab = B.bin_group + (size_t)t * L2_BINS;

    // Sort word: (keys below the edge << 1 | is boundary) << 18 | order of the key among the class
    // edges << 12 | item.  Class edges with the same number of keys below them have no key between
    // them, but they may lie in different bins, so they are put in key order.
    __shared__ u32 ckey[MAX_PAIRS * 4];
    if (tid < n_pairs * 4u)
        ckey[tid] = class_edge_key(tid & 3u, st->thr_mag[gd->pair_p[tid >> 2]],
                                   st->thr_mag[n_p + gd->pair_o[tid >> 2]]);
    __syncthreads();
    u64 w[MAX_EDGES / BLOCK]; // this thread's words: positions tid + m * BLOCK of the list
#pragma unroll
    for (int m = 0; m < MAX_EDGES / BLOCK; m++) {
        const u32 i = tid + (u32)m * BLOCK;
        u64 v = ~0ull;
        if (i < n_e) {
            const u32 q = i / epp, r = i % epp;
            const u32 e = r < n_bnd ? r : (u32)NBT + (r - n_bnd);
            u64 below, is_boundary, corder = 0ull;
            if (e < (u32)NBT) {
                below = trank[q * NBT + e];
                is_boundary = 1ull;
            } else {
                const u32 me = q * 4u + (e - NBT), key = ckey[me];
                for (u32 j = 0; j < n_pairs * 4u; j++)
                    corder += (ckey[j] < key || (ckey[j] == key && j < me)) ? 1ull : 0ull;
                switch (e - NBT) {
                case 0: below = st->pair_An[q]; break;                 // keys < first quantized negative
                case 1: below = n_neg - st->pair_Pn[q]; break;         // keys < first pruned
                case 2: below = n_neg + st->pair_Pp[q]; break;         // keys < first quantized positive
                default: below = n - st->pair_Ap[q]; break;            // keys < first protected positive
                }
                is_boundary = 0ull;
            }
            v = (((below << 1) | is_boundary) << 18) | (corder << 12) | (u64)(q * EPP + e);
        }
        w[m] = v;
    }
    // Bitonic sort.  Position i = tid + m * BLOCK: a partner i ^ j lies in the same thread for
    // j >= BLOCK (registers), in the same wave for j < 64 (a lane exchange), and only for the strides
    // in between in another wave (through LDS, two buffers in turn, one barrier per step): 18 of the
    // 78 steps.  With a barrier after every step the sort took two thirds of this kernel.
    {
        u64 *buf[2] = {srt, reinterpret_cast<u64 *>(smem + 2 * MAX_EDGES)}; // (ebin and segc are not in use yet)
        int cur = 0;
        for (u32 k = 2; k <= (u32)MAX_EDGES; k <<= 1) {
            for (u32 j = k >> 1; j > 0; j >>= 1) {
                if (j >= (u32)BLOCK) {
                    const u32 dm = j / BLOCK;
#pragma unroll
                    for (u32 m = 0; m < (u32)(MAX_EDGES / BLOCK); m++) {
                        const u32 mm = m ^ dm;
                        if (mm > m) {
                            const u32 i = tid + m * BLOCK;
                            const bool up = (i & k) == 0u;
                            const u64 a = w[m], b = w[mm];
                            if ((a > b) == up) {
                                w[m] = b;
                                w[mm] = a;
                            }
                        }
                    }
                } else if (j < 64u) {
#pragma unroll
                    for (u32 m = 0; m < (u32)(MAX_EDGES / BLOCK); m++) {
                        const u32 i = tid + m * BLOCK;
                        const u64 a = w[m], b = __shfl_xor(a, (int)j);
                        const bool keep_small = ((i & j) == 0u) == ((i & k) == 0u);
                        w[m] = keep_small ? (a < b ? a : b) : (a > b ? a : b);
                    }
                } else {
                    u64 *sb = buf[cur];
#pragma unroll
                    for (u32 m = 0; m < (u32)(MAX_EDGES / BLOCK); m++) sb[tid + m * BLOCK] = w[m];
                    __syncthreads();
#pragma unroll
                    for (u32 m = 0; m < (u32)(MAX_EDGES / BLOCK); m++) {
                        const u32 i = tid + m * BLOCK;
                        const u64 a = w[m], b = sb[i ^ j];
                        const bool keep_small = ((i & j) == 0u) == ((i & k) == 0u);
                        w[m] = keep_small ? (a < b ? a : b) : (a > b ? a : b);
                    }
                    cur ^= 1; // (the next exchange writes the other buffer: no second barrier)
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (u32 m = 0; m < (u32)(MAX_EDGES / BLOCK); m++) srt[tid + m * BLOCK] = w[m];
        __syncthreads();
    }
    u32 *E = B.edges + (size_t)t * MAX_EDGES;
    u32 *eb = B.edge_bin + (size_t)t * MAX_EDGES;
    u16 *ei = B.edge_item + (size_t)t * MAX_EDGES;
    u16 *pe = B.pair_eidx + (size_t)t * MAX_PAIRS * EIDX_STRIDE;
    u32 *elo = B.grp_elo + (size_t)t * MAX_GROUPS;
    u32 *ehi = B.grp_ehi + (size_t)t * MAX_GROUPS;
    for (u32 pos = tid; pos < (u32)MAX_EDGES; pos += BLOCK) {
        u32 bin = 0xFFFFFFFFu;
        if (pos < n_e) {
            const u32 item = (u32)(srt[pos] & 4095ull);
            const u32 q = item / EPP, e = item % EPP;
            u32 key = 0u; // a boundary's key is found later, from the gathered keys
            if (e < (u32)NBT) {
                bin = tb[q * NBT + e];
                if (bin == RESOLVED) {
                    bin = zbin;
                    key = ZERO_KEY;
                }
            } else {
                key = class_edge_key(e - NBT, st->thr_mag[gd->pair_p[q]], st->thr_mag[n_p + gd->pair_o[q]]);
                bin = l2_bin(key, tab[key >> COARSE_SHIFT]);
            }
            E[pos] = key;
            eb[pos] = bin;
            ei[pos] = (u16)item;
            pe[q * EIDX_STRIDE + e] = (u16)pos;
        }
        ebin[pos] = bin;
        segc[pos] = 0u;
    }
    for (u32 g = tid; g < (u32)MAX_GROUPS; g += BLOCK) {
        elo[g] = 0xFFFFFFFFu;
        ehi[g] = 0u;
    }
    __syncthreads();
    for (u32 pos = tid; pos < n_e; pos += BLOCK) {
        const u32 bin = ebin[pos];
        if (pos + 1u < n_e && ebin[pos + 1u] < bin) atomicOr(&st->internal_err, 512u);
        const u32 g = (bin < nb2) ? gtab[bin] : 0xFFFFu;
        if (g >= (u32)MAX_GROUPS) {
            atomicOr(&st->internal_err, 512u);
        } else {
            atomicMin(&elo[g], pos);
            atomicMax(&ehi[g], pos + 1u);
        }
    }
    // Slot and sub-slot of every bin.  A bin without an edge lies inside one slot; sweep 3 adds the
    // mantissas of its keys as integers, which is exact and linear in the value only among keys of
    // one sign and exponent, so a slot is cut further wherever the exponent changes: sub-slot =
    // (edges in lower bins) + (key >> 23 of the bin).  Both terms grow with the bin, so the sum
    // names the pair; it stays below n_e + 512.
    u32 *subc = smem;                 // [MAX_SUB] keys per sub-slot (the sort words are done with)
    __shared__ u32 bfirst[512];       // first bin of every sign and exponent
    __shared__ u32 s_err;
    const u32 n_sub = n_e + 512u;
    u32 *sub_code = B.sub_code + (size_t)t * MAX_SUB;
    // (a table prefix is sign, exponent and three mantissa bits; every prefix has a bin of its own)
    for (u32 k = tid; k < 512u; k += BLOCK) bfirst[k] = (tab[8u * k] >> 5) & 0x7fffu;
    for (u32 i = tid; i < (u32)MAX_SUB; i += BLOCK) {
        subc[i] = 0u;
        sub_code[i] = 0xFFFFFFFFu; // no bin has this sub-slot
    }
    if (tid == 0) s_err = 0u;
    __syncthreads();
    u16 *sl = B.sl + (size_t)t * (L2_BINS + 64);
    u32 x = 0u;
    for (u32 b = tid; b < nb2; b += BLOCK) {
        const u32 bi = binfo[b], hb = h2[b]; // (in flight during the searches)
        u32 lo = 0u, hi = n_e; // edges in lower bins
        while (lo < hi) {
            const u32 mid = (lo + hi) >> 1;
            if (ebin[mid] < b)
                lo = mid + 1u;
            else
                hi = mid;
        }
        u32 xh = 511u; // last exponent whose first bin is <= b (not below that of the thread's last bin)
        while (x < xh) {
            const u32 mid = (x + xh + 1u) >> 1;
            if (bfirst[mid] <= b)
                x = mid;
            else
                xh = mid - 1u;
        }
        const u32 ss = lo + x;
        if (bi != INACTIVE) {
            sl[b] = 0xFFFFu;
        } else if (ss >= (u32)MAX_SUB) {
            s_err = 1u;
            sl[b] = 0xFFFFu;
        } else {
            sl[b] = (u16)ss;
            if (hb) {
                atomicAdd(&segc[lo], hb);
                if (atomicAdd(&subc[ss], hb) == 0u) sub_code[ss] = (lo << 9) | x; // first bin to arrive
            }
        }
    }
    __syncthreads();
    if (tid == 0 && s_err) atomicOr(&st->internal_err, 512u);
    u32 *sc = B.seg_cnt + (size_t)t * MAX_EDGES;
    for (u32 i = tid; i <= n_e; i += BLOCK) sc[i] = segc[i];
    u32 *sub_cnt = B.sub_cnt + (size_t)t * MAX_SUB;
    for (u32 i = tid; i < (u32)MAX_SUB; i += BLOCK) sub_cnt[i] = subc[i];
    if (tid == 0) st->n_sub = min(n_sub, (u32)MAX_SUB);
    if (tid == 0) st->n_edges = n_e;
}

// ------------------------------------------------------------------------------------------
// slots -> bins -> centres, errors, choice
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float float_of_key(u32 k) { return __uint_as_float(bits_of_key(k)); }

__global__ __launch_bounds__(BLOCK) void k_final(const TDesc *__restrict__ td,
                                                 const GridDesc *__restrict__ gd,
                                                 const u32 *__restrict__ t_fu_off,
                                                 const u32 *__restrict__ t_fu_ids, Bufs B)
{
    extern __shared__ u32 smem[];
    double *V = reinterpret_cast<double *>(smem);              // [4096] sum of each slot
    u64 *C = reinterpret_cast<u64 *>(smem + 2 * MAX_EDGES);    // [4096] keys in slots 0..s
    double *S8 = reinterpret_cast<double *>(smem + 4 * MAX_EDGES); // [MAX_PAIRS][256] sums of 8-bit bins
    double *SV = S8 + MAX_PAIRS * 256;                         // [MAX_SUB] sum of each sub-slot
    __shared__ double s_qout[MAX_FRAC];
    __shared__ double s_sumsq;

    const int t = blockIdx.x;
    const u32 tid = threadIdx.x;
    TState *st = B.ts + t;
    const u64 n = td[t].n;
    const u32 m = st->n_edges;
    const u32 u0 = t_fu_off[t], u1 = t_fu_off[t + 1];
    const u32 n_cfg = gd->n_cfg, n_p = gd->n_p, n_o = gd->n_o;

    const u32 *segc = B.seg_cnt + (size_t)t * MAX_EDGES;
    const u32 *gc = B.grp_cnt + (size_t)t * 2 * MAX_EDGES;
    const double *gs = B.grp_sx + (size_t)t * 2 * MAX_EDGES;
    // Per slot: count and sum.  The counts are kept as inclusive prefixes over the slots (a bin is
    // a run of consecutive slots, so its count is a difference): every thread owns four consecutive
    // slots, the running totals of the threads before it come from a scan.  The sums are kept per
    // slot and added bin by bin: a difference of prefix sums would lose a bin of small values next
    // to large ones (fp64 carries 16 digits, fp32 values span 83).
    __shared__ u64 w_c[BLOCK / 64];
    // Keys of bins without an edge: sweep 3 left, per unit and sub-slot, the sum of their 23 mantissa
    // bits.  All keys of a sub-slot share sign and exponent E, so their values add up to
    // +-2^(E-150) (2^23 count + sum of mantissas), or +-2^-149 (sum) for E = 0; the integer is
    // below 2^51 and the conversion exact.
    const u32 n_sub = st->n_sub;
    const u32 *sub_code = B.sub_code + (size_t)t * MAX_SUB;
    const u32 *sub_cnt = B.sub_cnt + (size_t)t * MAX_SUB;
    // (first and last sub-slot of every slot: kept where the slot's sum goes afterwards)
    u32 *ss_lo = reinterpret_cast<u32 *>(V), *ss_hi = ss_lo + 1; // [2 * slot]
    for (u32 i = tid; i <= m; i += BLOCK) {
        ss_lo[2u * i] = 0xFFFFFFFFu;
        ss_hi[2u * i] = 0u;
    }
    __syncthreads();
    for (u32 ss = tid; ss < n_sub; ss += BLOCK) {
        const u32 code = sub_code[ss];
        double val = 0.0;
        if (code != 0xFFFFFFFFu) {
            u64 tot = 0ull;
            for (u32 u = u0; u < u1; u++) tot += B.mom_sx[(size_t)t_fu_ids[u] * MAX_SUB + ss];
            const u32 bx = code & 511u; // key >> 23: the top bit is set for values >= 0, else all bits are flipped
            const bool neg = (bx & 256u) == 0u;
            const int E = (int)((neg ? ~bx : bx) & 255u);
            if (E)
                val = ldexp((double)(((u64)sub_cnt[ss] << 23) + tot), E - 150);
            else
                val = ldexp((double)tot, -149);
            if (neg) val = -val;
            const u32 slot = code >> 9;
            if (slot <= m) {
                atomicMin(&ss_lo[2u * slot], ss);
                atomicMax(&ss_hi[2u * slot], ss);
            }
        }
        SV[ss] = val;
    }
    __syncthreads();
    {
        u64 pc[4];
        u64 run_c = 0;
        // a slot's sub-slots in ascending order (those in between that no bin has hold 0.0)
        double su[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int r = 0; r < 4; r++) {
            const u32 i = 4u * tid + (u32)r;
            if (i <= m) {
                const u32 a = ss_lo[2u * i], b = ss_hi[2u * i];
                for (u32 ss = a; ss <= b && a != 0xFFFFFFFFu; ss++) su[r] += SV[ss];
            }
        }
        __syncthreads(); // V is written next
#pragma unroll
        for (int r = 0; r < 4; r++) {
            const u32 i = 4u * tid + r;
            double sv = 0.0;
            u64 c = 0;
            if (i <= m) {
                // then the gathered keys from the group of the slot's lower edge and from the
                // group of its upper edge
                sv = su[r];
                sv += gs[i];
                sv += gs[MAX_EDGES + i];
                c = (u64)segc[i] + gc[i] + gc[MAX_EDGES + i];
            }
            V[i] = sv;
            run_c += c;
            pc[r] = run_c;
        }
        u64 inc_c = run_c;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const u64 b = __shfl_up(inc_c, o);
            if ((int)(tid & 63u) >= o) inc_c += b;
        }
        if ((tid & 63u) == 63u) w_c[tid >> 6] = inc_c;
        __syncthreads();
        u64 base_c = inc_c - run_c;
        for (u32 w = 0; w < (tid >> 6); w++) base_c += w_c[w];
#pragma unroll
        for (int r = 0; r < 4; r++) C[4u * tid + r] = base_c + pc[r];
    }
    if (tid <= n_o) {
        double s = 0.0;
        for (u32 u = u0; u < u1; u++) s += B.sq_part[(size_t)t_fu_ids[u] * SQ_STRIDE + tid];
        if (tid == 0) {
            s_sumsq = s;
            st->sumsq = s;
        } else {
            s_qout[tid - 1] = s;
            st->thr_sumsq[n_p + tid - 1] = s;
        }
    }
    __syncthreads();

    const u16 *pe = B.pair_eidx + (size_t)t * MAX_PAIRS * EIDX_STRIDE;
    // sums of the 8-bit bins of every pair, slot by slot; the bins for fewer bits are unions of them
    for (u32 w = tid; w < gd->n_pairs * 256u; w += BLOCK) {
        const u32 q = w >> 8, k = w & 255u;
        const u16 *e = pe + q * EIDX_STRIDE;
        // bin k covers slots idx(lo)+1 .. idx(hi) without those of the pruned gap (g_lo, g_hi]
        const u32 i_lo = (k == 0) ? e[NBT + 0] : e[k - 1u];
        const u32 i_hi = (k == 255u) ? e[NBT + 3] : e[k];
        const u32 g_lo = e[NBT + 1], g_hi = e[NBT + 2];
        double sk = 0.0;
        for (u32 i = i_lo + 1u; i <= min(i_hi, g_lo); i++) sk += V[i];
        for (u32 i = max(i_lo, g_hi) + 1u; i <= i_hi; i++) sk += V[i];
        S8[w] = sk;
    }
    __syncthreads();
    const u32 *tk = B.tgt_key + (size_t)t * TGT_STRIDE;
    float *cb = B.codebook + (size_t)t * n_cfg * CB_STRIDE;
    double *bt = B.bin_term + (size_t)t * n_cfg * CB_STRIDE;
    // one work item per (configuration, bin)
    for (u32 w = tid; w < n_cfg * (u32)CB_STRIDE; w += BLOCK) {
        const u32 g = w / CB_STRIDE, k = w % CB_STRIDE;
        const u32 K = gd->cfg_K[g];
        if (k >= K) continue;
        const u32 q = gd->cfg_pair[g];
        const u16 *e = pe + q * EIDX_STRIDE;
        // bin k covers keys [lo, hi): slots idx(lo)+1 .. idx(hi); the pruned gap [E2, E3) is left out
        const u32 i_lo = (k == 0) ? e[NBT + 0] : e[bnd_index(K, k)];
        const u32 i_hi = (k == K - 1u) ? e[NBT + 3] : e[bnd_index(K, k + 1u)];
        const u32 g_lo = e[NBT + 1], g_hi = e[NBT + 2];
        // slots i_lo+1 .. i_hi without those of the pruned gap (g_lo, g_hi]
        u64 nk = C[i_hi] - C[i_lo];
        const u32 a = max(i_lo, g_lo), b = min(i_hi, g_hi);
        if (a < b) nk -= C[b] - C[a];
        double sk = 0.0;
        if ((K & (K - 1u)) == 0u) { // a union of 8-bit bins
            const u32 per = 256u / K;
            for (u32 j = 0; j < per; j++) sk += S8[q * 256u + k * per + j];
        } else { // 3, 6 or 12 bins: slot by slot
            for (u32 i = i_lo + 1u; i <= min(i_hi, g_lo); i++) sk += V[i];
            for (u32 i = max(i_lo, g_hi) + 1u; i <= i_hi; i++) sk += V[i];
        }
        float c;
        if (nk)
            c = (float)(sk / (double)nk);
        else
            c = float_of_key(tk[q * NBT + bnd_index(K, k == 0 ? 1u : k)]);
        cb[g * CB_STRIDE + k] = c;
        const double cd = (double)c;
        bt[g * CB_STRIDE + k] = 2.0 * cd * sk - (double)nk * cd * cd;
    }
    __syncthreads();
    Score *sc = B.scores + (size_t)t * n_cfg;
    __shared__ double s_sse[MAX_CFG];
    __shared__ u64 s_cost[MAX_CFG];
    for (u32 g = tid; g < n_cfg; g += BLOCK) {
        const u32 K = gd->cfg_K[g], q = gd->cfg_pair[g];
        double acc = 0.0;
        for (u32 k = 0; k < K; k++) acc += bt[g * CB_STRIDE + k];
        double sse = s_sumsq - s_qout[gd->pair_o[q]] - acc;
        if (sse < 0.0) sse = 0.0;
        Score r;
        r.sse = sse;
        r.sumsq = s_sumsq;
        r.n_pruned = st->pair_Pn[q] + st->pair_Pp[q];
        r.n_outlier = st->pair_An[q] + st->pair_Ap[q];
        r.n_kept = st->pair_M[q];
        // payload model: log2 K bits per quantized value (in units of 2^-16, rounded up), 32 per
        // protected value and per centre
        r.cost_bits = ((r.n_kept * (u64)gd->cfg_l16[g] + 65535ull) >> 16) + 32ull * r.n_outlier + 32ull * (u64)K;
        sc[g] = r;
        s_sse[g] = sse;
        s_cost[g] = r.cost_bits;
        if (r.n_pruned + r.n_outlier + r.n_kept != n) atomicOr(&st->internal_err, 256u);
    }
    __syncthreads();
    if (tid == 0) { // Sec. 5: cheapest feasible configuration, else the most accurate one
        bool have_f = false, have_a = false;
        u32 best_f = 0, best_a = 0;
        u64 best_cost = 0;
        double best_sse = 0.0;
        const double eps = gd->eps, sumsq = s_sumsq;
        for (u32 g = 0; g < n_cfg; g++) {
            const double sse = s_sse[g];
            const double rel = (sumsq > 0.0) ? sse / sumsq : 0.0;
            if (rel <= eps && (!have_f || s_cost[g] < best_cost)) {
                have_f = true;
                best_f = g;
                best_cost = s_cost[g];
            }
            if (!have_a || sse < best_sse) {
                have_a = true;
                best_a = g;
                best_sse = sse;
            }
        }
        st->best = have_f ? best_f : best_a;
        st->feasible = have_f ? 1u : 0u;
    }
}

constexpr int SM_EDGES = (2 * MAX_EDGES + 2 * MAX_EDGES) * 4;
constexpr int SM_FINAL = (2 * MAX_EDGES + 2 * MAX_EDGES) * 4 + MAX_PAIRS * 256 * 8 + MAX_SUB * 8;

static bool g_attr_done = false;
static hipError_t set_attrs()
{
    if (g_attr_done) return hipSuccess;
    hipError_t e;
    if ((e = hipFuncSetAttribute((const void *)k_edges, hipFuncAttributeMaxDynamicSharedMemorySize, SM_EDGES))) return e;
    if ((e = hipFuncSetAttribute((const void *)k_final, hipFuncAttributeMaxDynamicSharedMemorySize, SM_FINAL))) return e;
    g_attr_done = true;
    return hipSuccess;
}

hipError_t launch_edges(const Batch &bt, hipStream_t s)
{
    hipError_t e = set_attrs();
    if (e) return e;
    PROF("k_edges", s, k_edges<<<bt.nT, BLOCK, SM_EDGES, s>>>(bt.td, bt.gd, bt.bufs));
    return hipGetLastError();
}

hipError_t launch_score(const Batch &bt, hipStream_t s)
{
    hipError_t e = set_attrs();
    if (e) return e;
    PROF("k_final", s, k_final<<<bt.nT, BLOCK, SM_FINAL, s>>>(bt.td, bt.gd, bt.t_fu_off, bt.t_fu_ids, bt.bufs));
    return hipGetLastError();
}

} // namespace inshr
