// Scoring of every grid configuration in one sweep (Sec. 5: the search evaluates a grid of
// configurations; here all of them share one pass over the data).
//
// All thresholds and boundaries of all (prune, protect) pairs are merged into one sorted list of
// distinct "edges"; an element's slot in that list fixes its class and bin under every
// configuration, because the boundaries for fewer bits are a subset of those for 8 bits
// (floor(j*M/2^b) = floor(j*2^(8-b)*M/2^8)).  The sweep accumulates (count, sum x) per slot; a
// small kernel turns slots into per-bin centres (Sec. 4.4, one centre update) and errors:
//   sse = sum_all x^2 - sum_protected x^2 - sum_bins (2 c S - n c^2)        (c rounded to fp32)
// (a pruned element's error x^2 is its own share of sum_all x^2).
#include "inshr_launch.h"

namespace inshr {

constexpr int EPP = NB8 + 4; // edges per pair: 255 boundaries + 4 class edges
constexpr int EIDX_STRIDE = 260;

// ------------------------------------------------------------------------------------------
// plan 3: merged edge list and its lookup accelerator
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_plan3(const GridDesc *__restrict__ gd, Bufs B)
{
    extern __shared__ u32 smem[];
    u32 *srt = smem;              // [4096]
    u32 *cnt = smem + MAX_EDGES;  // [32768 + 4]
    __shared__ u32 tmp[BLOCK / 64 + 1];

    const int t = blockIdx.x;
    const u32 tid = threadIdx.x;
    TState *st = B.ts + t;
    const u32 n_pairs = gd->n_pairs, n_p = gd->n_p;
    const u32 *tk = B.tgt_key + (size_t)t * TGT_STRIDE;
    const u32 n_in = n_pairs * EPP;

    auto edge_key = [&](u32 idx) -> u32 {
        const u32 q = idx / EPP, e = idx % EPP;
        if (e < (u32)NB8) return tk[q * NB8 + e];
        const u32 tp = st->thr_mag[gd->pair_p[q]], to = st->thr_mag[n_p + gd->pair_o[q]];
        switch (e - NB8) {
        case 0: return key_neg(to);           // first quantized negative key
        case 1: return key_neg(tp) + 1u;      // first pruned key
        case 2: return key_pos(tp);           // first quantized positive key
        default: return key_pos(to) + 1u;     // first protected positive key
        }
    };
    for (u32 i = tid; i < (u32)MAX_EDGES; i += BLOCK) srt[i] = (i < n_in) ? edge_key(i) : 0xFFFFFFFFu;
    __syncthreads();
    // bitonic sort of 4096 keys
    for (u32 k = 2; k <= (u32)MAX_EDGES; k <<= 1) {
        for (u32 j = k >> 1; j > 0; j >>= 1) {
            for (u32 i = tid; i < (u32)MAX_EDGES; i += BLOCK) {
                u32 l = i ^ j;
                if (l > i) {
                    u32 a = srt[i], b = srt[l];
                    bool up = (i & k) == 0;
                    if ((a > b) == up) {
                        srt[i] = b;
                        srt[l] = a;
                    }
                }
            }
            __syncthreads();
        }
    }
    // distinct values, in order
    for (u32 i = tid; i < (u32)MAX_EDGES; i += BLOCK)
        cnt[i] = (srt[i] != 0xFFFFFFFFu && (i == 0 || srt[i] != srt[i - 1])) ? 1u : 0u;
    __syncthreads();
    u32 *E = B.edges + (size_t)t * MAX_EDGES;
    u32 *Ec = cnt + 2 * MAX_EDGES; // LDS copy of the distinct list
    // the scan overwrites the flags with positions, so each thread keeps its own flags
    u32 flags[MAX_EDGES / BLOCK];
    for (int r = 0; r < MAX_EDGES / BLOCK; r++) flags[r] = cnt[tid + r * BLOCK];
    for (u32 i = tid; i < (u32)MAX_EDGES; i += BLOCK) Ec[i] = 0xFFFFFFFFu;
    __syncthreads();
    const u32 m = block_excl_scan(cnt, cnt, MAX_EDGES, tmp);
    for (int r = 0; r < MAX_EDGES / BLOCK; r++) {
        u32 i = tid + r * BLOCK;
        if (flags[r]) {
            E[cnt[i]] = srt[i];
            Ec[cnt[i]] = srt[i];
        }
    }
    if (tid == 0) st->n_edges = m;
    __syncthreads();
    for (u32 i = tid; i < (u32)MAX_EDGES; i += BLOCK) srt[i] = Ec[i];
    __syncthreads();
    u16 *pe = B.pair_eidx + (size_t)t * MAX_PAIRS * EIDX_STRIDE;
    for (u32 i = tid; i < n_in; i += BLOCK) {
        const u32 key = edge_key(i);
        u32 lo = 0, hi = m; // first index with srt[idx] >= key
        while (lo < hi) {
            u32 mid = (lo + hi) >> 1;
            if (srt[mid] < key)
                lo = mid + 1;
            else
                hi = mid;
        }
        pe[(i / EPP) * EIDX_STRIDE + (i % EPP)] = (u16)lo;
    }
    // edges below each second-level bin
    const u32 nb2 = st->nb2;
    const u32 *tab = B.table2 + (size_t)t * COARSE;
    for (u32 i = tid; i <= nb2; i += BLOCK) cnt[i] = 0u;
    __syncthreads();
    for (u32 i = tid; i < m; i += BLOCK) {
        u32 key = srt[i];
        atomicAdd(&cnt[l2_bin(key, tab[key >> COARSE_SHIFT])], 1u);
    }
    __syncthreads();
    block_excl_scan(cnt, cnt, (int)nb2, tmp);
    u16 *sl = B.sl + (size_t)t * (L2_BINS + 64);
    for (u32 i = tid; i <= nb2; i += BLOCK) sl[i] = (u16)cnt[i];
}

// ------------------------------------------------------------------------------------------
// sweep 4: per-slot count and sum
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_score(const TDesc *__restrict__ td, int nT,
                                                 const u64 *__restrict__ wg_tile0,
                                                 const u32 *__restrict__ wg_fu0, Bufs B)
{
    extern __shared__ u32 smem[];
    double *sx = reinterpret_cast<double *>(smem);         // [4096]
    u32 *cnt = smem + 2 * MAX_EDGES;                       // [4096]
    u32 *E = cnt + MAX_EDGES;                              // [4096]
    u32 *T = E + MAX_EDGES;                                // [4096]
    u16 *SL = reinterpret_cast<u16 *>(T + COARSE);         // [32768 + 64]

    const u32 tid = threadIdx.x;
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
        const TState *st = B.ts + t;
        const u32 m = st->n_edges, nb2 = st->nb2;
        for (u32 i = tid; i < (u32)MAX_EDGES; i += BLOCK) {
            sx[i] = 0.0;
            cnt[i] = 0u;
            E[i] = (i < m) ? B.edges[(size_t)t * MAX_EDGES + i] : 0xFFFFFFFFu;
            T[i] = B.table2[(size_t)t * COARSE + i];
        }
        const u16 *gsl = B.sl + (size_t)t * (L2_BINS + 64);
        for (u32 i = tid; i <= nb2; i += BLOCK) SL[i] = gsl[i];
        __syncthreads();
        for (; tile < stop; tile++) {
            const u64 e0 = (tile - d.tile0) * (u64)TILE;
            const u64 rem = d.n - e0;
            const u32 c = rem < (u64)TILE ? (u32)rem : (u32)TILE;
            float v[16];
            const u32 mask = load_tile(d, e0, c, v);
#pragma unroll
            for (int i = 0; i < 16; i++) {
                if (!((mask >> i) & 1u)) continue;
                const u32 key = key_of_bits(canon_bits(__float_as_uint(v[i])));
                const u32 b2 = l2_bin(key, T[key >> COARSE_SHIFT]);
                u32 s = SL[b2];
                const u32 hi = SL[b2 + 1];
                while (s < hi && E[s] <= key) s++;
                atomicAdd(&cnt[s], 1u);
                atomicAdd(&sx[s], (double)v[i]);
            }
        }
        __syncthreads();
        const u32 fu = wg_fu0[blockIdx.x] + (u32)(t - t_first);
        u32 *gc = B.mom_cnt + (size_t)fu * MAX_EDGES;
        double *gs = B.mom_sx + (size_t)fu * MAX_EDGES;
        for (u32 i = tid; i <= m; i += BLOCK) {
            gc[i] = cnt[i];
            gs[i] = sx[i];
        }
        __syncthreads();
        t++;
    }
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
    double *S = reinterpret_cast<double *>(smem);              // [4096]
    u64 *C = reinterpret_cast<u64 *>(smem + 2 * MAX_EDGES);    // [4096]
    __shared__ double s_qout[MAX_FRAC];
    __shared__ double s_sumsq;

    const int t = blockIdx.x;
    const u32 tid = threadIdx.x;
    TState *st = B.ts + t;
    const u64 n = td[t].n;
    const u32 m = st->n_edges;
    const u32 u0 = t_fu_off[t], u1 = t_fu_off[t + 1];
    const u32 n_cfg = gd->n_cfg, n_p = gd->n_p, n_o = gd->n_o;

    for (u32 i = tid; i < (u32)MAX_EDGES; i += BLOCK) {
        double s = 0.0;
        u64 c = 0;
        if (i <= m) {
            for (u32 u = u0; u < u1; u++) {
                const u32 fu = t_fu_ids[u];
                c += B.mom_cnt[(size_t)fu * MAX_EDGES + i];
                s += B.mom_sx[(size_t)fu * MAX_EDGES + i];
            }
        }
        S[i] = s;
        C[i] = c;
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
    const u32 *tk = B.tgt_key + (size_t)t * TGT_STRIDE;
    float *cb = B.codebook + (size_t)t * n_cfg * CB_STRIDE;
    double *bt = B.bin_term + (size_t)t * n_cfg * CB_STRIDE;
    // one work item per (configuration, bin)
    for (u32 w = tid; w < n_cfg * (u32)CB_STRIDE; w += BLOCK) {
        const u32 g = w / CB_STRIDE, k = w % CB_STRIDE;
        const u32 bits = gd->cfg_bits[g], K = 1u << bits;
        if (k >= K) continue;
        const u32 q = gd->cfg_pair[g];
        const u16 *e = pe + q * EIDX_STRIDE;
        const u32 sh = 8u - bits;
        // bin k covers keys [lo, hi): slots idx(lo)+1 .. idx(hi); the pruned gap [E2, E3) is left out
        const u32 i_lo = (k == 0) ? e[NB8 + 0] : e[(k << sh) - 1u];
        const u32 i_hi = (k == K - 1u) ? e[NB8 + 3] : e[((k + 1u) << sh) - 1u];
        const u32 g_lo = e[NB8 + 1], g_hi = e[NB8 + 2];
        u64 nk = 0;
        double sk = 0.0;
        for (u32 s = i_lo + 1u; s <= i_hi; s++) {
            if (s > g_lo && s <= g_hi) continue;
            nk += C[s];
            sk += S[s];
        }
        float c;
        if (nk)
            c = (float)(sk / (double)nk);
        else
            c = float_of_key(tk[q * NB8 + (((k == 0 ? 1u : k) << sh) - 1u)]);
        cb[g * CB_STRIDE + k] = c;
        const double cd = (double)c;
        bt[g * CB_STRIDE + k] = 2.0 * cd * sk - (double)nk * cd * cd;
    }
    __syncthreads();
    Score *sc = B.scores + (size_t)t * n_cfg;
    for (u32 g = tid; g < n_cfg; g += BLOCK) {
        const u32 bits = gd->cfg_bits[g], K = 1u << bits, q = gd->cfg_pair[g];
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
        r.cost_bits = r.n_kept * (u64)bits + 32ull * r.n_outlier + 32ull * (u64)K;
        sc[g] = r;
        if (r.n_pruned + r.n_outlier + r.n_kept != n) atomicOr(&st->internal_err, 256u);
    }
    __syncthreads();
    if (tid == 0) {
        bool have_f = false, have_a = false;
        u32 best_f = 0, best_a = 0;
        u64 best_cost = 0;
        double best_sse = 0.0;
        const double eps = gd->eps;
        for (u32 g = 0; g < n_cfg; g++) {
            const Score r = sc[g];
            const double rel = (r.sumsq > 0.0) ? r.sse / r.sumsq : 0.0;
            if (rel <= eps && (!have_f || r.cost_bits < best_cost)) {
                have_f = true;
                best_f = g;
                best_cost = r.cost_bits;
            }
            if (!have_a || r.sse < best_sse) {
                have_a = true;
                best_a = g;
                best_sse = r.sse;
            }
        }
        st->best = have_f ? best_f : best_a;
        st->feasible = have_f ? 1u : 0u;
    }
}

constexpr int SM_PLAN3 = (MAX_EDGES + L2_BINS + 4) * 4;
constexpr int SM_SCORE = (2 * MAX_EDGES + 3 * MAX_EDGES) * 4 + (L2_BINS + 64) * 2;
constexpr int SM_FINAL = (2 * MAX_EDGES + 2 * MAX_EDGES) * 4;

static bool g_attr_done = false;
hipError_t launch_score(const Batch &bt, hipStream_t s)
{
    if (!g_attr_done) {
        hipError_t e;
        if ((e = hipFuncSetAttribute((const void *)k_plan3, hipFuncAttributeMaxDynamicSharedMemorySize, SM_PLAN3))) return e;
        if ((e = hipFuncSetAttribute((const void *)k_score, hipFuncAttributeMaxDynamicSharedMemorySize, SM_SCORE))) return e;
        if ((e = hipFuncSetAttribute((const void *)k_final, hipFuncAttributeMaxDynamicSharedMemorySize, SM_FINAL))) return e;
        g_attr_done = true;
    }
    const Bufs &B = bt.bufs;
    PROF("k_plan3", s, k_plan3<<<bt.nT, BLOCK, SM_PLAN3, s>>>(bt.gd, B));
    PROF("k_score", s, k_score<<<bt.n_wg, BLOCK, SM_SCORE, s>>>(bt.td, bt.nT, bt.wg_tile0, bt.wg_fu0, B));
    PROF("k_final", s, k_final<<<bt.nT, BLOCK, SM_FINAL, s>>>(bt.td, bt.gd, bt.t_fu_off, bt.t_fu_ids, B));
    return hipGetLastError();
}

} // namespace inshr
