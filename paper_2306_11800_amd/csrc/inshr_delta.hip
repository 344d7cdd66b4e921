// Delta Encoder (Sec. 6): d = (s_prev - s_cur) mod B with B = max(K_prev, K_cur) + 2, regrouped in
// the stable order of the previous checkpoint's symbol (Algorithm 5) and bit-packed.
//
// The regrouping is a stable partition into at most 258 groups:
//   k_dhist     per tile of 16384 elements: population of every previous symbol
//   k_dchunk    per chunk of 64 tiles: totals;  k_dgroups: per tensor: group offsets and the start
//               of every chunk inside every group
//   k_dscatter  per tile: stable rank of every element inside (tile, group) from wavefront ballots
//               (each wave owns 1024 consecutive elements, 64 consecutive elements per step), the
//               tile's elements are laid out group by group in LDS and each group's run is written
//               to its place in the packed stream (whole words stored, the two end words OR-ed in)
#include "inshr_launch.h"

namespace inshr {

constexpr int DTILE = 16384;
constexpr int DCHUNK = 64;     // tiles per chunk
constexpr int SS = 264;        // symbol stride (258 symbols at most)

__device__ __forceinline__ u32 lds_extract(const u32 *W, u32 idx, u32 w)
{
    const u32 off = idx * w;
    const u32 wd = off >> 5, sh = off & 31u;
    const u64 two = ((u64)W[wd + 1] << 32) | (u64)W[wd];
    return (u32)(two >> sh) & ((1u << w) - 1u);
}

// lanes of this wave that hold the same symbol (among valid lanes)
__device__ __forceinline__ u64 wave_peers(u32 sym, u32 w, bool valid)
{
    u64 peers = __ballot(valid);
    for (u32 b = 0; b < w; b++) {
        const bool bit = (sym >> b) & 1u;
        const u64 m = __ballot(bit);
        peers &= bit ? m : ~m;
    }
    return peers;
}

__device__ __forceinline__ int find_dtensor(const DDesc *dd, int nT, u64 tile)
{
    int lo = 0, hi = nT - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (dd[mid].dtile0 <= tile)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

// stage the packed words of elements [e0, e0 + cnt) (e0 a multiple of 64) into LDS as u32 words
__device__ __forceinline__ void stage_words(const unsigned long long *src, u64 e0, u32 cnt, u32 w,
                                            u32 *dst)
{
    const u64 w0 = e0 * w / 64u; // exact: e0 is a multiple of 64
    const u32 nw = (cnt * w + 63u) >> 6;
    for (u32 k = threadIdx.x; k < nw; k += BLOCK) {
        unsigned long long x = src[w0 + k];
        dst[2 * k] = (u32)x;
        dst[2 * k + 1] = (u32)(x >> 32);
    }
    if (threadIdx.x < 2) dst[2 * nw + threadIdx.x] = 0u;
}

__global__ __launch_bounds__(BLOCK) void k_dhist(const DDesc *__restrict__ dd, int nT,
                                                 u16 *__restrict__ tile_hist)
{
    __shared__ u32 P[DTILE * 9 / 32 + 4];
    __shared__ u32 cntw[BLOCK / 64][SS];
    const u64 tile = blockIdx.x;
    const int t = find_dtensor(dd, nT, tile);
    const DDesc d = dd[t];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u64 e0 = (tile - d.dtile0) * (u64)DTILE;
    const u64 rem = d.n - e0;
    const u32 cnt = rem < (u64)DTILE ? (u32)rem : (u32)DTILE;
    const u32 S = d.Kp + 2u;
    stage_words(d.prev, e0, cnt, d.wp, P);
    for (u32 k = tid; k < (BLOCK / 64) * SS; k += BLOCK) (&cntw[0][0])[k] = 0u;
    __syncthreads();
    for (u32 r = 0; r < 16u; r++) {
        const u32 idx = wave * 1024u + r * 64u + lane;
        const bool valid = idx < cnt;
        const u32 sym = valid ? lds_extract(P, idx, d.wp) : 0u;
        const u64 peers = wave_peers(sym, d.wp, valid);
        if (valid && sym < S) {
            const u32 rank = __popcll(peers & ((1ull << lane) - 1ull));
            if (rank == 0u) cntw[wave][sym] += __popcll(peers);
        }
    }
    __syncthreads();
    for (u32 g = tid; g < S; g += BLOCK) {
        u32 s = 0;
        for (int wv = 0; wv < BLOCK / 64; wv++) s += cntw[wv][g];
        tile_hist[tile * SS + g] = (u16)s; // <= 16384
    }
}

// totals of each chunk of 64 tiles
__global__ __launch_bounds__(SS) void k_dchunk(const DDesc *__restrict__ dd, int nT,
                                               const u64 *__restrict__ chunk_tile0, // [n_chunks + 1] first tile of each chunk
                                               const u16 *__restrict__ tile_hist,
                                               u32 *__restrict__ chunk_tot)
{
    const u64 c = blockIdx.x;
    const u64 t0 = chunk_tile0[c], t1 = chunk_tile0[c + 1];
    const u32 g = threadIdx.x;
    u32 s = 0;
    for (u64 tile = t0; tile < t1; tile++) s += tile_hist[tile * SS + g];
    chunk_tot[c * SS + g] = s;
}

// per tensor: group offsets; chunk_tot becomes the start of each chunk inside its group
__global__ __launch_bounds__(SS) void k_dgroups(const DDesc *__restrict__ dd,
                                                u32 *__restrict__ chunk_tot)
{
    __shared__ u64 tot[SS];
    const int t = blockIdx.x;
    const DDesc d = dd[t];
    const u32 g = threadIdx.x;
    const u32 S = d.Kp + 2u;
    u64 run = 0;
    for (u64 c = d.chunk0; c < d.chunk0 + d.n_chunks; c++) {
        u32 v = chunk_tot[c * SS + g];
        chunk_tot[c * SS + g] = (u32)run; // n < 2^32
        run += v;
    }
    tot[g] = (g < S) ? run : 0ull;
    __syncthreads();
    if (g == 0) {
        u64 acc = 0;
        for (u32 k = 0; k < S; k++) {
            d.group_off[k] = acc;
            acc += tot[k];
        }
        d.group_off[S] = acc;
    }
}

__global__ __launch_bounds__(BLOCK) void k_dscatter(const DDesc *__restrict__ dd, int nT,
                                                    const u16 *__restrict__ tile_hist,
                                                    const u32 *__restrict__ chunk_tot)
{
    __shared__ u32 P[DTILE * 9 / 32 + 4];
    __shared__ u32 C[DTILE * 9 / 32 + 4];
    __shared__ u32 wst[BLOCK / 64][SS];     // counts, then local start of (wave, symbol)
    __shared__ u32 lbase[SS + 1];           // local start of each symbol's run
    __shared__ u32 gcnt[SS];                // tile population per symbol
    __shared__ u64 gbase[SS];               // global stream position of each run
    __shared__ u32 woff[SS + 1];            // first work item (output word) of each run
    __shared__ u16 sd[DTILE];               // deltas in regrouped order
    __shared__ u16 si[DTILE];               // local indices in regrouped order

    const u64 tile = blockIdx.x;
    const int t = find_dtensor(dd, nT, tile);
    const DDesc d = dd[t];
    if (d.prev_perm) return; // this tensor's regrouping is given: k_dgather writes its stream
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u64 lt = tile - d.dtile0;
    const u64 e0 = lt * (u64)DTILE;
    const u64 rem = d.n - e0;
    const u32 cnt = rem < (u64)DTILE ? (u32)rem : (u32)DTILE;
    const u32 S = d.Kp + 2u, Bm = d.B, wB = d.wB;
    stage_words(d.prev, e0, cnt, d.wp, P);
    stage_words(d.cur, e0, cnt, d.wc, C);
    for (u32 k = tid; k < (BLOCK / 64) * SS; k += BLOCK) (&wst[0][0])[k] = 0u;
    __syncthreads();
    // population of (wave, symbol)
    for (u32 r = 0; r < 16u; r++) {
        const u32 idx = wave * 1024u + r * 64u + lane;
        const bool valid = idx < cnt;
        const u32 sym = valid ? lds_extract(P, idx, d.wp) : 0u;
        const u64 peers = wave_peers(sym, d.wp, valid);
        if (valid && sym < S) {
            const u32 rank = __popcll(peers & ((1ull << lane) - 1ull));
            if (rank == 0u) wst[wave][sym] += __popcll(peers);
        }
    }
    __syncthreads();
    // global start of this tile's run of every symbol; totals
    if (tid < S) {
        const u32 g = tid;
        u32 s = 0;
        for (int wv = 0; wv < BLOCK / 64; wv++) s += wst[wv][g];
        gcnt[g] = s;
        const u64 chunk = d.chunk0 + lt / DCHUNK;
        u64 base = d.group_off[g] + chunk_tot[chunk * SS + g];
        const u64 first = d.dtile0 + (lt / DCHUNK) * DCHUNK;
        for (u64 tl = first; tl < tile; tl++) base += tile_hist[tl * SS + g];
        gbase[g] = base;
    }
    __syncthreads();
    if (tid == 0) {
        u32 acc = 0, wacc = 0;
        for (u32 g = 0; g < S; g++) {
            lbase[g] = acc;
            woff[g] = wacc;
            const u32 c = gcnt[g];
            if (c) {
                const u64 fb = gbase[g] * wB, lb = (gbase[g] + c) * wB;
                wacc += (u32)(((lb - 1) >> 6) - (fb >> 6) + 1);
            }
            acc += c;
        }
        lbase[S] = acc;
        woff[S] = wacc;
    }
    __syncthreads();
    if (tid < S) {
        u32 run = lbase[tid];
        for (int wv = 0; wv < BLOCK / 64; wv++) {
            u32 c = wst[wv][tid];
            wst[wv][tid] = run;
            run += c;
        }
    }
    __syncthreads();
    // stable ranks and regrouped layout
    for (u32 r = 0; r < 16u; r++) {
        const u32 idx = wave * 1024u + r * 64u + lane;
        const bool valid = idx < cnt;
        const u32 sp = valid ? lds_extract(P, idx, d.wp) : 0u;
        const u64 peers = wave_peers(sp, d.wp, valid);
        if (valid && sp < S) {
            const u32 sc = lds_extract(C, idx, d.wc);
            const u32 rank = __popcll(peers & ((1ull << lane) - 1ull));
            const u32 old = wst[wave][sp];
            if (rank == 0u) wst[wave][sp] = old + __popcll(peers);
            const u32 L = old + rank;
            u32 dv = sp + Bm - sc;
            if (dv >= Bm) dv -= Bm;
            sd[L] = (u16)dv;
            si[L] = (u16)idx;
        }
    }
    __syncthreads();
    // write the runs: one work item per (run, output word)
    const u32 n_items = woff[S];
    for (u32 it = tid; it < n_items; it += BLOCK) {
        u32 lo = 0, hi = S - 1u; // last g with woff[g] <= it and gcnt[g] > 0
        while (lo < hi) {
            u32 mid = (lo + hi + 1u) >> 1;
            if (woff[mid] <= it)
                lo = mid;
            else
                hi = mid - 1u;
        }
        // woff is flat over empty runs; lo is the last index with woff <= it, which is non-empty
        // unless followed by equal entries; step back to the run that owns the item
        u32 g = lo;
        while (gcnt[g] == 0u) g--;
        const u64 gb = gbase[g];
        const u64 fb = gb * wB, lb = (gb + gcnt[g]) * wB;
        const u64 W = (fb >> 6) + (it - woff[g]);
        const u64 wlo = W << 6, whi = wlo + 64u;
        const u64 a = fb > wlo ? fb : wlo, b = lb < whi ? lb : whi;
        const u64 ra = a / wB, rb = (b - 1u) / wB;
        unsigned long long word = 0ull;
        for (u64 rr = ra; rr <= rb; rr++) {
            const unsigned long long val = sd[lbase[g] + (u32)(rr - gb)];
            const long long bp = (long long)(rr * wB) - (long long)wlo;
            word |= (bp >= 0) ? (val << bp) : (val >> (-bp));
        }
        if (a == wlo && b == whi)
            d.out[W] = word;
        else if (word)
            atomicOr(&d.out[W], word);
    }
    if (d.perm) {
        for (u32 L = tid; L < cnt; L += BLOCK) {
            u32 lo = 0, hi = S - 1u; // last g with lbase[g] <= L
            while (lo < hi) {
                u32 mid = (lo + hi + 1u) >> 1;
                if (lbase[mid] <= L)
                    lo = mid;
                else
                    hi = mid - 1u;
            }
            u32 g = lo;
            while (gcnt[g] == 0u) g--;
            d.perm[gbase[g] + (L - lbase[g])] = (u32)(e0 + si[L]);
        }
    }
}

// regrouping given: e[r] = d[perm[r]] by gathering
__global__ __launch_bounds__(BLOCK) void k_dgather(const DDesc *__restrict__ dd, int nT)
{
    __shared__ unsigned long long pk[256 * 9];
    const u64 tile = blockIdx.x;
    const int t = find_dtensor(dd, nT, tile);
    const DDesc d = dd[t];
    if (!d.prev_perm) return;
    const u32 tid = threadIdx.x;
    const u64 r0 = (tile - d.dtile0) * (u64)DTILE;
    const u64 rem = d.n - r0;
    const u32 cnt = rem < (u64)DTILE ? (u32)rem : (u32)DTILE;
    const u32 wB = d.wB, Bm = d.B;
    for (u32 k = tid; k < 256u * wB; k += BLOCK) pk[k] = 0ull;
    __syncthreads();
    for (u32 j = 0; j < 16u; j++) {
        const u32 l = tid + j * BLOCK;
        if (l >= cnt) break;
        const u64 i = d.prev_perm[r0 + l];
        u32 sym[2];
        for (int which = 0; which < 2; which++) {
            const unsigned long long *src = which ? d.cur : d.prev;
            const u32 w = which ? d.wc : d.wp;
            const u64 off = i * w;
            const u64 wd = off >> 6;
            const u32 sh = (u32)(off & 63u);
            unsigned long long x = src[wd] >> sh;
            if (sh + w > 64u) x |= src[wd + 1] << (64u - sh);
            sym[which] = (u32)x & ((1u << w) - 1u);
        }
        u32 dv = sym[0] + Bm - sym[1];
        if (dv >= Bm) dv -= Bm;
        const u32 bitoff = l * wB;
        const u32 word = bitoff >> 6, shf = bitoff & 63u;
        if (dv) {
            atomicOr(&pk[word], (unsigned long long)dv << shf);
            if (shf + wB > 64u) atomicOr(&pk[word + 1u], (unsigned long long)dv >> (64u - shf));
        }
    }
    __syncthreads();
    const u32 n_words = (cnt * wB + 63u) >> 6;
    unsigned long long *dst = d.out + r0 * wB / 64u;
    for (u32 k = tid; k < n_words; k += BLOCK) dst[k] = pk[k];
}

__global__ void k_dzero(const DDesc *__restrict__ dd, int nT)
{
    // clears the packed outputs that k_dscatter ORs into (one block row per tensor)
    const int t = blockIdx.y;
    const DDesc d = dd[t];
    if (d.prev_perm) return;
    for (u64 k = (u64)blockIdx.x * blockDim.x + threadIdx.x; k < d.out_words;
         k += (u64)gridDim.x * blockDim.x)
        d.out[k] = 0ull;
}

hipError_t launch_delta(const DDesc *dd, int nT, u64 n_dtiles, u64 n_chunks,
                        const u64 *chunk_tile0, u16 *tile_hist, u32 *chunk_tot, bool any_scatter,
                        bool any_gather, hipStream_t s)
{
    PROF("k_dhist", s, k_dhist<<<(unsigned)n_dtiles, BLOCK, 0, s>>>(dd, nT, tile_hist));
    PROF("k_dchunk", s, k_dchunk<<<(unsigned)n_chunks, SS, 0, s>>>(dd, nT, chunk_tile0, tile_hist, chunk_tot));
    PROF("k_dgroups", s, k_dgroups<<<nT, SS, 0, s>>>(dd, chunk_tot));
    if (any_scatter) {
        PROF("k_dzero", s, k_dzero<<<dim3(64, nT), 256, 0, s>>>(dd, nT));
        PROF("k_dscatter", s, k_dscatter<<<(unsigned)n_dtiles, BLOCK, 0, s>>>(dd, nT, tile_hist, chunk_tot));
    }
    if (any_gather) PROF("k_dgather", s, k_dgather<<<(unsigned)n_dtiles, BLOCK, 0, s>>>(dd, nT));
    return hipGetLastError();
}

} // namespace inshr
