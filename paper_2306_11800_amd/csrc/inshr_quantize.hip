// Quantizer output (Sec. 4): symbols (0 pruned, 1 protected, 2 + bin) bit-packed at bits + 1 bits,
// the codebook of bin centres and the list of protected values in ascending index.
//
// The thresholds, boundaries and centres come from the per-tensor search state; this sweep only
// classifies, searches the boundary list, packs and gathers the protected values.  The position
// of a tile's protected values in the output list is the prefix sum of the per-tile counts that
// the gathering sweep of the search recorded.
#include "inshr_launch.h"

namespace inshr {

// per tensor: prefix of protected counts over its tiles, meta data, codebook / boundary copy
__global__ __launch_bounds__(BLOCK) void k_qprep(const TDesc *__restrict__ td,
                                                 const GridDesc *__restrict__ gd,
                                                 const QDesc *__restrict__ qd,
                                                 QInfo *__restrict__ qi, Bufs B)
{
    extern __shared__ u32 smem[]; // [32768 + 4]
    __shared__ u32 tmp[BLOCK / 64 + 1];
    const int i = blockIdx.x;
    const QDesc q = qd[i];
    if (q.packed == nullptr) return;
    const int t = i;
    const u32 tid = threadIdx.x;
    const TDesc d = td[t];
    const TState *st = B.ts + t;
    const u32 g = q.cfg, pair = gd->cfg_pair[g], K = gd->cfg_K[g];
    const u32 o = gd->pair_o[pair], n_p = gd->n_p;
    const u64 n_tiles = (d.n + TILE - 1) / TILE;
    u32 carry = 0;
    for (u64 base = 0; base < n_tiles; base += L2_BINS) {
        const u64 left = n_tiles - base;
        const int m = left < (u64)L2_BINS ? (int)left : L2_BINS;
        for (int k = tid; k < m; k += BLOCK) smem[k] = B.tile_out[(d.tile0 + base + k) * MAX_FRAC + o];
        __syncthreads();
        u32 tot = block_excl_scan(smem, smem, m, tmp);
        for (int k = tid; k < m; k += BLOCK) B.tile_off[d.tile0 + base + k] = carry + smem[k];
        carry += tot;
        __syncthreads();
    }
    // (boundary keys given from outside come as 256 entries, boundary j of K = 2^b at j * 256 / K - 1)
    const u32 *tk = q.alt_key ? q.alt_key : B.tgt_key + (size_t)t * TGT_STRIDE + pair * NBT;
    if (q.boundaries)
        for (u32 j = 1 + tid; j < K; j += BLOCK)
            gptr(q.boundaries)[j - 1] = __uint_as_float(bits_of_key(tk[bnd_index(K, j)]));
    const float *cb = q.alt_cb ? q.alt_cb : B.codebook + ((size_t)t * gd->n_cfg + g) * CB_STRIDE;
    for (u32 k = tid; k < K; k += BLOCK) gptr(q.codebook)[k] = cb[k];
    if (tid == 0) {
        QInfo r;
        r.n_pruned = st->pair_Pn[pair] + st->pair_Pp[pair];
        r.n_outlier = st->pair_An[pair] + st->pair_Ap[pair];
        r.n_kept = st->pair_M[pair];
        r.tau_p = st->thr_mag[gd->pair_p[pair]];
        r.tau_o = st->thr_mag[n_p + o];
        r.flags = 0u;
        if ((u64)carry != r.n_outlier) r.flags |= 1u;  // self-check
        if (r.n_outlier > q.out_cap) r.flags |= 2u;    // caller buffer too small
        qi[i] = r;
    }
}

// The symbol is a step function of the key: the 255 bin boundaries and the four class edges
// (first quantized negative key, first pruned key, first quantized positive key, first protected
// positive key) cut the key axis into at most 260 slots, each with one symbol.  The search's
// equal-population bins (32768 of them) are far finer than the slots, so a table gives the symbol
// of every bin that holds no breakpoint; in the few bins that do, the key is compared with the
// breakpoints from the bin's first one on.
constexpr int QBP = 264;          // breakpoints, padded
constexpr int PKW = 256 * 9;      // most packed words of a tile

struct QuantTables {
    u32 bp[QBP + 8];   // sorted breakpoints, then 0xFFFFFFFF
    u32 raw[QBP];      // boundaries of the configuration, then the class edges
    u16 symtab[QBP];   // symbol of slot s = #{breakpoints <= key}
    u32 wcnt[2][64];   // protected values per (quarter j, wave) of the tile, per buffer
};

struct QuantShared {
    u32 T[COARSE];                     // key prefix -> bins
    u16 symt[L2_BINS];                 // symbol, or 0x8000 | first breakpoint of the bin
    unsigned long long pk[2 * PKW];    // two bit buffers of packed symbols
    QuantTables qt;
};

template <bool FULL>
__device__ __forceinline__ void classify_tile(const float (&v)[16], u32 mask, const u32 *T,
                                              const u16 *symt, const QuantTables &qt, u32 n_bp, u32 w,
                                              unsigned long long *pk, u32 *wcnt, u32 &omask,
                                              u32 (&pre)[4])
{
    const u32 tid = threadIdx.x, lane = tid & 63u;
    omask = 0u;
#pragma unroll
    for (int j = 0; j < 4; j++) {
        u32 e[4], key[4];
#pragma unroll
        for (int c = 0; c < 4; c++) {
            key[c] = key_of_float(v[4 * j + c]);
            e[c] = T[key[c] >> COARSE_SHIFT];
        }
#pragma unroll
        for (int c = 0; c < 4; c++) e[c] = lookup_u16(symt, key[c], e[c]);
        u32 lo32 = 0u, s3 = 0u;
#pragma unroll
        for (int c = 0; c < 4; c++) {
            u32 sym = e[c];
            if (sym & 0x8000u) { // the bin holds breakpoints: count those at or below the key
                u32 s = sym & 0x7fffu;
                if (qt.bp[s] <= key[c]) { // (the bin's first breakpoint exists: s < n_bp)
                    s++;
                    if (qt.bp[s] <= key[c]) { // many equal values put many breakpoints into one bin
                        s++;
                        for (u32 step = 256u; step > 0u; step >>= 1)
                            if (s + step <= n_bp && qt.bp[s + step - 1u] <= key[c]) s += step;
                    }
                }
                sym = qt.symtab[s];
            }
            if (!FULL && !((mask >> (4 * j + c)) & 1u)) sym = 0u;
            if (c < 3)
                lo32 |= sym << (c * w);
            else
                s3 = sym;
            omask |= (sym == 1u ? 1u : 0u) << (4 * j + c);
        }
        const unsigned long long piece = (unsigned long long)lo32 | ((unsigned long long)s3 << (3u * w));
        const u32 bitoff = 4u * (tid + 1024u * j) * w;
        const u32 word = bitoff >> 6, shf = bitoff & 63u;
        if (piece) {
            atomicOr(&pk[word], piece << shf);
            if (shf + 4u * w > 64u) atomicOr(&pk[word + 1u], piece >> (64u - shf));
        }
        // protected values of this wave's 256 elements: total, and those of lower lanes
        const u32 cj = __popc((omask >> (4 * j)) & 0xFu);
        u32 tot = 0u;
        pre[j] = 0u;
        if (__ballot(cj != 0u)) {
            const u64 m0 = __ballot(cj & 1u), m1 = __ballot(cj & 2u), m2 = __ballot(cj & 4u);
            pre[j] = __builtin_amdgcn_mbcnt_hi((u32)(m0 >> 32), __builtin_amdgcn_mbcnt_lo((u32)m0, 0u)) +
                     2u * __builtin_amdgcn_mbcnt_hi((u32)(m1 >> 32), __builtin_amdgcn_mbcnt_lo((u32)m1, 0u)) +
                     4u * __builtin_amdgcn_mbcnt_hi((u32)(m2 >> 32), __builtin_amdgcn_mbcnt_lo((u32)m2, 0u));
            tot = (u32)__popcll(m0) + 2u * (u32)__popcll(m1) + 4u * (u32)__popcll(m2);
        }
        if (lane == 0u) wcnt[j * 16 + (tid >> 6)] = tot;
    }
}

__global__ __launch_bounds__(BLOCK) void k_quant(const TDesc *__restrict__ td, int nT,
                                                 const u64 *__restrict__ wg_tile0,
                                                 const GridDesc *__restrict__ gd,
                                                 const QDesc *__restrict__ qd_by_tensor, Bufs B)
{
    // one static LDS object (it starts at LDS address 0): table offsets then fold into the LDS
    // instructions, which the base of a dynamic array does not allow
    __shared__ QuantShared qs;
    u32 *T = qs.T;
    u16 *symt = qs.symt;
    unsigned long long *pk0 = qs.pk;
    QuantTables &qt = qs.qt;

    const u32 tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const u64 tile_lo = wg_tile0[blockIdx.x], tile_hi = wg_tile0[blockIdx.x + 1];
    if (tile_lo >= tile_hi) return;
    for (u32 k = tid; k < 2u * PKW; k += BLOCK) pk0[k] = 0ull;
    int t = find_tensor(td, nT, tile_lo);
    u64 tile = tile_lo;
    u32 buf = 0u;
    while (tile < tile_hi) {
        const TDesc d = td[t];
        const u64 n_tiles_t = (d.n + TILE - 1) / TILE;
        const u64 t_end = d.tile0 + n_tiles_t;
        const u64 stop = t_end < tile_hi ? t_end : tile_hi;
        const QDesc q = qd_by_tensor[t];
        if (q.packed == nullptr) { // tensor not part of this call
            tile = stop;
            t++;
            continue;
        }
        const TState *st = B.ts + t;
        const u32 g = q.cfg, pair = gd->cfg_pair[g], K = gd->cfg_K[g];
        const u32 w = symbol_bits(K);
        const u32 o = gd->pair_o[pair];
        const u32 tau_p = st->thr_mag[gd->pair_p[pair]], tau_o = st->thr_mag[gd->n_p + o];
        const u32 nb2 = st->nb2;
        const u32 *tk = q.alt_key ? q.alt_key : B.tgt_key + (size_t)t * TGT_STRIDE + pair * NBT;
        const u32 n_bnd = K - 1u, n_bp = n_bnd + 4u;
        __syncthreads();
        for (u32 i = tid; i < (u32)COARSE; i += BLOCK) T[i] = entry_for_u16(B.table2[(size_t)t * COARSE + i]);
        if (tid < n_bnd) qt.raw[tid] = tk[bnd_index(K, tid + 1u)];
        if (tid < 4u) qt.raw[n_bnd + tid] = class_edge_key(tid, tau_p, tau_o);
        __syncthreads();
        if (tid < n_bp) { // sort by counting the smaller ones
            const u32 x = qt.raw[tid];
            u32 r = 0u;
            for (u32 i = 0; i < n_bp; i++) {
                const u32 y = qt.raw[i];
                r += (y < x || (y == x && i < tid)) ? 1u : 0u;
            }
            qt.bp[r] = x;
        } else if (tid < (u32)QBP + 8u) {
            qt.bp[tid] = 0xFFFFFFFFu;
        }
        __syncthreads();
        if (tid <= n_bp) { // symbol of each slot, from its smallest key
            const u32 rep = tid ? qt.bp[tid - 1u] : 0u;
            const u32 m = mag_of_key(rep);
            u32 sym;
            if (m < tau_p) {
                sym = 0u;
            } else if (m > tau_o) {
                sym = 1u;
            } else {
                u32 lo = 0u, hi = n_bnd; // #{boundaries <= rep}
                while (lo < hi) {
                    const u32 mid = (lo + hi) >> 1;
                    if (qt.raw[mid] <= rep)
                        lo = mid + 1u;
                    else
                        hi = mid;
                }
                sym = 2u + lo;
            }
            qt.symtab[tid] = (u16)sym;
        }
        __syncthreads();
        for (u32 b = tid; b < nb2; b += BLOCK) { // symbol of every bin, or its first breakpoint
            u32 lo = 0u, hi = COARSE - 1u; // key prefix of the bin: last one that starts at or below it
            while (lo < hi) {
                const u32 mid = (lo + hi + 1u) >> 1;
                if ((T[mid] >> 6) <= b)
                    lo = mid;
                else
                    hi = mid - 1u;
            }
            const u32 e = T[lo], dd = e & 31u, sub = b - (e >> 6);
            const u32 first = (lo << COARSE_SHIFT) | (sub << (COARSE_SHIFT - dd));
            const u32 last = first + ((1u << (COARSE_SHIFT - dd)) - 1u);
            u32 below = 0u, upto = 0u; // breakpoints < first, breakpoints <= last
            for (u32 step = 256u; step > 0u; step >>= 1) {
                if (below + step <= n_bp && qt.bp[below + step - 1u] < first) below += step;
                if (upto + step <= n_bp && qt.bp[upto + step - 1u] <= last) upto += step;
            }
            symt[b] = (below == upto) ? qt.symtab[below] : (u16)(0x8000u | below);
        }
        __syncthreads();
        GLOBAL_AS unsigned long long *packed = gptr(q.packed);
        auto tile_cnt = [&](u64 tl) -> u32 {
            const u64 rem = d.n - (tl - d.tile0) * (u64)TILE;
            return rem < (u64)TILE ? (u32)rem : (u32)TILE;
        };
        // Software pipeline of one tile: (1) the tile's values, asked for during the tile before,
        // arrive; (2) the words and protected values of the tile before leave (their stores drain
        // while this tile is classified, and no load ever waits behind a store); (3) the next tile
        // is asked for; (4) this tile is classified into the other LDS buffer; barrier.
        float vn[16];
        bool ahead = false; // vn holds the tile about to be worked on (uniform)
        float vp[16];           // values of the tile before (its protected ones are still to be written)
        u32 omask_p = 0u, pre_p[4] = {0u, 0u, 0u, 0u}, obase_p = 0u;
        bool have_prev = false; // uniform
        auto write_out = [&](u64 tl, u32 bf) { // phase 2 of tile tl, classified into buffer bf
            const u64 e0 = (tl - d.tile0) * (u64)TILE;
            const u32 cnt = tile_cnt(tl);
            const u32 w_ = w;
            unsigned long long *pk = pk0 + bf * PKW;
            const u32 *wcnt = qt.wcnt[bf];
            // the tile's words leave, and the buffer is clean for the tile after the next
            const u32 n_words = (cnt * w_ + 63u) >> 6;
            GLOBAL_AS unsigned long long *dst = packed + (tl - d.tile0) * (u64)(256u * w_);
            // (at most 9 * 256 words: three per thread, read together, so the LDS latency is paid once)
            unsigned long long xw[3];
#pragma unroll
            for (u32 j = 0; j < 3u; j++) {
                const u32 k = tid + j * BLOCK;
                xw[j] = k < 256u * w_ ? pk[k] : 0ull;
            }
#pragma unroll
            for (u32 j = 0; j < 3u; j++) {
                const u32 k = tid + j * BLOCK;
                if (k < n_words) dst[k] = xw[j];
                if (k < 256u * w_) pk[k] = 0ull;
            }
            // protected values in ascending index: quarter j, wave, lane, c
            const u32 wc = wcnt[lane];
            u32 inc = wc;
#pragma unroll
            for (int ofs = 1; ofs < 64; ofs <<= 1) {
                const u32 y = __shfl_up(inc, ofs);
                if ((int)lane >= ofs) inc += y;
            }
            if (__builtin_amdgcn_readlane(inc, 63) != 0u) {
                const u32 excl = inc - wc;
                const u64 obase = obase_p;
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    u32 r = __builtin_amdgcn_readlane(excl, j * 16 + wave) + pre_p[j];
#pragma unroll
                    for (int c = 0; c < 4; c++) {
                        const int i = 4 * j + c;
                        if ((omask_p >> i) & 1u) {
                            const u64 pos = obase + r;
                            if (pos < q.out_cap) {
                                gptr(q.out_idx)[pos] = (u32)(e0 + 4u * (tid + 1024u * j) + c);
                                if (q.val_bf16) { // upper 16 bits, rounded to nearest even
                                    const u32 b = __float_as_uint(vp[i]);
                                    ((GLOBAL_AS u16 *)gptr(q.out_val))[pos] = (u16)((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
                                } else {
                                    gptr(q.out_val)[pos] = vp[i];
                                }
                            }
                            r++;
                        }
                    }
                }
            }
        };
        for (; tile < stop; tile++) {
            const u64 e0 = (tile - d.tile0) * (u64)TILE;
            const u32 cnt = tile_cnt(tile);
            float v[16];
            u32 mask = 0xFFFFu;
            if (ahead) {
#pragma unroll
                for (int i = 0; i < 16; i++) v[i] = vn[i];
            } else {
                mask = load_tile(d, e0, cnt, v);
            }
#pragma unroll
            for (int i = 0; i < 16; i++)
                asm volatile("" : "+v"(v[i])); // the values are taken here, before any store below
            // offset of this tile's protected values in the list (needed one tile later)
            const u32 obase = __builtin_amdgcn_readfirstlane(B.tile_off[tile]);
            if (have_prev) write_out(tile - 1, buf ^ 1u);
            // a whole, aligned next tile is asked for now and used one iteration later
            ahead = tile + 1 < stop && d.aligned16 && tile_cnt(tile + 1) == (u32)TILE;
            if (ahead) load_tile_ahead(d, e0 + TILE, vn);
            u32 omask, pre[4];
            if (cnt == (u32)TILE) // the same for every lane: the tile code uses ballots
                classify_tile<true>(v, mask, T, symt, qt, n_bp, w, pk0 + buf * PKW, qt.wcnt[buf], omask, pre);
            else
                classify_tile<false>(v, mask, T, symt, qt, n_bp, w, pk0 + buf * PKW, qt.wcnt[buf], omask, pre);
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 16; i++) vp[i] = v[i];
            omask_p = omask;
            obase_p = obase;
#pragma unroll
            for (int j = 0; j < 4; j++) pre_p[j] = pre[j];
            have_prev = true;
            buf ^= 1u;
        }
        if (have_prev) write_out(stop - 1, buf ^ 1u);
        t++;
    }
}

hipError_t launch_quantize(const Batch &bt, const QDesc *qd, QInfo *qi, hipStream_t s)
{
    static bool attr = false;
    if (!attr) {
        hipError_t e = hipFuncSetAttribute((const void *)k_qprep,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (L2_BINS + 4) * 4);
        if (e) return e;
        attr = true;
    }
    PROF("k_qprep", s, k_qprep<<<bt.nT, BLOCK, (L2_BINS + 4) * 4, s>>>(bt.td, bt.gd, qd, qi, bt.bufs));
    PROF("k_quant", s, k_quant<<<bt.n_wg, BLOCK, 0, s>>>(bt.td, bt.nT, bt.wg_tile0, bt.gd, qd, bt.bufs));
    return hipGetLastError();
}

} // namespace inshr
