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
    const u32 g = q.cfg, pair = gd->cfg_pair[g], bits = gd->cfg_bits[g], K = 1u << bits;
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
    const u32 *tk = B.tgt_key + (size_t)t * TGT_STRIDE + pair * NB8;
    const u32 sh = 8u - bits;
    if (q.boundaries)
        for (u32 j = 1 + tid; j < K; j += BLOCK)
            gptr(q.boundaries)[j - 1] = __uint_as_float(bits_of_key(tk[(j << sh) - 1u]));
    const float *cb = B.codebook + ((size_t)t * gd->n_cfg + g) * CB_STRIDE;
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

__global__ __launch_bounds__(BLOCK) void k_quant(const TDesc *__restrict__ td, int nT,
                                                 const u64 *__restrict__ wg_tile0,
                                                 const GridDesc *__restrict__ gd,
                                                 const QDesc *__restrict__ qd_by_tensor, Bufs B)
{
    __shared__ u32 bnd[256];
    __shared__ u16 ctab[COARSE]; // per 12-bit key prefix: boundaries below it | boundaries up to its end << 8
    __shared__ unsigned long long pk[256 * 9];
    __shared__ u32 wtot[4][BLOCK / 64];
    __shared__ u32 wbase[4][BLOCK / 64];

    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u64 tile_lo = wg_tile0[blockIdx.x], tile_hi = wg_tile0[blockIdx.x + 1];
    if (tile_lo >= tile_hi) return;
    int t = find_tensor(td, nT, tile_lo);
    u64 tile = tile_lo;
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
        const u32 g = q.cfg, pair = gd->cfg_pair[g], bits = gd->cfg_bits[g], K = 1u << bits;
        const u32 w = bits + 1u, sh = 8u - bits;
        const u32 o = gd->pair_o[pair];
        const u32 tau_p = st->thr_mag[gd->pair_p[pair]], tau_o = st->thr_mag[gd->n_p + o];
        const u32 *tk = B.tgt_key + (size_t)t * TGT_STRIDE + pair * NB8;
        __syncthreads();
        if (tid < 256u) bnd[tid] = (tid + 1u < K) ? tk[((tid + 1u) << sh) - 1u] : 0xFFFFFFFFu;
        __syncthreads();
        for (u32 c = tid; c < (u32)COARSE; c += BLOCK) {
            const u32 first = c << COARSE_SHIFT, last = first | ((1u << COARSE_SHIFT) - 1u);
            u32 lo = 0u, hi = 0u; // lo = #{t < first}, hi = #{t <= last}
            for (u32 step = K >> 1; step > 0u; step >>= 1) {
                if (bnd[lo + step - 1u] < first) lo += step;
                if (bnd[hi + step - 1u] <= last) hi += step;
            }
            ctab[c] = (u16)(lo | (hi << 8));
        }
        __syncthreads();
        for (; tile < stop; tile++) {
            const u64 e0 = (tile - d.tile0) * (u64)TILE;
            const u64 rem = d.n - e0;
            const u32 cnt = rem < (u64)TILE ? (u32)rem : (u32)TILE;
            const u32 n_words = (cnt * w + 63u) >> 6;
            for (u32 k = tid; k < 256u * w; k += BLOCK) pk[k] = 0ull;
            float v[16];
            const u32 mask = load_tile(d, e0, cnt, v);
            const u32 n_out_tile = B.tile_out[tile * MAX_FRAC + o];
            __syncthreads();
            u32 omask = 0u;
#pragma unroll
            for (int j = 0; j < 4; j++) {
                unsigned long long piece = 0ull;
#pragma unroll
                for (int c = 0; c < 4; c++) {
                    const int i = 4 * j + c;
                    u32 s = 0u;
                    if ((mask >> i) & 1u) {
                        const u32 b = canon_bits(__float_as_uint(v[i]));
                        const u32 m = b & 0x7fffffffu;
                        if (m < tau_p) {
                            s = 0u;
                        } else if (m > tau_o) {
                            s = 1u;
                            omask |= 1u << i;
                        } else {
                            const u32 key = key_of_bits(b);
                            const u32 e = ctab[key >> COARSE_SHIFT];
                            u32 lo = e & 255u, hi = e >> 8;
                            while (lo < hi) { // bin = #{t <= key}, known to lie in [lo, hi]
                                const u32 mid = (lo + hi) >> 1;
                                if (bnd[mid] <= key)
                                    lo = mid + 1u;
                                else
                                    hi = mid;
                            }
                            s = 2u + lo;
                        }
                    }
                    piece |= (unsigned long long)s << (c * w);
                }
                const u32 bitoff = 4u * (tid + 1024u * j) * w;
                const u32 word = bitoff >> 6, shf = bitoff & 63u;
                if (piece) {
                    atomicOr(&pk[word], piece << shf);
                    if (shf + 4u * w > 64u) atomicOr(&pk[word + 1u], piece >> (64u - shf));
                }
            }
            if (n_out_tile) {
                // rank of each protected value in index order: (j, thread, c)
                u32 incl[4], cj[4];
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    cj[j] = __popc((omask >> (4 * j)) & 0xFu);
                    u32 x = cj[j];
#pragma unroll
                    for (int ofs = 1; ofs < 64; ofs <<= 1) {
                        u32 y = __shfl_up(x, ofs);
                        if ((int)lane >= ofs) x += y;
                    }
                    incl[j] = x;
                    if (lane == 63u) wtot[j][wave] = x;
                }
                __syncthreads();
                if (tid < 64u) {
                    const u32 j = tid >> 4, wv = tid & 15u;
                    u32 x = wtot[j][wv], inc = x;
#pragma unroll
                    for (int ofs = 1; ofs < 64; ofs <<= 1) {
                        u32 y = __shfl_up(inc, ofs);
                        if ((int)tid >= ofs) inc += y;
                    }
                    wbase[j][wv] = inc - x;
                }
                __syncthreads();
                const u64 obase = B.tile_off[tile];
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    u32 r = wbase[j][wave] + incl[j] - cj[j];
#pragma unroll
                    for (int c = 0; c < 4; c++) {
                        const int i = 4 * j + c;
                        if ((omask >> i) & 1u) {
                            const u64 pos = obase + r;
                            if (pos < q.out_cap) {
                                gptr(q.out_idx)[pos] = (u32)(e0 + 4u * (tid + 1024u * j) + c);
                                gptr(q.out_val)[pos] = v[i];
                            }
                            r++;
                        }
                    }
                }
            }
            __syncthreads();
            GLOBAL_AS unsigned long long *dst = gptr(q.packed) + (tile - d.tile0) * (u64)(256u * w);
            for (u32 k = tid; k < n_words; k += BLOCK) dst[k] = pk[k];
            __syncthreads();
        }
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
