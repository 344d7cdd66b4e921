// Partition by magnitude and sensitivity (Sec. 4.1-4.2) for one configuration per tensor.
//
// The sensitivity score of a weight is s = |gradient * weight|.  A weight is protected when its
// magnitude or its score lies above the respective threshold, pruned when it is not protected and
// its pruning metric (magnitude or score) lies below the prune threshold; the rest is quantized.
// The classes are then no rank ranges of one key any more, so the bins are not found by the grid
// search's shared order statistics: the quantized values are copied out in index order and searched
// as a tensor of their own (no pruning, no protection), and a last pass writes the symbols of all
// elements from the thresholds and the boundaries found.
//
//   k_sens_score     s = |g * w| for every element (the thresholds of s come from the ordinary
//                    threshold search over s)
//   k_sens_count     per block of 1024 consecutive elements (one wave): quantized and protected
//                    counts, squares of the pruned and of the protected values
//   k_sens_scan      per tensor: exclusive prefixes over its blocks, totals
//   k_sens_compact   quantized values -> the compact tensor, in index order
//   k_sens_quant     symbols (packed), protected list in index order, boundaries and centres
#include "inshr_launch.h"

namespace inshr {

constexpr int SBLK = 1024;      // elements per wave-block
constexpr int SWG = 1024;       // threads per workgroup: 16 wave-blocks

__device__ __forceinline__ int sens_tensor_of(const SDesc *sd, int nT, u64 blk)
{
    int lo = 0, hi = nT - 1; // last tensor whose first block is <= blk
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (sd[mid].blk0 <= blk)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

// class of an element: 0 pruned, 1 protected, 2 quantized
__device__ __forceinline__ u32 sens_class(const SDesc &d, float w, float s)
{
    const u32 mag = __float_as_uint(w) & 0x7fffffffu;
    const u32 sc = __float_as_uint(s); // non-negative: its bits order like the value
    if (mag > d.tau_om || sc > d.tau_os) return 1u;
    const u32 m = d.by_sens ? sc : mag;
    return m < d.tau_p ? 0u : 2u;
}

__global__ __launch_bounds__(SWG) void k_sens_score(const SDesc *__restrict__ sd, int nT, u64 n_blocks)
{
    const u32 lane = threadIdx.x & 63u;
    const u64 blk = (u64)blockIdx.x * (SWG / 64) + (threadIdx.x >> 6);
    if (blk >= n_blocks) return;
    const SDesc d = sd[sens_tensor_of(sd, nT, blk)];
    const u64 e0 = (blk - d.blk0) * (u64)SBLK;
#pragma unroll 4
    for (int r = 0; r < SBLK / 64; r++) {
        const u64 i = e0 + (u64)r * 64u + lane;
        if (i < d.n) d.S[i] = fabsf(d.g[i] * d.w[i]);
    }
}

__global__ __launch_bounds__(SWG) void k_sens_count(const SDesc *__restrict__ sd, int nT, u64 n_blocks,
                                                    u32 *__restrict__ blk_kept, u32 *__restrict__ blk_prot,
                                                    double *__restrict__ blk_sq)
{
    const u32 lane = threadIdx.x & 63u;
    const u64 blk = (u64)blockIdx.x * (SWG / 64) + (threadIdx.x >> 6);
    if (blk >= n_blocks) return;
    const SDesc d = sd[sens_tensor_of(sd, nT, blk)];
    const u64 e0 = (blk - d.blk0) * (u64)SBLK;
    u32 kept = 0u, prot = 0u;
    double q_pruned = 0.0, q_prot = 0.0;
    for (int r = 0; r < SBLK / 64; r++) {
        const u64 i = e0 + (u64)r * 64u + lane;
        const bool valid = i < d.n;
        const float w = valid ? d.w[i] : 0.0f, s = valid ? d.S[i] : 0.0f;
        const u32 c = valid ? sens_class(d, w, s) : 3u;
        kept += (u32)__popcll(__ballot(c == 2u));
        prot += (u32)__popcll(__ballot(c == 1u));
        const double xd = (double)w;
        if (c == 0u) q_pruned = fma(xd, xd, q_pruned);
        if (c == 1u) q_prot = fma(xd, xd, q_prot);
    }
    q_pruned = wave_sum_f64(q_pruned);
    q_prot = wave_sum_f64(q_prot);
    if (lane == 0u) {
        blk_kept[blk] = kept;
        blk_prot[blk] = prot;
        blk_sq[2u * blk] = q_pruned;
        blk_sq[2u * blk + 1u] = q_prot;
    }
}

// one workgroup per tensor: block counts -> exclusive prefixes (in place), totals
__global__ __launch_bounds__(SWG) void k_sens_scan(const SDesc *__restrict__ sd, u32 *__restrict__ blk_kept,
                                                   u32 *__restrict__ blk_prot, const double *__restrict__ blk_sq,
                                                   SInfo *__restrict__ info)
{
    __shared__ u32 sk[SWG], sp[SWG];
    const int t = blockIdx.x;
    const SDesc d = sd[t];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const u64 nb = (d.n + SBLK - 1) / SBLK;
    const u64 per = (nb + SWG - 1) / SWG;
    const u64 b0 = d.blk0 + (u64)tid * per, b1 = min(d.blk0 + nb, b0 + per);
    u32 ck = 0u, cp = 0u;
    for (u64 b = b0; b < b1; b++) {
        ck += blk_kept[b];
        cp += blk_prot[b];
    }
    sk[tid] = ck;
    sp[tid] = cp;
    __syncthreads();
    if (tid == 0) { // serial over 1024 partial sums
        u32 rk = 0u, rp = 0u;
        for (int i = 0; i < SWG; i++) {
            const u32 a = sk[i], b = sp[i];
            sk[i] = rk;
            sp[i] = rp;
            rk += a;
            rp += b;
        }
        info[t].n_kept = rk;
        info[t].n_outlier = rp;
        info[t].n_pruned = d.n - rk - rp;
    }
    __syncthreads();
    u32 rk = sk[tid], rp = sp[tid];
    for (u64 b = b0; b < b1; b++) {
        const u32 a = blk_kept[b], c = blk_prot[b];
        blk_kept[b] = rk;
        blk_prot[b] = rp;
        rk += a;
        rp += c;
    }
    // squares of the pruned and of the protected values, added in block order by one wave
    if (wave == 0u) {
        double a = 0.0, c = 0.0;
        for (u64 b = d.blk0; b < d.blk0 + nb; b += 64u) { // 64 blocks at a time, lanes in order
            const double x = (b + lane < d.blk0 + nb) ? blk_sq[2u * (b + lane)] : 0.0;
            const double y = (b + lane < d.blk0 + nb) ? blk_sq[2u * (b + lane) + 1u] : 0.0;
            a += wave_sum_f64(x);
            c += wave_sum_f64(y);
        }
        if (lane == 0u) {
            info[t].sq_pruned = a;
            info[t].sq_prot = c;
        }
    }
}

__global__ __launch_bounds__(SWG) void k_sens_compact(const SDesc *__restrict__ sd, int nT, u64 n_blocks,
                                                      const u32 *__restrict__ blk_kept)
{
    const u32 lane = threadIdx.x & 63u;
    const u64 blk = (u64)blockIdx.x * (SWG / 64) + (threadIdx.x >> 6);
    if (blk >= n_blocks) return;
    const SDesc d = sd[sens_tensor_of(sd, nT, blk)];
    const u64 e0 = (blk - d.blk0) * (u64)SBLK;
    u64 pos = (u64)blk_kept[blk]; // wave-uniform
    for (int r = 0; r < SBLK / 64; r++) {
        const u64 i = e0 + (u64)r * 64u + lane;
        const bool valid = i < d.n;
        const float w = valid ? d.w[i] : 0.0f, s = valid ? d.S[i] : 0.0f;
        const bool keep = valid && sens_class(d, w, s) == 2u;
        const u64 m = __ballot(keep);
        if (keep) d.Wm[pos + __builtin_amdgcn_mbcnt_hi((u32)(m >> 32), __builtin_amdgcn_mbcnt_lo((u32)m, 0u))] = w;
        pos += (u64)__popcll(m);
    }
}

__global__ __launch_bounds__(SWG) void k_sens_quant(const SDesc *__restrict__ sd, int nT, u64 n_blocks,
                                                    const u32 *__restrict__ blk_prot, u32 *__restrict__ flags)
{
    __shared__ u32 skey[SWG / 64][256];  // this wave's tensor: boundary keys, ascending
    __shared__ u16 ssym[SWG / 64][SBLK]; // symbols of the wave's block
    const u32 lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const u64 blk = (u64)blockIdx.x * (SWG / 64) + wave;
    const bool live = blk < n_blocks; // (every wave reaches the barriers)
    const int t = sens_tensor_of(sd, nT, live ? blk : 0ull);
    const SDesc d = sd[t];
    const u32 K = d.K, wb = d.sym_bits;
    u32 *bk = skey[wave];
    u16 *sy = ssym[wave];
    if (live) {
        for (u32 j = lane; j + 1u < K; j += 64u) bk[j] = d.bkeys[bnd_index(K, j + 1u)];
        if (blk == d.blk0) { // the tensor's first block also hands out boundaries and centres
            for (u32 j = lane; j + 1u < K; j += 64u)
                if (d.boundaries) d.boundaries[j] = __uint_as_float(bits_of_key(d.bkeys[bnd_index(K, j + 1u)]));
            for (u32 j = lane; j < K; j += 64u) d.codebook[j] = d.cb[j];
        }
    }
    __syncthreads();
    const u64 e0 = live ? (blk - d.blk0) * (u64)SBLK : 0ull;
    u64 ppos = live ? (u64)blk_prot[blk] : 0ull;
    bool overflow = false;
    for (int r = 0; r < SBLK / 64; r++) {
        const u64 i = e0 + (u64)r * 64u + lane;
        const bool valid = live && i < d.n;
        const float w = valid ? d.w[i] : 0.0f, s = valid ? d.S[i] : 0.0f;
        u32 sym = valid ? sens_class(d, w, s) : 0u;
        if (sym == 2u) { // number of boundaries at or below the key
            const u32 key = key_of_float(w);
            u32 lo = 0u, hi = K - 1u;
            while (lo < hi) {
                const u32 mid = (lo + hi) >> 1;
                if (bk[mid] <= key)
                    lo = mid + 1u;
                else
                    hi = mid;
            }
            sym = 2u + lo;
        }
        const bool prot = valid && sym == 1u;
        const u64 m = __ballot(prot);
        if (prot) {
            const u64 at = ppos + __builtin_amdgcn_mbcnt_hi((u32)(m >> 32), __builtin_amdgcn_mbcnt_lo((u32)m, 0u));
            if (at < d.out_cap) {
                d.out_idx[at] = (u32)i;
                d.out_val[at] = w;
            } else {
                overflow = true;
            }
        }
        ppos += (u64)__popcll(m);
        sy[r * 64 + lane] = (u16)sym;
    }
    if (__ballot(overflow) && lane == 0u) atomicOr(flags, 2u);
    __syncthreads();
    if (!live) return;
    // 1024 symbols of wb bits are 16 * wb whole words; the tensor's last block may end earlier
    const u64 n_here = (d.n - e0 < (u64)SBLK) ? d.n - e0 : (u64)SBLK;
    const u32 n_words = (u32)((n_here * wb + 63u) >> 6);
    unsigned long long *dst = d.packed + (e0 * wb >> 6); // e0 * wb is a multiple of 64
    for (u32 k = lane; k < n_words; k += 64u) {
        const u32 bit0 = k * 64u;
        u32 e = bit0 / wb;                 // first element with bits in this word
        unsigned long long word = 0ull;
        for (; e < (u32)n_here && e * wb < bit0 + 64u; e++) {
            const unsigned long long v = sy[e];
            const int sh = (int)(e * wb) - (int)bit0;
            word |= sh >= 0 ? v << sh : v >> (-sh);
        }
        dst[k] = word;
    }
}

hipError_t launch_sens_score(const SDesc *sd, int nT, u64 n_blocks, hipStream_t s)
{
    const unsigned grid = (unsigned)((n_blocks + SWG / 64 - 1) / (SWG / 64));
    PROF("k_sens_score", s, k_sens_score<<<grid, SWG, 0, s>>>(sd, nT, n_blocks));
    return hipGetLastError();
}

hipError_t launch_sens_partition(const SDesc *sd, int nT, u64 n_blocks, u32 *blk_kept, u32 *blk_prot,
                                 double *blk_sq, SInfo *info, hipStream_t s)
{
    const unsigned grid = (unsigned)((n_blocks + SWG / 64 - 1) / (SWG / 64));
    PROF("k_sens_count", s, k_sens_count<<<grid, SWG, 0, s>>>(sd, nT, n_blocks, blk_kept, blk_prot, blk_sq));
    PROF("k_sens_scan", s, k_sens_scan<<<nT, SWG, 0, s>>>(sd, blk_kept, blk_prot, blk_sq, info));
    PROF("k_sens_compact", s, k_sens_compact<<<grid, SWG, 0, s>>>(sd, nT, n_blocks, blk_kept));
    return hipGetLastError();
}

hipError_t launch_sens_quant(const SDesc *sd, int nT, u64 n_blocks, const u32 *blk_prot, u32 *flags,
                             hipStream_t s)
{
    const unsigned grid = (unsigned)((n_blocks + SWG / 64 - 1) / (SWG / 64));
    PROF("k_sens_quant", s, k_sens_quant<<<grid, SWG, 0, s>>>(sd, nT, n_blocks, blk_prot, flags));
    return hipGetLastError();
}

} // namespace inshr
