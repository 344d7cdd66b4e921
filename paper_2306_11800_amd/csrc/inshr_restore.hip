// Decoding a quantized tensor (Sec. 4, the inverse of the Quantizer): symbol 0 gives +0.0, symbol
// 2 + b gives the centre of bin b, and the elements with symbol 1 take their original values from
// the protected list.
//
//   k_dequant            workgroups of 256 threads (eight per CU) walk runs of tiles of 16384 elements:
//                        the tile's packed words (asked for one tile ahead) and the codebook are
//                        staged in LDS, every thread decodes 4 consecutive elements at a time and
//                        stores them as one 16-byte piece, 16 pieces per tile.  Waiting for the next
//                        tile's words also waits for this tile's stores, so a tile has to be long
//                        enough to hide that.  Elements with symbol 1 are counted (ballots) and left
//                        at +0.0.
//   k_dequant_protected  one thread per entry of the protected list: checks that the element's symbol
//                        is 1 and stores the value.
#include "inshr_launch.h"

namespace inshr {

__device__ __forceinline__ int find_rdesc(const RDesc *rd, int nT, u64 tile)
{
    int lo = 0, hi = nT - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (rd[mid].tile0 <= tile)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

constexpr int DQ_BLOCK = 256;
constexpr int DQ_TILE = DEQUANT_TILE; // 64 elements per thread
constexpr int DQ_ROUNDS = DQ_TILE / (4 * DQ_BLOCK);

__global__ __launch_bounds__(DQ_BLOCK) void k_dequant(const RDesc *__restrict__ rd, int nT, u64 n_tiles,
                                                      u32 *__restrict__ flags, u32 *__restrict__ ones)
{
    __shared__ u32 W[((DQ_TILE * 9 / 32 + DQ_BLOCK - 1) / DQ_BLOCK) * DQ_BLOCK + 4];
    __shared__ float cb[256];
    const u32 tid = threadIdx.x;
    // every workgroup takes a run of consecutive tiles: the tensor of the first is searched for, the
    // others follow from it
    const u64 per = (n_tiles + gridDim.x - 1) / gridDim.x;
    const u64 tile_lo = (u64)blockIdx.x * per;
    const u64 tile_hi = tile_lo + per < n_tiles ? tile_lo + per : n_tiles;
    if (tile_lo >= tile_hi) return;
    int t = __builtin_amdgcn_readfirstlane(find_rdesc(rd, nT, tile_lo));
    int t_cb = -1; // tensor whose codebook is in LDS
    u32 bad = 0u;
    constexpr int PRE = (DQ_TILE * 9 / 32 + DQ_BLOCK - 1) / DQ_BLOCK; // dwords per thread and tile
    u32 pre[PRE]; // the next tile's packed words, asked for one tile ahead
    auto fetch = [&](int tt, u64 tile) {
        const RDesc d = rd[tt];
        const u64 e0 = (tile - d.tile0) * DQ_TILE;
        const u32 cnt = (d.n - e0 < (u64)DQ_TILE) ? (u32)(d.n - e0) : (u32)DQ_TILE;
        const u32 nd = 2u * ((cnt * d.w + 63u) >> 6); // dwords of the tile, all inside the packed array
        const GLOBAL_AS u32 *src = (const GLOBAL_AS u32 *)(gptr(d.packed) + e0 * d.w / 64u);
#pragma unroll
        for (int j = 0; j < PRE; j++) {
            const u32 k = tid + (u32)DQ_BLOCK * j;
            pre[j] = k < nd ? src[k] : 0u;
        }
    };
    fetch(t, tile_lo);
    for (u64 tile = tile_lo; tile < tile_hi; tile++) {
        const RDesc d = rd[t];
        const u64 e0 = (tile - d.tile0) * DQ_TILE;
        const u32 cnt = (d.n - e0 < (u64)DQ_TILE) ? (u32)(d.n - e0) : (u32)DQ_TILE;
        const u32 w = d.w, K = d.K;
        __syncthreads(); // the previous tile has been decoded
#pragma unroll
        for (int j = 0; j < PRE; j++) W[tid + (u32)DQ_BLOCK * j] = pre[j]; // zero past the tile's words
        if (t != t_cb) {
            if (tid < 256u) cb[tid] = tid < K ? gptr(d.codebook)[tid] : 0.0f;
            t_cb = t;
        }
        __syncthreads();
        const int t_now = t;
        if (tile + 1 < tile_hi) {
            while (t + 1 < nT && rd[t + 1].tile0 <= tile + 1) t++;
            fetch(t, tile + 1);
        }
        GLOBAL_AS float *dst = gptr(d.dst) + e0;
        const bool vec = cnt == (u32)DQ_TILE && ((((u64)dst) & 15u) == 0u);
        const u32 mask = (1u << w) - 1u;
        u32 n_one = 0u;
#pragma unroll
        for (u32 j = 0; j < (u32)DQ_ROUNDS; j++) {
            const u32 i0 = 4u * (tid + (u32)DQ_BLOCK * j);
            // four symbols are 4 w <= 36 bits from bit i0 * w on
            const u32 off = i0 * w, wd = off >> 5, sh = off & 31u;
            const u64 lo = ((u64)W[wd + 1] << 32) | (u64)W[wd];
            const u64 bits = (lo >> sh) | (sh ? ((u64)W[wd + 2] << (64u - sh)) : 0ull);
            float x[4];
#pragma unroll
            for (u32 c = 0; c < 4u; c++) {
                const u32 sym = (u32)(bits >> (c * w)) & mask;
                const bool valid = i0 + c < cnt;
                n_one += (u32)__popcll(__ballot(valid && sym == 1u));
                if (valid && sym >= K + 2u) bad = 1u;
                const u32 b = sym - 2u;
                x[c] = (sym >= 2u && b < K) ? cb[b] : 0.0f;
            }
            if (vec) {
                typedef float f4 __attribute__((ext_vector_type(4)));
                f4 q = {x[0], x[1], x[2], x[3]};
                ((GLOBAL_AS f4 *)dst)[tid + (u32)DQ_BLOCK * j] = q;
            } else {
#pragma unroll
                for (u32 c = 0; c < 4u; c++)
                    if (i0 + c < cnt) dst[i0 + c] = x[c];
            }
        }
        if ((tid & 63u) == 0u && n_one) atomicAdd(&ones[t_now], n_one);
    }
    if (__ballot(bad != 0u) && (tid & 63u) == 0u) atomicOr(flags, RF_SYMBOL);
}

__global__ __launch_bounds__(256) void k_dequant_protected(const RDesc *__restrict__ rd,
                                                           u32 *__restrict__ flags,
                                                           const u32 *__restrict__ ones)
{
    const RDesc d = rd[blockIdx.y];
    if (blockIdx.x == 0 && threadIdx.x == 0 && (u64)ones[blockIdx.y] != d.n_outlier)
        atomicOr(flags, RF_LIST);
    const u32 mask = (1u << d.w) - 1u;
    for (u64 j = (u64)blockIdx.x * 256u + threadIdx.x; j < d.n_outlier; j += (u64)gridDim.x * 256u) {
        const u64 i = gptr(d.out_idx)[j];
        bool ok = i < d.n && (j == 0 || gptr(d.out_idx)[j - 1] < i); // ascending, hence distinct
        if (ok) {
            const u64 off = i * d.w, wd = off >> 6;
            const u32 sh = (u32)(off & 63u);
            unsigned long long x = gptr(d.packed)[wd] >> sh;
            if (sh + d.w > 64u) x |= gptr(d.packed)[wd + 1] << (64u - sh);
            ok = ((u32)x & mask) == 1u;
        }
        if (ok)
            gptr(d.dst)[i] = d.val_bf16
                                 ? __uint_as_float((u32)((const GLOBAL_AS u16 *)gptr(d.out_val))[j] << 16)
                                 : gptr(d.out_val)[j];
        else
            atomicOr(flags, RF_LIST);
    }
}

hipError_t launch_dequantize(const RDesc *rd, int nT, u64 n_tiles, u64 max_outlier, u32 *flags,
                             u32 *ones, int n_cu, hipStream_t s)
{
    u64 grid = (u64)n_cu * 64u; // 8 resident workgroups per CU, 8 rounds
    if (grid > n_tiles) grid = n_tiles;
    PROF("k_dequant", s, k_dequant<<<(unsigned)grid, DQ_BLOCK, 0, s>>>(rd, nT, n_tiles, flags, ones));
    u64 blocks = (max_outlier + 255u) / 256u;
    if (blocks < 1) blocks = 1;
    if (blocks > 1024) blocks = 1024;
    PROF("k_dequant_protected", s,
         k_dequant_protected<<<dim3((unsigned)blocks, (unsigned)nT), 256, 0, s>>>(rd, flags, ones));
    return hipGetLastError();
}

} // namespace inshr
