// Delta Encoder (Sec. 6): d = (s_prev - s_cur) mod B with B = max(K_prev, K_cur) + 2, regrouped in
// the stable order of the previous checkpoint's symbol (Algorithm 5) and bit-packed.
//
// The regrouping is a stable partition into at most 258 groups:
//   k_dhist     per chunk (64 tiles of 12288 elements): population of every previous symbol
//   k_dgroups   per tensor: group offsets and the start of every chunk inside every group
//   k_dscatter  one workgroup of 12 waves per chunk walks its tiles in order.  Per tile each wave
//               owns 1024 consecutive elements, 64 consecutive elements per step; a returning LDS
//               add per element (or lane bits OR-ed into the symbol's LDS slot) gives the stable
//               rank.  The tile's deltas are OR-ed into an LDS image of the output words of every
//               group's run, and one thread per word stores it (first / last word of a chunk's run
//               are OR-ed into words that k_dzero cleared).
#include "inshr_launch.h"

namespace inshr {

constexpr int DTILE = DELTA_TILE;   // elements per tile = 1024 per wave of the scatter workgroup
constexpr int DCHUNK = DELTA_CHUNK; // tiles per chunk
constexpr int SS = DELTA_SS;        // symbol stride (258 symbols at most)
constexpr int NWAVE = DTILE / 1024; // waves of a scatter workgroup (two workgroups share a CU)
constexpr int DBLOCK = NWAVE * 64;
constexpr int TWORDS = DTILE * 9 / 64;            // most packed u64 words of one tile
constexpr u64 CHUNK_ELEMS = (u64)DTILE * DCHUNK;  // 786432, a multiple of 16384
constexpr int HTILE = 16384;                      // step of the counting and gathering kernels
static_assert(CHUNK_ELEMS % HTILE == 0, "chunks are whole counting steps");

__device__ __forceinline__ u32 lds_extract(const u32 *W, u32 idx, u32 w)
{
    const u32 off = idx * w;
    const u32 wd = off >> 5, sh = off & 31u;
    const u64 two = ((u64)W[wd + 1] << 32) | (u64)W[wd];
    return (u32)(two >> sh) & ((1u << w) - 1u);
}

// Symbols of one chunk counted by width W: every lane takes runs of 64 consecutive symbols (W whole
// words), extracts them from registers with compile-time shifts and counts the non-zero ones in its
// wave's LDS histogram.  Symbol 0 (pruned: the most frequent one when pruning is on) is not counted:
// its population is what the others leave of the chunk.
// Narrow symbols (few clusters, unequal populations: the bins of the sketch quantizer) make many
// lanes of a wave hit the same counter at once; their lanes are spread over DH_COPIES rows.
constexpr int DH_COPIES = 4;
template <int W, bool WHOLE>
__device__ __forceinline__ void count_run(const u32 (&x)[2 * W + 1], u32 nvalid, u32 S, u32 *hrow)
{
    if (W <= 7) hrow += (threadIdx.x & (u32)(DH_COPIES - 1)) * (u32)SS;
#pragma unroll
    for (int i = 0; i < 64; i++) {
        constexpr u32 mask = (1u << W) - 1u;
        const int p = i * W, dw = p >> 5, sh = p & 31;
        u32 sym = (sh + W <= 32) ? (x[dw] >> sh) & mask
                                 : __builtin_amdgcn_alignbit(x[dw + 1], x[dw], sh) & mask;
        sym = sym < S ? sym : S; // a malformed stream counts into the unused entry S
        if (sym != 0u && (WHOLE || (u32)i < nvalid)) atomicAdd(&hrow[sym], 1u);
    }
}

template <int W>
__device__ __forceinline__ void count_symbols(const DDesc &d, u64 c0, u64 c1, u32 S, u32 *hrow)
{
    const u32 tid = threadIdx.x;
    const GLOBAL_AS unsigned long long *src = gptr(d.prev);
    const u64 total_words = (d.n * W + 63u) >> 6;
    const u32 n_runs = (u32)((c1 - c0 + 63u) >> 6);
    for (u32 u = tid; u < n_runs; u += BLOCK) {
        const u64 e = c0 + 64ull * u;
        const u32 nvalid = (c1 - e < 64ull) ? (u32)(c1 - e) : 64u;
        const u64 w0 = (e >> 6) * W; // e is a multiple of 64
        u32 x[2 * W + 1];
#pragma unroll
        for (int k = 0; k < W; k++) {
            const unsigned long long v = (w0 + k < total_words) ? src[w0 + k] : 0ull;
            x[2 * k] = (u32)v;
            x[2 * k + 1] = (u32)(v >> 32);
        }
        x[2 * W] = 0u;
        if (__ballot(nvalid < 64u) == 0ull) // the same for every active lane
            count_run<W, true>(x, nvalid, S, hrow);
        else
            count_run<W, false>(x, nvalid, S, hrow);
    }
}

// population of every previous symbol in one chunk
__global__ __launch_bounds__(BLOCK) void k_dhist(const DDesc *__restrict__ dd,
                                                 const u32 *__restrict__ chunk_tensor,
                                                 u32 *__restrict__ chunk_tot)
{
    __shared__ u32 hw[BLOCK / 64][DH_COPIES * SS];
    __shared__ u32 s_nonzero;
    const u64 chunk = blockIdx.x;
    const DDesc d = dd[__builtin_amdgcn_readfirstlane(chunk_tensor[chunk])];
    const u32 tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const u32 S = d.Kp + 2u;
    const u64 c0 = (chunk - d.chunk0) * CHUNK_ELEMS;
    const u64 c1 = (c0 + CHUNK_ELEMS < d.n) ? c0 + CHUNK_ELEMS : d.n;
    for (u32 k = tid; k < (BLOCK / 64) * DH_COPIES * SS; k += BLOCK) (&hw[0][0])[k] = 0u;
    if (tid == 0u) s_nonzero = 0u;
    __syncthreads();
    switch (d.wp) {
    case 2: count_symbols<2>(d, c0, c1, S, hw[wave]); break;
    case 3: count_symbols<3>(d, c0, c1, S, hw[wave]); break;
    case 4: count_symbols<4>(d, c0, c1, S, hw[wave]); break;
    case 5: count_symbols<5>(d, c0, c1, S, hw[wave]); break;
    case 6: count_symbols<6>(d, c0, c1, S, hw[wave]); break;
    case 7: count_symbols<7>(d, c0, c1, S, hw[wave]); break;
    case 8: count_symbols<8>(d, c0, c1, S, hw[wave]); break;
    default: count_symbols<9>(d, c0, c1, S, hw[wave]); break;
    }
    __syncthreads();
    u32 mine = 0u; // population of symbol tid (symbols above S - 1 are in entry S)
    if (tid >= 1u && tid <= S) {
        for (int wv = 0; wv < BLOCK / 64; wv++)
            for (int cp = 0; cp < DH_COPIES; cp++) mine += hw[wv][cp * SS + tid];
        if (mine) atomicAdd(&s_nonzero, mine);
    }
    __syncthreads();
    if (tid == 0u) mine = (u32)(c1 - c0) - s_nonzero;
    if (tid < SS) chunk_tot[chunk * SS + tid] = tid < S ? mine : 0u;
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
            gptr(d.group_off)[k] = acc;
            acc += tot[k];
        }
        gptr(d.group_off)[S] = acc;
    }
}

// The packed words of one tile's symbols go from device memory straight into LDS (no registers in
// between, nothing waits here): every lane moves 16 bytes per instruction when the source is
// 16-byte aligned, 4 bytes otherwise; a wave's lanes write consecutive LDS addresses.  NW waves
// share the work, the calling wave being number widx of them.  The words are complete after
// `s_waitcnt vmcnt(0)` and a barrier.
template <int NW>
__device__ __forceinline__ void lds_fetch(const GLOBAL_AS unsigned long long *src, u64 e0, u32 cnt,
                                          u32 w, u32 *dst, u32 widx)
{
    u32 lane = threadIdx.x & 63u;
    asm volatile("" : "+v"(lane)); // the addresses below are cheap: recomputing them in every tile
                                   // beats keeping them in (spilled) registers across the loop
    const GLOBAL_AS u32 *g = (const GLOBAL_AS u32 *)(src + e0 * w / 64u); // exact: e0 % 64 == 0
    LDS_AS u32 *l = (LDS_AS u32 *)dst;
    const u32 nd = 2u * ((cnt * w + 63u) >> 6); // dwords of the tile, all inside the packed array
    constexpr u32 MAXD = DTILE * 9 / 32;        // at most 3456 dwords
    constexpr u32 R16 = (MAXD / 4 + NW * 64 - 1) / (NW * 64), R4 = (MAXD + NW * 64 - 1) / (NW * 64);
    u32 done = 0u;
    if ((((u64)g) & 15u) == 0u) {
        const u32 n16 = nd >> 2;
#pragma unroll
        for (u32 it = 0; it < R16; it++) {
            const u32 c0 = (it * NW + widx) * 64u;
            if (c0 + lane < n16)
                __builtin_amdgcn_global_load_lds(g + (c0 + lane) * 4u, l + c0 * 4u, 16, 0, 0);
        }
        done = n16 << 2;
    }
    if (done < nd) { // (the same for the whole workgroup: nothing is left after the 16-byte pieces
                     // of a whole tile)
#pragma unroll
        for (u32 it = 0; it < R4; it++) {
            const u32 c0 = done + (it * NW + widx) * 64u;
            if (c0 + lane < nd) __builtin_amdgcn_global_load_lds(g + (c0 + lane), l + c0, 4, 0, 0);
        }
    }
}

// Words of the LDS image of one tile's output: every group's run starts at the bit of its first
// stream word that the stream position dictates, so LDS word k is stream word dbase[g] + k.  A run
// of b bits touches at most b / 64 + 2 words.
constexpr int BWORDS = TWORDS + 2 * SS + 2;
constexpr int WST = NWAVE * SS;       // per-(wave, symbol) counters; the row stride is S + 1
constexpr int CIDX = BWORDS / 8 + 2;  // one entry per 8 image words: the group of the first of them

constexpr int LINE = 4; // stream words (32 bytes) per output line

struct ScatterShared {
    u32 wst[WST];                   // counts, then bit position in the image of (wave, symbol)
    u32 wstart[SS + 8];             // first image word of each group's run; [S] = words in use
    unsigned long long lw[SS][LINE]; // per group: the words of its current, incomplete output line
    u32 fo[SS];                     // first stream word that this chunk's run of the group owns
                                    // alone; bit 31: the word before it is shared with the run before
    u32 gb[SS];                     // stream position after each group's runs so far (n < 2^32)
    u32 gWf[SS], gWe[SS];           // the group's run of the current tile: stream word of its first
                                    // bit; first word that is still incomplete after it
    u32 gtl[SS];                    // bits of word gWe that are filled; bit 31: the run is not empty
    u32 wtot[8], etot[8];
    unsigned long long hotkey;      // population << 9 | symbol, maximum over the tensor's groups
    u16 cidx[CIDX];
};

// Where a group's run of `cnt` symbols that starts at stream position `pos` lies in the stream.
struct RunWords {
    u32 Wf, We; // word of its first bit; first word that is still incomplete after it
    u32 tail;   // bits of word We that are filled
};
__device__ __forceinline__ RunWords run_words(u32 pos, u32 cnt, u32 wB)
{
    RunWords r;
    const u64 fb = (u64)pos * wB, fe = fb + (u64)cnt * wB;
    r.Wf = (u32)(fb >> 6);
    r.We = (u32)(fe >> 6);
    r.tail = (u32)(fe & 63u);
    return r;
}

// Cross-check of the ordered ranking, once per chunk and wave, before the tile loop: the 64 previous
// symbols of the wave's first row of the chunk's first tile are ranked once with returning adds into
// the wave's (zero) counter row and once from ballots; the counters are zero again afterwards.  Returns 1 when the two disagree (the
// device did not serve same-address LDS atomics in lane order).
__device__ __forceinline__ u32 ordered_rank_check(const u32 *P, u32 *wrow, u32 ebase, u32 cnt, u32 S, u32 wp)
{
    const u32 lane = threadIdx.x & 63u;
    const u32 off = ebase * wp;
    u32 sp = S; // lanes past the end share the unused symbol S
    if (ebase < cnt) {
        sp = __builtin_amdgcn_alignbit(P[(off >> 5) + 1u], P[off >> 5], off & 31u) & ((1u << wp) - 1u);
        sp = sp < S - 1u ? sp : S - 1u;
    }
    const u32 got = atomicAdd(&wrow[sp], 1u);
    u64 peers = ~0ull;
#pragma unroll
    for (int b = 0; b < 9; b++) {
        const bool bit = (sp >> b) & 1u;
        const u64 m = __ballot(bit);
        peers &= bit ? m : ~m;
    }
    const u32 bad = got != (u32)__popcll(peers & ((1ull << lane) - 1ull)) ? 1u : 0u;
    wrow[sp] = 0u; // (after the add: the wave's LDS operations complete in order)
    return bad;
}

// Sweep 1 of a tile: stable rank of every element among the equal symbols of its wave's 1024
// elements.  Row r of a lane is element ebase + 64 r: its bit offset in the packed words moves
// by 64 w per row, so the shift is a lane constant and the word address advances by 2 w.
// reg[r] = symbol | rank << 9 | delta << 19 | valid << 31, or with BITPOS (needs wB): symbol |
// (rank * wB) << 9 | delta << 23, where an element past the end has delta 0.
template <bool FULL, bool ORDERED, bool BITPOS = false>
__device__ __forceinline__ void rank_rows(const u32 *P, const u32 *C, u32 *wrow,
                                          unsigned long long *myslot, u32 ebase, u32 cnt, u32 S,
                                          u32 Bm, u32 wp, u32 wc, u32 hot, u32 (&reg)[16], u32 wB = 0u)
{
    u32 hot_seen = 0u; // elements of the wave so far that hold the most frequent symbol
    const u32 lane = threadIdx.x & 63u;
    const u64 ltmask = (1ull << lane) - 1ull;
    const unsigned long long lanebit = 1ull << lane;
    const u32 offP = ebase * wp, offC = ebase * wc;
    const u32 shP = offP & 31u, shC = offC & 31u;
    const u32 mP = (1u << wp) - 1u, mC = (1u << wc) - 1u;
    const u32 *pp = P + (offP >> 5), *pc = C + (offC >> 5);
#pragma unroll
    for (u32 rb = 0; rb < 16u; rb += 4u) {
        u32 xp[4][2], xc[4][2];
#pragma unroll
        for (u32 q = 0; q < 4u; q++) { // the reads of four rows are in flight together
            const u32 r = rb + q;
            xp[q][0] = pp[r * 2u * wp];
            xp[q][1] = pp[r * 2u * wp + 1u];
            xc[q][0] = pc[r * 2u * wc];
            xc[q][1] = pc[r * 2u * wc + 1u];
        }
#pragma unroll
        for (u32 q = 0; q < 4u; q++) {
            const u32 r = rb + q;
            const bool valid = FULL || (ebase + r * 64u < cnt);
            u32 sp = S, sc = 0u; // lanes past the end share the unused symbol S
            if (valid) {
                sp = __builtin_amdgcn_alignbit(xp[q][1], xp[q][0], shP) & mP;
                sc = __builtin_amdgcn_alignbit(xc[q][1], xc[q][0], shC) & mC;
                sp = sp < S - 1u ? sp : S - 1u; // clamps a malformed stream
            }
            u32 within; // elements of this wave with the same symbol and a lower index
            if (ORDERED) {
                // the most frequent symbol (the pruned one, typically a fifth of all elements) would
                // serialise the atomic: its lanes rank themselves from the ballot instead
                const bool is_hot = sp == hot;
                const u64 hm = __ballot(is_hot);
                const u32 hrank = __builtin_amdgcn_mbcnt_hi((u32)(hm >> 32),
                                                            __builtin_amdgcn_mbcnt_lo((u32)hm, hot_seen));
                hot_seen += (u32)__popcll(hm);
                within = hrank;
                if (!is_hot) within = atomicAdd(&wrow[sp], 1u);
            } else {
                atomicOr(&myslot[sp], lanebit);
                const unsigned long long peers = myslot[sp];
                const u32 rank = __popcll(peers & ltmask);
                const u32 old = wrow[sp];
                if (rank == 0u) {
                    myslot[sp] = 0ull;
                    wrow[sp] = old + (u32)__popcll(peers);
                }
                within = old + rank;
            }
            u32 dv = sp - sc;
            if (sp < sc) dv += Bm;
            if (BITPOS)
                reg[r] = (__umul24(within, wB << 9) + sp) | ((valid ? dv : 0u) << 23);
            else
                reg[r] = sp | (within << 9) | (dv << 19) | ((valid ? 1u : 0u) << 31);
        }
    }
    if (ORDERED && lane == 0u) wrow[hot] = hot_seen;
}

// After a tile's output phase, one thread per (group, word j of a line): word j of the line that
// the tile completed, if earlier tiles had buffered it, is stored; then word j of the group's open
// line, if it came from this tile's image (a complete word of a line that is the chunk's own, or the
// partial last word), moves into the group's line buffer.  A thread touches no other thread's
// buffer word, and nothing else touches the buffers or the image meanwhile.
__device__ __forceinline__ void flush_and_commit(ScatterShared &sh, const unsigned long long *image,
                                                 GLOBAL_AS unsigned long long *out, u32 item)
{
    asm volatile("" : "+v"(item)); // the item's addresses are recomputed here, not kept across the
                                   // tile loop in spilled registers (a reload would wait for stores)
    const u32 g = item / LINE, j = item % LINE;
    const u32 meta = sh.gtl[g];
    if (!(meta >> 31)) return; // the group had no element in the tile
    const u32 Wf = sh.gWf[g], We = sh.gWe[g], tail = meta & 63u;
    const u32 own = sh.fo[g] & 0x7fffffffu;
    const u32 Lf = Wf / LINE, Le = We / LINE;
    if (Lf * LINE >= own && Lf < Le && j < (Wf & (LINE - 1u))) out[Lf * LINE + j] = sh.lw[g][j];
    const u32 Wt = Le * LINE + j;      // word j of the line that is open after the tile
    if (Wt > We || Wt < Wf) return;    // not written yet / buffered by an earlier tile
    unsigned long long v = 0ull;
    if (Wt < We || tail) {
        v = image[sh.wstart[g] + (Wt - Wf)];
        if (Wt == Wf) v |= sh.lw[g][j]; // bits of earlier tiles in the run's first word
    }
    sh.lw[g][j] = v;
}

// ORDERED: same-address LDS atomics with return are served in ascending lane order on this device
// (checked by k_lds_order_check before the library relies on it); one returning add then ranks an
// element.  Otherwise equal symbols of a step find each other through the slot array.
//
// Output: a group's run of one tile is a few dozen bytes, and 258 groups interleave, so storing it
// as it comes would reach memory as partial lines.  Each group therefore keeps the words of its
// current 64-byte line in LDS until the line is complete; complete lines are stored whole.  Only the
// ends of a (chunk, group) run are different: its first partial line is stored word by word, its
// first word, when shared with the run before, and its last partial word are OR-ed into words that
// k_dzero cleared.
template <bool PERM, bool ORDERED>
__global__ __launch_bounds__(DBLOCK, 6) void k_dscatter(const DDesc *__restrict__ dd,
                                                     const u32 *__restrict__ chunk_tensor,
                                                     const u32 *__restrict__ chunk_tot,
                                                     u32 *__restrict__ flags)
{
    __shared__ ScatterShared sh;
    // packed symbols of the current tile (variables of their own: the loads that fill them are
    // asynchronous, and only reads of these two arrays have to wait for them)
    __shared__ __attribute__((aligned(16))) u32 Pw[DTILE * 9 / 32 + 8];
    __shared__ __attribute__((aligned(16))) u32 Cw[DTILE * 9 / 32 + 8];
    // slot[wave][symbol]: lanes of the wave's current step that hold the symbol (sweep 1);
    // the same memory then holds the image of the tile's output words (sweep 2, output)
    __shared__ unsigned long long slot[ORDERED ? BWORDS : NWAVE * SS];
    __shared__ u32 wel[PERM ? WST : 1];  // local regrouped index of (wave, symbol)
    __shared__ u32 lbase[PERM ? SS : 1]; // local regrouped index of each group's run; [S] = elements
    __shared__ u16 si[PERM ? DTILE : 1]; // local indices in regrouped order
    u32 *img = (u32 *)slot;
    static_assert(NWAVE * SS >= BWORDS, "output image fits the slot array");

    const u64 chunk = blockIdx.x;
    const DDesc d = dd[__builtin_amdgcn_readfirstlane(chunk_tensor[chunk])];
    if (d.prev_perm) return; // this tensor's regrouping is given: k_dgather writes its stream
    if (PERM != (d.perm != nullptr)) return;
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const u32 S = d.Kp + 2u, Bm = d.B, wB = d.wB, wp = d.wp, wc = d.wc;
    const u32 srow = S + 1u; // row stride of the (wave, symbol) tables
    const u64 n_tiles = (d.n + DTILE - 1) / DTILE;
    const u64 lt0 = (chunk - d.chunk0) * DCHUNK;
    const u64 lt1 = (lt0 + DCHUNK < n_tiles) ? lt0 + DCHUNK : n_tiles;
    GLOBAL_AS unsigned long long *out = gptr(d.out);
    if (tid < S) {
        const u32 g0 = (u32)gptr(d.group_off)[tid] + chunk_tot[chunk * SS + tid];
        sh.gb[tid] = g0;
        sh.gtl[tid] = 0u;
        const u64 sb = (u64)g0 * wB;
        sh.fo[tid] = (u32)((sb + 63u) >> 6) | ((sb & 63u) ? 0x80000000u : 0u);
    }
    for (u32 k = tid; k < S * LINE; k += DBLOCK) (&sh.lw[0][0])[k] = 0ull;
    if (tid < SS + 8u) sh.wstart[tid] = 0xFFFFFFFFu;
    if (tid == 0u) sh.hotkey = 0ull;
    for (u32 k = tid; k < (u32)WST; k += DBLOCK) sh.wst[k] = 0u;
    __syncthreads();
    if (tid < S)
        atomicMax(&sh.hotkey, ((gptr(d.group_off)[tid + 1u] - gptr(d.group_off)[tid]) << 9) | tid);
    __syncthreads();
    const u32 hot = __builtin_amdgcn_readfirstlane((u32)sh.hotkey & 511u);
    u32 *wrow = sh.wst + wave * srow;
    u32 order_bad = 0u;

    auto tile_cnt = [&](u64 lt) -> u32 {
        const u64 rem = d.n - lt * (u64)DTILE;
        return rem < (u64)DTILE ? (u32)rem : (u32)DTILE;
    };
    lds_fetch<NWAVE>(gptr(d.prev), lt0 * (u64)DTILE, tile_cnt(lt0), wp, Pw, wave);
    lds_fetch<NWAVE>(gptr(d.cur), lt0 * (u64)DTILE, tile_cnt(lt0), wc, Cw, wave);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // this wave's share of the first tile's words
    if (ORDERED) {
        __syncthreads(); // all shares of the first tile's words are in LDS
        order_bad = ordered_rank_check(Pw, wrow, wave * 1024u + lane, tile_cnt(lt0), S, wp);
    }
    for (u64 lt = lt0; lt < lt1; lt++) {
        const u64 e0 = lt * (u64)DTILE;
        const u32 cnt = tile_cnt(lt);
        __syncthreads(); // all shares of the tile's words are in LDS (every wave waited for its own
                         // before its output phase); the previous tile's output phase is over
        // the previous tile's lines
        if (tid < S * LINE) flush_and_commit(sh, slot, out, tid);
        if (tid + (u32)DBLOCK < S * LINE) flush_and_commit(sh, slot, out, tid + (u32)DBLOCK);
        if (!ORDERED) { // sweep 1 uses the slots
            __syncthreads();
            for (u32 k = tid; k < (u32)(NWAVE * SS); k += DBLOCK) slot[k] = 0ull;
            __syncthreads();
        }
        u32 reg[16];
        u32 ebase = wave * 1024u + lane;
        asm volatile("" : "+v"(ebase)); // keeps the per-row LDS addresses from being hoisted out of
                                        // the tile loop and spilled
        if (cnt == (u32)DTILE)
            rank_rows<true, ORDERED, !PERM>(Pw, Cw, wrow, slot + wave * SS, ebase, cnt, S, Bm, wp, wc, hot, reg, wB);
        else
            rank_rows<false, ORDERED, !PERM>(Pw, Cw, wrow, slot + wave * SS, ebase, cnt, S, Bm, wp, wc, hot, reg, wB);
        __syncthreads();
        if (ORDERED) { // the image of the previous tile has been taken over; clear it for sweep 2
            const u32 nz = ((cnt * wB) >> 6) + 2u * S + 2u;
            u32 k0 = tid;
            asm volatile("" : "+v"(k0)); // (address recomputed here, not reloaded from a spill slot:
                                         // a reload would wait for the words in flight)
            for (u32 k = k0; k < nz; k += DBLOCK) slot[k] = 0ull;
        }
        // counts -> positions: population of each symbol, the stream words its run touches,
        // exclusive scans over symbols, start of every (wave, symbol)
        u32 tot = 0, nW = 0, s0 = 0, preW = 0, preE = 0;
        u64 fb = 0;
        u32 sy = tid;  // this thread's symbol
        asm volatile("" : "+v"(sy)); // its table addresses are recomputed per tile, not kept (and
                                     // spilled: a reload would wait for the words in flight)
        if (tid < 320u) { // waves 0..4 hold the 258 symbols
            if (tid < S) {
#pragma unroll
                for (int wv = 0; wv < NWAVE; wv++) tot += sh.wst[wv * srow + sy];
                const u32 pos = sh.gb[sy]; // after the previous tile's run
                fb = (u64)pos * wB;
                s0 = (u32)(fb & 63u);
                nW = tot ? (s0 + tot * wB + 63u) >> 6 : 0u;
            }
            const u32 incW = wave_incl_scan(nW), incE = PERM ? wave_incl_scan(tot) : 0u;
            preW = incW - nW;
            preE = incE - tot;
            if (lane == 63u) {
                sh.wtot[wave] = incW;
                sh.etot[wave] = incE;
            }
        }
        __syncthreads();
        // the symbols are in registers: the next tile's words start travelling, asked for by the
        // waves that have no scan to do
        if (lt + 1 < lt1 && wave >= 5u) {
            lds_fetch<NWAVE - 5>(gptr(d.prev), e0 + DTILE, tile_cnt(lt + 1), wp, Pw, wave - 5u);
            lds_fetch<NWAVE - 5>(gptr(d.cur), e0 + DTILE, tile_cnt(lt + 1), wc, Cw, wave - 5u);
        }
        if (tid < S) {
            u32 ws = preW, es = preE;
#pragma unroll
            for (u32 w2 = 0; w2 < 4u; w2++) { // (all read together, the needed ones added)
                const u32 a = sh.wtot[w2], b = PERM ? sh.etot[w2] : 0u;
                ws += w2 < wave ? a : 0u;
                es += w2 < wave ? b : 0u;
            }
            const u64 fe = fb + (u64)tot * wB;
            sh.gb[sy] += tot;
            sh.gWf[sy] = (u32)(fb >> 6);
            sh.gWe[sy] = (u32)(fe >> 6);
            sh.gtl[sy] = (u32)(fe & 63u) | (tot ? 0x80000000u : 0u);
            sh.wstart[sy] = ws;
            if (tid == S - 1u) {
                sh.wstart[S] = ws + nW;
                if (PERM) lbase[S] = es + tot;
            }
            for (u32 k = (ws + 7u) & ~7u; k < ws + nW; k += 8u) sh.cidx[k >> 3] = (u16)tid;
            if (PERM) lbase[sy] = es;
            u32 bitpos = ws * 64u + s0;
            static_assert(NWAVE % 4 == 0, "the waves are taken four at a time");
#pragma unroll
            for (int w0 = 0; w0 < NWAVE; w0 += 4) { // four counts are read together, then replaced
                u32 c4[4];
#pragma unroll
                for (int j = 0; j < 4; j++) c4[j] = sh.wst[(w0 + j) * srow + sy];
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    sh.wst[(w0 + j) * srow + sy] = bitpos;
                    bitpos += c4[j] * wB;
                    if (PERM) {
                        wel[(w0 + j) * srow + sy] = es;
                        es += c4[j];
                    }
                }
            }
        }
        __syncthreads();
        // sweep 2: the image of the tile's output words (all slots are zero again)
#pragma unroll
        for (u32 rb = 0; rb < 16u; rb += 8u) {
            u32 start[8];
#pragma unroll
            for (u32 q = 0; q < 8u; q++) start[q] = wrow[reg[rb + q] & 511u];
#pragma unroll
            for (u32 q = 0; q < 8u; q++) {
                const u32 r = rb + q;
                const u32 v = reg[r];
                const u32 dv = PERM ? (v >> 19) & 511u : v >> 23;
                const u32 within = (v >> 9) & 1023u; // (PERM)
                if ((!PERM || (v >> 31)) && dv) {
                    const u32 bo = start[q] + (PERM ? within * wB : (v >> 9) & 0x3FFFu);
                    const u32 word = bo >> 5, shf = bo & 31u;
                    atomicOr(&img[word], dv << shf);
                    if (shf + wB > 32u) atomicOr(&img[word + 1u], dv >> (32u - shf));
                }
                if (PERM && (v >> 31))
                    si[wel[wave * srow + (v & 511u)] + within] = (u16)(wave * 1024u + r * 64u + lane);
            }
        }
        // The next tile's words were asked for a while ago: waiting for them here is free, while at
        // the top of the loop it would also wait for the stores of the output phase below.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        // one thread per image word: complete words leave now, unless their line is still open
        const u32 n_img = sh.wstart[S];
        for (u32 k = tid; k < n_img; k += DBLOCK) {
            u32 g = sh.cidx[k >> 3];
            while (sh.wstart[g + 1u] <= k) g++;
            const u32 Wf = sh.gWf[g], We = sh.gWe[g];
            const u32 j = k - sh.wstart[g], Wg = Wf + j;
            if (Wg >= We) continue; // the run's last, partial word: taken over at the next tile
            unsigned long long val = slot[k];
            if (j == 0u) val |= sh.lw[g][Wf & (LINE - 1u)]; // bits of earlier tiles in this word
            const u32 fo = sh.fo[g], own = fo & 0x7fffffffu;
            const u32 L = Wg / LINE;
            if ((fo >> 31) && Wg + 1u == own) { // shared with the run before this chunk's
                if (val) __hip_atomic_fetch_or(out + Wg, val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else if (L * LINE >= own && L == We / LINE) {
                // a line of this chunk's own that is not complete yet: it waits in LDS
            } else {
                out[Wg] = val;
            }
        }
        for (u32 k = tid; k < NWAVE * srow; k += DBLOCK) sh.wst[k] = 0u; // for the next tile's counts
        if (PERM) {
            for (u32 g = wave; g < S; g += NWAVE) {
                const u32 c = lbase[g + 1u] - lbase[g];
                const u32 p0 = sh.gb[g] - c;
                for (u32 i = lane; i < c; i += 64u)
                    gptr(d.perm)[p0 + i] = (u32)(e0 + si[lbase[g] + i]);
            }
        }
    }
    __syncthreads();
    for (u32 i = tid; i < S * LINE; i += DBLOCK) flush_and_commit(sh, slot, out, i);
    __syncthreads();
    if (tid < S) { // what the chunk leaves behind: the words of an open line, the last partial word
        const RunWords r = run_words(sh.gb[tid], 0u, wB);
        const u32 Le = r.We / LINE, wl = r.We & (LINE - 1u);
        if (Le * LINE >= (sh.fo[tid] & 0x7fffffffu))
            for (u32 j = 0; j < wl; j++) out[Le * LINE + j] = sh.lw[tid][j];
        const unsigned long long part = sh.lw[tid][wl];
        if (r.tail && part)
            __hip_atomic_fetch_or(out + r.We, part, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (ORDERED && order_bad) atomicOr(flags, DF_ORDER);
}

// regrouping given: e[r] = d[perm[r]] by gathering
// A given permutation is checked as it is used: an index outside the tensor is skipped and raises
// DF_PERM; symbols are clamped like those of the scatter, so a delta always fits its field.
__global__ __launch_bounds__(BLOCK) void k_dgather(const DDesc *__restrict__ dd,
                                                   const u32 *__restrict__ chunk_tensor,
                                                   u32 *__restrict__ flags)
{
    __shared__ unsigned long long pk[256 * 9];
    const u64 chunk = blockIdx.x;
    const DDesc d = dd[__builtin_amdgcn_readfirstlane(chunk_tensor[chunk])];
    if (!d.prev_perm) return;
    const u32 tid = threadIdx.x;
    const u32 wB = d.wB, Bm = d.B;
    const u32 smax[2] = {d.Kp + 1u, Bm - 1u}; // largest symbol of either stream that is taken as it is
    bool bad_index = false;
    const u64 c0 = (chunk - d.chunk0) * CHUNK_ELEMS;
    const u64 c1 = (c0 + CHUNK_ELEMS < d.n) ? c0 + CHUNK_ELEMS : d.n;
    for (u64 r0 = c0; r0 < c1; r0 += HTILE) {
        const u32 cnt = (c1 - r0 < (u64)HTILE) ? (u32)(c1 - r0) : (u32)HTILE;
        __syncthreads();
        for (u32 k = tid; k < 256u * wB; k += BLOCK) pk[k] = 0ull;
        __syncthreads();
        for (u32 j = 0; j < 16u; j++) {
            const u32 l = tid + j * BLOCK;
            if (l >= cnt) break;
            const u64 i = gptr(d.prev_perm)[r0 + l];
            if (i >= d.n) { // not a permutation of this tensor
                bad_index = true;
                continue;
            }
            u32 sym[2];
            for (int which = 0; which < 2; which++) {
                const GLOBAL_AS unsigned long long *src = which ? gptr(d.cur) : gptr(d.prev);
                const u32 w = which ? d.wc : d.wp;
                const u64 off = i * w;
                const u64 wd = off >> 6;
                const u32 sh = (u32)(off & 63u);
                unsigned long long x = src[wd] >> sh;
                if (sh + w > 64u) x |= src[wd + 1] << (64u - sh);
                sym[which] = (u32)x & ((1u << w) - 1u);
                sym[which] = sym[which] < smax[which] ? sym[which] : smax[which];
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
        GLOBAL_AS unsigned long long *dst = gptr(d.out) + r0 * wB / 64u;
        for (u32 k = tid; k < n_words; k += BLOCK) dst[k] = pk[k];
    }
    if (bad_index) atomicOr(flags, DF_PERM);
}

// clears the stream words that k_dscatter ORs into: the first word of every (chunk, group) run,
// which is also where the run before it ends, and the word where the stream ends
__global__ __launch_bounds__(SS) void k_dzero(const DDesc *__restrict__ dd,
                                              const u32 *__restrict__ chunk_tensor,
                                              const u32 *__restrict__ chunk_tot)
{
    const u64 chunk = blockIdx.x;
    const DDesc d = dd[__builtin_amdgcn_readfirstlane(chunk_tensor[chunk])];
    if (d.prev_perm) return;
    const u32 g = threadIdx.x, S = d.Kp + 2u;
    u64 pos;
    if (g < S)
        pos = gptr(d.group_off)[g] + chunk_tot[chunk * SS + g];
    else if (g == S && chunk == d.chunk0)
        pos = d.n;
    else
        return;
    const u64 word = (pos * d.wB) >> 6;
    if (word < d.out_words) gptr(d.out)[word] = 0ull;
}

// Restore side (Algorithm 6): s_cur[i] = (s_prev[i] - e[r]) mod B, where r is the position of element
// i in the stable order of s_prev.  Same chunk and tile walk as k_dscatter, with the data flowing the
// other way: sweep 1 ranks the elements of a tile; the stream words of every group's run of the tile
// are copied into an LDS image (one thread per word, consecutive words of a run by consecutive
// threads); sweep 2 takes every element's delta from the image and ORs the current symbol into an
// LDS image of the tile's packed words, which is stored whole.
struct RestoreShared {
    u32 wst[WST];       // counts, then bit position in the stream image of (wave, symbol)
    u32 wstart[SS + 8]; // first image word of each group's run; [S] = words in use
    u32 gWf[SS];        // stream word of the first bit of each group's run of this tile
    u32 gb[SS];         // stream position after each group's runs so far
    u32 wtot[8];
    unsigned long long hotkey;
    u16 cidx[CIDX];
};

template <bool ORDERED>
__global__ __launch_bounds__(DBLOCK, 6) void k_drestore(const DDesc *__restrict__ dd,
                                                        const XDesc *__restrict__ xd,
                                                        const u32 *__restrict__ chunk_tensor,
                                                        const u32 *__restrict__ chunk_tot,
                                                        u32 *__restrict__ flags)
{
    __shared__ RestoreShared sh;
    __shared__ __attribute__((aligned(16))) u32 Pw[DTILE * 9 / 32 + 8];
    __shared__ u32 Ci[DTILE * 9 / 32 + 8]; // image of the tile's current symbols
    // slots of sweep 1 (ballot ranking only); then the image of the tile's stream words
    __shared__ unsigned long long slot[NWAVE * SS];
    static_assert(NWAVE * SS >= BWORDS, "stream image fits the slot array");
    const u32 *img = (const u32 *)slot;
    const u64 chunk = blockIdx.x;
    const u32 t = __builtin_amdgcn_readfirstlane(chunk_tensor[chunk]);
    const DDesc d = dd[t];
    const XDesc x = xd[t];
    const u32 tid = threadIdx.x, lane = tid & 63u, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const u32 S = d.Kp + 2u, Bm = d.B, wB = d.wB, wp = d.wp, wc = d.wc;
    const u32 srow = S + 1u;
    const u64 n_tiles = (d.n + DTILE - 1) / DTILE;
    const u64 lt0 = (chunk - d.chunk0) * DCHUNK;
    const u64 lt1 = (lt0 + DCHUNK < n_tiles) ? lt0 + DCHUNK : n_tiles;
    if (tid < S) sh.gb[tid] = (u32)gptr(d.group_off)[tid] + chunk_tot[chunk * SS + tid];
    if (tid < SS + 8u) sh.wstart[tid] = 0xFFFFFFFFu;
    if (tid == 0u) sh.hotkey = 0ull;
    for (u32 k = tid; k < (u32)WST; k += DBLOCK) sh.wst[k] = 0u;
    __syncthreads();
    if (tid < S)
        atomicMax(&sh.hotkey, ((gptr(d.group_off)[tid + 1u] - gptr(d.group_off)[tid]) << 9) | tid);
    __syncthreads();
    const u32 hot = __builtin_amdgcn_readfirstlane((u32)sh.hotkey & 511u);
    u32 *wrow = sh.wst + wave * srow;
    const GLOBAL_AS unsigned long long *stream = gptr(d.out);
    const u32 mB = (1u << wB) - 1u;
    u32 bad = 0u, order_bad = 0u;
    auto tile_cnt = [&](u64 lt) -> u32 {
        const u64 rem = d.n - lt * (u64)DTILE;
        return rem < (u64)DTILE ? (u32)rem : (u32)DTILE;
    };
    lds_fetch<NWAVE>(gptr(d.prev), lt0 * (u64)DTILE, tile_cnt(lt0), wp, Pw, wave);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (ORDERED) {
        __syncthreads(); // all shares of the first tile's words are in LDS
        order_bad = ordered_rank_check(Pw, wrow, wave * 1024u + lane, tile_cnt(lt0), S, wp);
    }
    for (u64 lt = lt0; lt < lt1; lt++) {
        const u64 e0 = lt * (u64)DTILE;
        const u32 cnt = tile_cnt(lt);
        __syncthreads(); // the tile's previous symbols are in LDS; the previous tile has been stored
        if (!ORDERED) {
            for (u32 k = tid; k < (u32)(NWAVE * SS); k += DBLOCK) slot[k] = 0ull;
            __syncthreads();
        }
        u32 reg[16];
        u32 ebase = wave * 1024u + lane;
        asm volatile("" : "+v"(ebase)); // (the per-row LDS addresses are not kept across tiles)
        if (cnt == (u32)DTILE)
            rank_rows<true, ORDERED>(Pw, Pw, wrow, slot + wave * SS, ebase, cnt, S, Bm, wp, wp, hot, reg);
        else
            rank_rows<false, ORDERED>(Pw, Pw, wrow, slot + wave * SS, ebase, cnt, S, Bm, wp, wp, hot, reg);
        __syncthreads();
        {
            const u32 ndc = 2u * ((cnt * wc + 63u) >> 6) + 2u;
            u32 k0 = tid;
            asm volatile("" : "+v"(k0));
            for (u32 k = k0; k < ndc; k += DBLOCK) Ci[k] = 0u;
        }
        // counts -> positions, as in the scatter: the stream words each group's run touches,
        // exclusive scan over symbols, bit position of every (wave, symbol) in the image
        u32 tot = 0, nW = 0, s0 = 0, preW = 0;
        u64 fb = 0;
        u32 sy = tid;
        asm volatile("" : "+v"(sy));
        if (tid < 320u) { // waves 0..4 hold the 258 symbols
            if (tid < S) {
#pragma unroll
                for (int wv = 0; wv < NWAVE; wv++) tot += sh.wst[wv * srow + sy];
                fb = (u64)sh.gb[sy] * wB;
                s0 = (u32)(fb & 63u);
                nW = tot ? (s0 + tot * wB + 63u) >> 6 : 0u;
            }
            const u32 incW = wave_incl_scan(nW);
            preW = incW - nW;
            if (lane == 63u) sh.wtot[wave] = incW;
        }
        __syncthreads();
        // the next tile's previous symbols start travelling, asked for by the waves without a scan
        if (lt + 1 < lt1 && wave >= 5u)
            lds_fetch<NWAVE - 5>(gptr(d.prev), e0 + DTILE, tile_cnt(lt + 1), wp, Pw, wave - 5u);
        if (tid < S) {
            u32 ws = preW;
#pragma unroll
            for (u32 w2 = 0; w2 < 4u; w2++) ws += w2 < wave ? sh.wtot[w2] : 0u;
            sh.gb[sy] += tot;
            sh.gWf[sy] = (u32)(fb >> 6);
            sh.wstart[sy] = ws;
            if (tid == S - 1u) sh.wstart[S] = ws + nW;
            for (u32 k = (ws + 7u) & ~7u; k < ws + nW; k += 8u) sh.cidx[k >> 3] = (u16)tid;
            u32 bitpos = ws * 64u + s0;
#pragma unroll
            for (int w0 = 0; w0 < NWAVE; w0 += 4) { // four counts are read together, then replaced
                u32 c4[4];
#pragma unroll
                for (int j = 0; j < 4; j++) c4[j] = sh.wst[(w0 + j) * srow + sy];
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    sh.wst[(w0 + j) * srow + sy] = bitpos;
                    bitpos += c4[j] * wB;
                }
            }
        }
        __syncthreads();
        { // the stream words of the tile: image word k is stream word gWf[g] + k - wstart[g]
            const u32 n_img = sh.wstart[S];
            for (u32 k = tid; k < n_img; k += DBLOCK) {
                u32 g = sh.cidx[k >> 3];
                while (sh.wstart[g + 1u] <= k) g++;
                const u64 W = (u64)sh.gWf[g] + (k - sh.wstart[g]);
                slot[k] = W < d.out_words ? stream[W] : 0ull;
            }
            if (tid < 2u) slot[n_img + tid] = 0ull; // sweep 2 reads one dword past a run's last bit
        }
        __syncthreads();
#pragma unroll
        for (u32 r = 0; r < 16u; r++) {
            const u32 v = reg[r];
            if (!(v >> 31)) continue;
            const u32 sp = v & 511u, within = (v >> 9) & 1023u;
            const u32 bo = wrow[sp] + within * wB;
            const u32 e = __builtin_amdgcn_alignbit(img[(bo >> 5) + 1u], img[bo >> 5], bo & 31u) & mB;
            u32 sc = sp >= e ? sp - e : sp + Bm - e;
            if (e >= Bm || sc >= x.Sc) {
                bad = 1u;
                sc = 0u;
            }
            const u32 co = (ebase + 64u * r) * wc;
            const u32 word = co >> 5, shf = co & 31u;
            if (sc) {
                atomicOr(&Ci[word], sc << shf);
                if (shf + wc > 32u) atomicOr(&Ci[word + 1u], sc >> (32u - shf));
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // this wave's share of the next tile's words
        __syncthreads();
        {
            const u32 ndc = 2u * ((cnt * wc + 63u) >> 6);
            GLOBAL_AS u32 *dst = (GLOBAL_AS u32 *)(gptr(x.cur_out) + e0 * wc / 64u);
            for (u32 k = tid; k < ndc; k += DBLOCK) dst[k] = Ci[k];
            for (u32 k = tid; k < NWAVE * srow; k += DBLOCK) sh.wst[k] = 0u; // for the next tile's counts
        }
    }
    if (__ballot(bad != 0u) && lane == 0u) atomicOr(flags, RF_DELTA);
    if (ORDERED && order_bad) atomicOr(flags, RF_ORDER);
}

// group offsets that came with the stream against those of the previous symbols
__global__ __launch_bounds__(SS) void k_dcheck_groups(const DDesc *__restrict__ dd,
                                                      const XDesc *__restrict__ xd,
                                                      u32 *__restrict__ flags)
{
    const DDesc d = dd[blockIdx.x];
    const XDesc x = xd[blockIdx.x];
    const u32 g = threadIdx.x;
    if (x.group_off_in && g <= d.Kp + 2u && gptr(x.group_off_in)[g] != gptr(d.group_off)[g])
        atomicOr(flags, RF_GROUPS);
}

hipError_t launch_reconstruct(const DDesc *dd, const XDesc *xd, int nT, u64 n_chunks,
                              const u32 *chunk_tensor, u32 *chunk_tot, u32 *flags, bool lds_ordered,
                              hipStream_t s)
{
    PROF("k_dhist", s, k_dhist<<<(unsigned)n_chunks, BLOCK, 0, s>>>(dd, chunk_tensor, chunk_tot));
    PROF("k_dgroups", s, k_dgroups<<<nT, SS, 0, s>>>(dd, chunk_tot));
    PROF("k_dcheck_groups", s, k_dcheck_groups<<<nT, SS, 0, s>>>(dd, xd, flags));
    if (lds_ordered)
        PROF("k_drestore", s, k_drestore<true><<<(unsigned)n_chunks, DBLOCK, 0, s>>>(dd, xd, chunk_tensor, chunk_tot, flags));
    else
        PROF("k_drestore_slots", s, k_drestore<false><<<(unsigned)n_chunks, DBLOCK, 0, s>>>(dd, xd, chunk_tensor, chunk_tot, flags));
    return hipGetLastError();
}

// 1 if same-address LDS atomics with return are served in ascending lane order, for every pattern
// tried: all lanes on one address, few addresses, many addresses, with inactive lanes
__global__ __launch_bounds__(256) void k_lds_order_check(u32 *__restrict__ violations)
{
    __shared__ u32 cnt[4][SS];
    const u32 lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    for (u32 i = threadIdx.x; i < 4 * SS; i += 256) (&cnt[0][0])[i] = 0u;
    __syncthreads();
    u32 bad = 0;
    const u32 mods[6] = {1u, 2u, 5u, 18u, 66u, 258u};
    for (u32 t = 0; t < 600u; t++) {
        u32 x = lane * 7919u + t * 104729u + blockIdx.x * 31u + wave * 977u;
        x ^= x >> 16;
        x *= 0x7feb352du;
        x ^= x >> 15;
        x *= 0x846ca68bu;
        x ^= x >> 16;
        const u32 sym = x % mods[t % 6u];
        const bool active = ((x >> 20) & 7u) != 0u;
        const u32 before = cnt[wave][sym];
        u32 got = 0;
        if (active) got = atomicAdd(&cnt[wave][sym], 1u);
        u64 peers = __ballot(active);
        for (int b = 0; b < 9; b++) {
            const bool bit = (sym >> b) & 1u;
            const u64 m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        const u32 rank = __popcll(peers & ((1ull << lane) - 1ull));
        if (active && got != before + rank) bad++;
    }
    if (bad) atomicAdd(violations, bad);
}

hipError_t launch_lds_order_check(u32 *violations, hipStream_t s)
{
    k_lds_order_check<<<64, 256, 0, s>>>(violations);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// The delta without any allocation: descriptors, the chunk -> tensor table, the per-chunk symbol
// populations and the flag word live in one file-scope device array.  Every GPU holds its own copy
// at its own address; delta_static_init asks for it once per device, and host code uses that
// pointer only (the array's name is not a device address on the host side).
// ------------------------------------------------------------------------------------------
constexpr size_t DST_DD = 0;                                                   // DDesc[MAX_TENSORS]
constexpr size_t DST_FLAGS = DST_DD + sizeof(DDesc) * DELTA_STATIC_MAX_TENSORS; // u32 flag word
constexpr size_t DST_CT = (DST_FLAGS + 256) & ~(size_t)255;                    // u32[MAX_CHUNKS]
constexpr size_t DST_CK = DST_CT + sizeof(u32) * DELTA_STATIC_MAX_CHUNKS;      // u32[MAX_CHUNKS][SS]
constexpr size_t DST_BYTES = DST_CK + sizeof(u32) * (size_t)DELTA_STATIC_MAX_CHUNKS * DELTA_SS;
static __device__ __align__(256) unsigned char scratch[DST_BYTES];

constexpr int MAX_DEVICES = 64;
static unsigned char *g_scratch_ptr[MAX_DEVICES]; // per device: where its copy of `scratch` lies

hipError_t delta_static_init(int device)
{
    if (device < 0 || device >= MAX_DEVICES) return hipErrorInvalidDevice;
    if (g_scratch_ptr[device]) return hipSuccess;
    void *p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)); // (the current device's copy)
    if (e != hipSuccess) return e;
    g_scratch_ptr[device] = (unsigned char *)p;
    return hipSuccess;
}

u32 *delta_static_flags(int device)
{
    if (device < 0 || device >= MAX_DEVICES || !g_scratch_ptr[device]) return nullptr;
    return (u32 *)(g_scratch_ptr[device] + DST_FLAGS);
}

// descriptors from the kernel arguments into the scratch array; tensor of every chunk; flags cleared
__global__ __launch_bounds__(256) void k_dstatic_setup(DeltaStaticArgs a, DDesc *__restrict__ dd,
                                                       u32 *__restrict__ chunk_tensor,
                                                       u32 *__restrict__ flags)
{
    const u32 tid = threadIdx.x;
    if (tid < a.n_tensors) dd[tid] = a.dd[tid];
    if (tid == 0u) *flags = 0u;
    for (u32 t = 0; t < a.n_tensors; t++) {
        const u64 c0 = a.dd[t].chunk0, c1 = c0 + a.dd[t].n_chunks;
        for (u64 c = c0 + tid; c < c1; c += 256u) chunk_tensor[c] = t;
    }
}

hipError_t launch_delta_static(int device, const DeltaStaticArgs &a, u64 n_dtiles, u64 n_chunks,
                               bool any_scatter, bool any_perm, bool lds_ordered, hipStream_t s)
{
    if (device < 0 || device >= MAX_DEVICES || !g_scratch_ptr[device]) return hipErrorNotInitialized;
    if (a.n_tensors > (u32)DELTA_STATIC_MAX_TENSORS || n_chunks > (u64)DELTA_STATIC_MAX_CHUNKS)
        return hipErrorInvalidValue;
    unsigned char *base = g_scratch_ptr[device];
    DDesc *dd = (DDesc *)(base + DST_DD);
    u32 *flags = (u32 *)(base + DST_FLAGS);
    u32 *chunk_tensor = (u32 *)(base + DST_CT);
    u32 *chunk_tot = (u32 *)(base + DST_CK); // every entry of the chunks in use is written by k_dhist
    PROF("k_dstatic_setup", s, k_dstatic_setup<<<1, 256, 0, s>>>(a, dd, chunk_tensor, flags));
    return launch_delta(dd, (int)a.n_tensors, n_dtiles, n_chunks, chunk_tensor, chunk_tot, flags,
                        any_scatter, any_perm, false, lds_ordered, s);
}

hipError_t launch_delta(const DDesc *dd, int nT, u64 n_dtiles, u64 n_chunks,
                        const u32 *chunk_tensor, u32 *chunk_tot, u32 *flags, bool any_scatter,
                        bool any_perm, bool any_gather, bool lds_ordered, hipStream_t s)
{
    PROF("k_dhist", s, k_dhist<<<(unsigned)n_chunks, BLOCK, 0, s>>>(dd, chunk_tensor, chunk_tot));
    PROF("k_dgroups", s, k_dgroups<<<nT, SS, 0, s>>>(dd, chunk_tot));
    if (any_scatter || any_perm)
        PROF("k_dzero", s, k_dzero<<<(unsigned)n_chunks, SS, 0, s>>>(dd, chunk_tensor, chunk_tot));
    if (any_scatter) {
        if (lds_ordered)
            PROF("k_dscatter", s, k_dscatter<false, true><<<(unsigned)n_chunks, DBLOCK, 0, s>>>(dd, chunk_tensor, chunk_tot, flags));
        else
            PROF("k_dscatter_slots", s, k_dscatter<false, false><<<(unsigned)n_chunks, DBLOCK, 0, s>>>(dd, chunk_tensor, chunk_tot, flags));
    }
    if (any_perm) {
        if (lds_ordered)
            PROF("k_dscatter_perm", s, k_dscatter<true, true><<<(unsigned)n_chunks, DBLOCK, 0, s>>>(dd, chunk_tensor, chunk_tot, flags));
        else
            PROF("k_dscatter_perm_slots", s, k_dscatter<true, false><<<(unsigned)n_chunks, DBLOCK, 0, s>>>(dd, chunk_tensor, chunk_tot, flags));
    }
    if (any_gather) PROF("k_dgather", s, k_dgather<<<(unsigned)n_chunks, BLOCK, 0, s>>>(dd, chunk_tensor, flags));
    return hipGetLastError();
}

} // namespace inshr
