// Host side of the C ABI (include/inshr.h): argument checks, work partition, scratch memory and
// kernel sequencing.  No arithmetic of the method runs here.
#include "../../include/inshr.h"
#include "inshr_launch.h"
#include "inshr_sketch.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <string>
#include <unordered_map>
#include <vector>

using namespace inshr;

namespace {

struct DevBuf { // grow-only device allocation
    void *p = nullptr;
    size_t cap = 0;
};

struct HostBuf { // grow-only pinned host allocation
    void *p = nullptr;
    size_t cap = 0;
};

} // namespace

struct inshr_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    uint64_t scratch_limit = 0;
    int n_cu = 256;
    int wg_per_cu = 2;
    bool lds_ordered = false; // same-address LDS atomics return in lane order (checked at creation)
    // tensors of at least this many elements get a sampled first sweep (INSHR_SAMPLE_MIN_N; 0 = never)
    uint64_t sample_min_n = 16ull << 20;
    bool sample_force_miss = false; // INSHR_SAMPLE_FORCE_MISS=1 (tests): always take the exact sweeps again
    // keys a wave may gather per tile of its 1024 elements, on average over its tiles (of 1024): the
    // gather pools are sized by it; a search that finds them too small doubles it and runs again
    // (INSHR_POOL_WCAP sets the start)
    uint32_t pool_wcap = 136;
    std::vector<char> batch_sampled;
    std::string last_err;

    u32 *delta_flags = nullptr; // flag word of the delta kernels (DF_*), allocated with the context
    bool delta_pending = false; // an asynchronous delta call has not had its flags read yet
    bool static_pending = false; // the same for inshr_delta_static (its flag word is in its own scratch)
    DevBuf search_mem; // everything a search leaves behind for inshr_quantize
    DevBuf aux_mem;    // quantize descriptors, delta scratch
    DevBuf sketch_mem; // sketch tables, histograms, bucket lists and the centres they give
    DevBuf sens_mem;   // scores, compacted values and block counts of inshr_quantize_sens
    double sketch_alpha = 0.0;                 // the bucket tables last built, and for which alpha
    int sketch_i_lo = 0;
    std::vector<u32> sketch_cell, sketch_tops;
    std::vector<double> sketch_rep;
    HostBuf h_up;      // staging for descriptor uploads
    HostBuf h_down;    // staging for result downloads

    // state of the last search
    bool have_search = false;
    Batch batch{};
    GridDesc grid{};
    std::vector<inshr_config> grid_cfgs;
    std::vector<inshr_tensor> tensors;
    size_t ts_off = 0, scores_off = 0;
};

// ------------------------------------------------------------------------------------------
// optional per-kernel timing (HIP events on the launch stream)
// ------------------------------------------------------------------------------------------
namespace {
struct ProfState {
    bool on = false;
    std::vector<hipEvent_t> pool;       // event pairs, reused
    std::vector<const char *> pending;  // name of each recorded pair
    std::vector<std::string> names;
    std::vector<double> total_ms;
    std::vector<uint64_t> launches;
} g_prof;
} // namespace

namespace inshr {
void prof_begin(const char *name, hipStream_t s)
{
    if (!g_prof.on) return;
    const size_t k = g_prof.pending.size();
    while (g_prof.pool.size() < 2 * (k + 1)) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return;
        g_prof.pool.push_back(e);
    }
    g_prof.pending.push_back(name);
    (void)hipEventRecord(g_prof.pool[2 * k], s);
}
void prof_end(hipStream_t s)
{
    if (!g_prof.on || g_prof.pending.empty()) return;
    const size_t k = g_prof.pending.size() - 1;
    (void)hipEventRecord(g_prof.pool[2 * k + 1], s);
}
} // namespace inshr

namespace {

void prof_collect()
{
    for (size_t k = 0; k < g_prof.pending.size(); k++) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_prof.pool[2 * k], g_prof.pool[2 * k + 1]) != hipSuccess) continue;
        size_t i = 0;
        for (; i < g_prof.names.size(); i++)
            if (g_prof.names[i] == g_prof.pending[k]) break;
        if (i == g_prof.names.size()) {
            g_prof.names.push_back(g_prof.pending[k]);
            g_prof.total_ms.push_back(0.0);
            g_prof.launches.push_back(0);
        }
        g_prof.total_ms[i] += ms;
        g_prof.launches[i]++;
    }
    g_prof.pending.clear();
}

#define HIPCHK(ctx, call)                                                                         \
    do {                                                                                          \
        hipError_t e__ = (call);                                                                  \
        if (e__ != hipSuccess) {                                                                  \
            (ctx)->last_err = std::string(#call) + ": " + hipGetErrorString(e__);                 \
            return INSHR_E_DEVICE;                                                                \
        }                                                                                         \
    } while (0)

int ensure_dev(inshr_ctx *c, DevBuf &b, size_t bytes)
{
    if (bytes <= b.cap) return INSHR_OK;
    if (c->scratch_limit && bytes > c->scratch_limit) return INSHR_E_CAPACITY;
    if (b.p) HIPCHK(c, hipFree(b.p));
    b.p = nullptr;
    b.cap = 0;
    hipError_t e = hipMalloc(&b.p, bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        c->last_err = std::string("hipMalloc of scratch: ") + hipGetErrorString(e);
        b.p = nullptr;
        return INSHR_E_CAPACITY;
    }
    b.cap = bytes;
    return INSHR_OK;
}

// After the stream has been synchronised: the flags that the kernels of the last inshr_delta raised.
int take_delta_flags(inshr_ctx *c)
{
    if (!c->delta_pending && !c->static_pending) return INSHR_OK;
    u32 f = 0, g = 0;
    if (c->delta_pending) HIPCHK(c, hipMemcpy(&f, c->delta_flags, sizeof(u32), hipMemcpyDeviceToHost));
    if (c->static_pending)
        HIPCHK(c, hipMemcpy(&g, delta_static_flags(c->device), sizeof(u32), hipMemcpyDeviceToHost));
    c->delta_pending = c->static_pending = false;
    f |= g;
    if (f & DF_ORDER) {
        c->last_err = "delta: ranks from returning LDS atomics disagree with ballot ranks (set INSHR_NO_LDS_ORDER=1)";
        return INSHR_E_INTERNAL;
    }
    if (f & DF_PERM) return INSHR_E_ARG;
    return INSHR_OK;
}

int ensure_host(inshr_ctx *c, HostBuf &b, size_t bytes)
{
    if (bytes <= b.cap) return INSHR_OK;
    if (b.p) HIPCHK(c, hipHostFree(b.p));
    b.p = nullptr;
    b.cap = 0;
    HIPCHK(c, hipHostMalloc(&b.p, bytes, hipHostMallocDefault));
    b.cap = bytes;
    return INSHR_OK;
}

struct Carver { // lays sub-buffers out in one allocation, 256-byte aligned
    size_t off = 0;
    size_t take(size_t bytes)
    {
        size_t o = off;
        off = (off + bytes + 255) & ~(size_t)255;
        return o;
    }
};

uint32_t bins_of(const inshr_config &c) { return c.bins ? c.bins : (1u << c.bits); }
bool same_config(const inshr_config &a, const inshr_config &b)
{
    return bins_of(a) == bins_of(b) && a.prune_ppm == b.prune_ppm && a.outlier_ppm == b.outlier_ppm;
}

int check_config(const inshr_config &c)
{
    if (c.bins) {
        if (!bins_supported(c.bins)) return INSHR_E_CONFIG;
    } else if (c.bits < 1 || c.bits > 8) {
        return INSHR_E_CONFIG;
    }
    if ((uint64_t)c.prune_ppm + (uint64_t)c.outlier_ppm >= 1000000ull) return INSHR_E_CONFIG;
    return INSHR_OK;
}

int build_grid(const inshr_config *grid, uint32_t n_cfg, double eps, GridDesc &g)
{
    if (n_cfg == 0 || n_cfg > (uint32_t)MAX_CFG) return INSHR_E_CONFIG;
    memset(&g, 0, sizeof(g));
    g.n_cfg = n_cfg;
    g.eps = eps;
    g.n_bnd = NB8;
    for (uint32_t i = 0; i < n_cfg; i++) {
        int rc = check_config(grid[i]);
        if (rc) return rc;
        uint32_t ip = 0, io = 0;
        for (ip = 0; ip < g.n_p; ip++)
            if (g.p_ppm[ip] == grid[i].prune_ppm) break;
        if (ip == g.n_p) {
            if (g.n_p == (uint32_t)MAX_FRAC) return INSHR_E_CONFIG;
            g.p_ppm[g.n_p++] = grid[i].prune_ppm;
        }
        for (io = 0; io < g.n_o; io++)
            if (g.o_ppm[io] == grid[i].outlier_ppm) break;
        if (io == g.n_o) {
            if (g.n_o == (uint32_t)MAX_FRAC) return INSHR_E_CONFIG;
            g.o_ppm[g.n_o++] = grid[i].outlier_ppm;
        }
        uint32_t q = 0;
        for (q = 0; q < g.n_pairs; q++)
            if (g.pair_p[q] == ip && g.pair_o[q] == io) break;
        if (q == g.n_pairs) {
            if (g.n_pairs == (uint32_t)MAX_PAIRS) return INSHR_E_CONFIG;
            g.pair_p[q] = ip;
            g.pair_o[q] = io;
            g.n_pairs++;
        }
        g.cfg_pair[i] = q;
        const uint32_t K = bins_of(grid[i]);
        g.cfg_K[i] = K;
        g.cfg_bits[i] = symbol_bits(K) - 1u;
        g.cfg_l16[i] = (uint32_t)std::floor(std::log2((double)K) * 65536.0 + 0.5);
        if (K & (K - 1u)) g.n_bnd = NBT; // 3, 6 or 12 bins: the twelfths are boundaries too
    }
    return INSHR_OK;
}

// light: thresholds, class counts and the second-level table only (for the sketch quantizer, which
// brings its own bins and takes the protected counts per tile in its own sweep); the state is then
// not offered to INSHR_REUSE_SEARCH.
// group: NULL, or one number per tensor; tensors with equal numbers share their thresholds, which
// are then order statistics of the group's pooled magnitudes (Sec. 4.2, per-layer-type pruning).
int run_search(inshr_ctx *c, const inshr_tensor *tensors, uint32_t nT, const inshr_config *grid,
               uint32_t n_cfg, double eps, bool light = false, const uint32_t *group = nullptr)
{
    c->have_search = false;
    if (!tensors || !grid || nT == 0) return INSHR_E_ARG;
    // leader of every tensor's group and the group's size
    std::vector<u32> leader(nT);
    std::vector<u64> n_pool(nT, 0);
    std::vector<u32> members(nT, 0);
    bool any_pooled = false;
    {
        std::unordered_map<uint32_t, u32> first;
        for (uint32_t t = 0; t < nT; t++) {
            leader[t] = group ? first.emplace(group[t], t).first->second : t;
            n_pool[leader[t]] += tensors[t].n;
            members[leader[t]]++;
        }
        for (uint32_t t = 0; t < nT; t++) {
            if (members[leader[t]] > 1) any_pooled = true;
            if (n_pool[leader[t]] >= (1ull << 32)) {
                c->last_err = "a group of tensors that share thresholds holds 2^32 values or more";
                return INSHR_E_ARG;
            }
        }
    }
    GridDesc g;
    int rc = build_grid(grid, n_cfg, eps, g);
    if (rc) return rc;
    uint64_t total_tiles = 0;
    for (uint32_t t = 0; t < nT; t++) {
        if (!tensors[t].data || tensors[t].n == 0 || tensors[t].n >= (1ull << 32)) return INSHR_E_ARG;
        if ((uintptr_t)tensors[t].data & 3u) return INSHR_E_ARG;
        total_tiles += (tensors[t].n + TILE - 1) / TILE;
    }
    HIPCHK(c, hipSetDevice(c->device));
    HIPCHK(c, hipStreamSynchronize(c->stream)); // staging buffers may be in flight (inshr_delta)

    // work partition: tiles are dealt out evenly to workgroups in order
    const int n_wg = (int)std::min<uint64_t>(total_tiles, (uint64_t)c->n_cu * c->wg_per_cu);
    std::vector<TDesc> td(nT);
    std::vector<u64> wg_tile0(n_wg + 1);
    std::vector<u32> wg_fu0(n_wg);
    std::vector<std::vector<u32>> t_units(nT);
    {
        u64 tile = 0, pool = 0;
        bool any_sampled = false;
        for (uint32_t t = 0; t < nT; t++) {
            td[t].data = tensors[t].data;
            td[t].n = tensors[t].n;
            td[t].tile0 = tile;
            const u64 padded = (tensors[t].n + TILE - 1) / TILE * TILE;
            td[t].aligned16 = (((uintptr_t)tensors[t].data & 15u) == 0) ? 1u : 0u;
            td[t].leader = leader[t];
            td[t].pooled = members[leader[t]] > 1 ? 1u : 0u;
            td[t].n_pool = n_pool[leader[t]];
            // (a sampled first sweep predicts where a tensor's own order statistics lie; a group's
            // come from the exact histograms of all its tensors)
            td[t].sampled = (!td[t].pooled && c->sample_min_n && tensors[t].n >= c->sample_min_n &&
                             tensors[t].n < (1ull << 31)) ? 1u : 0u;
            any_sampled = any_sampled || td[t].sampled;
            c->batch_sampled.resize(nT);
            c->batch_sampled[t] = (char)td[t].sampled;
            tile += padded / TILE;
        }
        for (int w = 0; w <= n_wg; w++) wg_tile0[w] = total_tiles * (u64)w / (u64)n_wg;
        // Gather pools: every wave of a (workgroup, tensor) unit owns a share of each pool, sized for
        // pool_wcap keys per tile of the unit plus one full tile (the sweeps stop gathering when the
        // share cannot take a whole tile any more), and never more than the wave's elements.
        std::vector<u64> unit_off;
        std::vector<u32> unit_capw;
        u32 units = 0;
        uint32_t t = 0;
        for (int w = 0; w < n_wg; w++) {
            wg_fu0[w] = units;
            const u64 lo = wg_tile0[w], hi = wg_tile0[w + 1];
            if (lo >= hi) continue;
            while (t + 1 < nT && td[t + 1].tile0 <= lo) t++;
            uint32_t tt = t;
            while (true) {
                t_units[tt].push_back(units++);
                const u64 t_end = (tt + 1 < nT) ? td[tt + 1].tile0 : total_tiles;
                const u64 u_lo = std::max(lo, td[tt].tile0), u_hi = std::min(hi, t_end);
                const u64 tiles_u = u_hi - u_lo;
                const u64 per_wave = TILE / (BLOCK / 64);
                const u64 capw = std::min(tiles_u * per_wave, tiles_u * (u64)c->pool_wcap + per_wave);
                if (t_units[tt].size() == 1) {
                    td[tt].pool_grp = pool;
                    td[tt].pool_len = 0;
                }
                unit_off.push_back(pool);
                unit_capw.push_back((u32)capw);
                td[tt].pool_len += capw * (BLOCK / 64);
                pool += capw * (BLOCK / 64);
                if (t_end >= hi) break;
                tt++;
            }
        }
        // device layout
        Carver cv;
        const size_t o_td = cv.take(sizeof(TDesc) * nT);
        const size_t o_gd = cv.take(sizeof(GridDesc));
        const size_t o_wt = cv.take(sizeof(u64) * (n_wg + 1));
        const size_t o_wf = cv.take(sizeof(u32) * n_wg);
        const size_t o_tfo = cv.take(sizeof(u32) * (nT + 1));
        const size_t o_tfi = cv.take(sizeof(u32) * units);
        const size_t o_fut = cv.take(sizeof(u32) * units);
        const size_t o_us = cv.take((size_t)units * 8);
        const size_t o_usb = cv.take((size_t)units * 4);
        const size_t up_bytes = cv.off;
        const size_t o_ts = cv.take(sizeof(TState) * nT);
        const size_t o_h1 = cv.take((size_t)nT * L1_BINS * 4);
        const size_t o_h2 = cv.take((size_t)nT * L2_BINS * 4);
        const size_t o_ngt = cv.take(256);
        const size_t o_gcn = cv.take((size_t)nT * 2 * MAX_EDGES * 4);
        const size_t o_gsx = cv.take((size_t)nT * 2 * MAX_EDGES * 8);
        const size_t o_to = cv.take((size_t)total_tiles * MAX_FRAC * 4);
        const size_t o_ph1 = cv.take(any_pooled ? (size_t)nT * L1_BINS * 4 : 0);
        const size_t zero_end = cv.off; // [o_ts, zero_end) is cleared before the sweeps
        const size_t o_psel = cv.take(any_pooled ? (size_t)nT * 2 * SEL_WORDS * 4 : 0);
        const size_t o_tab = cv.take((size_t)nT * COARSE * 4);
        const size_t o_ut = cv.take((size_t)units * 16 * 4);
        const size_t o_bi = cv.take((size_t)nT * L2_BINS * 4);
        const size_t o_cur = cv.take((size_t)nT * CURSOR_STRIDE * 4);
        const size_t o_tb = cv.take((size_t)nT * TGT_STRIDE * 4);
        const size_t o_tr = cv.take((size_t)nT * TGT_STRIDE * 4);
        const size_t o_tk = cv.take((size_t)nT * TGT_STRIDE * 4);
        const size_t o_tf = cv.take((size_t)total_tiles * 4);
        const size_t o_sq = cv.take((size_t)units * SQ_STRIDE * 8);
        const size_t o_ed = cv.take((size_t)nT * MAX_EDGES * 4);
        const size_t o_sl = cv.take((size_t)nT * (L2_BINS + 64) * 2);
        const size_t o_pe = cv.take((size_t)nT * MAX_PAIRS * EIDX_STRIDE * 2);
        const size_t o_eb = cv.take((size_t)nT * MAX_EDGES * 4);
        const size_t o_ei = cv.take((size_t)nT * MAX_EDGES * 2);
        const size_t o_gel = cv.take((size_t)nT * MAX_GROUPS * 4);
        const size_t o_geh = cv.take((size_t)nT * MAX_GROUPS * 4);
        const size_t o_sgc = cv.take((size_t)nT * MAX_EDGES * 4);
        const size_t o_ms = cv.take((size_t)units * MAX_SUB * 8);
        const size_t o_sbc = cv.take((size_t)nT * MAX_SUB * 4);
        const size_t o_sbn = cv.take((size_t)nT * MAX_SUB * 4);
        const size_t o_cb = cv.take((size_t)nT * n_cfg * CB_STRIDE * 4);
        const size_t o_sc = cv.take((size_t)nT * n_cfg * sizeof(Score));
        const size_t o_bt = cv.take((size_t)nT * n_cfg * CB_STRIDE * 8);
        const size_t o_uc = cv.take((size_t)units * 16 * 4);
        const size_t o_bg = cv.take((size_t)nT * L2_BINS * 2);
        const size_t o_go = cv.take((size_t)nT * MAX_GROUPS * 4);
        const size_t o_ge = cv.take((size_t)nT * MAX_GROUPS * 4);
        const size_t o_gc = cv.take((size_t)nT * MAX_GROUPS * 4);
        const size_t o_tgg = cv.take((size_t)nT * TGT_STRIDE * 4);
        const size_t o_tkl = cv.take((size_t)nT * TGT_STRIDE * 4);
        const size_t o_tkh = cv.take((size_t)nT * TGT_STRIDE * 4);
        const size_t o_gl = cv.take((size_t)nT * MAX_GROUPS * 4);
        const size_t o_pool = cv.take((size_t)pool * 4);
        const size_t o_pool2 = cv.take((size_t)pool * 4);
        rc = ensure_dev(c, c->search_mem, cv.off);
        if (rc) return rc;
        rc = ensure_host(c, c->h_up, up_bytes);
        if (rc) return rc;
        char *hb = (char *)c->h_up.p;
        char *db = (char *)c->search_mem.p;
        memcpy(hb + o_td, td.data(), sizeof(TDesc) * nT);
        memcpy(hb + o_gd, &g, sizeof(GridDesc));
        memcpy(hb + o_wt, wg_tile0.data(), sizeof(u64) * (n_wg + 1));
        memcpy(hb + o_wf, wg_fu0.data(), sizeof(u32) * n_wg);
        {
            u32 *tfo = (u32 *)(hb + o_tfo), *tfi = (u32 *)(hb + o_tfi);
            u32 k = 0;
            for (uint32_t tt = 0; tt < nT; tt++) {
                tfo[tt] = k;
                for (u32 u : t_units[tt]) tfi[k++] = u;
            }
            tfo[nT] = k;
            u32 *fut = (u32 *)(hb + o_fut);
            for (uint32_t tt = 0; tt < nT; tt++)
                for (u32 u : t_units[tt]) fut[u] = tt;
            memcpy(hb + o_us, unit_off.data(), sizeof(u64) * units);
            memcpy(hb + o_usb, unit_capw.data(), sizeof(u32) * units);
        }
        HIPCHK(c, hipMemcpyAsync(db, hb, up_bytes, hipMemcpyHostToDevice, c->stream));
        HIPCHK(c, hipMemsetAsync(db + o_ts, 0, zero_end - o_ts, c->stream));

        Batch &bt = c->batch;
        bt.td = (const TDesc *)(db + o_td);
        bt.gd = (const GridDesc *)(db + o_gd);
        bt.wg_tile0 = (const u64 *)(db + o_wt);
        bt.wg_fu0 = (const u32 *)(db + o_wf);
        bt.t_fu_off = (const u32 *)(db + o_tfo);
        bt.t_fu_ids = (const u32 *)(db + o_tfi);
        bt.fu_tensor = (const u32 *)(db + o_fut);
        bt.grp_list = (u32 *)(db + o_gl);
        bt.n_grp_total = (u32 *)(db + o_ngt);
        bt.n_units = (int)units;
        bt.n_bucket_blocks = c->n_cu * 4;
        bt.lds_ordered = c->lds_ordered;
        bt.any_sampled = any_sampled;
        bt.any_pooled = any_pooled;
        bt.force_miss = c->sample_force_miss;
        bt.nT = (int)nT;
        bt.n_wg = n_wg;
        bt.n_pairs = g.n_pairs;
        bt.n_cfg = n_cfg;
        bt.n_tiles = total_tiles;
        Bufs &B = bt.bufs;
        B.ts = (TState *)(db + o_ts);
        B.hist1 = (u32 *)(db + o_h1);
        B.pool_h1 = (u32 *)(db + o_ph1);
        B.pool_sel = (u32 *)(db + o_psel);
        B.hist2 = (u32 *)(db + o_h2);
        B.table2 = (u32 *)(db + o_tab);
        B.unit_off = (const u64 *)(db + o_us);
        B.unit_thr = (u32 *)(db + o_ut);
        B.unit_capw = (const u32 *)(db + o_usb);
        B.binfo = (u32 *)(db + o_bi);
        B.cursor2 = (u32 *)(db + o_cur);
        B.tgt_bin = (u32 *)(db + o_tb);
        B.tgt_res = (u32 *)(db + o_tr);
        B.tgt_key = (u32 *)(db + o_tk);
        B.pool = (u32 *)(db + o_pool);
        B.pool2 = (u32 *)(db + o_pool2);
        B.unit_cand = (u32 *)(db + o_uc);
        B.bin_group = (u16 *)(db + o_bg);
        B.grp_off = (u32 *)(db + o_go);
        B.grp_end = (u32 *)(db + o_ge);
        B.grp_cur = (u32 *)(db + o_gc);
        B.tgt_rank = (u32 *)(db + o_tgg);
        B.tgt_klo = (u32 *)(db + o_tkl);
        B.tgt_khi = (u32 *)(db + o_tkh);
        B.tile_out = (u32 *)(db + o_to);
        B.tile_off = (u32 *)(db + o_tf);
        B.sq_part = (double *)(db + o_sq);
        B.edges = (u32 *)(db + o_ed);
        B.sl = (u16 *)(db + o_sl);
        B.pair_eidx = (u16 *)(db + o_pe);
        B.edge_bin = (u32 *)(db + o_eb);
        B.edge_item = (u16 *)(db + o_ei);
        B.grp_elo = (u32 *)(db + o_gel);
        B.grp_ehi = (u32 *)(db + o_geh);
        B.seg_cnt = (u32 *)(db + o_sgc);
        B.grp_cnt = (u32 *)(db + o_gcn);
        B.grp_sx = (double *)(db + o_gsx);
        B.mom_sx = (u64 *)(db + o_ms);
        B.sub_code = (u32 *)(db + o_sbc);
        B.sub_cnt = (u32 *)(db + o_sbn);
        B.codebook = (float *)(db + o_cb);
        B.scores = (Score *)(db + o_sc);
        B.bin_term = (double *)(db + o_bt);
        c->ts_off = o_ts;
        c->scores_off = o_sc;
    }
    c->batch.light = light;
    HIPCHK(c, launch_select(c->batch, c->stream));
    if (!light) HIPCHK(c, launch_score(c->batch, c->stream));

    // results: per-tensor state and scores
    const size_t ts_bytes = sizeof(TState) * nT, sc_bytes = sizeof(Score) * (size_t)nT * n_cfg;
    rc = ensure_host(c, c->h_down, ts_bytes + sc_bytes);
    if (rc) return rc;
    char *db = (char *)c->search_mem.p;
    HIPCHK(c, hipMemcpyAsync(c->h_down.p, db + c->ts_off, ts_bytes, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipMemcpyAsync((char *)c->h_down.p + ts_bytes, db + c->scores_off, sc_bytes,
                             hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    const TState *hts = (const TState *)c->h_down.p;
    for (uint32_t t = 0; t < nT; t++) {
        if (hts[t].nonfinite) return INSHR_E_NONFINITE;
    }
    for (uint32_t t = 0; t < nT; t++) {
        if (any_pooled && (hts[t].internal_err & 32u)) { // (a tensor alone always keeps the value of rank P)
            c->last_err = "the shared thresholds leave tensor " + std::to_string(t) + " without quantized values";
            return INSHR_E_CONFIG;
        }
    }
    for (uint32_t t = 0; t < nT; t++) {
        if (!hts[t].pool_overflow) continue;
        // some wave gathered more keys than its share of a pool holds: larger pools, once more
        const uint32_t full = TILE / (BLOCK / 64);
        if (c->pool_wcap >= full) {
            c->last_err = "gather pool overflow with full-size pools on tensor " + std::to_string(t);
            return INSHR_E_INTERNAL;
        }
        c->pool_wcap = std::min<uint32_t>(full, c->pool_wcap * 2);
        if (getenv("INSHR_SAMPLE_DEBUG"))
            fprintf(stderr, "inshr_search: gather pools too small (tensor %u, code %u): again with %u keys per wave and tile\n",
                    t, hts[t].pool_overflow, c->pool_wcap);
        return run_search(c, tensors, nT, grid, n_cfg, eps, light, group);
    }
    if (getenv("INSHR_SAMPLE_DEBUG")) { // how many sampled first sweeps had to be repeated exactly
        uint32_t n_sampled = 0, n_redo = 0;
        for (uint32_t t = 0; t < nT; t++) {
            n_sampled += c->batch_sampled.size() > t && c->batch_sampled[t] ? 1u : 0u;
            n_redo += hts[t].redo ? 1u : 0u;
            if (hts[t].redo)
                fprintf(stderr, "inshr_search: tensor %u (n = %llu) repeated, thresholds missed: 0x%x\n", t,
                        (unsigned long long)tensors[t].n, hts[t].redo >> 1);
        }
        fprintf(stderr, "inshr_search: %u tensors, %u with a sampled first sweep, %u of them repeated\n",
                nT, n_sampled, n_redo);
    }
    for (uint32_t t = 0; t < nT; t++) {
        if (hts[t].internal_err) {
            c->last_err = "kernel self-check failed on tensor " + std::to_string(t) + ", code " +
                          std::to_string(hts[t].internal_err);
            return INSHR_E_INTERNAL;
        }
    }
    c->grid = g;
    c->grid_cfgs.assign(grid, grid + n_cfg);
    c->tensors.assign(tensors, tensors + nT);
    c->have_search = !light;
    return INSHR_OK;
}

} // namespace

extern "C" {

int inshr_create(inshr_ctx **out, int device, void *hip_stream, uint64_t scratch_bytes)
{
    if (!out) return INSHR_E_ARG;
    *out = nullptr;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || device < 0 || device >= n_dev) return INSHR_E_DEVICE;
    inshr_ctx *c = new inshr_ctx();
    c->device = device;
    c->stream = (hipStream_t)hip_stream;
    c->scratch_limit = scratch_bytes;
    hipDeviceProp_t pr;
    if (hipSetDevice(device) != hipSuccess || hipGetDeviceProperties(&pr, device) != hipSuccess) {
        delete c;
        return INSHR_E_DEVICE;
    }
    c->n_cu = pr.multiProcessorCount > 0 ? pr.multiProcessorCount : 256;
    if (const char *e = getenv("INSHR_WG_PER_CU")) {
        int v = atoi(e);
        if (v >= 1 && v <= 16) c->wg_per_cu = v;
    }
    // the delta scatter and the group sort have a fast path that needs same-address LDS atomics to
    // be served in lane order; it is used only if this device passes the check
    // (INSHR_NO_LDS_ORDER=1, or its older name INSHR_DELTA_SLOTS=1, forces it off)
    {
        u32 *viol = nullptr;
        u32 h = 1;
        if (hipMalloc(&viol, 4) == hipSuccess) {
            if (hipMemsetAsync(viol, 0, 4, c->stream) == hipSuccess &&
                launch_lds_order_check(viol, c->stream) == hipSuccess &&
                hipMemcpyAsync(&h, viol, 4, hipMemcpyDeviceToHost, c->stream) == hipSuccess &&
                hipStreamSynchronize(c->stream) == hipSuccess)
                c->lds_ordered = (h == 0);
            (void)hipFree(viol);
        }
        for (const char *name : {"INSHR_NO_LDS_ORDER", "INSHR_DELTA_SLOTS"})
            if (const char *e = getenv(name))
                if (atoi(e) != 0) c->lds_ordered = false;
    }
    if (hipMalloc(&c->delta_flags, 256) != hipSuccess || delta_static_init(device) != hipSuccess) {
        delete c;
        return INSHR_E_DEVICE;
    }
    if (const char *e = getenv("INSHR_SAMPLE_MIN_N")) c->sample_min_n = strtoull(e, nullptr, 10);
    if (const char *e = getenv("INSHR_SAMPLE_FORCE_MISS")) c->sample_force_miss = atoi(e) != 0;
    if (const char *e = getenv("INSHR_POOL_WCAP")) {
        const long v = atol(e);
        if (v >= 1 && v <= TILE / (BLOCK / 64)) c->pool_wcap = (uint32_t)v;
    }
    *out = c;
    return INSHR_OK;
}

void inshr_destroy(inshr_ctx *c)
{
    if (!c) return;
    (void)hipSetDevice(c->device);
    (void)hipStreamSynchronize(c->stream);
    if (c->search_mem.p) (void)hipFree(c->search_mem.p);
    if (c->aux_mem.p) (void)hipFree(c->aux_mem.p);
    if (c->sketch_mem.p) (void)hipFree(c->sketch_mem.p);
    if (c->sens_mem.p) (void)hipFree(c->sens_mem.p);
    if (c->delta_flags) (void)hipFree(c->delta_flags);
    if (c->h_up.p) (void)hipHostFree(c->h_up.p);
    if (c->h_down.p) (void)hipHostFree(c->h_down.p);
    delete c;
}

const char *inshr_strerror(int code)
{
    switch (code) {
    case INSHR_OK: return "ok";
    case INSHR_E_ARG: return "bad argument";
    case INSHR_E_CONFIG: return "bad configuration or grid too large";
    case INSHR_E_NONFINITE: return "NaN or Inf in a tensor";
    case INSHR_E_CAPACITY: return "buffer or scratch too small";
    case INSHR_E_SHAPE: return "shape mismatch";
    case INSHR_E_DEVICE: return "HIP error";
    case INSHR_E_INTERNAL: return "internal self-check failed";
    default: return "unknown error";
    }
}

const char *inshr_last_device_error(const inshr_ctx *c) { return c ? c->last_err.c_str() : ""; }

int inshr_sync(inshr_ctx *c)
{
    if (!c) return INSHR_E_ARG;
    HIPCHK(c, hipSetDevice(c->device));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    return take_delta_flags(c);
}

int inshr_lds_ordered(const inshr_ctx *c) { return (c && c->lds_ordered) ? 1 : 0; }

int inshr_profile(inshr_ctx *c, int enable)
{
    if (!c) return INSHR_E_ARG;
    HIPCHK(c, hipSetDevice(c->device));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    prof_collect();
    g_prof.on = enable != 0;
    if (enable) {
        g_prof.names.clear();
        g_prof.total_ms.clear();
        g_prof.launches.clear();
    }
    return INSHR_OK;
}

int inshr_profile_read(inshr_ctx *c, inshr_kernel_time *out, uint32_t cap, uint32_t *n)
{
    if (!c || !n) return INSHR_E_ARG;
    HIPCHK(c, hipSetDevice(c->device));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    prof_collect();
    *n = (uint32_t)g_prof.names.size();
    for (uint32_t i = 0; i < *n && i < cap && out; i++) {
        memset(&out[i], 0, sizeof(out[i]));
        strncpy(out[i].name, g_prof.names[i].c_str(), sizeof(out[i].name) - 1);
        out[i].total_ms = g_prof.total_ms[i];
        out[i].launches = g_prof.launches[i];
    }
    return INSHR_OK;
}

int inshr_search(inshr_ctx *c, const inshr_tensor *tensors, uint32_t n_tensors,
                 const inshr_config *grid, uint32_t n_cfg, double eps, uint32_t *best,
                 uint8_t *feasible, inshr_score *scores)
{
    if (!c || !best || !feasible) return INSHR_E_ARG;
    int rc = run_search(c, tensors, n_tensors, grid, n_cfg, eps);
    if (rc) return rc;
    const TState *hts = (const TState *)c->h_down.p;
    const Score *hsc = (const Score *)((const char *)c->h_down.p + sizeof(TState) * n_tensors);
    for (uint32_t t = 0; t < n_tensors; t++) {
        best[t] = hts[t].best;
        feasible[t] = (uint8_t)hts[t].feasible;
    }
    if (scores) {
        static_assert(sizeof(Score) == sizeof(inshr_score), "score layout");
        memcpy(scores, hsc, sizeof(Score) * (size_t)n_tensors * n_cfg);
    }
    return INSHR_OK;
}

int inshr_search_pooled(inshr_ctx *c, const inshr_tensor *tensors, const uint32_t *group,
                        uint32_t n_tensors, const inshr_config *grid, uint32_t n_cfg, double eps,
                        uint32_t *best, uint8_t *feasible, inshr_score *scores)
{
    if (!c || !best || !feasible || !group) return INSHR_E_ARG;
    int rc = run_search(c, tensors, n_tensors, grid, n_cfg, eps, false, group);
    if (rc) return rc;
    const TState *hts = (const TState *)c->h_down.p;
    const Score *hsc = (const Score *)((const char *)c->h_down.p + sizeof(TState) * n_tensors);
    for (uint32_t t = 0; t < n_tensors; t++) {
        best[t] = hts[t].best;
        feasible[t] = (uint8_t)hts[t].feasible;
    }
    if (scores) memcpy(scores, hsc, sizeof(Score) * (size_t)n_tensors * n_cfg);
    return INSHR_OK;
}

int inshr_quantize_bound(uint64_t n, const inshr_config *cfg, uint64_t *packed_words,
                         uint64_t *outlier_cap)
{
    if (!cfg || n == 0 || n >= (1ull << 32)) return INSHR_E_ARG;
    int rc = check_config(*cfg);
    if (rc) return rc;
    if (packed_words) *packed_words = (n * (uint64_t)symbol_bits(bins_of(*cfg)) + 63) / 64;
    if (outlier_cap) *outlier_cap = n * (uint64_t)cfg->outlier_ppm / 1000000ull;
    return INSHR_OK;
}

static int quantize_with_state(inshr_ctx *c, const inshr_config *cfg, inshr_quantized *out,
                               const uint32_t *which, uint32_t n_sel, const u32 *alt_key = nullptr,
                               const float *alt_cb = nullptr, bool val_bf16 = false)
{
    // alt_key / alt_cb: device arrays with 256 entries per tensor of the batch that replace the
    // search's boundaries and centres
    // which[k] = position in the search batch of the k-th tensor to quantize (cfg / out indexed by k)
    const uint32_t nT = (uint32_t)c->batch.nT;
    std::vector<QDesc> qd(nT);
    for (auto &q : qd) memset(&q, 0, sizeof(q));
    for (uint32_t k = 0; k < n_sel; k++) {
        const uint32_t t = which[k];
        uint32_t gi = 0;
        for (gi = 0; gi < c->grid.n_cfg; gi++)
            if (same_config(c->grid_cfgs[gi], cfg[k])) break;
        if (gi == c->grid.n_cfg) return INSHR_E_SHAPE;
        uint64_t words = 0, cap = 0;
        inshr_quantize_bound(c->tensors[t].n, &cfg[k], &words, &cap);
        if (!out[k].packed || !out[k].codebook || out[k].packed_words < words) return INSHR_E_CAPACITY;
        if (out[k].outlier_cap && (!out[k].outlier_idx || !out[k].outlier_val)) return INSHR_E_ARG;
        qd[t].packed = (unsigned long long *)out[k].packed;
        qd[t].codebook = out[k].codebook;
        qd[t].boundaries = out[k].boundaries;
        qd[t].out_idx = out[k].outlier_idx;
        qd[t].out_val = out[k].outlier_val;
        qd[t].out_cap = out[k].outlier_cap;
        qd[t].cfg = gi;
        qd[t].val_bf16 = val_bf16 ? 1u : 0u;
        qd[t].alt_key = alt_key ? alt_key + (size_t)t * 256 : nullptr;
        qd[t].alt_cb = alt_cb ? alt_cb + (size_t)t * 256 : nullptr;
    }
    Carver cv;
    const size_t o_qd = cv.take(sizeof(QDesc) * nT);
    const size_t o_qi = cv.take(sizeof(QInfo) * nT);
    int rc = ensure_dev(c, c->aux_mem, cv.off);
    if (rc) return rc;
    rc = ensure_host(c, c->h_up, sizeof(QDesc) * nT);
    if (rc) return rc;
    rc = ensure_host(c, c->h_down, sizeof(QInfo) * nT);
    if (rc) return rc;
    char *db = (char *)c->aux_mem.p;
    HIPCHK(c, hipStreamSynchronize(c->stream)); // staging buffers may be in flight (inshr_delta)
    memcpy(c->h_up.p, qd.data(), sizeof(QDesc) * nT);
    HIPCHK(c, hipMemcpyAsync(db + o_qd, c->h_up.p, sizeof(QDesc) * nT, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, launch_quantize(c->batch, (const QDesc *)(db + o_qd), (QInfo *)(db + o_qi), c->stream));
    HIPCHK(c, hipMemcpyAsync(c->h_down.p, db + o_qi, sizeof(QInfo) * nT, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    const QInfo *qi = (const QInfo *)c->h_down.p;
    int result = INSHR_OK;
    for (uint32_t k = 0; k < n_sel; k++) {
        const QInfo &r = qi[which[k]];
        out[k].n_pruned = r.n_pruned;
        out[k].n_outlier = r.n_outlier;
        out[k].n_kept = r.n_kept;
        out[k].n_bins = bins_of(cfg[k]);
        out[k].sym_bits = symbol_bits(out[k].n_bins);
        uint32_t tp = r.tau_p, to = r.tau_o;
        memcpy(&out[k].tau_prune, &tp, 4);
        memcpy(&out[k].tau_outlier, &to, 4);
        if (r.flags & 1u) {
            c->last_err = "protected-value count self-check failed";
            result = INSHR_E_INTERNAL;
        } else if ((r.flags & 2u) && result == INSHR_OK) {
            result = INSHR_E_CAPACITY;
        }
    }
    return result;
}

int inshr_quantize(inshr_ctx *c, const inshr_tensor *tensors, const inshr_config *cfg,
                   inshr_quantized *out, uint32_t n_tensors, uint32_t flags)
{
    if (!c || !tensors || !cfg || !out || n_tensors == 0) return INSHR_E_ARG;
    for (uint32_t t = 0; t < n_tensors; t++) {
        int rc = check_config(cfg[t]);
        if (rc) return rc;
    }
    HIPCHK(c, hipSetDevice(c->device));
    if (flags & INSHR_REUSE_SEARCH) {
        if (!c->have_search || c->tensors.size() != n_tensors) return INSHR_E_SHAPE;
        std::vector<uint32_t> which(n_tensors);
        for (uint32_t t = 0; t < n_tensors; t++) {
            if (c->tensors[t].data != tensors[t].data || c->tensors[t].n != tensors[t].n) return INSHR_E_SHAPE;
            which[t] = t;
        }
        return quantize_with_state(c, cfg, out, which.data(), n_tensors, nullptr, nullptr,
                                   (flags & INSHR_PROTECT_BF16) != 0);
    }
    // stand-alone: one internal single-configuration search per distinct configuration
    std::vector<char> done(n_tensors, 0);
    for (uint32_t t0 = 0; t0 < n_tensors; t0++) {
        if (done[t0]) continue;
        std::vector<inshr_tensor> sub;
        std::vector<inshr_config> subcfg;
        std::vector<uint32_t> idx;
        for (uint32_t t = t0; t < n_tensors; t++) {
            if (!done[t] && same_config(cfg[t], cfg[t0])) {
                done[t] = 1;
                sub.push_back(tensors[t]);
                subcfg.push_back(cfg[t]);
                idx.push_back(t);
            }
        }
        int rc = run_search(c, sub.data(), (uint32_t)sub.size(), &cfg[t0], 1, 0.0);
        if (rc) return rc;
        std::vector<inshr_quantized> subout(sub.size());
        std::vector<uint32_t> which(sub.size());
        for (size_t k = 0; k < sub.size(); k++) {
            subout[k] = out[idx[k]];
            which[k] = (uint32_t)k;
        }
        rc = quantize_with_state(c, subcfg.data(), subout.data(), which.data(), (uint32_t)sub.size(), nullptr,
                                 nullptr, (flags & INSHR_PROTECT_BF16) != 0);
        for (size_t k = 0; k < sub.size(); k++) out[idx[k]] = subout[k];
        if (rc) return rc;
    }
    return INSHR_OK;
}

// ------------------------------------------------------------------------------------------
// sketch + weighted K-Means boundaries
// ------------------------------------------------------------------------------------------
namespace {

struct SketchTables {
    std::vector<u32> cell, tops;
    std::vector<double> rep;
    int i_lo = 0; // tops[b] belongs to bucket index i_lo + b
};

// Tables of the bucket law ceil(log_gamma |x|): tops[b] = magnitude image of the largest fp32
// number <= gamma^(i_lo + b) (extended precision; a value x lies in the first bucket whose top
// reaches it), rep[b] = the bucket's value, cell[c] = first bucket and its top for the magnitudes
// c << 17 .. (c << 17) + 2^17 - 1.
int build_sketch_tables(inshr_ctx *ctx, double alpha, SketchTables &T)
{
    if (!(alpha >= 0.01 && alpha <= 0.5)) return INSHR_E_CONFIG;
    if (ctx && ctx->sketch_alpha == alpha) { // the tables of the call before
        T.i_lo = ctx->sketch_i_lo;
        T.cell = ctx->sketch_cell;
        T.tops = ctx->sketch_tops;
        T.rep = ctx->sketch_rep;
        return INSHR_OK;
    }
    const double gamma = (1.0 + alpha) / (1.0 - alpha);
    const long double lg = logl((long double)gamma);
    const int i_lo = (int)floorl(-149.0L * logl(2.0L) / lg) - 2;
    const int i_hi = (int)ceill(128.0L * logl(2.0L) / lg) + 1;
    const int n_idx = i_hi - i_lo + 1;
    if (n_idx > SK_MAX_IDX) return INSHR_E_CONFIG;
    T.i_lo = i_lo;
    T.tops.resize(n_idx);
    T.rep.resize(n_idx);
    for (int b = 0; b < n_idx; b++) {
        const int i = i_lo + b;
        const long double v = powl((long double)gamma, (long double)i);
        float f;
        if (v >= (long double)3.402823466e+38F) {
            f = 3.402823466e+38F;
        } else {
            f = (float)v;
            if ((long double)f > v) f = nextafterf(f, -1.0f); // round down (v > 0)
        }
        u32 bits;
        memcpy(&bits, &f, 4);
        T.tops[b] = bits;
        T.rep[b] = 2.0 * pow(gamma, (double)i) / (gamma + 1.0);
    }
    T.cell.assign(SK_CELLS, (u32)(n_idx - 1) << 17);
    for (u32 c = 64; c < (0x7f800000u >> 17); c++) { // normal numbers
        const u32 first = c << 17, last = first | 0x1FFFFu;
        const u32 b0 = (u32)(std::lower_bound(T.tops.begin(), T.tops.end(), first) - T.tops.begin());
        if (b0 + 1u >= (u32)n_idx || T.tops[b0 + 1u] < last) return INSHR_E_CONFIG; // more than two buckets
        const u32 split = T.tops[b0] <= last ? (T.tops[b0] & 0x1FFFFu) : 0x1FFFFu;
        T.cell[c] = (b0 << 17) | (0x1FFFFu - split); // adding the low magnitude bits carries above the split
    }
    if (ctx) {
        ctx->sketch_cell = T.cell;
        ctx->sketch_tops = T.tops;
        ctx->sketch_rep = T.rep;
        ctx->sketch_i_lo = i_lo;
        ctx->sketch_alpha = alpha;
    }
    return INSHR_OK;
}

} // namespace

namespace {

// Sketch and clustering for tensors which[k] of the searched batch with configurations cfg[k] (all
// in the search's grid); src[k] = the tensor's position in the caller's arrays (uniforms, info).
// Leaves 256 boundary keys and centres per tensor of the batch in *alt_key / *alt_cb (device).
int sketch_with_state(inshr_ctx *c, const inshr_config *cfg, const uint32_t *which, const uint32_t *src,
                      uint32_t n_sel, const inshr_sketch_params *params, const SketchTables &T,
                      inshr_sketch_info *info, const u32 **alt_key, const float **alt_cb,
                      bool multi = false, double eps = 0.0, inshr_sketch_choice *choice = nullptr)
{
    // multi: centres for 2 .. 8 bits, their exact errors and the choice (cfg[k].bits must be 8 then:
    // it names the grid entry that carries the tensor's prune / protect fractions)
    const uint32_t nT = (uint32_t)c->batch.nT;
    std::vector<SketchDesc> sd(nT);
    for (auto &d : sd) d.active = d.cfg = 0u;
    for (uint32_t k = 0; k < n_sel; k++) {
        uint32_t gi = 0;
        for (gi = 0; gi < c->grid.n_cfg; gi++)
            if (c->grid_cfgs[gi].bits == cfg[k].bits && c->grid_cfgs[gi].prune_ppm == cfg[k].prune_ppm &&
                c->grid_cfgs[gi].outlier_ppm == cfg[k].outlier_ppm)
                break;
        if (gi == c->grid.n_cfg) return INSHR_E_SHAPE;
        sd[which[k]].active = 1u;
        sd[which[k]].cfg = gi;
    }
    const size_t n_idx = T.tops.size();
    Carver cv;
    const size_t o_cell = cv.take(sizeof(u32) * SK_CELLS);
    const size_t o_tops = cv.take(sizeof(u32) * n_idx);
    const size_t o_rep = cv.take(sizeof(double) * n_idx);
    const size_t o_uni = cv.take(sizeof(double) * 256 * nT);
    const size_t o_sd = cv.take(sizeof(SketchDesc) * nT);
    const size_t upload = cv.off; // everything up to here comes from the host
    const size_t o_info = cv.take(sizeof(SketchInfo) * nT);
    const size_t o_hist = cv.take(sizeof(u32) * SK_HIST * nT);
    const size_t o_xq = cv.take(sizeof(double) * SK_HIST * nT);
    const size_t o_w = cv.take(sizeof(double) * SK_HIST * nT);
    const size_t o_d = cv.take(sizeof(double) * SK_HIST * nT);
    const size_t n_sets = multi ? SK_SETS : 1;
    const size_t o_key = cv.take(sizeof(u32) * 256 * n_sets * nT);
    const size_t o_cb = cv.take(sizeof(float) * 256 * n_sets * nT);
    const size_t o_sr = cv.take(sizeof(u32) * SK_SETS * nT);
    const size_t o_ch = cv.take(sizeof(SketchChoice) * nT);
    const size_t o_fk = cv.take(sizeof(u32) * 256 * nT);
    const size_t o_fc = cv.take(sizeof(float) * 256 * nT);
    const size_t o_se = cv.take(sizeof(u32) * SK_SLOTS * nT);
    const size_t o_slot = cv.off; // slot moments, cleared before the scoring sweep
    const size_t o_sc = cv.take(sizeof(u32) * SK_SLOTS * nT);
    const size_t o_sx = cv.take(sizeof(double) * SK_SLOTS * nT);
    const size_t slot_end = cv.off;
    int rc = ensure_dev(c, c->sketch_mem, cv.off);
    if (rc) return rc;
    rc = ensure_host(c, c->h_up, upload);
    if (rc) return rc;
    rc = ensure_host(c, c->h_down, (sizeof(SketchInfo) + sizeof(SketchChoice)) * nT);
    if (rc) return rc;
    char *hb = (char *)c->h_up.p, *db = (char *)c->sketch_mem.p;
    HIPCHK(c, hipStreamSynchronize(c->stream)); // the staging buffer may still be in flight
    memcpy(hb + o_cell, T.cell.data(), sizeof(u32) * SK_CELLS);
    memcpy(hb + o_tops, T.tops.data(), sizeof(u32) * n_idx);
    memcpy(hb + o_rep, T.rep.data(), sizeof(double) * n_idx);
    memset(hb + o_uni, 0, sizeof(double) * 256 * nT);
    for (uint32_t k = 0; k < n_sel; k++)
        memcpy(hb + o_uni + sizeof(double) * 256 * which[k], params->uniforms + (size_t)src[k] * 256,
               sizeof(double) * 256);
    memcpy(hb + o_sd, sd.data(), sizeof(SketchDesc) * nT);
    HIPCHK(c, hipMemcpyAsync(db, hb, upload, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipMemsetAsync(db + o_hist, 0, sizeof(u32) * SK_HIST * nT, c->stream));
    SketchParams P;
    P.sigma = params->sigma;
    P.max_iter = params->max_iter;
    P.n_idx = (u32)n_idx;
    P.cell = (const u32 *)(db + o_cell);
    P.tops = (const u32 *)(db + o_tops);
    P.rep = (const double *)(db + o_rep);
    P.uniforms = (const double *)(db + o_uni);
    P.hist = (u32 *)(db + o_hist);
    P.xq = (double *)(db + o_xq);
    P.w = (double *)(db + o_w);
    P.d = (double *)(db + o_d);
    P.alt_key = (u32 *)(db + o_key);
    P.alt_cb = (float *)(db + o_cb);
    P.info = (SketchInfo *)(db + o_info);
    P.multi = multi ? 1u : 0u;
    P.light = c->batch.light ? 1u : 0u;
    P.eps = eps;
    P.set_rounds = (u32 *)(db + o_sr);
    P.slot_cnt = (u32 *)(db + o_sc);
    P.slot_sx = (double *)(db + o_sx);
    P.slot_edge = (u32 *)(db + o_se);
    P.choice = (SketchChoice *)(db + o_ch);
    P.final_key = (u32 *)(db + o_fk);
    P.final_cb = (float *)(db + o_fc);
    if (multi) HIPCHK(c, hipMemsetAsync(db + o_slot, 0, slot_end - o_slot, c->stream));
    HIPCHK(c, launch_sketch(c->batch, (const SketchDesc *)(db + o_sd), P, c->stream));
    if (multi)
        HIPCHK(c, hipMemcpyAsync((char *)c->h_down.p + sizeof(SketchInfo) * nT, db + o_ch,
                                 sizeof(SketchChoice) * nT, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipMemcpyAsync(c->h_down.p, db + o_info, sizeof(SketchInfo) * nT, hipMemcpyDeviceToHost,
                             c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    if (info) {
        const SketchInfo *si = (const SketchInfo *)c->h_down.p;
        for (uint32_t k = 0; k < n_sel; k++) {
            info[src[k]].n_buckets = si[which[k]].n_buckets;
            info[src[k]].rounds = si[which[k]].rounds;
        }
    }
    if (multi && choice) {
        const SketchChoice *sc = (const SketchChoice *)((const char *)c->h_down.p + sizeof(SketchInfo) * nT);
        for (uint32_t k = 0; k < n_sel; k++) {
            const SketchChoice &r = sc[which[k]];
            inshr_sketch_choice &o = choice[src[k]];
            for (int b = 0; b < SK_SETS; b++) {
                o.sse[b] = r.sse[b];
                o.rounds[b] = r.rounds[b];
            }
            o.sumsq = r.sumsq;
            o.best_bits = r.best_bits;
            o.feasible = r.feasible;
        }
    }
    *alt_key = multi ? P.final_key : P.alt_key;
    *alt_cb = multi ? P.final_cb : P.alt_cb;
    return INSHR_OK;
}

} // namespace

int inshr_quantize_sketch(inshr_ctx *c, const inshr_tensor *tensors, const inshr_config *cfg,
                          const inshr_sketch_params *params, inshr_quantized *out,
                          inshr_sketch_info *info, uint32_t n_tensors, uint32_t flags)
{
    if (!c || !tensors || !cfg || !params || !out || n_tensors == 0 || !params->uniforms) return INSHR_E_ARG;
    if (!(params->sigma >= 0.0 && params->sigma <= 1.0)) return INSHR_E_CONFIG;
    for (uint32_t t = 0; t < n_tensors; t++) {
        int rc = check_config(cfg[t]);
        if (rc) return rc;
        if (cfg[t].bins) return INSHR_E_CONFIG; // the clustered bins come in powers of two, by bits
        for (int r = 0; r < (1 << cfg[t].bits); r++) {
            const double u = params->uniforms[(size_t)t * 256 + r];
            if (!(u >= 0.0 && u < 1.0)) return INSHR_E_ARG;
        }
    }
    SketchTables T;
    int rc = build_sketch_tables(c, params->alpha, T);
    if (rc) return rc;
    HIPCHK(c, hipSetDevice(c->device));
    const u32 *alt_key = nullptr;
    const float *alt_cb = nullptr;
    if (flags & INSHR_REUSE_SEARCH) {
        if (!c->have_search || c->tensors.size() != n_tensors) return INSHR_E_SHAPE;
        std::vector<uint32_t> which(n_tensors);
        for (uint32_t t = 0; t < n_tensors; t++) {
            if (c->tensors[t].data != tensors[t].data || c->tensors[t].n != tensors[t].n) return INSHR_E_SHAPE;
            which[t] = t;
        }
        rc = sketch_with_state(c, cfg, which.data(), which.data(), n_tensors, params, T, info, &alt_key, &alt_cb);
        if (rc) return rc;
        return quantize_with_state(c, cfg, out, which.data(), n_tensors, alt_key, alt_cb);
    }
    // stand-alone: one single-configuration search per distinct configuration gives the thresholds
    std::vector<char> done(n_tensors, 0);
    for (uint32_t t0 = 0; t0 < n_tensors; t0++) {
        if (done[t0]) continue;
        std::vector<inshr_tensor> sub;
        std::vector<inshr_config> subcfg;
        std::vector<uint32_t> idx;
        for (uint32_t t = t0; t < n_tensors; t++) {
            if (!done[t] && cfg[t].bits == cfg[t0].bits && cfg[t].prune_ppm == cfg[t0].prune_ppm &&
                cfg[t].outlier_ppm == cfg[t0].outlier_ppm) {
                done[t] = 1;
                sub.push_back(tensors[t]);
                subcfg.push_back(cfg[t]);
                idx.push_back(t);
            }
        }
        const uint32_t nS = (uint32_t)sub.size();
        rc = run_search(c, sub.data(), nS, &cfg[t0], 1, 0.0, true);
        if (rc) return rc;
        std::vector<inshr_quantized> subout(nS);
        std::vector<uint32_t> which(nS);
        for (uint32_t k = 0; k < nS; k++) {
            subout[k] = out[idx[k]];
            which[k] = k;
        }
        rc = sketch_with_state(c, subcfg.data(), which.data(), idx.data(), nS, params, T, info, &alt_key, &alt_cb);
        if (rc) return rc;
        rc = quantize_with_state(c, subcfg.data(), subout.data(), which.data(), nS, alt_key, alt_cb);
        for (uint32_t k = 0; k < nS; k++) out[idx[k]] = subout[k];
        if (rc) return rc;
    }
    return INSHR_OK;
}

int inshr_search_sketch(inshr_ctx *c, const inshr_tensor *tensors, const inshr_config *cfg,
                        const inshr_sketch_params *params, double eps, inshr_quantized *out,
                        inshr_sketch_choice *choice, inshr_sketch_info *info, uint32_t n_tensors,
                        uint32_t flags)
{
    if (!c || !tensors || !cfg || !params || !out || !choice || n_tensors == 0 || !params->uniforms)
        return INSHR_E_ARG;
    if (!(params->sigma >= 0.0 && params->sigma <= 1.0) || !(eps >= 0.0)) return INSHR_E_CONFIG;
    std::vector<inshr_config> wide(n_tensors); // the tensor's fractions with 8 bits
    for (uint32_t t = 0; t < n_tensors; t++) {
        if (cfg[t].bins) return INSHR_E_CONFIG;
        wide[t] = cfg[t];
        wide[t].bits = 8;
        int rc = check_config(wide[t]);
        if (rc) return rc;
        for (int r = 0; r < 256; r++) {
            const double u = params->uniforms[(size_t)t * 256 + r];
            if (!(u >= 0.0 && u < 1.0)) return INSHR_E_ARG;
        }
    }
    SketchTables T;
    int rc = build_sketch_tables(c, params->alpha, T);
    if (rc) return rc;
    HIPCHK(c, hipSetDevice(c->device));
    const u32 *alt_key = nullptr;
    const float *alt_cb = nullptr;
    auto finish = [&](const inshr_config *sub_wide, inshr_quantized *sub_out, const uint32_t *which,
                      const uint32_t *src, uint32_t n) -> int {
        int r = sketch_with_state(c, sub_wide, which, src, n, params, T, info, &alt_key, &alt_cb, true, eps, choice);
        if (r) return r;
        std::vector<inshr_config> chosen(n);
        for (uint32_t k = 0; k < n; k++) {
            chosen[k] = sub_wide[k];
            chosen[k].bits = (uint8_t)choice[src[k]].best_bits;
        }
        return quantize_with_state(c, chosen.data(), sub_out, which, n, alt_key, alt_cb);
    };
    if (flags & INSHR_REUSE_SEARCH) {
        if (!c->have_search || c->tensors.size() != n_tensors) return INSHR_E_SHAPE;
        std::vector<uint32_t> which(n_tensors);
        for (uint32_t t = 0; t < n_tensors; t++) {
            if (c->tensors[t].data != tensors[t].data || c->tensors[t].n != tensors[t].n) return INSHR_E_SHAPE;
            which[t] = t;
        }
        return finish(wide.data(), out, which.data(), which.data(), n_tensors);
    }
    // stand-alone: one search over 2 .. 8 bits per distinct pair of fractions gives the thresholds
    std::vector<char> done(n_tensors, 0);
    for (uint32_t t0 = 0; t0 < n_tensors; t0++) {
        if (done[t0]) continue;
        std::vector<inshr_tensor> sub;
        std::vector<inshr_config> subcfg;
        std::vector<uint32_t> idx;
        for (uint32_t t = t0; t < n_tensors; t++) {
            if (!done[t] && cfg[t].prune_ppm == cfg[t0].prune_ppm && cfg[t].outlier_ppm == cfg[t0].outlier_ppm) {
                done[t] = 1;
                sub.push_back(tensors[t]);
                subcfg.push_back(wide[t]);
                idx.push_back(t);
            }
        }
        const uint32_t nS = (uint32_t)sub.size();
        inshr_config grid7[SK_SETS];
        for (int b = 0; b < SK_SETS; b++) {
            grid7[b] = wide[t0];
            grid7[b].bits = (uint8_t)(2 + b);
        }
        rc = run_search(c, sub.data(), nS, grid7, SK_SETS, eps, true);
        if (rc) return rc;
        std::vector<inshr_quantized> subout(nS);
        std::vector<uint32_t> which(nS);
        for (uint32_t k = 0; k < nS; k++) {
            subout[k] = out[idx[k]];
            which[k] = k;
        }
        rc = finish(subcfg.data(), subout.data(), which.data(), idx.data(), nS);
        for (uint32_t k = 0; k < nS; k++) out[idx[k]] = subout[k];
        if (rc) return rc;
    }
    return INSHR_OK;
}

int inshr_search_sketch_grid(inshr_ctx *c, const inshr_tensor *tensors, const inshr_config *pairs,
                             uint32_t n_pairs, const inshr_sketch_params *params, double eps,
                             inshr_quantized *out, uint32_t *best_pair, inshr_sketch_choice *choice,
                             inshr_sketch_choice *table, uint32_t n_tensors)
{
    if (!c || !tensors || !pairs || !params || !out || !best_pair || !choice || n_tensors == 0 || n_pairs == 0)
        return INSHR_E_ARG;
    const uint32_t nT = n_tensors;
    std::vector<inshr_config> cfg(nT);
    std::vector<inshr_sketch_choice> ch(nT);
    std::vector<inshr_quantized> tmp(nT);
    struct Best {
        bool any = false, feasible = false;
        uint64_t cost = 0;
        double sse8 = 0.0;
        uint32_t pair = 0;
    };
    std::vector<Best> best(nT);
    // every pair in turn: all widths of the pair scored for all tensors (the outputs are scratch here)
    for (uint32_t q = 0; q < n_pairs; q++) {
        for (uint32_t t = 0; t < nT; t++) {
            cfg[t] = pairs[q];
            cfg[t].bits = 8;
            cfg[t].bins = 0;
            tmp[t] = out[t];
        }
        int rc = inshr_search_sketch(c, tensors, cfg.data(), params, eps, tmp.data(), ch.data(), nullptr, nT, 0);
        if (rc) return rc;
        for (uint32_t t = 0; t < nT; t++) {
            if (table) table[(size_t)t * n_pairs + q] = ch[t];
            Best &b = best[t];
            if (ch[t].feasible) {
                const uint32_t bits = ch[t].best_bits; // the fewest feasible bits of a pair are its cheapest
                const uint64_t cost = tmp[t].n_kept * bits + 32ull * tmp[t].n_outlier + (32ull << bits);
                if (!b.feasible || cost < b.cost) {
                    b.feasible = true;
                    b.cost = cost;
                    b.pair = q;
                }
            } else if (!b.feasible && (!b.any || ch[t].sse[6] < b.sse8)) {
                b.sse8 = ch[t].sse[6];
                b.pair = q;
            }
            b.any = true;
        }
    }
    // the winners once more, pair by pair, into the caller's buffers (same uniforms: same result)
    std::vector<char> done(nT, 0);
    for (uint32_t t0 = 0; t0 < nT; t0++) {
        if (done[t0]) continue;
        std::vector<inshr_tensor> sub;
        std::vector<inshr_config> subcfg;
        std::vector<inshr_quantized> subout;
        std::vector<uint32_t> idx;
        std::vector<double> uni;
        for (uint32_t t = t0; t < nT; t++) {
            if (!done[t] && best[t].pair == best[t0].pair) {
                done[t] = 1;
                sub.push_back(tensors[t]);
                inshr_config k = pairs[best[t].pair];
                k.bits = 8;
                k.bins = 0;
                subcfg.push_back(k);
                subout.push_back(out[t]);
                idx.push_back(t);
                uni.insert(uni.end(), params->uniforms + (size_t)t * 256, params->uniforms + (size_t)t * 256 + 256);
            }
        }
        inshr_sketch_params p2 = *params;
        p2.uniforms = uni.data();
        std::vector<inshr_sketch_choice> ch2(sub.size());
        int rc = inshr_search_sketch(c, sub.data(), subcfg.data(), &p2, eps, subout.data(), ch2.data(), nullptr,
                                     (uint32_t)sub.size(), 0);
        if (rc) return rc;
        for (size_t k = 0; k < sub.size(); k++) {
            out[idx[k]] = subout[k];
            choice[idx[k]] = ch2[k];
            best_pair[idx[k]] = best[idx[k]].pair;
        }
    }
    return INSHR_OK;
}

int inshr_sketch_buckets(double alpha, int32_t *i_lo, uint32_t *n_buckets, float *tops, double *values,
                         uint32_t cap)
{
    if (!i_lo || !n_buckets) return INSHR_E_ARG;
    SketchTables T;
    int rc = build_sketch_tables(nullptr, alpha, T);
    if (rc) return rc;
    *i_lo = T.i_lo;
    *n_buckets = (uint32_t)T.tops.size();
    if (cap < T.tops.size() && (tops || values)) return INSHR_E_CAPACITY;
    for (size_t b = 0; b < T.tops.size(); b++) {
        if (tops) memcpy(&tops[b], &T.tops[b], 4);
        if (values) values[b] = T.rep[b];
    }
    return INSHR_OK;
}

int inshr_sketch_quantiles(inshr_ctx *c, const inshr_tensor *tensors, uint32_t n_tensors, const double *q,
                           uint32_t n_q, double alpha, double *estimates)
{
    if (!c || !tensors || !q || !estimates || n_tensors == 0 || n_q == 0 || n_q > 4096u) return INSHR_E_ARG;
    SketchTables T;
    int rc = build_sketch_tables(c, alpha, T);
    if (rc) return rc;
    const uint32_t nT = n_tensors;
    const size_t n_idx = T.tops.size();
    std::vector<MagDesc> md(nT);
    std::vector<u64> ranks((size_t)nT * n_q);
    u64 chunks = 0;
    for (uint32_t t = 0; t < nT; t++) {
        if (!tensors[t].data || tensors[t].n == 0 || tensors[t].n >= (1ull << 32)) return INSHR_E_ARG;
        if ((uintptr_t)tensors[t].data & 3u) return INSHR_E_ARG;
        md[t].x = tensors[t].data;
        md[t].n = tensors[t].n;
        md[t].chunk0 = chunks;
        md[t].aligned16 = (((uintptr_t)tensors[t].data & 15u) == 0) ? 1u : 0u;
        md[t].pad = 0u;
        chunks += (tensors[t].n + SK_MAG_CHUNK - 1) / SK_MAG_CHUNK;
        for (uint32_t k = 0; k < n_q; k++) {
            if (!(q[k] >= 0.0 && q[k] <= 1.0)) return INSHR_E_ARG;
            ranks[(size_t)t * n_q + k] = (u64)floor(q[k] * (double)(tensors[t].n - 1)); // rank floor(q (n - 1))
        }
    }
    HIPCHK(c, hipSetDevice(c->device));
    Carver cv;
    const size_t o_cell = cv.take(sizeof(u32) * SK_CELLS);
    const size_t o_tops = cv.take(sizeof(u32) * n_idx);
    const size_t o_rep = cv.take(sizeof(double) * n_idx);
    const size_t o_md = cv.take(sizeof(MagDesc) * nT);
    const size_t o_rk = cv.take(sizeof(u64) * ranks.size());
    const size_t upload = cv.off;
    const size_t o_hist = cv.take(sizeof(u32) * SK_MAG_HIST * nT);
    const size_t o_nf = cv.take(256);
    const size_t zero_end = cv.off;
    const size_t o_est = cv.take(sizeof(double) * ranks.size());
    rc = ensure_dev(c, c->sketch_mem, cv.off);
    if (rc) return rc;
    rc = ensure_host(c, c->h_up, upload);
    if (rc) return rc;
    rc = ensure_host(c, c->h_down, sizeof(double) * ranks.size() + 256);
    if (rc) return rc;
    char *hb = (char *)c->h_up.p, *db = (char *)c->sketch_mem.p;
    HIPCHK(c, hipStreamSynchronize(c->stream)); // the staging buffer may still be in flight
    memcpy(hb + o_cell, T.cell.data(), sizeof(u32) * SK_CELLS);
    memcpy(hb + o_tops, T.tops.data(), sizeof(u32) * n_idx);
    memcpy(hb + o_rep, T.rep.data(), sizeof(double) * n_idx);
    memcpy(hb + o_md, md.data(), sizeof(MagDesc) * nT);
    memcpy(hb + o_rk, ranks.data(), sizeof(u64) * ranks.size());
    HIPCHK(c, hipMemcpyAsync(db, hb, upload, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipMemsetAsync(db + o_hist, 0, zero_end - o_hist, c->stream));
    HIPCHK(c, launch_sketch_quantiles((const MagDesc *)(db + o_md), (int)nT, chunks, c->n_cu, (const u32 *)(db + o_cell),
                                      (const u32 *)(db + o_tops), (const double *)(db + o_rep), (u32)n_idx,
                                      (u32 *)(db + o_hist), (u32 *)(db + o_nf), (const u64 *)(db + o_rk), n_q,
                                      (double *)(db + o_est), c->stream));
    HIPCHK(c, hipMemcpyAsync(c->h_down.p, db + o_est, sizeof(double) * ranks.size(), hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipMemcpyAsync((char *)c->h_down.p + sizeof(double) * ranks.size(), db + o_nf, 4,
                             hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    u32 nf = 0;
    memcpy(&nf, (const char *)c->h_down.p + sizeof(double) * ranks.size(), 4);
    if (nf) return INSHR_E_NONFINITE;
    memcpy(estimates, c->h_down.p, sizeof(double) * ranks.size());
    return INSHR_OK;
}

// number of bins of a symbol stream; nonzero return: not a valid description
static int codes_bins(const inshr_codes &c, uint32_t &K)
{
    if (c.bins) {
        if (c.bins < 2 || c.bins > 256) return 1;
        K = c.bins;
    } else {
        if (c.bits < 1 || c.bits > 8) return 1;
        K = 1u << c.bits;
    }
    return 0;
}

int inshr_quantize_sens(inshr_ctx *c, const inshr_tensor *tensors, const float *const *grads,
                        const inshr_config *cfg, const uint8_t *prune_by_sensitivity,
                        inshr_quantized *out, inshr_sens_info *info, uint32_t n_tensors)
{
    if (!c || !tensors || !grads || !cfg || !out || n_tensors == 0 || n_tensors > 65535u) return INSHR_E_ARG;
    const uint32_t nT = n_tensors;
    c->have_search = false;
    // the distinct configurations: their fractions for the two threshold searches, their numbers
    // of bins for the search over the quantized values
    std::vector<inshr_config> frac_grid, bin_grid;
    std::vector<uint32_t> frac_of(nT), bin_of_t(nT);
    u64 n_total = 0, n_blocks = 0;
    for (uint32_t t = 0; t < nT; t++) {
        int rc = check_config(cfg[t]);
        if (rc) return rc;
        if (!tensors[t].data || !grads[t] || tensors[t].n == 0 || tensors[t].n >= (1ull << 32)) return INSHR_E_ARG;
        if (((uintptr_t)tensors[t].data | (uintptr_t)grads[t]) & 3u) return INSHR_E_ARG;
        if (!out[t].packed || !out[t].codebook) return INSHR_E_ARG;
        if (out[t].outlier_cap && (!out[t].outlier_idx || !out[t].outlier_val)) return INSHR_E_ARG;
        if (out[t].packed_words < (tensors[t].n * (u64)symbol_bits(bins_of(cfg[t])) + 63) / 64) return INSHR_E_CAPACITY;
        inshr_config f = cfg[t], b = cfg[t];
        f.bits = 1;
        f.bins = 0;
        b.prune_ppm = b.outlier_ppm = 0;
        size_t i;
        for (i = 0; i < frac_grid.size(); i++)
            if (same_config(frac_grid[i], f)) break;
        if (i == frac_grid.size()) frac_grid.push_back(f);
        frac_of[t] = (uint32_t)i;
        for (i = 0; i < bin_grid.size(); i++)
            if (same_config(bin_grid[i], b)) break;
        if (i == bin_grid.size()) bin_grid.push_back(b);
        bin_of_t[t] = (uint32_t)i;
        n_total += tensors[t].n;
        n_blocks += (tensors[t].n + 1023) / 1024;
    }
    HIPCHK(c, hipSetDevice(c->device));
    Carver cv;
    const size_t o_sd = cv.take(sizeof(SDesc) * nT);
    const size_t o_si = cv.take(sizeof(SInfo) * nT);
    const size_t o_fl = cv.take(256);
    const size_t o_bk = cv.take(n_blocks * 4);
    const size_t o_bp = cv.take(n_blocks * 4);
    const size_t o_bq = cv.take(n_blocks * 16);
    const size_t o_S = cv.take(n_total * 4 + 64ull * nT);
    const size_t o_W = cv.take(n_total * 4 + 64ull * nT);
    int rc = ensure_dev(c, c->sens_mem, cv.off);
    if (rc) return rc;
    char *db = (char *)c->sens_mem.p;
    std::vector<SDesc> sd(nT);
    {
        u64 blk = 0, off = 0;
        for (uint32_t t = 0; t < nT; t++) {
            memset(&sd[t], 0, sizeof(SDesc));
            sd[t].w = tensors[t].data;
            sd[t].g = grads[t];
            sd[t].n = tensors[t].n;
            sd[t].blk0 = blk;
            sd[t].S = (float *)(db + o_S) + off;
            sd[t].Wm = (float *)(db + o_W) + off;
            sd[t].by_sens = (prune_by_sensitivity && prune_by_sensitivity[t]) ? 1u : 0u;
            blk += (tensors[t].n + 1023) / 1024;
            off += (tensors[t].n + 15) / 16 * 16; // every tensor's scratch starts 64-byte aligned
        }
    }
    auto upload = [&]() -> int {
        HIPCHK(c, hipStreamSynchronize(c->stream));
        HIPCHK(c, hipMemcpy(db + o_sd, sd.data(), sizeof(SDesc) * nT, hipMemcpyHostToDevice));
        return INSHR_OK;
    };
    if ((rc = upload())) return rc;
    HIPCHK(c, launch_sens_score((const SDesc *)(db + o_sd), (int)nT, n_blocks, c->stream));

    // thresholds: order statistics of the scores, then of the weights (threshold searches only)
    std::vector<inshr_tensor> sub(nT);
    for (int pass = 0; pass < 2; pass++) {
        for (uint32_t t = 0; t < nT; t++) {
            sub[t].data = pass == 0 ? sd[t].S : tensors[t].data;
            sub[t].n = tensors[t].n;
        }
        rc = run_search(c, sub.data(), nT, frac_grid.data(), (uint32_t)frac_grid.size(), 0.0, true);
        if (rc) return rc;
        const TState *hts = (const TState *)c->h_down.p;
        for (uint32_t t = 0; t < nT; t++) {
            uint32_t qp = 0, qo = 0;
            while (qp < c->grid.n_p && c->grid.p_ppm[qp] != cfg[t].prune_ppm) qp++;
            while (qo < c->grid.n_o && c->grid.o_ppm[qo] != cfg[t].outlier_ppm) qo++;
            if (qp == c->grid.n_p || qo == c->grid.n_o) return INSHR_E_INTERNAL;
            const u32 tp = hts[t].thr_mag[qp], to = hts[t].thr_mag[c->grid.n_p + qo];
            if (pass == 0) {
                sd[t].tau_os = to;
                if (sd[t].by_sens) sd[t].tau_p = tp;
            } else {
                sd[t].tau_om = to;
                if (!sd[t].by_sens) sd[t].tau_p = tp;
            }
        }
    }
    c->have_search = false;
    if ((rc = upload())) return rc;
    HIPCHK(c, launch_sens_partition((const SDesc *)(db + o_sd), (int)nT, n_blocks, (u32 *)(db + o_bk),
                                    (u32 *)(db + o_bp), (double *)(db + o_bq), (SInfo *)(db + o_si), c->stream));
    std::vector<SInfo> si(nT);
    HIPCHK(c, hipStreamSynchronize(c->stream));
    HIPCHK(c, hipMemcpy(si.data(), db + o_si, sizeof(SInfo) * nT, hipMemcpyDeviceToHost));
    for (uint32_t t = 0; t < nT; t++) {
        if (si[t].n_kept == 0) {
            c->last_err = "the thresholds leave tensor " + std::to_string(t) + " without quantized values";
            return INSHR_E_CONFIG;
        }
        if (si[t].n_outlier > out[t].outlier_cap) return INSHR_E_CAPACITY;
        sub[t].data = sd[t].Wm;
        sub[t].n = si[t].n_kept;
    }
    // the bins: the quantized values as tensors of their own, nothing pruned, nothing protected
    rc = run_search(c, sub.data(), nT, bin_grid.data(), (uint32_t)bin_grid.size(), 0.0, false);
    if (rc) return rc;
    c->have_search = false; // (the state describes the compacted values, not the caller's tensors)
    const Score *hsc = (const Score *)((const char *)c->h_down.p + sizeof(TState) * nT);
    const uint32_t n_bg = (uint32_t)bin_grid.size();
    std::vector<double> sse_q(nT), sq_q(nT);
    for (uint32_t t = 0; t < nT; t++) {
        const uint32_t gi = bin_of_t[t];
        sse_q[t] = hsc[(size_t)t * n_bg + gi].sse;
        sq_q[t] = hsc[(size_t)t * n_bg + gi].sumsq;
        sd[t].packed = (unsigned long long *)out[t].packed;
        sd[t].out_idx = out[t].outlier_idx;
        sd[t].out_val = out[t].outlier_val;
        sd[t].out_cap = out[t].outlier_cap;
        sd[t].codebook = out[t].codebook;
        sd[t].boundaries = out[t].boundaries;
        sd[t].bkeys = c->batch.bufs.tgt_key + (size_t)t * TGT_STRIDE; // (one pair: nothing pruned or protected)
        sd[t].cb = c->batch.bufs.codebook + ((size_t)t * n_bg + gi) * CB_STRIDE;
        sd[t].K = bins_of(cfg[t]);
        sd[t].sym_bits = symbol_bits(sd[t].K);
    }
    if ((rc = upload())) return rc;
    HIPCHK(c, hipMemsetAsync(db + o_fl, 0, 4, c->stream));
    HIPCHK(c, launch_sens_quant((const SDesc *)(db + o_sd), (int)nT, n_blocks, (const u32 *)(db + o_bp),
                                (u32 *)(db + o_fl), c->stream));
    u32 fl = 0;
    HIPCHK(c, hipStreamSynchronize(c->stream));
    HIPCHK(c, hipMemcpy(&fl, db + o_fl, 4, hipMemcpyDeviceToHost));
    if (fl & 2u) return INSHR_E_CAPACITY;
    for (uint32_t t = 0; t < nT; t++) {
        out[t].n_pruned = si[t].n_pruned;
        out[t].n_outlier = si[t].n_outlier;
        out[t].n_kept = si[t].n_kept;
        out[t].n_bins = sd[t].K;
        out[t].sym_bits = sd[t].sym_bits;
        memcpy(&out[t].tau_prune, &sd[t].tau_p, 4);
        memcpy(&out[t].tau_outlier, &sd[t].tau_om, 4);
        if (info) {
            memcpy(&info[t].tau_outlier_sens, &sd[t].tau_os, 4);
            info[t].sse = sse_q[t] + si[t].sq_pruned;
            info[t].sumsq = sq_q[t] + si[t].sq_pruned + si[t].sq_prot;
        }
    }
    return INSHR_OK;
}

int inshr_delta_bound(const inshr_codes *prev, const inshr_codes *cur, uint64_t *packed_words)
{
    if (!prev || !cur || !packed_words) return INSHR_E_ARG;
    if (prev->n != cur->n) return INSHR_E_SHAPE;
    uint32_t Kp = 0, Kc = 0;
    if (codes_bins(*prev, Kp) || codes_bins(*cur, Kc)) return INSHR_E_CONFIG;
    const uint32_t wB = symbol_bits(std::max(Kp, Kc));
    *packed_words = (prev->n * (uint64_t)wB + 63) / 64;
    return INSHR_OK;
}

int inshr_delta(inshr_ctx *c, const inshr_codes *prev, const uint32_t *const *prev_perm,
                const inshr_codes *cur, inshr_delta_out *out, uint32_t n_tensors)
{
    if (!c || !prev || !cur || !out || n_tensors == 0) return INSHR_E_ARG;
    std::vector<DDesc> dd(n_tensors);
    std::vector<u32> chunk_tensor;
    u64 dtile = 0, chunk = 0;
    bool any_scatter = false, any_gather = false, any_perm = false;
    for (uint32_t t = 0; t < n_tensors; t++) {
        uint64_t words = 0;
        int rc = inshr_delta_bound(&prev[t], &cur[t], &words);
        if (rc) return rc;
        const uint64_t n = prev[t].n;
        if (n == 0 || n >= (1ull << 32) || !prev[t].packed || !cur[t].packed) return INSHR_E_ARG;
        uint32_t Kp = 0, Kc = 0;
        (void)codes_bins(prev[t], Kp); // (checked by inshr_delta_bound)
        (void)codes_bins(cur[t], Kc);
        if (prev[t].sym_bits != symbol_bits(Kp) || cur[t].sym_bits != symbol_bits(Kc)) return INSHR_E_CONFIG;
        if (!out[t].packed || !out[t].group_off || out[t].packed_words < words) return INSHR_E_CAPACITY;
        if (out[t].group_off_entries && out[t].group_off_entries < Kp + 3u) return INSHR_E_CAPACITY;
        if (prev_perm && prev_perm[t] && out[t].perm) return INSHR_E_ARG; // a given permutation is not written again
        DDesc &d = dd[t];
        memset(&d, 0, sizeof(d));
        d.prev = (const unsigned long long *)prev[t].packed;
        d.cur = (const unsigned long long *)cur[t].packed;
        d.out = (unsigned long long *)out[t].packed;
        d.group_off = out[t].group_off;
        d.perm = out[t].perm;
        d.prev_perm = prev_perm ? prev_perm[t] : nullptr;
        d.n = n;
        d.out_words = words;
        d.wp = prev[t].sym_bits;
        d.wc = cur[t].sym_bits;
        d.Kp = Kp;
        d.B = std::max(Kp, Kc) + 2u;
        d.wB = symbol_bits(std::max(Kp, Kc));
        out[t].delta_bits = d.wB;
        d.dtile0 = dtile;
        d.chunk0 = chunk;
        const u64 nt = (n + DELTA_TILE - 1) / DELTA_TILE;
        d.n_chunks = (nt + DELTA_CHUNK - 1) / DELTA_CHUNK;
        for (u64 k = 0; k < d.n_chunks; k++) chunk_tensor.push_back(t);
        dtile += nt;
        chunk += d.n_chunks;
        if (d.prev_perm)
            any_gather = true;
        else if (d.perm)
            any_perm = true;
        else
            any_scatter = true;
    }
    HIPCHK(c, hipSetDevice(c->device));
    Carver cv;
    const size_t o_dd = cv.take(sizeof(DDesc) * n_tensors);
    const size_t o_ct = cv.take(sizeof(u32) * chunk_tensor.size());
    const size_t up_bytes = cv.off;
    const size_t o_ck = cv.take((size_t)chunk * DELTA_SS * 4);
    int rc = ensure_dev(c, c->aux_mem, cv.off);
    if (rc) return rc;
    rc = ensure_host(c, c->h_up, up_bytes);
    if (rc) return rc;
    // the staging buffer may still be in flight from an earlier asynchronous delta call
    HIPCHK(c, hipStreamSynchronize(c->stream));
    rc = take_delta_flags(c); // (of a call whose flags nobody has asked for yet)
    if (rc) return rc;
    char *hb = (char *)c->h_up.p, *db = (char *)c->aux_mem.p;
    memcpy(hb + o_dd, dd.data(), sizeof(DDesc) * n_tensors);
    memcpy(hb + o_ct, chunk_tensor.data(), sizeof(u32) * chunk_tensor.size());
    HIPCHK(c, hipMemcpyAsync(db, hb, up_bytes, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipMemsetAsync(c->delta_flags, 0, sizeof(u32), c->stream));
    c->delta_pending = true;
    HIPCHK(c, launch_delta((const DDesc *)(db + o_dd), (int)n_tensors, dtile, chunk,
                           (const u32 *)(db + o_ct), (u32 *)(db + o_ck), c->delta_flags, any_scatter,
                           any_perm, any_gather, c->lds_ordered, c->stream));
    return INSHR_OK;
}

int inshr_delta_static(inshr_ctx *c, const inshr_codes *prev, const inshr_codes *cur,
                       inshr_delta_out *out, uint32_t n_tensors)
{
    if (!c || !prev || !cur || !out || n_tensors == 0) return INSHR_E_ARG;
    if (n_tensors > (uint32_t)DELTA_STATIC_MAX_TENSORS) {
        c->last_err = "inshr_delta_static: more than " + std::to_string(DELTA_STATIC_MAX_TENSORS) + " tensors";
        return INSHR_E_CAPACITY;
    }
    DeltaStaticArgs a;
    memset(&a, 0, sizeof(a));
    a.n_tensors = n_tensors;
    u64 dtile = 0, chunk = 0;
    bool any_scatter = false, any_perm = false;
    for (uint32_t t = 0; t < n_tensors; t++) {
        uint64_t words = 0;
        int rc = inshr_delta_bound(&prev[t], &cur[t], &words);
        if (rc) return rc;
        const uint64_t n = prev[t].n;
        if (n == 0 || n >= (1ull << 32) || !prev[t].packed || !cur[t].packed) return INSHR_E_ARG;
        uint32_t Kp = 0, Kc = 0;
        (void)codes_bins(prev[t], Kp); // (checked by inshr_delta_bound)
        (void)codes_bins(cur[t], Kc);
        if (prev[t].sym_bits != symbol_bits(Kp) || cur[t].sym_bits != symbol_bits(Kc)) return INSHR_E_CONFIG;
        if (!out[t].packed || !out[t].group_off || out[t].packed_words < words) return INSHR_E_CAPACITY;
        if (out[t].group_off_entries && out[t].group_off_entries < Kp + 3u) return INSHR_E_CAPACITY;
        DDesc &d = a.dd[t];
        d.prev = (const unsigned long long *)prev[t].packed;
        d.cur = (const unsigned long long *)cur[t].packed;
        d.out = (unsigned long long *)out[t].packed;
        d.group_off = out[t].group_off;
        d.perm = out[t].perm;
        d.n = n;
        d.out_words = words;
        d.wp = prev[t].sym_bits;
        d.wc = cur[t].sym_bits;
        d.Kp = Kp;
        d.B = std::max(Kp, Kc) + 2u;
        d.wB = symbol_bits(std::max(Kp, Kc));
        out[t].delta_bits = d.wB;
        d.dtile0 = dtile;
        d.chunk0 = chunk;
        const u64 nt = (n + DELTA_TILE - 1) / DELTA_TILE;
        d.n_chunks = (nt + DELTA_CHUNK - 1) / DELTA_CHUNK;
        dtile += nt;
        chunk += d.n_chunks;
        if (d.perm)
            any_perm = true;
        else
            any_scatter = true;
    }
    if (chunk > (u64)DELTA_STATIC_MAX_CHUNKS) {
        c->last_err = "inshr_delta_static: the tensors need " + std::to_string(chunk) + " chunks of " +
                      std::to_string((u64)DELTA_TILE * DELTA_CHUNK) + " elements, the static scratch holds " +
                      std::to_string(DELTA_STATIC_MAX_CHUNKS);
        return INSHR_E_CAPACITY;
    }
    HIPCHK(c, hipSetDevice(c->device));
    c->static_pending = true;
    HIPCHK(c, launch_delta_static(c->device, a, dtile, chunk, any_scatter, any_perm, c->lds_ordered, c->stream));
    return INSHR_OK;
}

int inshr_dequantize(inshr_ctx *c, const inshr_dequant_in *in, float *const *out, uint32_t n_tensors)
{
    if (!c || !in || !out || n_tensors == 0 || n_tensors > 65535u) return INSHR_E_ARG;
    std::vector<RDesc> rd(n_tensors);
    u64 tile = 0, max_out = 0;
    for (uint32_t t = 0; t < n_tensors; t++) {
        const inshr_dequant_in &q = in[t];
        inshr_codes as_codes;
        as_codes.bits = q.bits;
        as_codes.bins = q.bins;
        uint32_t K = 0;
        if (codes_bins(as_codes, K)) return INSHR_E_CONFIG;
        if (q.n == 0 || q.n >= (1ull << 32) || !q.packed || !q.codebook || !out[t]) return INSHR_E_ARG;
        if (q.n_outlier && (!q.outlier_idx || !q.outlier_val)) return INSHR_E_ARG;
        if (q.n_outlier > q.n) return INSHR_E_SHAPE;
        RDesc &d = rd[t];
        memset(&d, 0, sizeof(d));
        d.packed = (const unsigned long long *)q.packed;
        d.codebook = q.codebook;
        d.out_idx = q.outlier_idx;
        d.out_val = q.outlier_val;
        d.dst = out[t];
        d.n = q.n;
        d.n_outlier = q.n_outlier;
        d.tile0 = tile;
        d.w = symbol_bits(K);
        d.K = K;
        d.val_bf16 = q.protected_bf16 ? 1u : 0u;
        tile += (q.n + DEQUANT_TILE - 1) / DEQUANT_TILE;
        max_out = std::max<u64>(max_out, q.n_outlier);
    }
    HIPCHK(c, hipSetDevice(c->device));
    Carver cv;
    const size_t o_rd = cv.take(sizeof(RDesc) * n_tensors);
    const size_t o_fl = cv.take(sizeof(u32) * (n_tensors + 1)); // flags, then symbol-1 counts
    const size_t up_bytes = cv.off;
    int rc = ensure_dev(c, c->aux_mem, cv.off);
    if (rc) return rc;
    rc = ensure_host(c, c->h_up, up_bytes);
    if (rc) return rc;
    rc = ensure_host(c, c->h_down, sizeof(u32));
    if (rc) return rc;
    HIPCHK(c, hipStreamSynchronize(c->stream)); // the staging buffer may still be in flight
    char *hb = (char *)c->h_up.p, *db = (char *)c->aux_mem.p;
    memset(hb, 0, up_bytes);
    memcpy(hb + o_rd, rd.data(), sizeof(RDesc) * n_tensors);
    HIPCHK(c, hipMemcpyAsync(db, hb, up_bytes, hipMemcpyHostToDevice, c->stream));
    u32 *flags = (u32 *)(db + o_fl);
    HIPCHK(c, launch_dequantize((const RDesc *)(db + o_rd), (int)n_tensors, tile, max_out, flags,
                                flags + 1, c->n_cu, c->stream));
    HIPCHK(c, hipMemcpyAsync(c->h_down.p, flags, sizeof(u32), hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    const u32 f = *(const u32 *)c->h_down.p;
    if (f & RF_SYMBOL) return INSHR_E_ARG;
    if (f & RF_LIST) return INSHR_E_SHAPE;
    return INSHR_OK;
}

int inshr_reconstruct(inshr_ctx *c, const inshr_codes *prev, const inshr_delta_out *delta,
                      inshr_codes_out *cur, uint32_t n_tensors)
{
    if (!c || !prev || !delta || !cur || n_tensors == 0) return INSHR_E_ARG;
    std::vector<DDesc> dd(n_tensors);
    std::vector<XDesc> xd(n_tensors);
    std::vector<u32> chunk_tensor;
    u64 dtile = 0, chunk = 0;
    for (uint32_t t = 0; t < n_tensors; t++) {
        const uint64_t n = prev[t].n;
        inshr_codes cur_codes;
        cur_codes.bits = cur[t].bits;
        cur_codes.bins = cur[t].bins;
        uint32_t Kp = 0, Kc = 0;
        if (codes_bins(prev[t], Kp) || codes_bins(cur_codes, Kc)) return INSHR_E_CONFIG;
        if (prev[t].sym_bits != symbol_bits(Kp)) return INSHR_E_CONFIG;
        if (n == 0 || n >= (1ull << 32) || !prev[t].packed || !delta[t].packed || !cur[t].packed) return INSHR_E_ARG;
        const uint32_t wB = symbol_bits(std::max(Kp, Kc));
        if (delta[t].delta_bits != wB) return INSHR_E_CONFIG;
        if (delta[t].packed_words < (n * wB + 63) / 64) return INSHR_E_CAPACITY;
        const uint32_t wc = symbol_bits(Kc);
        if (cur[t].packed_words < (n * wc + 63) / 64) return INSHR_E_CAPACITY;
        DDesc &d = dd[t];
        memset(&d, 0, sizeof(d));
        d.prev = (const unsigned long long *)prev[t].packed;
        d.out = (unsigned long long *)delta[t].packed; // read only on this side
        d.n = n;
        d.out_words = (n * wB + 63) / 64;
        d.wp = prev[t].sym_bits;
        d.wc = wc;
        d.Kp = Kp;
        d.B = std::max(Kp, Kc) + 2u;
        d.wB = wB;
        d.dtile0 = dtile;
        d.chunk0 = chunk;
        const u64 nt = (n + DELTA_TILE - 1) / DELTA_TILE;
        d.n_chunks = (nt + DELTA_CHUNK - 1) / DELTA_CHUNK;
        for (u64 k = 0; k < d.n_chunks; k++) chunk_tensor.push_back(t);
        dtile += nt;
        chunk += d.n_chunks;
        XDesc &x = xd[t];
        memset(&x, 0, sizeof(x));
        x.cur_out = (unsigned long long *)cur[t].packed;
        x.group_off_in = delta[t].group_off;
        x.Sc = Kc + 2u;
    }
    HIPCHK(c, hipSetDevice(c->device));
    Carver cv;
    const size_t o_dd = cv.take(sizeof(DDesc) * n_tensors);
    const size_t o_xd = cv.take(sizeof(XDesc) * n_tensors);
    const size_t o_ct = cv.take(sizeof(u32) * chunk_tensor.size());
    const size_t o_fl = cv.take(sizeof(u32));
    const size_t up_bytes = cv.off;
    const size_t o_go = cv.take(sizeof(u64) * (DELTA_SS + 8) * n_tensors); // group offsets from prev
    const size_t o_ck = cv.take((size_t)chunk * DELTA_SS * 4);
    int rc = ensure_dev(c, c->aux_mem, cv.off);
    if (rc) return rc;
    rc = ensure_host(c, c->h_up, up_bytes);
    if (rc) return rc;
    rc = ensure_host(c, c->h_down, sizeof(u32));
    if (rc) return rc;
    HIPCHK(c, hipStreamSynchronize(c->stream));
    char *hb = (char *)c->h_up.p, *db = (char *)c->aux_mem.p;
    for (uint32_t t = 0; t < n_tensors; t++) dd[t].group_off = (u64 *)(db + o_go) + (size_t)t * (DELTA_SS + 8);
    memset(hb, 0, up_bytes);
    memcpy(hb + o_dd, dd.data(), sizeof(DDesc) * n_tensors);
    memcpy(hb + o_xd, xd.data(), sizeof(XDesc) * n_tensors);
    memcpy(hb + o_ct, chunk_tensor.data(), sizeof(u32) * chunk_tensor.size());
    HIPCHK(c, hipMemcpyAsync(db, hb, up_bytes, hipMemcpyHostToDevice, c->stream));
    u32 *flags = (u32 *)(db + o_fl);
    HIPCHK(c, launch_reconstruct((const DDesc *)(db + o_dd), (const XDesc *)(db + o_xd),
                                 (int)n_tensors, chunk, (const u32 *)(db + o_ct),
                                 (u32 *)(db + o_ck), flags, c->lds_ordered, c->stream));
    HIPCHK(c, hipMemcpyAsync(c->h_down.p, flags, sizeof(u32), hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    const u32 f = *(const u32 *)c->h_down.p;
    if (f & RF_ORDER) {
        c->last_err = "reconstruct: ranks from returning LDS atomics disagree with ballot ranks (set INSHR_NO_LDS_ORDER=1)";
        return INSHR_E_INTERNAL;
    }
    if (f & RF_GROUPS) return INSHR_E_SHAPE;
    if (f & RF_DELTA) return INSHR_E_ARG;
    return INSHR_OK;
}

} // extern "C"
