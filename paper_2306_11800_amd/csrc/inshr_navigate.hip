// Search-space navigation over a score table (Sec. 5): guided exhaustive search (Alg. 4) and
// delta-neighbourhood search.  Host code only: the sweeps have already scored every configuration
// of the grid, so a "trial" here is one read of the table; the calls say which configurations a
// caller that pays per trial would have evaluated, and which one it ends up with.
#include "../../include/inshr.h"
#include <algorithm>
#include <cstdint>
#include <vector>

namespace {

struct Cube {
    const inshr_score *scores;
    const uint32_t *cell_cfg;
    uint32_t d[3];
    double eps;
    std::vector<uint8_t> seen;
    uint32_t trials = 0;

    size_t at(const uint32_t c[3]) const { return ((size_t)c[0] * d[1] + c[1]) * d[2] + c[2]; }
    const inshr_score &read(const uint32_t c[3])
    {
        const size_t i = at(c);
        if (!seen[i]) {
            seen[i] = 1;
            trials++;
        }
        return scores[cell_cfg[i]];
    }
    bool feasible(const inshr_score &s) const { return s.sse <= eps * s.sumsq; }
};

struct Found {
    bool any = false;
    uint32_t c[3] = {0, 0, 0};
    uint64_t cost = 0;
    uint32_t cfg = 0;
    void offer(const uint32_t p[3], uint64_t cost_, uint32_t cfg_)
    { // a strictly better cell replaces the incumbent (ties: the lower configuration index)
        if (!any || cost_ < cost || (cost_ == cost && cfg_ < cfg)) {
            any = true;
            cost = cost_;
            cfg = cfg_;
            std::copy(p, p + 3, c);
        }
    }
};

// box [lo, hi) along every axis
void guided(Cube &q, const uint32_t lo[3], const uint32_t hi[3], Found &best)
{
    uint32_t len[3], L = 0;
    for (int a = 0; a < 3; a++) {
        if (hi[a] <= lo[a]) return;
        len[a] = hi[a] - lo[a];
        L = std::max(L, len[a]);
    }
    // the diagonal, scaled to the longest axis: from the most aggressive corner to the most
    // conservative one, no axis ever steps back
    Found diag;
    for (uint32_t t = 0; t < L; t++) {
        uint32_t p[3];
        for (int a = 0; a < 3; a++) p[a] = lo[a] + (uint32_t)(((uint64_t)t * len[a]) / L);
        if (t == L - 1)
            for (int a = 0; a < 3; a++) p[a] = hi[a] - 1;
        const inshr_score &s = q.read(p);
        if (q.feasible(s)) diag.offer(p, s.cost_bits, q.cell_cfg[q.at(p)]);
    }
    if (!diag.any) return; // the most conservative corner is infeasible: so is the box
    best.offer(diag.c, diag.cost, diag.cfg);
    // split at the incumbent; of the eight parts, the all-high one (which holds the incumbent) only
    // costs more and the all-low one is more aggressive than the infeasible diagonal cell before
    for (int m = 1; m < 7; m++) {
        uint32_t l2[3], h2[3];
        for (int a = 0; a < 3; a++) {
            if ((m >> a) & 1) {
                l2[a] = diag.c[a];
                h2[a] = hi[a];
            } else {
                l2[a] = lo[a];
                h2[a] = diag.c[a];
            }
        }
        guided(q, l2, h2, best);
    }
}

bool check(const inshr_score *scores, const uint32_t *cell_cfg, const uint32_t *dims)
{
    if (!scores || !cell_cfg || !dims) return false;
    for (int a = 0; a < 3; a++)
        if (dims[a] == 0 || dims[a] > 255) return false;
    return true;
}

} // namespace

extern "C" int inshr_guided_search(const inshr_score *scores, const uint32_t *cell_cfg,
                                   const uint32_t dims[3], double eps, uint32_t *best_cell,
                                   uint32_t *feasible, uint32_t *trials, uint8_t *visited)
{
    if (!check(scores, cell_cfg, dims) || !best_cell || !feasible || !trials) return INSHR_E_ARG;
    Cube q{scores, cell_cfg, {dims[0], dims[1], dims[2]}, eps, {}, 0};
    q.seen.assign((size_t)dims[0] * dims[1] * dims[2], 0);
    const uint32_t lo[3] = {0, 0, 0};
    Found best;
    guided(q, lo, q.d, best);
    if (best.any) {
        *best_cell = best.c[0] << 16 | best.c[1] << 8 | best.c[2];
    } else {
        *best_cell = (dims[0] - 1) << 16 | (dims[1] - 1) << 8 | (dims[2] - 1);
    }
    *feasible = best.any ? 1u : 0u;
    *trials = q.trials;
    if (visited) std::copy(q.seen.begin(), q.seen.end(), visited);
    return INSHR_OK;
}

extern "C" int inshr_neighbourhood_search(const inshr_score *scores, const uint32_t *cell_cfg,
                                          const uint32_t dims[3], uint32_t prev_cell, uint32_t e,
                                          double eps, uint32_t *best_cell, uint32_t *feasible,
                                          uint32_t *trials)
{
    if (!check(scores, cell_cfg, dims) || !best_cell || !feasible || !trials) return INSHR_E_ARG;
    const uint32_t pc[3] = {prev_cell >> 16, (prev_cell >> 8) & 255u, prev_cell & 255u};
    for (int a = 0; a < 3; a++)
        if (pc[a] >= dims[a]) return INSHR_E_ARG;
    Cube q{scores, cell_cfg, {dims[0], dims[1], dims[2]}, eps, {}, 0};
    q.seen.assign((size_t)dims[0] * dims[1] * dims[2], 0);
    struct Cand {
        uint64_t cost;
        uint32_t cfg, c[3];
    };
    std::vector<Cand> cand;
    uint32_t c[3];
    for (c[0] = 0; c[0] < dims[0]; c[0]++)
        for (c[1] = 0; c[1] < dims[1]; c[1]++)
            for (c[2] = 0; c[2] < dims[2]; c[2]++) {
                uint32_t dist = 0;
                bool none_above = true, some_below = false;
                for (int a = 0; a < 3; a++) {
                    dist += c[a] > pc[a] ? c[a] - pc[a] : pc[a] - c[a];
                    none_above &= c[a] <= pc[a];
                    some_below |= c[a] < pc[a];
                }
                if (dist > e || (none_above && some_below)) continue;
                // (the order of the trials comes from the cost model, which needs no trial: it
                // depends on the class counts alone)
                const uint32_t cfg = cell_cfg[q.at(c)];
                cand.push_back({scores[cfg].cost_bits, cfg, {c[0], c[1], c[2]}});
            }
    std::sort(cand.begin(), cand.end(), [](const Cand &x, const Cand &y) {
        return x.cost != y.cost ? x.cost < y.cost : x.cfg < y.cfg;
    });
    *feasible = 0u;
    *best_cell = prev_cell;
    for (const Cand &k : cand) {
        if (q.feasible(q.read(k.c))) {
            *feasible = 1u;
            *best_cell = k.c[0] << 16 | k.c[1] << 8 | k.c[2];
            break;
        }
    }
    *trials = q.trials;
    return INSHR_OK;
}
