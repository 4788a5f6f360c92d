// Exact solver for the resource-allocation model of Sec. III-B ("Optimization Formulation"),
// at kernel-group ("unit") granularity.  CPU only, integer arithmetic only.
//
// Structure used: the workers couple only through S_D = D * sum_w CUAverage_w (D = lcm of the
// workers' kernel counts), the objective is  (sum_w B_w) * phi(S_D)  with phi non-decreasing in all
// three overlap modes, and for a fixed S_D it increases with sum_w B_w.  Hence
//   1. per worker, a dynamic programme over (unit, previous configuration, switches left, CU-sum)
//      yields  f_w[U] = min B_w  subject to the switch budget, U = sum_g n_g * c_g;
//   2. only Pareto-optimal (U smaller, B smaller) points of f_w can be part of an optimum (ties
//      prefer the smaller S_D), so workers are combined front by front (a Minkowski sum, pruned);
//   3. the optimum of (sum B) * phi(S) over the combined front is the answer;
//   4. the lexicographically smallest optimal assignment is rebuilt worker by worker, unit by unit,
//      taking at every position the smallest configuration index from which the remaining target
//      is still reachable exactly.
#include <algorithm>
#include <cstdint>
#include <functional>
#include <limits>
#include <map>
#include <numeric>
#include <string>
#include <vector>

#include "eclip.h"

namespace eclip {

typedef unsigned __int128 u128;
static const uint64_t INF = std::numeric_limits<uint64_t>::max();

struct Point { uint64_t s; uint64_t b; };            // (scaled CU sum, latency sum)

// Pareto front: s strictly increasing, b strictly decreasing.
static std::vector<Point> prune(std::vector<Point> v)
{
    std::sort(v.begin(), v.end(), [](const Point &x, const Point &y) { return x.s != y.s ? x.s < y.s : x.b < y.b; });
    std::vector<Point> out;
    uint64_t best = INF;
    for (const Point &p : v)
        if (p.b < best) { out.push_back(p); best = p.b; }
    return out;
}

struct WorkerDP {
    int G = 0, C = 0, SM = 0;                 // units, configs, switch budget
    std::vector<uint32_t> n;                  // kernels per unit
    std::vector<uint32_t> cq;                 // config CU counts divided by their gcd
    const uint64_t *beta = nullptr;           // [G][C]
    uint64_t switch_cost = 0;                 // added to the latency at every configuration switch
    std::vector<int> allowed;                 // configurations this run may use (all, or a subset)
    uint32_t umax = 0;                        // largest reduced CU sum
    // h[g][c_prev][s_left][u] = min latency of units g..G-1 given unit g-1 used c_prev, s_left switches
    // remain and the units g..G-1 must add up to reduced CU sum u.  g = 0 uses c_prev = C ("none").
    std::vector<uint64_t> h;
    std::vector<uint32_t> rem_max;            // rem_max[g] = max reduced CU sum of units g..G-1
    size_t idx(int g, int cp, int sl, uint32_t u) const
    {
        return (((size_t)g * (C + 1) + cp) * (SM + 1) + sl) * (umax + 1) + u;
    }
    bool is_allowed(int c) const { return std::find(allowed.begin(), allowed.end(), c) != allowed.end(); }
    size_t states() const { return (size_t)(G + 1) * (C + 1) * (SM + 1) * ((size_t)umax + 1); }

    void run()
    {
        h.assign(states(), INF);
        for (int cp = 0; cp <= C; ++cp)
            for (int sl = 0; sl <= SM; ++sl) h[idx(G, cp, sl, 0)] = 0;
        for (int g = G - 1; g >= 0; --g)
            for (int cp = 0; cp <= C; ++cp) {
                if (g == 0 && cp != C) continue;
                if (g > 0 && (cp == C || !is_allowed(cp))) continue;
                for (int sl = 0; sl <= SM; ++sl)
                    for (uint32_t u = 0; u <= rem_max[g]; ++u) {
                        uint64_t best = INF;
                        for (int c : allowed) {
                            const bool sw = (g > 0 && c != cp);
                            if (sw && sl == 0) continue;
                            const uint32_t du = n[g] * cq[c];
                            if (du > u) continue;
                            const uint64_t t = h[idx(g + 1, c, sl - (sw ? 1 : 0), u - du)];
                            if (t == INF) continue;
                            const uint64_t v = t + beta[(size_t)g * C + c] + (sw ? switch_cost : 0);
                            if (v < best) best = v;
                        }
                        h[idx(g, cp, sl, u)] = best;
                    }
            }
    }
    uint64_t f(uint32_t u) const { return h[idx(0, C, SM, u)]; }
    // lexicographically smallest assignment reaching exactly (u, f(u))
    void rebuild(uint32_t u, uint32_t *out, uint32_t *switches) const
    {
        int cp = C, sl = SM;
        uint32_t sw_count = 0;
        for (int g = 0; g < G; ++g) {
            const uint64_t target = h[idx(g, cp, sl, u)];
            for (int c : allowed) {                 // ascending: the first match is the lexicographic minimum
                const bool sw = (g > 0 && c != cp);
                if (sw && sl == 0) continue;
                const uint32_t du = n[g] * cq[c];
                if (du > u) continue;
                const uint64_t t = h[idx(g + 1, c, sl - (sw ? 1 : 0), u - du)];
                if (t == INF || t + beta[(size_t)g * C + c] + (sw ? switch_cost : 0) != target) continue;
                out[g] = (uint32_t)c;
                if (sw) { --sl; ++sw_count; }
                cp = c;
                u -= du;
                break;
            }
        }
        *switches = sw_count;
    }
};

static bool mul_overflows(uint64_t a, uint64_t b) { return b != 0 && a > INF / b; }

// returns "" on success, otherwise an error text; *limit set when the failure is a capacity limit
std::string solve_alloc(const eclip_alloc_problem *p, uint32_t *cfg_out, eclip_u128 *obj_out, uint32_t *sw_out, bool *limit)
{
    *limit = false;
    if (!p || !cfg_out) return "null problem or output";
    if (!p->configs || !p->units_of_worker || !p->n_kernels || !p->beta) return "null array in problem";
    if (p->n_configs == 0 || p->n_configs > 64) return "n_configs must be 1..64";
    if (p->n_workers == 0 || p->n_workers > 16) return "n_workers must be 1..16";
    if (p->total_cus == 0) return "total_cus must be positive";
    if (p->overlap_mode > ECLIP_OVERLAP_TABLE) return "unknown overlap mode";
    for (uint32_t c = 0; c < p->n_configs; ++c) {
        if (p->configs[c] == 0) return "configuration with zero CUs";
        if (c && p->configs[c] <= p->configs[c - 1]) return "configs must be strictly increasing";
    }
    if (p->overlap_mode == ECLIP_OVERLAP_TABLE) {
        if (!p->alpha_ppm || p->n_alpha == 0 || p->granule == 0) return "TABLE mode needs alpha_ppm and granule";
        for (uint32_t i = 1; i < p->n_alpha; ++i)
            if (p->alpha_ppm[i] < p->alpha_ppm[i - 1]) return "alpha_ppm must be non-decreasing";
    }
    const int W = (int)p->n_workers, C = (int)p->n_configs;
    // configuration subsets a worker may draw from: all of them, or every subset of at most K configurations, K being the
    // worker's own limit (max_configs_of_worker) or the common one (max_configs)
    auto subsets_for = [&](int K, std::vector<std::vector<int>> &subsets) -> bool {
        subsets.clear();
        if (K <= 0 || K >= C) {
            std::vector<int> all(C);
            std::iota(all.begin(), all.end(), 0);
            subsets.push_back(all);
            return true;
        }
        std::vector<int> cur;
        // subsets of exactly K configurations (smaller ones are contained in them), in lexicographic order
        std::function<void(int)> rec = [&](int start) {
            if ((int)cur.size() == K) { subsets.push_back(cur); return; }
            for (int c = start; c < C; ++c) { cur.push_back(c); rec(c + 1); cur.pop_back(); }
        };
        rec(0);
        return subsets.size() <= 4096;
    };
    std::vector<std::vector<std::vector<int>>> subsets_w(W);
    for (int w = 0; w < W; ++w) {
        const int K = p->max_configs_of_worker ? (int)p->max_configs_of_worker[w] : (int)p->max_configs;
        if (!subsets_for(K, subsets_w[w])) { *limit = true; return "too many configuration subsets (max_configs)"; }
    }
    uint32_t cg = 0;
    for (int c = 0; c < C; ++c) cg = std::gcd(cg, p->configs[c]);

    std::vector<WorkerDP> dp(W);
    std::vector<uint64_t> Nw(W);
    size_t unit0 = 0;
    uint64_t D = 1;
    uint64_t beta_total_max = 0;
    for (int w = 0; w < W; ++w) {
        WorkerDP &d = dp[w];
        d.G = (int)p->units_of_worker[w];
        if (d.G == 0) return "worker with no units";
        d.C = C;
        d.SM = (int)std::min<uint32_t>(p->switch_max, (uint32_t)(d.G - 1));
        d.n.assign(p->n_kernels + unit0, p->n_kernels + unit0 + d.G);
        d.beta = p->beta + unit0 * C;
        d.switch_cost = p->switch_cost_ns;
        d.cq.resize(C);
        for (int c = 0; c < C; ++c) d.cq[c] = p->configs[c] / cg;
        uint64_t nsum = 0, bmax = 0;
        for (int g = 0; g < d.G; ++g) {
            if (d.n[g] == 0) return "unit with zero kernels";
            nsum += d.n[g];
            uint64_t m = 0;
            for (int c = 0; c < C; ++c) m = std::max(m, d.beta[(size_t)g * C + c]);
            if (bmax > INF - m) { *limit = true; return "latency sum overflows 64 bits"; }
            bmax += m;
            if (g > 0) {
                if (bmax > INF - p->switch_cost_ns) { *limit = true; return "latency sum overflows 64 bits"; }
                bmax += p->switch_cost_ns;
            }
        }
        if (beta_total_max > INF - bmax) { *limit = true; return "latency sum overflows 64 bits"; }
        beta_total_max += bmax;
        if (nsum * d.cq[C - 1] > (1u << 24)) { *limit = true; return "CU-sum range too large"; }
        d.umax = (uint32_t)(nsum * d.cq[C - 1]);
        d.rem_max.assign(d.G + 1, 0);
        for (int g = d.G - 1; g >= 0; --g) d.rem_max[g] = d.rem_max[g + 1] + d.n[g] * d.cq[C - 1];
        if (d.states() > ((size_t)1 << 25)) { *limit = true; return "instance exceeds the solver's state budget (2^25 states per worker)"; }
        Nw[w] = nsum;
        const uint64_t l = D / std::gcd(D, nsum);
        if (mul_overflows(l, nsum)) { *limit = true; return "lcm of kernel counts overflows"; }
        D = l * nsum;
        unit0 += d.G;
    }
    // S_D <= D * W * cmax ; objective <= beta_total_max * (T*D + S_D): keep within 128 bits with margin
    {
        const u128 smax = (u128)D * (u128)W * p->configs[C - 1];
        const u128 fac = (u128)p->total_cus * D + smax;
        if (smax >> 62 || fac >> 63) { *limit = true; return "scaled CU sums exceed 62 bits"; }
    }
    // per-worker fronts in the common scale: s = U_reduced * cg * (D / N_w); with a subset limit the front is the
    // Pareto union over the subsets
    std::vector<std::vector<Point>> front(W);
    std::vector<uint64_t> mult(W);
    for (int w = 0; w < W; ++w) {
        mult[w] = (uint64_t)cg * (D / Nw[w]);
        std::vector<Point> v;
        for (const std::vector<int> &sub : subsets_w[w]) {
            dp[w].allowed = sub;
            dp[w].run();
            for (uint32_t u = 0; u <= dp[w].umax; ++u) {
                const uint64_t b = dp[w].f(u);
                if (b != INF) v.push_back(Point{(uint64_t)u * mult[w], b});
            }
        }
        front[w] = prune(std::move(v));
    }
    // suffix fronts R[w] = front[w] (+) front[w+1] (+) ... ; R[W] = {(0,0)}
    std::vector<std::vector<Point>> R(W + 1);
    R[W] = {Point{0, 0}};
    for (int w = W - 1; w >= 0; --w) {
        if (front[w].size() * R[w + 1].size() > ((size_t)1 << 27)) { *limit = true; return "front product exceeds the solver's budget"; }
        std::vector<Point> v;
        v.reserve(front[w].size() * R[w + 1].size());
        for (const Point &a : front[w])
            for (const Point &b : R[w + 1]) v.push_back(Point{a.s + b.s, a.b + b.b});
        R[w] = prune(std::move(v));
    }
    // objective over the combined front
    const u128 TD = (u128)p->total_cus * D;
    auto phi = [&](uint64_t s) -> u128 {
        const u128 excess = (u128)s > TD ? (u128)s - TD : 0;
        if (p->overlap_mode == ECLIP_OVERLAP_EXCESS) return TD + excess;
        if (p->overlap_mode == ECLIP_OVERLAP_LITERAL) return TD + s;
        u128 gi = excess / ((u128)D * p->granule);
        if (gi > p->n_alpha - 1) gi = p->n_alpha - 1;
        return (u128)1000000u + p->alpha_ppm[(size_t)gi];
    };
    if (p->overlap_mode == ECLIP_OVERLAP_TABLE && p->alpha_ppm[p->n_alpha - 1] > (INF >> 2)) { *limit = true; return "alpha_ppm too large"; }
    u128 best = 0;
    Point bp{0, 0};
    bool have = false;
    for (const Point &q : R[0]) {           // s ascending: the first minimum has the smallest S_D
        const u128 j = (u128)q.b * phi(q.s);
        if (!have || j < best) { best = j; bp = q; have = true; }
    }
    if (!have) return "no feasible assignment";
    if (obj_out) { obj_out->lo = (uint64_t)best; obj_out->hi = (uint64_t)(best >> 64); }

    // rebuild, worker-major lexicographic
    uint64_t s_left = bp.s, b_left = bp.b;
    unit0 = 0;
    for (int w = 0; w < W; ++w) {
        // candidate front points of worker w whose remainder lies exactly on R[w+1]
        std::vector<uint32_t> best_assign, cur(dp[w].G);
        uint32_t best_sw = 0, cur_sw = 0;
        Point chosen{0, 0};
        bool found = false;
        for (const Point &a : front[w]) {
            if (a.s > s_left || a.b > b_left) continue;
            const Point need{s_left - a.s, b_left - a.b};
            auto it = std::lower_bound(R[w + 1].begin(), R[w + 1].end(), need,
                                       [](const Point &x, const Point &y) { return x.s < y.s; });
            if (it == R[w + 1].end() || it->s != need.s || it->b != need.b) continue;
            for (const std::vector<int> &sub : subsets_w[w]) {
                dp[w].allowed = sub;
                dp[w].run();
                const uint32_t u = (uint32_t)(a.s / mult[w]);
                if (dp[w].f(u) != a.b) continue;
                dp[w].rebuild(u, cur.data(), &cur_sw);
                if (!found || cur < best_assign) { best_assign = cur; best_sw = cur_sw; chosen = a; found = true; }
            }
        }
        if (!found) return "internal error: optimum not reconstructible";
        for (int g = 0; g < dp[w].G; ++g) cfg_out[unit0 + g] = best_assign[g];
        if (sw_out) sw_out[w] = best_sw;
        s_left -= chosen.s;
        b_left -= chosen.b;
        unit0 += dp[w].G;
    }
    return "";
}

// ------------------------------------------------------------------------------------------------------------------
// The two comparison policies of Sec. IV ("Spatial Partitioning Scenarios"), on the same tables as the optimizer.
// Both are direct rules, no search; all comparisons are exact integer arithmetic.
// ------------------------------------------------------------------------------------------------------------------
static std::string check_tables(const eclip_alloc_problem *p, const uint32_t *cfg_out)
{
    if (!p || !cfg_out) return "null problem or output";
    if (!p->configs || !p->units_of_worker || !p->beta) return "null array in problem";
    if (p->n_configs == 0 || p->n_configs > 64) return "n_configs must be 1..64";
    if (p->n_workers == 0 || p->n_workers > 16) return "n_workers must be 1..16";
    for (uint32_t c = 0; c < p->n_configs; ++c) {
        if (p->configs[c] == 0) return "configuration with zero CUs";
        if (c && p->configs[c] <= p->configs[c - 1]) return "configs must be strictly increasing";
    }
    for (uint32_t w = 0; w < p->n_workers; ++w)
        if (p->units_of_worker[w] == 0) return "worker with no units";
    return "";
}

// Model-Wise (Sec. II-A, Sec. IV): one configuration per worker for the whole request -- the smallest CU count whose
// request latency (sum of the worker's unit latencies at that configuration) stays within slo_num / slo_den times
// the latency at the largest configuration (the QoS convention of Sec. II-A: 3x the solo latency).
std::string policy_model_wise(const eclip_alloc_problem *p, uint32_t slo_num, uint32_t slo_den, uint32_t *cfg_out, uint32_t *sw_out)
{
    std::string err = check_tables(p, cfg_out);
    if (!err.empty()) return err;
    if (slo_den == 0 || slo_num < slo_den) return "the latency target must be a ratio >= 1";
    const uint32_t C = p->n_configs;
    size_t unit0 = 0;
    for (uint32_t w = 0; w < p->n_workers; ++w) {
        const uint32_t G = p->units_of_worker[w];
        std::vector<u128> tot(C, 0);
        for (uint32_t g = 0; g < G; ++g)
            for (uint32_t c = 0; c < C; ++c) tot[c] += p->beta[(unit0 + g) * C + c];
        uint32_t pick = C - 1;
        for (uint32_t c = 0; c < C; ++c)
            if (tot[c] * slo_den <= tot[C - 1] * slo_num) { pick = c; break; }
        for (uint32_t g = 0; g < G; ++g) cfg_out[unit0 + g] = pick;
        if (sw_out) sw_out[w] = 0;
        unit0 += G;
    }
    return "";
}

// Kernel-Wise on pre-allocated streams (Sec. IV, KW-Prealloc): every unit runs at its own minimum-CU threshold
// (Sec. III-B, "Minimum CU Threshold Profiling": the fewest CUs with no noticeable slowdown), read here as the
// smallest configuration c with 100 * beta[c] <= (100 + tol_pct) * beta[largest configuration]; a switch is charged
// wherever consecutive units differ (the KW-Prealloc column of Table I).
std::string policy_kernel_wise(const eclip_alloc_problem *p, uint32_t tol_pct, uint32_t *cfg_out, uint32_t *sw_out)
{
    std::string err = check_tables(p, cfg_out);
    if (!err.empty()) return err;
    if (tol_pct > 10000) return "tolerance above 10000 percent";
    const uint32_t C = p->n_configs;
    size_t unit0 = 0;
    for (uint32_t w = 0; w < p->n_workers; ++w) {
        const uint32_t G = p->units_of_worker[w];
        uint32_t sw = 0;
        for (uint32_t g = 0; g < G; ++g) {
            const uint64_t *b = p->beta + (unit0 + g) * C;
            uint32_t pick = C - 1;
            for (uint32_t c = 0; c < C; ++c)
                if ((u128)b[c] * 100u <= (u128)b[C - 1] * (100u + tol_pct)) { pick = c; break; }
            cfg_out[unit0 + g] = pick;
            if (g && pick != cfg_out[unit0 + g - 1]) ++sw;
        }
        if (sw_out) sw_out[w] = sw;
        unit0 += G;
    }
    return "";
}

}  // namespace eclip
