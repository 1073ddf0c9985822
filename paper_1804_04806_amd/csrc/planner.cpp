#include "planner.h"

#include <algorithm>
#include <numeric>

namespace ucd {

bool policy_allows(int policy, int B, int b)
{
    if (b < 1 || b > B) return false;
    switch (policy) {
    case 0: return b == B;                 // undivided
    case 1: return (b & (b - 1)) == 0 || b == B;  // powerOfTwo: {2^0, 2^1, ..., B}: powers of two and B itself
    case 2: return true;                   // all
    default: return false;
    }
}

std::vector<int> policy_sizes(int policy, int B)
{
    std::vector<int> s;
    for (int b = 1; b <= B; ++b)
        if (policy_allows(policy, B, b)) s.push_back(b);
    return s;
}

static inline bool feasible(const Table &tab, int a, int b, size_t limit)
{
    return tab.time(a, b) != kTimeInf && tab.wsize(a, b) != kWsNa && tab.wsize(a, b) <= limit;
}

// ---- WR ------------------------------------------------------------------------------------
// T(b) = min_{b_mu = 1..b} T_mu(b_mu) + T(b - b_mu), T(0) = 0 (Section 3.2, step 2).
bool wr_plan(const Table &tab, size_t ws_limit, int policy, Config &out)
{
    const int B = tab.B;
    std::vector<uint64_t> t_mu(B + 1, kTimeInf);  // fastest fitting algorithm per size (step 1's c_mu)
    std::vector<int> a_mu(B + 1, -1);
    for (int b : policy_sizes(policy, B))
        for (int a = 0; a < tab.n_algo; ++a)
            if (feasible(tab, a, b, ws_limit) && tab.time(a, b) < t_mu[b]) {
                t_mu[b] = tab.time(a, b);
                a_mu[b] = a;
            }
    std::vector<uint64_t> T(B + 1, kTimeInf);
    std::vector<int> first(B + 1, 0);
    T[0] = 0;
    for (int b = 1; b <= B; ++b)
        for (int bm = b; bm >= 1; --bm) {  // descending: ties keep the largest first part
            if (t_mu[bm] == kTimeInf || T[b - bm] == kTimeInf) continue;
            uint64_t c = t_mu[bm] + T[b - bm];
            if (c < T[b]) {
                T[b] = c;
                first[b] = bm;
            }
        }
    if (T[B] == kTimeInf) return false;
    out.micro.clear();
    out.cost = T[B];
    out.ws = 0;
    for (int b = B; b > 0; b -= first[b]) {
        int bm = first[b];
        out.micro.push_back({a_mu[bm], bm});
        out.ws = std::max(out.ws, tab.wsize(a_mu[bm], bm));
    }
    return true;
}

// ---- desirable sets ------------------------------------------------------------------------
namespace {
struct Cand {
    uint64_t t;
    size_t m;
    int parts;
    int b_mu, algo, prev;  // {c_mu} + C(b - b_mu)[prev]
};
}  // namespace

// D(C): drop c iff a different point is no slower and no bigger; equal points keep the one with
// the fewest micro-batches.  Result sorted by m ascending, t strictly descending.
static void prune(std::vector<Cand> &c)
{
    std::sort(c.begin(), c.end(), [](const Cand &x, const Cand &y) {
        if (x.m != y.m) return x.m < y.m;
        if (x.t != y.t) return x.t < y.t;
        return x.parts < y.parts;
    });
    std::vector<Cand> keep;
    uint64_t best_t = kTimeInf;
    for (const Cand &x : c)
        if (x.t < best_t) {
            keep.push_back(x);
            best_t = x.t;
        }
    c.swap(keep);
}

bool desirable_set(const Table &tab, size_t ws_limit, int policy, std::vector<Config> &front)
{
    const int B = tab.B;
    std::vector<std::vector<Cand>> C(B + 1);
    C[0].push_back({0, 0, 0, 0, -1, -1});
    const std::vector<int> sizes = policy_sizes(policy, B);
    for (int b = 1; b <= B; ++b) {
        std::vector<Cand> cand;
        for (int bm : sizes) {
            if (bm > b) break;
            const std::vector<Cand> &rest = C[b - bm];
            if (rest.empty()) continue;
            for (int a = 0; a < tab.n_algo; ++a) {
                if (!feasible(tab, a, bm, ws_limit)) continue;
                const uint64_t t = tab.time(a, bm);
                const size_t m = tab.wsize(a, bm);
                for (int i = 0; i < (int)rest.size(); ++i)
                    cand.push_back({t + rest[i].t, std::max(m, rest[i].m), rest[i].parts + 1, bm, a, i});
            }
        }
        prune(cand);
        C[b].swap(cand);
    }
    front.clear();
    if (C[B].empty()) return false;
    for (const Cand &top : C[B]) {
        Config cfg;
        cfg.cost = top.t;
        cfg.ws = top.m;
        const Cand *p = &top;
        for (int b = B; b > 0;) {
            cfg.micro.push_back({p->algo, p->b_mu});
            int nb = b - p->b_mu;
            p = &C[nb][p->prev];
            b = nb;
        }
        front.push_back(std::move(cfg));
    }
    return true;
}

// ---- WD 0-1 programme (multiple-choice knapsack) ---------------------------------------------
// Exact: a sweep over kernels that keeps the Pareto set of (sum m, sum t) partial choices, cut
// down by the LP-relaxation bound of the kernels still to come (greedy over the convex-hull
// segments of every remaining kernel in order of time saved per byte).
namespace {
typedef __int128 i128;

struct Seg {
    uint64_t dm, dt;  // extra bytes, time saved (both > 0)
    int kernel;
};

struct State {
    size_t m;
    uint64_t t;
    int parent, pick;
};

struct Suffix {                  // kernels k..n-1
    size_t base_m = 0;           // every kernel at its smallest point
    uint64_t base_t = 0;
    std::vector<uint64_t> pm, pt;  // prefix sums over segments in greedy order (pm[0]=pt[0]=0)
    std::vector<Seg> seg;
    // least LP time with r bytes (rounded down), and the time of the integral greedy prefix
    bool bounds(size_t r, uint64_t &lb, uint64_t &ub) const
    {
        if (r < base_m) return false;
        uint64_t rr = r - base_m;
        size_t i = std::upper_bound(pm.begin(), pm.end(), rr) - pm.begin() - 1;
        ub = base_t - pt[i];
        lb = ub;
        if (i < seg.size()) {
            i128 num = (i128)seg[i].dt * (i128)(rr - pm[i]);
            uint64_t frac = (uint64_t)((num + seg[i].dm - 1) / seg[i].dm);  // ceil: keeps lb a lower bound
            lb -= std::min<uint64_t>(frac, seg[i].dt);
        }
        return true;
    }
};
}  // namespace

bool wd_solve(const std::vector<std::vector<FrontPoint>> &fronts_in, size_t budget,
              std::vector<int> &choice, uint64_t &total_t)
{
    const int n = (int)fronts_in.size();
    // Pareto-filter each kernel's points (keeps the caller's indices), sorted by m ascending.
    std::vector<std::vector<int>> idx(n);
    for (int k = 0; k < n; ++k) {
        const auto &f = fronts_in[k];
        if (f.empty()) return false;
        std::vector<int> o(f.size());
        std::iota(o.begin(), o.end(), 0);
        std::sort(o.begin(), o.end(), [&](int a, int b) {
            if (f[a].m != f[b].m) return f[a].m < f[b].m;
            if (f[a].t != f[b].t) return f[a].t < f[b].t;
            return a < b;
        });
        uint64_t best = kTimeInf;
        for (int i : o)
            if (f[i].t < best || (best == kTimeInf && idx[k].empty())) {
                idx[k].push_back(i);
                best = f[i].t;
            }
    }
    auto P = [&](int k, int j) -> const FrontPoint & { return fronts_in[k][idx[k][j]]; };

    // convex-hull segments per kernel
    std::vector<Seg> all;
    for (int k = 0; k < n; ++k) {
        std::vector<int> hull;
        for (int j = 0; j < (int)idx[k].size(); ++j) {
            while (hull.size() >= 2) {
                const FrontPoint &a = P(k, hull[hull.size() - 2]), &b = P(k, hull.back()), &c = P(k, j);
                // b is on or above segment a-c  <=>  (a.t-b.t)/(b.m-a.m) <= (a.t-c.t)/(c.m-a.m)
                i128 lhs = (i128)(a.t - b.t) * (i128)(c.m - a.m);
                i128 rhs = (i128)(a.t - c.t) * (i128)(b.m - a.m);
                if (lhs <= rhs) hull.pop_back(); else break;
            }
            hull.push_back(j);
        }
        for (size_t h = 1; h < hull.size(); ++h) {
            const FrontPoint &a = P(k, hull[h - 1]), &b = P(k, hull[h]);
            all.push_back({(uint64_t)(b.m - a.m), a.t - b.t, k});
        }
    }
    std::stable_sort(all.begin(), all.end(), [](const Seg &x, const Seg &y) {
        return (i128)x.dt * (i128)y.dm > (i128)y.dt * (i128)x.dm;  // more time saved per byte first
    });
    std::vector<Suffix> suf(n + 1);
    for (int k = n; k >= 0; --k) {
        Suffix &s = suf[k];
        if (k < n) {
            s.base_m = suf[k + 1].base_m + P(k, 0).m;
            s.base_t = suf[k + 1].base_t + P(k, 0).t;
        }
        s.pm.push_back(0);
        s.pt.push_back(0);
        for (const Seg &g : all)
            if (g.kernel >= k) {
                s.seg.push_back(g);
                s.pm.push_back(s.pm.back() + g.dm);
                s.pt.push_back(s.pt.back() + g.dt);
            }
    }

    uint64_t lb0, ub;
    if (!suf[0].bounds(budget, lb0, ub)) return false;

    std::vector<std::vector<State>> level(n + 1);
    level[0].push_back({0, 0, -1, -1});
    for (int k = 0; k < n; ++k) {
        std::vector<State> next;
        for (int si = 0; si < (int)level[k].size(); ++si) {
            const State &s = level[k][si];
            for (int j = 0; j < (int)idx[k].size(); ++j) {
                const FrontPoint &p = P(k, j);
                if (p.m > budget - s.m) break;  // points are sorted by m
                size_t m = s.m + p.m;
                uint64_t t = s.t + p.t, lb, u;
                if (!suf[k + 1].bounds(budget - m, lb, u)) continue;
                if (t + lb > ub) continue;
                ub = std::min(ub, t + u);
                next.push_back({m, t, si, j});
            }
        }
        std::sort(next.begin(), next.end(), [](const State &a, const State &b) {
            if (a.m != b.m) return a.m < b.m;
            return a.t < b.t;
        });
        uint64_t best = kTimeInf;
        for (const State &s : next)
            if (s.t < best) {
                level[k + 1].push_back(s);
                best = s.t;
            }
        if (level[k + 1].empty()) return false;
    }
    int bi = 0;
    for (int i = 1; i < (int)level[n].size(); ++i)
        if (level[n][i].t < level[n][bi].t) bi = i;
    total_t = level[n][bi].t;
    choice.assign(n, 0);
    for (int k = n; k > 0; --k) {
        const State &s = level[k][bi];
        choice[k - 1] = idx[k - 1][s.pick];
        bi = s.parent;
    }
    return true;
}

}  // namespace ucd
