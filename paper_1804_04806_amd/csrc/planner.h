// Host-side planners of the micro-batch method (arXiv 1804.04806, Section 3): the WR dynamic
// programme, the desirable-set (Pareto) programme and an exact solver for the WD 0-1 programme.
// Pure host code: integer nanoseconds and bytes, no GPU calls.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

namespace ucd {

constexpr uint64_t kTimeInf = UINT64_MAX;
constexpr size_t kWsNa = SIZE_MAX;

struct Micro {
    int algo;
    int batch;
};

// Timing table view: t[a*(B+1)+b], ws[a*(B+1)+b], b = 1..B.
struct Table {
    int B;
    int n_algo;
    const uint64_t *t;
    const size_t *ws;
    uint64_t time(int a, int b) const { return t[(size_t)a * (B + 1) + b]; }
    size_t wsize(int a, int b) const { return ws[(size_t)a * (B + 1) + b]; }
};

struct Config {
    std::vector<Micro> micro;
    uint64_t cost = 0;  // sum of table times
    size_t ws = 0;      // largest workspace over the parts
};

// Section 3.4: micro-batch sizes a policy lets the benchmark step try.
bool policy_allows(int policy, int B, int b);
std::vector<int> policy_sizes(int policy, int B);

// Section 3.2 steps 2-3.  Returns false if no division of B is feasible.
bool wr_plan(const Table &tab, size_t ws_limit, int policy, Config &out);

// Section 3.3: desirable set C(B), sorted by increasing workspace / decreasing time.
bool desirable_set(const Table &tab, size_t ws_limit, int policy, std::vector<Config> &front);

struct FrontPoint {
    uint64_t t;
    size_t m;
};

// Section 3.3 Eq. 1-4: one point per kernel, sum m <= budget, least sum t.  Exact.
// Returns false if infeasible.
bool wd_solve(const std::vector<std::vector<FrontPoint>> &fronts, size_t budget,
              std::vector<int> &choice, uint64_t &total_t);

}  // namespace ucd
