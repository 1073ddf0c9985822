// Test driver: the host planners (planner.cpp) behind a text protocol on stdin, so that they can
// be built with -fsanitize=address,undefined as a plain executable and fed from the Python tests.
//
//   wr    B n_algo limit policy  t[n_algo*(B+1)] ws[n_algo*(B+1)]   -> "ok cost ws n a0 b0 a1 b1 ..." | "infeasible"
//   front B n_algo limit policy  t[...] ws[...]                     -> "ok n t0 m0 t1 m1 ..."          | "infeasible"
//   wd    n_kernels budget  n_0 (t m)*n_0  n_1 ...                  -> "ok total c0 c1 ..."            | "infeasible"
// Table holes are written as -1.
#include <cstdio>
#include <iostream>
#include <string>
#include <vector>

#include "planner.h"

using namespace ucd;

static bool read_table(int B, int n_algo, std::vector<uint64_t> &t, std::vector<size_t> &ws)
{
    const size_t n = (size_t)n_algo * (B + 1);
    t.resize(n);
    ws.resize(n);
    long long v;
    for (size_t i = 0; i < n; ++i) {
        if (!(std::cin >> v)) return false;
        t[i] = v < 0 ? kTimeInf : (uint64_t)v;
    }
    for (size_t i = 0; i < n; ++i) {
        if (!(std::cin >> v)) return false;
        ws[i] = v < 0 ? kWsNa : (size_t)v;
    }
    return true;
}

int main()
{
    std::string cmd;
    while (std::cin >> cmd) {
        if (cmd == "wr" || cmd == "front") {
            int B, n_algo, policy;
            long long limit;
            std::vector<uint64_t> t;
            std::vector<size_t> ws;
            if (!(std::cin >> B >> n_algo >> limit >> policy) || !read_table(B, n_algo, t, ws)) return 2;
            Table tab{B, n_algo, t.data(), ws.data()};
            if (cmd == "wr") {
                Config c;
                if (!wr_plan(tab, (size_t)limit, policy, c)) { std::puts("infeasible"); continue; }
                std::printf("ok %llu %zu %zu", (unsigned long long)c.cost, c.ws, c.micro.size());
                for (const Micro &m : c.micro) std::printf(" %d %d", m.algo, m.batch);
                std::puts("");
            } else {
                std::vector<Config> f;
                if (!desirable_set(tab, (size_t)limit, policy, f)) { std::puts("infeasible"); continue; }
                std::printf("ok %zu", f.size());
                for (const Config &c : f) std::printf(" %llu %zu", (unsigned long long)c.cost, c.ws);
                std::puts("");
            }
        } else if (cmd == "wd") {
            int nk;
            long long budget;
            if (!(std::cin >> nk >> budget) || nk < 1) return 2;
            std::vector<std::vector<FrontPoint>> fronts(nk);
            for (int k = 0; k < nk; ++k) {
                int n;
                if (!(std::cin >> n)) return 2;
                for (int i = 0; i < n; ++i) {
                    long long tt, mm;
                    if (!(std::cin >> tt >> mm)) return 2;
                    fronts[k].push_back({(uint64_t)tt, (size_t)mm});
                }
            }
            std::vector<int> choice;
            uint64_t total;
            if (!wd_solve(fronts, (size_t)budget, choice, total)) { std::puts("infeasible"); continue; }
            std::printf("ok %llu", (unsigned long long)total);
            for (int c : choice) std::printf(" %d", c);
            std::puts("");
        } else {
            return 2;
        }
    }
    return 0;
}
