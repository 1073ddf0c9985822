"""Host planners behind the C-ABI (no GPU needed) against the exhaustive oracle: exact integer
equality of the optimum cost, validity of the returned configuration, Pareto fronts and the
WD programme against full enumeration."""
import random

import pytest

from oracle import planner as P
from paper_1804_04806_amd import ucd

INF = P.INF


def random_table(r, B, n_algo=3, holes=True):
    """Synthetic timings shaped like measured ones: an overhead plus a per-sample cost that
    differs by algorithm, workspace growing with b for the faster algorithms."""
    t, ws = [], []
    for a in range(n_algo):
        over, per = r.randint(0, 400), r.randint(20, 200) // (a + 1) + 1
        wpb = 0 if a == 0 else r.randint(1, 50) * a
        base = 0 if a == 0 else r.randint(0, 100)
        ta, wa = [INF], [INF]
        for b in range(1, B + 1):
            if holes and a > 0 and r.random() < 0.1:
                ta.append(INF); wa.append(INF)
            else:
                ta.append(over + per * b + r.randint(0, 30)); wa.append(base + wpb * b)
        t.append(ta); ws.append(wa)
    return t, ws


def check_config(micro, cost, wsb, B, M, policy, t, ws):
    assert sum(b for _, b in micro) == B
    allowed = set(P.policy_sizes(B, policy))
    total, peak = 0, 0
    for a, b in micro:
        assert b in allowed and t[a][b] != INF and ws[a][b] <= M
        total += t[a][b]
        peak = max(peak, ws[a][b])
    assert total == cost and peak == wsb


@pytest.mark.parametrize("seed", range(25))
def test_wr_equals_brute_force_small(seed):
    r = random.Random(seed)
    B = r.randint(1, 14)
    t, ws = random_table(r, B)
    for M in (0, r.randint(0, 200), r.randint(0, 2000), 10 ** 9):
        for pol in (ucd.POLICY_UNDIVIDED, ucd.POLICY_POW2, ucd.POLICY_ALL):
            ref = P.wr_optimum(B, M, pol, t, ws)
            if B <= 9:
                assert ref == P.wr_optimum_explicit(B, M, pol, t, ws)
            plan = ucd.ucd_plan_from_table(B, M, pol, t, ws)
            micro, cost, wsb = plan.query()
            assert cost == ref
            check_config(micro, cost, wsb, B, M, pol, t, ws)


@pytest.mark.parametrize("seed", range(4))
def test_wr_equals_brute_force_b32_all(seed):
    r = random.Random(100 + seed)
    t, ws = random_table(r, 32)
    M = r.randint(100, 3000)
    plan = ucd.ucd_plan_from_table(32, M, ucd.POLICY_ALL, t, ws)
    assert plan.cost_ns == P.wr_optimum(32, M, P.ALL, t, ws)


def test_wr_equals_brute_force_b48_all():
    r = random.Random(4848)
    t, ws = random_table(r, 48)
    plan = ucd.ucd_plan_from_table(48, 1500, ucd.POLICY_ALL, t, ws)
    assert plan.cost_ns == P.wr_optimum(48, 1500, P.ALL, t, ws)   # p(48) = 147,273 divisions


def test_wr_equals_brute_force_b256_pow2():
    r = random.Random(256)
    t, ws = random_table(r, 256, holes=False)
    plan = ucd.ucd_plan_from_table(256, 4000, ucd.POLICY_POW2, t, ws)
    micro, cost, wsb = plan.query()
    assert cost == P.wr_optimum(256, 4000, P.POW2, t, ws)         # 692,004 binary partitions
    check_config(micro, cost, wsb, 256, 4000, ucd.POLICY_POW2, t, ws)


def test_undivided_picks_the_fastest_fitting_algorithm():
    r = random.Random(5)
    t, ws = random_table(r, 20, holes=False)
    for M in (0, 300, 10 ** 6):
        micro, cost, _ = ucd.ucd_plan_from_table(20, M, ucd.POLICY_UNDIVIDED, t, ws).query()
        assert len(micro) == 1 and micro[0][1] == 20
        assert cost == min(t[a][20] for a in range(3) if ws[a][20] <= M)


def test_policy_and_limit_monotonicity_at_256():
    r = random.Random(9)
    t, ws = random_table(r, 256, holes=False)
    prev = None
    for M in (0, 500, 2000, 8000, 10 ** 7):
        u, p, a = (ucd.ucd_plan_from_table(256, M, pol, t, ws).cost_ns for pol in (0, 1, 2))
        assert a <= p <= u
        if prev is not None:
            assert a <= prev
        prev = a


def test_paper_examples_through_the_library():
    B = 256
    t = [[INF] + [1000 * b for b in range(1, B + 1)], [INF] + [1000 + 100 * b for b in range(1, B + 1)]]
    ws = [[INF] + [0] * B, [INF] + list(range(1, B + 1))]
    micro, cost, wsb = ucd.ucd_plan_from_table(B, 64, ucd.POLICY_POW2, t, ws).query()
    assert micro == [(1, 64)] * 4 and cost == 4 * 7400 and wsb == 64
    f = lambda a, b: 10 * b if (a == 4 and b == 60) else 100 * b + a
    t = [[INF] + [f(a, b) for b in range(1, B + 1)] for a in range(5)]
    ws = [[INF] + [0] * B for _ in range(5)]
    micro, cost, _ = ucd.ucd_plan_from_table(B, 0, ucd.POLICY_ALL, t, ws).query()
    assert micro.count((4, 60)) == 4 and cost == 4 * 600 + 1600


def test_infeasible_and_bad_arguments():
    t, ws = [[INF, INF, INF]], [[INF, INF, INF]]
    with pytest.raises(ucd.UcdError) as e:
        ucd.ucd_plan_from_table(2, 10, ucd.POLICY_ALL, t, ws)
    assert e.value.status == ucd.E_INFEASIBLE
    with pytest.raises(ucd.UcdError) as e:
        ucd.ucd_plan_from_table(2, 10, 7, [[INF, 1, 2]], [[INF, 0, 0]])
    assert e.value.status == ucd.E_INVALID


@pytest.mark.parametrize("seed", range(12))
def test_desirable_set_equals_pareto_front_of_all_configurations(seed):
    r = random.Random(1000 + seed)
    B = r.randint(1, 7)
    t, ws = random_table(r, B)
    M = r.choice([0, 150, 10 ** 9])
    for pol in (ucd.POLICY_ALL, ucd.POLICY_POW2):
        cfgs = P.all_configurations(B, M, pol, t, ws)
        ref = P.desirable([(c[0], c[1]) for c in cfgs])
        got = ucd.ucd_desirable_from_table(B, M, pol, t, ws)
        assert got == ref
        # the WR optimum is the fastest point of the front
        assert min(p[0] for p in got) == P.wr_optimum(B, M, pol, t, ws)


@pytest.mark.parametrize("seed", range(10))
def test_wd_equals_full_enumeration(seed):
    r = random.Random(2000 + seed)
    nk = r.randint(2, 4)
    B = r.randint(2, 4 if nk > 3 else 5)
    tabs = [random_table(r, B, holes=False) for _ in range(nk)]
    big = 10 ** 9
    unpruned = [P.all_configurations(B, big, P.ALL, t, ws) for t, ws in tabs]
    fronts = [ucd.ucd_desirable_from_table(B, big, ucd.POLICY_ALL, t, ws) for t, ws in tabs]
    for budget in (0, r.randint(0, 300), r.randint(0, 1500), big):
        # proof-as-test: optimum over pruned fronts == optimum over every configuration
        ref_unpruned, _ = P.wd_optimum([[(c[0], c[1]) for c in k] for k in unpruned], budget)
        ref_pruned, _ = P.wd_optimum(fronts, budget)
        assert ref_unpruned == ref_pruned
        choice, total = ucd.ucd_wd_solve(fronts, budget)
        assert total == ref_pruned
        assert sum(fronts[k][i][1] for k, i in enumerate(choice)) <= budget
        assert sum(fronts[k][i][0] for k, i in enumerate(choice)) == total


def test_wd_budget_extremes_and_wr_comparison():
    r = random.Random(77)
    nk, B = 6, 16
    tabs = [random_table(r, B, holes=False) for _ in range(nk)]
    fronts = [ucd.ucd_desirable_from_table(B, 10 ** 9, ucd.POLICY_ALL, t, ws) for t, ws in tabs]
    # budget 0: everything on zero-workspace points; huge budget: every kernel at its fastest
    _, total0 = ucd.ucd_wd_solve(fronts, 0)
    assert total0 == sum(max(p[0] for p in f if p[1] == 0) for f in fronts)
    _, total_inf = ucd.ucd_wd_solve(fronts, 10 ** 12)
    assert total_inf == sum(min(p[0] for p in f) for f in fronts)
    # WD with nk*M in total is never worse than WR with M per kernel
    for M in (50, 200, 800):
        wr = sum(ucd.ucd_plan_from_table(B, M, ucd.POLICY_ALL, t, ws).cost_ns for t, ws in tabs)
        fr = [ucd.ucd_desirable_from_table(B, nk * M, ucd.POLICY_ALL, t, ws) for t, ws in tabs]
        _, wd = ucd.ucd_wd_solve(fr, nk * M)
        assert wd <= wr


def test_wd_many_kernels_is_fast_and_consistent():
    """159 kernels as in a ResNet-50 sized problem: solve, then verify feasibility and that no
    single-kernel change improves the solution."""
    r = random.Random(159)
    fronts = []
    for k in range(159):
        n = r.choice([1, 1, 1, 5, 20, 60])
        t0, pts = r.randint(10 ** 5, 10 ** 7), []
        m = 0
        for i in range(n):
            pts.append((t0, m))
            t0 -= r.randint(1, max(2, t0 // 20)); m += r.randint(1, 64) * 65536
        fronts.append(pts)
    budget = 512 << 20
    choice, total = ucd.ucd_wd_solve(fronts, budget)
    used = sum(fronts[k][i][1] for k, i in enumerate(choice))
    assert used <= budget and total == sum(fronts[k][i][0] for k, i in enumerate(choice))
    for k in range(159):
        for i, (t, m) in enumerate(fronts[k]):
            if used - fronts[k][choice[k]][1] + m <= budget:
                assert t >= fronts[k][choice[k]][0]


def test_plan_wd_from_tables_returns_plans_and_disjoint_segments():
    r = random.Random(31)
    Bs = [8, 8, 4]
    tabs = [random_table(r, B, holes=False) for B in Bs]
    # scale workspaces so that 256-byte rounding matters
    tabs = [(t, [[w if w == INF else w * 100 for w in row] for row in ws]) for t, ws in tabs]
    total = 30000
    plans, offs = ucd.ucd_plan_wd_from_tables(Bs, [t for t, _ in tabs], [w for _, w in tabs], total, ucd.POLICY_ALL)
    end = 0
    for k, (plan, off) in enumerate(zip(plans, offs)):
        micro, cost, wsb = plan.query()
        check_config(micro, cost, wsb, Bs[k], total, ucd.POLICY_ALL, *tabs[k])
        assert off % 256 == 0 and off >= end
        end = off + wsb
    assert end <= total
