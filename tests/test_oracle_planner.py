"""Pins for the exhaustive planner oracle: known partition counts, closed-form optima on
synthetic timing tables, the paper's two configuration examples, hand-worked Pareto and
knapsack cases."""
import json
import os

import pytest

from oracle import planner as P
from oracle.planner import INF, ALL, POW2, UNDIVIDED

GOLDEN = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "planner_examples.json")))


def table(B, n_algo, f_t, f_ws):
    t = [[INF] + [f_t(a, b) for b in range(1, B + 1)] for a in range(n_algo)]
    ws = [[INF] + [f_ws(a, b) for b in range(1, B + 1)] for a in range(n_algo)]
    return t, ws


def test_partition_counts_match_number_theory():
    # p(n): 1,2,3,5,7,11,15,22,...; binary partitions b(16)=36, b(32)=202
    assert [sum(1 for _ in P.partitions(n, range(1, n + 1))) for n in range(1, 9)] == [1, 2, 3, 5, 7, 11, 15, 22]
    assert sum(1 for _ in P.partitions(32, range(1, 33))) == 8349
    assert sum(1 for _ in P.partitions(16, P.policy_sizes(16, POW2))) == 36
    assert sum(1 for _ in P.partitions(32, P.policy_sizes(32, POW2))) == 202
    assert sum(1 for _ in P.compositions(7, range(1, 8))) == 2 ** 6
    assert all(sum(p) == 12 for p in P.partitions(12, range(1, 13)))


def test_policy_sizes():
    assert P.policy_sizes(6, ALL) == [1, 2, 3, 4, 5, 6]
    assert P.policy_sizes(12, POW2) == [1, 2, 4, 8, 12]      # Section 3.4 writes the set as ending in B
    assert P.policy_sizes(1, POW2) == [1] and P.policy_sizes(2, POW2) == [1, 2]
    assert P.policy_sizes(256, POW2) == [1, 2, 4, 8, 16, 32, 64, 128, 256]
    assert P.policy_sizes(12, UNDIVIDED) == [12]


def test_linear_cost_makes_every_division_equal():
    t, ws = table(12, 1, lambda a, b: 7 * b, lambda a, b: 0)
    for pol in (ALL, POW2, UNDIVIDED):
        assert P.wr_optimum(12, 0, pol, t, ws) == 84


def test_fixed_overhead_makes_undivided_optimal():
    t, ws = table(16, 1, lambda a, b: 100 + 3 * b, lambda a, b: 0)
    assert P.wr_optimum(16, 0, ALL, t, ws) == 100 + 48
    assert P.wr_optimum(16, 0, POW2, t, ws) == 100 + 48


def test_workspace_limit_forces_the_split():
    # fast algorithm 1 needs 10 bytes per sample; slow algorithm 0 needs none
    t, ws = table(12, 2, lambda a, b: (50 + 10 * b) if a == 0 else (5 + 2 * b), lambda a, b: 0 if a == 0 else 10 * b)
    assert P.wr_optimum(12, 120, ALL, t, ws) == 5 + 24          # fits undivided
    assert P.wr_optimum(12, 119, UNDIVIDED, t, ws) == 50 + 120  # one byte short: slow algorithm
    assert P.wr_optimum(12, 60, ALL, t, ws) == 2 * (5 + 12)     # two micro-batches of 6
    assert P.wr_optimum(12, 40, ALL, t, ws) == 3 * (5 + 8)      # three of 4
    assert P.wr_optimum(12, 50, ALL, t, ws) == 3 * 5 + 24       # e.g. 5+5+2: three parts
    assert P.wr_optimum(12, 9, ALL, t, ws) == 50 + 120          # nothing fits even at b=1
    assert P.wr_optimum(12, 40, POW2, t, ws) == 3 * (5 + 8)     # 4+4+4 are powers of two
    assert P.wr_optimum(12, 50, POW2, t, ws) == 3 * 5 + 24      # 4+4+4 again


def test_paper_example_equal_division_into_four():
    g = GOLDEN["equal_division"]
    B, X, s = g["B"], g["algo"], g["size"]
    # algorithm X needs 1 byte per sample and the limit is 64 bytes; algorithm 0 is 10x slower
    t, ws = table(B, 2, lambda a, b: 1000 * b if a == 0 else 1000 + 100 * b, lambda a, b: 0 if a == 0 else b)
    assert P.wr_optimum(B, s, POW2, t, ws) == g["count"] * (1000 + 100 * s)


def test_paper_example_size_60_used_repeatedly():
    g = GOLDEN["repeated_60"]
    B = g["B"]
    # five algorithms; algorithm 4 at size 60 has by far the least per-sample cost
    f = lambda a, b: 10 * b if (a == 4 and b == 60) else 100 * b + a
    t, ws = table(B, 5, f, lambda a, b: 0)
    rest = P.wr_optimum(g["rest"], 0, ALL, *table(g["rest"], 5, f, lambda a, b: 0))
    assert rest == 100 * g["rest"]
    # p(256) is out of reach: restrict sizes to 60 and a few sizes the rest can use
    best = INF
    for parts in P.partitions(B, [60, 16, 8, 4]):
        best = min(best, sum(P.micro_best(t, ws, b, 0) for b in parts))
    assert best == g["count"] * 600 + rest


@pytest.mark.parametrize("seed", range(6))
def test_explicit_algorithm_enumeration_agrees(seed):
    import random
    r = random.Random(seed)
    B = r.randint(3, 8)
    t, ws = table(B, 3, lambda a, b: r.randint(1, 100) * b + r.randint(0, 50), lambda a, b: a * b * r.randint(1, 4))
    M = r.randint(0, 3 * B)
    for pol in (ALL, POW2, UNDIVIDED):
        assert P.wr_optimum(B, M, pol, t, ws) == P.wr_optimum_explicit(B, M, pol, t, ws)


def test_monotone_in_policy_and_limit():
    import random
    r = random.Random(7)
    B = 10
    t, ws = table(B, 3, lambda a, b: r.randint(1, 100) * b + r.randint(0, 50), lambda a, b: a * b * 3)
    prev = None
    for M in range(0, 70, 5):
        u, p, a = (P.wr_optimum(B, M, pol, t, ws) for pol in (UNDIVIDED, POW2, ALL))
        assert a <= p <= u       # undivided's set is inside powerOfTwo's, which is inside all's
        if prev is not None:
            assert a <= prev
        prev = a


def test_desirable_set_by_hand():
    pts = [(10, 0), (8, 5), (8, 7), (9, 5), (6, 9), (6, 9), (7, 20), (5, 30)]
    # (8,7) loses to (8,5); (9,5) loses to (8,5); (7,20) loses to (6,9); duplicates collapse
    assert P.desirable(pts) == [(10, 0), (8, 5), (6, 9), (5, 30)]
    assert P.desirable([(3, 3)]) == [(3, 3)]


def test_all_configurations_counts_and_costs():
    # B=3, two algorithms, everything feasible: compositions (3),(1,2),(2,1),(1,1,1) -> 2+4+4+8
    t, ws = table(3, 2, lambda a, b: (a + 1) * b, lambda a, b: a * b)
    cfgs = P.all_configurations(3, 100, ALL, t, ws)
    assert len(cfgs) == 18
    assert (6, 3, ((1, 3),)) in cfgs and (3, 0, ((0, 1), (0, 1), (0, 1))) in cfgs
    assert (1 * 1 + 2 * 2, 2, ((0, 1), (1, 2))) in cfgs      # T adds, workspace is the max


def test_wd_optimum_by_hand():
    k0 = [(10, 0), (6, 4), (3, 8)]
    k1 = [(20, 0), (9, 5)]
    assert P.wd_optimum([k0, k1], 0) == (30, (0, 0))
    assert P.wd_optimum([k0, k1], 4) == (26, (1, 0))
    assert P.wd_optimum([k0, k1], 5) == (19, (0, 1))
    assert P.wd_optimum([k0, k1], 9) == (15, (1, 1))
    assert P.wd_optimum([k0, k1], 13) == (12, (2, 1))
    assert P.wd_optimum([[(1, 5)]], 4) == (INF, None)
