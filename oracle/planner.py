"""TEST INFRASTRUCTURE ONLY: exhaustive planners for the micro-batch method
(arXiv 1804.04806, Section 3).

The method's planners (the WR dynamic programme of Section 3.2, the desirable-set
programme and the 0-1 ILP of Section 3.3) reach the exact optimum of a problem
with a plain definition, so the oracle is that definition enumerated:

* WR: every division of the mini-batch B into micro-batches whose sizes the
  batch-size policy (Section 3.4) allows, every part running the fastest
  algorithm that fits the workspace limit M; the answer is the least total time.
* WD: every configuration (ordered list of (algorithm, micro-batch size)) of
  every kernel, every combination of one configuration per kernel whose
  workspaces (a configuration needs the largest of its parts, kernels get
  disjoint segments, Eq. 2) sum to at most the budget; the answer is the least
  total time (Eq. 1).

Times are integers (ns), so all sums are exact and order-free.  ``INF`` marks a
(algorithm, size) pair that was not benchmarked or does not apply.
Tables are indexed ``t[a][b]`` / ``ws[a][b]`` with b = 0..B (entry 0 unused).
"""
import itertools

INF = (1 << 64) - 1

UNDIVIDED, POW2, ALL = 0, 1, 2


def policy_sizes(B, policy):
    """Micro-batch sizes a batch-size policy lets the benchmark step try (Section 3.4)."""
    if policy == ALL:
        return list(range(1, B + 1))
    if policy == POW2:
        # the set is printed as {2^0, 2^1, 2^2, ..., B}: the powers of two below B, and B itself
        out, b = [], 1
        while b < B:
            out.append(b)
            b *= 2
        return out + [B]
    if policy == UNDIVIDED:
        return [B]
    raise ValueError("unknown policy")


def partitions(B, sizes):
    """All multisets of parts from ``sizes`` summing to B, as non-increasing tuples."""
    sizes = sorted(set(s for s in sizes if 1 <= s <= B), reverse=True)

    def rec(rest, start):
        if rest == 0:
            yield ()
            return
        for i in range(start, len(sizes)):
            s = sizes[i]
            if s <= rest:
                for tail in rec(rest - s, i):
                    yield (s,) + tail

    return rec(B, 0)


def compositions(B, sizes):
    """All ordered lists of parts from ``sizes`` summing to B."""
    sizes = sorted(set(s for s in sizes if 1 <= s <= B))

    def rec(rest):
        if rest == 0:
            yield ()
            return
        for s in sizes:
            if s <= rest:
                for tail in rec(rest - s):
                    yield (s,) + tail

    return rec(B)


def _feasible(t, ws, a, b, M):
    return t[a][b] != INF and ws[a][b] != INF and ws[a][b] <= M


def micro_best(t, ws, b, M):
    """T_mu(b): time of the fastest algorithm that fits M at micro-batch size b, or INF."""
    best = INF
    for a in range(len(t)):
        if _feasible(t, ws, a, b, M) and t[a][b] < best:
            best = t[a][b]
    return best


def wr_optimum(B, M, policy, t, ws):
    """Least total time over every division of B (WR problem). INF if none is feasible."""
    best = INF
    sizes = policy_sizes(B, policy)
    t_mu = {b: micro_best(t, ws, b, M) for b in sizes}
    for parts in partitions(B, sizes):
        total = 0
        for b in parts:
            c = t_mu[b]
            if c == INF:
                total = INF
                break
            total += c
        if total < best:
            best = total
    return best


def wr_optimum_explicit(B, M, policy, t, ws):
    """Same optimum, but the algorithm of every part is enumerated too (tiny B only)."""
    n_algo = len(t)
    best = INF
    for parts in partitions(B, policy_sizes(B, policy)):
        for algos in itertools.product(range(n_algo), repeat=len(parts)):
            if all(_feasible(t, ws, a, b, M) for a, b in zip(algos, parts)):
                total = sum(t[a][b] for a, b in zip(algos, parts))
                if total < best:
                    best = total
    return best


def all_configurations(B, M, policy, t, ws):
    """Every configuration of one kernel as (T, M_needed, ((algo, size), ...)), unpruned.

    T adds over the micro-batches; the workspace a configuration needs is the
    largest of its parts, since they run one after another in one segment.
    """
    n_algo = len(t)
    out = []
    for parts in compositions(B, policy_sizes(B, policy)):
        for algos in itertools.product(range(n_algo), repeat=len(parts)):
            if all(_feasible(t, ws, a, b, M) for a, b in zip(algos, parts)):
                out.append((sum(t[a][b] for a, b in zip(algos, parts)),
                            max(ws[a][b] for a, b in zip(algos, parts)),
                            tuple(zip(algos, parts))))
    return out


def desirable(points):
    """Pareto front of (T, M) pairs by the definition of Section 3.3: drop a point
    iff another, different point is no slower and no bigger; equal points count once.
    Returned sorted by workspace."""
    pts = sorted(set(points), key=lambda p: (p[1], p[0]))
    keep = []
    for p in pts:
        dominated = any(q != p and q[0] <= p[0] and q[1] <= p[1] for q in pts)
        if not dominated:
            keep.append(p)
    return keep


def wd_optimum(kernel_configs, budget):
    """Least total time choosing one (T, M) per kernel with sum of M <= budget (Eq. 1-4).

    ``kernel_configs`` is a list (one entry per kernel) of lists of (T, M, ...) tuples.
    Full cartesian product; returns (best_T, chosen index tuple) or (INF, None)."""
    best, arg = INF, None
    for choice in itertools.product(*[range(len(c)) for c in kernel_configs]):
        m = sum(kernel_configs[k][i][1] for k, i in enumerate(choice))
        if m > budget:
            continue
        tt = sum(kernel_configs[k][i][0] for k, i in enumerate(choice))
        if tt < best:
            best, arg = tt, choice
    return best, arg
