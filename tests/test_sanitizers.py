"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer: the planners (planner.cpp) and
the convolution oracle (conv_oracle.c) are built as plain executables with
-fsanitize=address,undefined and driven over a spread of inputs; any report fails the test, and
the results must equal those of the exhaustive Python planner / of the regular oracle build."""
import os
import random
import subprocess

import numpy as np
import pytest

from oracle import conv as oc
from oracle import planner as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NATIVE = os.path.join(ROOT, "tests", "native")
CSRC = os.path.join(ROOT, "paper_1804_04806_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


@pytest.fixture(scope="module")
def planner_bin(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("san") / "planner_asan")
    subprocess.check_call(["g++", "-std=c++17", *SAN, "-I", CSRC, os.path.join(NATIVE, "planner_driver.cpp"),
                           os.path.join(CSRC, "planner.cpp"), "-o", out])
    return out


@pytest.fixture(scope="module")
def oracle_bin(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("san") / "oracle_asan")
    subprocess.check_call(["gcc", "-std=c99", *SAN, "-fopenmp", os.path.join(NATIVE, "oracle_driver.c"),
                           os.path.join(ROOT, "oracle", "conv_oracle.c"), "-o", out])
    return out


def run(binary, text):
    r = subprocess.run([binary], input=text, capture_output=True, text=True, env=ENV, timeout=300)
    assert r.returncode == 0 and r.stderr == "", (r.returncode, r.stderr[-2000:])
    return r.stdout.splitlines()


def flat(table):
    return " ".join(str(-1 if v == P.INF else v) for row in table for v in row)


def random_table(rng, B, n_algo, holes=0.2):
    t = [[P.INF] + [P.INF if rng.random() < holes else rng.randint(1, 1000) * b + rng.randint(0, 300) for b in range(1, B + 1)]
         for _ in range(n_algo)]
    ws = [[P.INF] + [P.INF if rng.random() < 0.1 else a * b * rng.randint(0, 9) for b in range(1, B + 1)] for a in range(n_algo)]
    t[0] = [P.INF] + [rng.randint(500, 1500) * b for b in range(1, B + 1)]   # a zero-workspace algorithm always applies
    ws[0] = [P.INF] + [0] * B
    return t, ws


def test_planners_under_sanitizers_equal_the_exhaustive_optimum(planner_bin):
    rng = random.Random(7)
    lines, expect = [], []
    for case in range(60):
        B, n_algo = rng.randint(1, 14), rng.randint(1, 4)
        t, ws = random_table(rng, B, n_algo)
        limit, pol = rng.choice([0, 5, 20, 60, 10 ** 6]), rng.choice([P.UNDIVIDED, P.POW2, P.ALL])
        lines.append(f"wr {B} {n_algo} {limit} {pol} {flat(t)} {flat(ws)}")
        expect.append(("wr", P.wr_optimum(B, limit, pol, t, ws), (B, limit, pol, t, ws)))
        if B <= 8:
            lines.append(f"front {B} {n_algo} {limit} {pol} {flat(t)} {flat(ws)}")
            cfgs = [(c[0], c[1]) for c in P.all_configurations(B, limit, pol, t, ws)]
            expect.append(("front", sorted(set(P.desirable(cfgs)), key=lambda p: p[1]), None))
    # a large problem (B = 256, every size) for the quadratic programme's indexing
    t, ws = random_table(rng, 256, 5)
    lines.append(f"wr 256 5 4000 {P.ALL} {flat(t)} {flat(ws)}")
    expect.append(("wr-invariant", P.wr_optimum(256, 4000, P.POW2, t, ws), (256, 4000, P.ALL, t, ws)))
    # WD programmes over random fronts, against the full enumeration
    for case in range(25):
        nk = rng.randint(1, 5)
        fronts = []
        for _ in range(nk):
            pts = sorted({(rng.randint(1, 500), rng.randint(0, 60)) for _ in range(rng.randint(1, 6))})
            fronts.append(P.desirable(pts) if rng.random() < 0.7 else pts)
        budget = rng.randint(0, 120)
        lines.append(f"wd {nk} {budget} " + " ".join(f"{len(f)} " + " ".join(f"{a} {b}" for a, b in f) for f in fronts))
        best = P.wd_optimum([[(a, b) for a, b in f] for f in fronts], budget)
        expect.append(("wd", best, fronts))
    got = run(planner_bin, "\n".join(lines) + "\n")
    assert len(got) == len(expect)
    for line, (kind, want, ctx) in zip(got, expect):
        tok = line.split()
        if kind == "wr":
            if want == P.INF:
                assert tok[0] == "infeasible", line
                continue
            B, limit, pol, t, ws = ctx
            cost, need, n = int(tok[1]), int(tok[2]), int(tok[3])
            micro = [(int(tok[4 + 2 * i]), int(tok[5 + 2 * i])) for i in range(n)]
            assert cost == want and sum(b for _, b in micro) == B
            assert sum(t[a][b] for a, b in micro) == cost and max(ws[a][b] for a, b in micro) == need <= limit
            assert all(b in P.policy_sizes(B, pol) for _, b in micro)
        elif kind == "wr-invariant":
            assert tok[0] == "ok" and int(tok[1]) <= want        # all <= powerOfTwo on the same table
        elif kind == "front":
            if not want:
                assert tok[0] == "infeasible", line
                continue
            n = int(tok[1])
            assert [(int(tok[2 + 2 * i]), int(tok[3 + 2 * i])) for i in range(n)] == [tuple(p) for p in want]
        else:
            if want[0] == P.INF:
                assert tok[0] == "infeasible", line
            else:
                assert tok[0] == "ok" and int(tok[1]) == want[0], (line, want)


SHAPES = [(2, 3, 7, 6, 4, 3, 3, 1, 1, 1, 1), (1, 2, 9, 9, 3, 5, 4, 2, 3, 2, 1), (3, 1, 5, 5, 2, 1, 1, 2, 2, 0, 0),
          (2, 4, 6, 8, 5, 2, 4, 1, 2, 3, 0), (1, 1, 3, 3, 1, 3, 3, 1, 1, 0, 0)]


@pytest.mark.parametrize("dims", SHAPES, ids=lambda d: "x".join(map(str, d)))
def test_oracle_under_sanitizers_equals_the_regular_build(oracle_bin, tmp_path, dims):
    L = oc.Layer(*dims)
    rng = np.random.default_rng(sum(dims))
    x, w, dy = rng.standard_normal(L.x_shape), rng.standard_normal(L.w_shape), rng.standard_normal(L.y_shape)
    nidx = 9
    idx = [rng.integers(0, n, size=nidx, dtype=np.int64) for n in (dy.size, x.size, w.size)]
    src, dst = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(src, "wb") as f:
        for a in (x, w, dy, *idx):
            f.write(np.ascontiguousarray(a).tobytes())
    r = subprocess.run([oracle_bin, *map(str, dims), str(nidx), str(src), str(dst)], capture_output=True, text=True,
                       env=ENV, timeout=300)
    assert r.returncode == 0 and r.stderr == "", (r.returncode, r.stderr[-2000:])
    out = np.fromfile(dst, dtype=np.float64)
    parts = np.split(out, np.cumsum([dy.size, x.size, w.size, nidx, nidx]))
    want = [oc.conv_fwd(L, x, w), oc.conv_bwd_data(L, dy, w), oc.conv_bwd_filter(L, x, dy),
            oc.conv_fwd_at(L, x, w, idx[0]), oc.conv_bwd_data_at(L, dy, w, idx[1]), oc.conv_bwd_filter_at(L, x, dy, idx[2])]
    for got, ref in zip(parts, want):
        np.testing.assert_allclose(got, np.asarray(ref).ravel(), rtol=1e-12, atol=1e-12)
