"""File-backed benchmark database and planning from the cache alone (host only, no GPU)."""
import random

import pytest

from oracle import planner as P
from paper_1804_04806_amd import ucd


def fill(desc, op, B, seed):
    r = random.Random(seed)
    t = [[ucd.TIME_INF] * (B + 1) for _ in range(ucd.N_ALGO)]
    for a in range(ucd.N_ALGO):
        for b in range(1, B + 1):
            if ucd.ucd_workspace_size(desc, op, a, b) == ucd.WS_NA:
                continue
            t[a][b] = 1000 * (ucd.N_ALGO - a) * b + r.randint(0, 5000) + 20000
            ucd.ucd_bench_put(desc, op, a, b, t[a][b])
    return t


def test_put_table_save_load_roundtrip_and_cached_plan(tmp_path):
    ucd.ucd_bench_clear()
    L = ucd.layer(N=12, C=16, H=16, W=16, K=32, R=3, S=3, pad_h=1, pad_w=1)
    L2 = ucd.layer(N=12, C=16, H=16, W=16, K=32, R=3, S=3, pad_h=1, pad_w=1, stride_h=2, stride_w=2)
    t_fwd = fill(L, ucd.FWD, 12, 1)
    t_bf = fill(L, ucd.BWD_FILTER, 12, 2)
    fill(L2, ucd.BWD_DATA, 12, 3)
    got, ws = ucd.ucd_bench_table(L, ucd.FWD, 12)
    assert got == t_fwd
    path = tmp_path / "bench.txt"
    ucd.ucd_bench_save(path)
    ucd.ucd_bench_clear()
    assert ucd.ucd_bench_table(L, ucd.FWD, 12)[0] == [[ucd.TIME_INF] * 13 for _ in range(ucd.N_ALGO)]
    n_rows = sum(1 for a in range(ucd.N_ALGO) for b in range(1, 13) if t_fwd[a][b] != ucd.TIME_INF)
    n = ucd.ucd_bench_load(path)
    assert n > n_rows and ucd.ucd_bench_table(L, ucd.FWD, 12)[0] == t_fwd
    assert ucd.ucd_bench_table(L, ucd.BWD_FILTER, 12)[0] == t_bf
    # planning from the cache alone equals brute force on that table, under several limits
    for limit in (0, 300 * 1024, 1 << 20, 1 << 30):
        for pol in (ucd.POLICY_UNDIVIDED, ucd.POLICY_POW2, ucd.POLICY_ALL):
            plan = ucd.ucd_plan_cached(L, ucd.FWD, limit, pol)
            micro, cost, need = plan.query()
            assert cost == P.wr_optimum(12, limit, pol, t_fwd, ws) and need <= limit
            assert sum(b for _, b in micro) == 12
    # a layer that was never benchmarked cannot be planned offline
    other = ucd.layer(N=4, C=8, H=9, W=9, K=8, R=3, S=3)
    with pytest.raises(ucd.UcdError) as e:
        ucd.ucd_plan_cached(other, ucd.FWD, 1 << 20, ucd.POLICY_ALL)
    assert e.value.status == ucd.E_INFEASIBLE
    ucd.ucd_bench_clear()


def test_load_rejects_garbage(tmp_path):
    bad = tmp_path / "bad.txt"
    bad.write_text("not a benchmark file\n")
    with pytest.raises(ucd.UcdError) as e:
        ucd.ucd_bench_load(bad)
    assert e.value.status == ucd.E_INVALID
    trunc = tmp_path / "trunc.txt"
    trunc.write_text("ucd-bench 1 none\n16 16 16 32 3 3 1 1 1 1 0 0 0 4\n")
    with pytest.raises(ucd.UcdError):
        ucd.ucd_bench_load(trunc)
    with pytest.raises(ucd.UcdError):
        ucd.ucd_bench_load(tmp_path / "missing.txt")
    other_device = tmp_path / "dev.txt"
    other_device.write_text("ucd-bench 1 gfx000/1cu\n16 16 16 32 3 3 1 1 1 1 0 0 0 4 12345\n")
    # without a GPU in this process any device tag is accepted; with one, a foreign tag is refused
    try:
        assert ucd.ucd_bench_load(other_device) == 1
    except ucd.UcdError as err:
        assert err.status == ucd.E_UNSUPPORTED
    ucd.ucd_bench_clear()


def test_put_validation():
    L = ucd.layer(N=4, C=8, H=9, W=9, K=8, R=3, S=3)
    for args in ((ucd.FWD, ucd.N_ALGO, 1, 10), (5, 0, 1, 10), (ucd.FWD, 0, 0, 10), (ucd.FWD, 0, 1, 0)):
        with pytest.raises(ucd.UcdError):
            ucd.ucd_bench_put(L, *args)
