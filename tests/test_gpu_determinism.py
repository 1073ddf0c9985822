"""Run-to-run reproducibility on the device.  Launches that add every output element once must be
bit-identical from run to run in the default mode; in the reproducible mode
(ucd_set_deterministic) every operation of every algorithm it offers must be, and must still
match the oracle."""
import numpy as np
import pytest

from paper_1804_04806_amd import ucd
from paper_1804_04806_amd.synth import Shape
from hip_helpers import inputs, l2_tol, rel_l2, run_hip, run_oracle

pytestmark = pytest.mark.gpu

OPS = (ucd.FWD, ucd.BWD_DATA, ucd.BWD_FILTER)


@pytest.fixture
def deterministic():
    prev = ucd.ucd_set_deterministic(1)
    yield
    ucd.ucd_set_deterministic(prev)


def launches(s, op, algo, b):
    return ucd.ucd_describe_micro(ucd.layer(s), op, algo, b)[0]


# shapes of the parity tests whose default launches split reductions (deep: few output tiles) and
# one with many tiles and a tail (tiles not a multiple of the CU count)
DEEP = Shape(3, 120, 7, 7, 136, 3, 3, 1, 1, "deep")
DEEP_S2 = Shape(3, 130, 10, 10, 72, 3, 3, 2, 1, "deep-s2")
TAIL = Shape(8, 32, 112, 112, 128, 3, 3, 1, 1, "tail-split")
SMALL = Shape(8, 16, 16, 16, 32, 3, 3, 1, 1, "small3x3")
LONG = Shape(8, 32, 28, 28, 48, 3, 3, 1, 1, "long-reduction")   # BackwardFilter reduces 6272 rows: many chunks


def test_paths_without_atomics_are_bit_reproducible_in_the_default_mode():
    assert ucd.ucd_set_deterministic(-1) == 0
    s = SMALL
    x, w, dy = inputs(s, seed=31)
    cases = [(op, algo) for op in (ucd.FWD, ucd.BWD_DATA)
             for algo in (ucd.ALGO_IM2COL, ucd.ALGO_WINOGRAD, ucd.ALGO_WINOGRAD4, ucd.ALGO_FFT)]
    cases.append((ucd.FWD, ucd.ALGO_IMPLICIT))       # one tile row, no split: plain stores
    for op, algo in cases:
        text = launches(s, op, algo, s.N)
        assert "Atomic" not in text and "tail=" not in text, text
        runs = [run_hip(s, op, [(algo, 5), (algo, 3)], x=x, w=w, dy=dy) for _ in range(3)]
        assert all(np.array_equal(runs[0], r) for r in runs[1:]), (op, algo)


def test_default_mode_splits_are_what_the_header_says():
    # the launches the reproducible mode exists for really do use atomics by default
    assert "EpiNCHWAtomic" in launches(DEEP, ucd.FWD, ucd.ALGO_IMPLICIT, DEEP.N)
    assert "tail=" in launches(TAIL, ucd.FWD, ucd.ALGO_IMPLICIT, TAIL.N)
    assert "EpiAtomic" in launches(DEEP, ucd.BWD_FILTER, ucd.ALGO_IMPLICIT, DEEP.N)


@pytest.mark.parametrize("s", [DEEP, DEEP_S2, TAIL, SMALL, LONG], ids=lambda s: s.name)
def test_reproducible_mode_is_bit_identical_and_right(deterministic, s):
    desc = ucd.layer(s)
    x, w, dy = inputs(s, seed=32)
    for op in OPS:
        text = launches(s, op, ucd.ALGO_IMPLICIT, s.N)
        # no split outputs, no spread tails; a single-chunk BackwardFilter adds each element once
        assert "EpiNCHWAtomic" not in text and "tail=" not in text, text
        assert "EpiAtomic" not in text or "splits=1 " in text, text
        for algo in range(ucd.N_ALGO):
            if ucd.ucd_workspace_size(desc, op, algo, s.N) == ucd.WS_NA:
                continue
            assert not (op == ucd.BWD_FILTER and algo != ucd.ALGO_IMPLICIT)
            parts = [s.N] if s.N < 3 else [s.N - 2, 2]
            micro = [(algo, b) for b in parts]
            ref = run_oracle(s, op, x=x, w=w, dy=dy)
            runs = [run_hip(s, op, micro, x=x, w=w, dy=dy) for _ in range(3)]
            assert all(np.array_equal(runs[0], r) for r in runs[1:]), (s.name, op, algo)
            assert rel_l2(runs[0], ref) <= l2_tol(micro), (s.name, op, algo)


def test_reproducible_backward_filter_uses_workspace_partials_and_accumulates(deterministic):
    s = LONG
    desc = ucd.layer(s)
    need = ucd.ucd_workspace_size(desc, ucd.BWD_FILTER, ucd.ALGO_IMPLICIT, s.N)
    text = launches(s, ucd.BWD_FILTER, ucd.ALGO_IMPLICIT, s.N)
    splits = int(text.split("splits=")[1].split()[0])
    assert splits > 1 and need == 4 * splits * s.K * s.C * s.R * s.S
    assert "EpiPartial" in text and "reduce_partials_kernel" in text
    x, w, dy = inputs(s, seed=33)
    dw0 = np.random.default_rng(5).standard_normal(s.w_shape).astype(np.float32)
    ref = run_oracle(s, ucd.BWD_FILTER, x=x, dy=dy, beta=1.0, dw0=dw0)
    runs = [run_hip(s, ucd.BWD_FILTER, [(ucd.ALGO_IMPLICIT, 3), (ucd.ALGO_IMPLICIT, 5)], x=x, dy=dy, beta=1.0, dw0=dw0)
            for _ in range(2)]
    assert np.array_equal(runs[0], runs[1])
    assert rel_l2(runs[0], ref) <= 1e-5


def test_reproducible_mode_plans_and_runs_a_layer(deterministic):
    """WR planning in the mode (its own timings), then two executions of the planned configuration."""
    import torch
    s = Shape(32, 64, 14, 14, 96, 3, 3, 1, 1, "b32")
    desc = ucd.layer(s)
    x, w, dy = inputs(s, seed=34)
    dev = torch.device("cuda:0")
    xd, wd, dyd = (torch.from_numpy(a).to(dev) for a in (x, w, dy))
    limit = 8 << 20
    ws = torch.empty(limit // 4, dtype=torch.float32, device=dev)
    outs = {ucd.FWD: torch.empty(s.y_shape, device=dev), ucd.BWD_DATA: torch.empty(s.x_shape, device=dev),
            ucd.BWD_FILTER: torch.empty(s.w_shape, device=dev)}
    bufs = {ucd.FWD: (xd, wd, outs[ucd.FWD]), ucd.BWD_DATA: (outs[ucd.BWD_DATA], wd, dyd),
            ucd.BWD_FILTER: (xd, outs[ucd.BWD_FILTER], dyd)}
    for op in OPS:
        plan = ucd.ucd_plan(desc, op, limit, ucd.POLICY_POW2, *bufs[op], ws)
        assert plan.ws_bytes <= limit
        res = []
        for _ in range(2):
            outs[op].fill_(float("nan"))
            if op == ucd.FWD:
                ucd.ucd_conv_fwd(plan, xd, wd, outs[op], ws)
            elif op == ucd.BWD_DATA:
                ucd.ucd_conv_bwd_data(plan, dyd, wd, outs[op], ws)
            else:
                ucd.ucd_conv_bwd_filter(plan, xd, dyd, outs[op], 0.0, ws)
            torch.cuda.synchronize()
            res.append(outs[op].cpu().numpy())
        assert np.array_equal(res[0], res[1])
        assert rel_l2(res[0], run_oracle(s, op, x=x, w=w, dy=dy)) <= l2_tol(plan.micro)
