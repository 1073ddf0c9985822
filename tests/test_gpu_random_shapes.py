"""GPU parity on seeded random layer shapes: every algorithm that applies, fp32 and bf16 tensors, whole
and divided micro-batches, against the fp64 oracle.  The hand-picked shapes of the other files aim at
known tile and border cases; these catch the combinations nobody thought of (a strided layer whose
BackwardData phase grid is three columns wider than dy was found this way)."""
import numpy as np
import pytest

from paper_1804_04806_amd import ucd
from paper_1804_04806_amd.synth import Shape
from hip_helpers import inputs, rel_l2, run_hip, run_oracle
from test_gpu_bf16 import bf16_inputs, run_hip_bf16
from test_gpu_conv import TOL

pytestmark = pytest.mark.gpu

MAX_WS = 1 << 28


def random_shape(rng, i):
    n = int(rng.choice([1, 2, 3, 5, 8, 9]))
    r = int(rng.choice([1, 1, 2, 3, 3, 3, 4, 5, 5, 7, 11]))
    s = r if rng.random() < 0.8 else int(rng.choice([1, 2, 3, 4, 5]))
    stride = int(rng.choice([1, 1, 1, 2, 3, 4]))
    c, k = int(rng.integers(1, 90)), int(rng.integers(1, 150))
    h, w = int(rng.integers(max(r, 2), r + 24)), int(rng.integers(max(s, 2), s + 24))
    pad = int(rng.integers(0, max(r, s) // 2 + 2))
    pad = min(pad, r - 1, s - 1) if min(r, s) > 1 else 0
    return Shape(n, c, h, w, k, r, s, stride, pad, f"random{i}")


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_shapes_all_algorithms(seed):
    rng = np.random.default_rng(seed)
    ran = 0
    for i in range(40):
        s = random_shape(rng, i)
        if s.P < 1 or s.Q < 1:
            continue
        bf = i % 3 == 2
        desc = ucd.layer(s, dtype=1 if bf else 0)
        if bf:
            bits, (x, w, dy) = bf16_inputs(s, seed=300 + i)
        else:
            x, w, dy = inputs(s, seed=300 + i)
        for op in (ucd.FWD, ucd.BWD_DATA, ucd.BWD_FILTER):
            ref = None
            for algo in range(ucd.N_ALGO):
                parts = [s.N] if s.N < 2 or (i + algo) % 2 else [1, s.N - 1]
                sizes = [ucd.ucd_workspace_size(desc, op, algo, b) for b in parts]
                if any(z == ucd.WS_NA or z > MAX_WS for z in sizes):
                    continue
                if ref is None:
                    ref = run_oracle(s, op, x=x, w=w, dy=dy)
                micro = [(algo, b) for b in parts]
                got = run_hip_bf16(s, op, micro, bits) if bf else run_hip(s, op, micro, x=x, w=w, dy=dy)
                ctx = (s, "bf16" if bf else "f32", ucd.OP_NAMES[op], ucd.ALGO_NAMES[algo], parts)
                assert np.isfinite(got).all(), ctx
                tol = 5e-3 if bf and op != ucd.BWD_FILTER else TOL[algo]   # y / dx stored as bf16: the output rounding
                assert rel_l2(got, ref) <= tol, (ctx, rel_l2(got, ref))
                ran += 1
    assert ran >= 200
