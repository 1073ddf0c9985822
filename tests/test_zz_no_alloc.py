"""The Forward entry point that allocates nothing (its workspace is an array the library's code
object holds on the GPU) against ucd_conv_fwd with a caller's workspace, through the C-ABI: two
calls in a row on the same array, the second on a smaller layer, plus the size limit."""
import numpy as np
import pytest

from paper_1804_04806_amd import ucd
from paper_1804_04806_amd.synth import Shape
from hip_helpers import inputs, rel_l2, run_oracle

pytestmark = pytest.mark.gpu


def both_ways(s, micro, seed):
    """(static-workspace result, caller-workspace result, oracle) of one forced configuration."""
    import torch
    dev = torch.device("cuda:0")
    desc = ucd.layer(s)
    x, w, dy = inputs(s, seed=seed)
    xd, wd = torch.from_numpy(x).to(dev), torch.from_numpy(w).to(dev)
    plan = ucd.ucd_plan_fixed(desc, ucd.FWD, micro)
    assert 0 < plan.ws_bytes <= ucd.STATIC_WS_BYTES
    ws = torch.full((plan.ws_bytes // 4,), float("nan"), dtype=torch.float32, device=dev)
    y_ref = torch.full(s.y_shape, float("nan"), dtype=torch.float32, device=dev)
    y_got = torch.full(s.y_shape, float("nan"), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    ucd.ucd_conv_fwd(plan, xd, wd, y_ref, ws)
    ucd.ucd_conv_fwd_static_ws(plan, xd, wd, y_got)
    torch.cuda.synchronize()
    return y_got.cpu().numpy(), y_ref.cpu().numpy(), run_oracle(s, ucd.FWD, x=x, w=w)


def test_static_workspace_forward_matches_the_caller_workspace_entry_point():
    big = Shape(8, 16, 16, 16, 32, 3, 3, 1, 1, "small3x3")
    small = Shape(3, 6, 9, 11, 10, 3, 3, 1, 1, "smaller")
    # first call: Winograd then im2col micro-batches (filter transform, V, Z, column matrix all in
    # the array); second call, right after, on a smaller layer: it finds the first call's contents
    calls = [(big, [(ucd.ALGO_WINOGRAD, 5), (ucd.ALGO_IM2COL, 3)], 21),
             (small, [(ucd.ALGO_WINOGRAD4, 2), (ucd.ALGO_FFT, 1)], 22)]
    for s, micro, seed in calls:
        got, ref, exact = both_ways(s, micro, seed)
        assert np.isfinite(got).all()
        # no atomics in these Forward paths: the two entry points run the same kernels on the same
        # bits, only the workspace address differs
        assert np.array_equal(got, ref), s.name
        assert rel_l2(got, exact) <= 1e-4, s.name


def test_static_workspace_refuses_a_plan_beyond_its_size():
    import torch
    dev = torch.device("cuda:0")
    s = Shape(16, 96, 27, 27, 256, 5, 5, 1, 2, "conv2-b16")
    desc = ucd.layer(s)
    plan = ucd.ucd_plan_fixed(desc, ucd.FWD, [(ucd.ALGO_IM2COL, 16)])
    assert plan.ws_bytes > ucd.STATIC_WS_BYTES
    x = torch.zeros(s.x_shape, device=dev)
    w = torch.zeros(s.w_shape, device=dev)
    y = torch.zeros(s.y_shape, device=dev)
    with pytest.raises(ucd.UcdError) as e:
        ucd.ucd_conv_fwd_static_ws(plan, x, w, y)
    assert e.value.status == ucd.E_WS_TOO_SMALL
    # a zero-workspace plan runs without touching the array
    plan0 = ucd.ucd_plan_fixed(desc, ucd.FWD, [(ucd.ALGO_IMPLICIT, 16)])
    ucd.ucd_conv_fwd_static_ws(plan0, x, w, y)
    torch.cuda.synchronize()
    assert float(y.abs().sum()) == 0.0
