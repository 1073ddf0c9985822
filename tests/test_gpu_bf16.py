"""GPU parity of the bf16-storage variant (descriptor dtype 1): x, w, dy, y, dx are bfloat16, dw is
fp32.  The oracle runs in fp64 on exactly the values the library is handed (the bf16-rounded
inputs widened), so the only differences are fp32 accumulation order and the rounding of y / dx
to bf16 on store.

Tolerances: the paper states none for reduced precision.  bfloat16 keeps 8 significant bits, so
rounding an output to nearest moves it by at most half a unit in the last place, 2^-8 of its
magnitude; over a tensor that is a relative L2 error of about 2^-8 / sqrt(3) = 2.3e-3, so 5e-3 is
asserted for y and dx, together with the elementwise bound
|got - ref| <= 2^-8 |ref| + 1e-5 rms(ref) (half an ulp plus the fp32 accumulation error).
dw stays fp32 and keeps the fp32 path's tolerances (1e-5; 1e-4 for Winograd).
"""
import numpy as np
import pytest

from paper_1804_04806_amd import synth, ucd
from paper_1804_04806_amd.synth import Shape
from hip_helpers import GuardedWorkspace, inputs, l2_tol, rel_l2, run_oracle

pytestmark = pytest.mark.gpu

SHAPES = [
    Shape(8, 16, 16, 16, 32, 3, 3, 1, 1, "small3x3"),
    Shape(5, 3, 37, 35, 20, 11, 11, 4, 0, "conv1-like"),
    Shape(3, 24, 13, 13, 40, 5, 5, 1, 2, "conv2-like"),
    Shape(4, 70, 13, 13, 136, 3, 3, 1, 1, "conv3-like"),
    Shape(3, 8, 30, 30, 16, 7, 7, 2, 3, "stem-like"),
    Shape(2, 3, 30, 31, 16, 7, 7, 2, 3, "stem-c3"),
    Shape(3, 20, 14, 14, 36, 3, 3, 2, 1, "down3x3"),
    Shape(2, 64, 10, 10, 40, 3, 3, 2, 1, "c64-s2"),
    Shape(3, 20, 14, 14, 36, 1, 1, 2, 0, "proj1x1"),
    Shape(2, 40, 9, 9, 130, 1, 1, 1, 0, "1x1"),
    Shape(2, 6, 9, 12, 7, 2, 4, 1, 1, "evenfilter"),
    Shape(2, 96, 9, 9, 192, 3, 3, 1, 1, "c96k192"),
    Shape(3, 120, 7, 7, 136, 3, 3, 1, 1, "deep"),
    Shape(3, 5, 7, 7, 9, 3, 3, 1, 1, "odd-chw"),               # second micro-batch starts at an odd element: 2-byte aligned tensors
    Shape(9, 20, 13, 13, 24, 3, 3, 1, 1, "t49-n9"),            # fused BackwardFilter with the last tile group spread over 8 images
    Shape(2, 5, 11, 14, 7, 3, 3, 1, 0, "pad0-3x3"),
    Shape(2, 5, 6, 9, 7, 3, 3, 1, 2, "pad2-3x3"),
]
DIVISIONS = {9: [[9], [1, 8]], 8: [[8], [3, 5]], 5: [[5], [2, 3]], 4: [[4], [1, 3]], 3: [[3], [1, 2]], 2: [[2], [1, 1]]}


def bf16_inputs(s, seed):
    """(bits, values): uint16 storage handed to the library, and the exact fp32 values it holds."""
    arrs = inputs(s, seed)
    bits = [synth.to_bf16_bits(a) for a in arrs]
    vals = [synth.from_bf16_bits(b) for b in bits]
    return bits, vals


def dev_bf16(bits):
    import torch
    return torch.from_numpy(bits.view(np.int16)).to("cuda:0").view(torch.bfloat16)


def run_hip_bf16(s, op, micro, bits, beta=0.0, dw0=None):
    import torch
    dev = torch.device("cuda:0")
    desc = ucd.layer(s, dtype=1)
    plan = ucd.ucd_plan_fixed(desc, op, micro)
    need = plan.ws_bytes
    guarded = GuardedWorkspace(need)   # exactly the plan's bytes, a guard region behind them
    ws = guarded.tensor
    xb, wb, dyb = (dev_bf16(b) for b in bits)
    if op == ucd.FWD:
        out = torch.full(s.y_shape, float("nan"), dtype=torch.bfloat16, device=dev)
        ucd.ucd_conv_fwd(plan, xb, wb, out, ws, need)
    elif op == ucd.BWD_DATA:
        out = torch.full(s.x_shape, float("nan"), dtype=torch.bfloat16, device=dev)
        ucd.ucd_conv_bwd_data(plan, dyb, wb, out, ws, need)
    else:
        out = (torch.from_numpy(dw0).to(dev).clone() if dw0 is not None
               else torch.full(s.w_shape, float("nan"), dtype=torch.float32, device=dev))
        ucd.ucd_conv_bwd_filter(plan, xb, dyb, out, beta, ws, need)
    torch.cuda.synchronize()
    guarded.check_guard(need)
    return out.float().cpu().numpy()


def check_bf16_output(got, ref, ctx, slack=1e-5):
    """`slack` (in units of the tensor's rms) is what an element may be off beyond its own rounding to
    bf16: 1e-5 where the products are exact (bf16 operands, fp32 sums); 3e-2 for the fused Winograd
    kernel on the bf16 matrix pipe, which rounds the transformed filter and the transformed patches to
    bf16 (a relative 2^-9 each on 16 x Ci products per output: 4.2e-3 relative L2 in a numpy model of
    it, elements up to 1.8e-2 rms off)."""
    assert np.isfinite(got).all(), ctx
    assert rel_l2(got, ref) <= 5e-3, (ctx, rel_l2(got, ref))
    rms = float(np.sqrt(np.mean(np.square(ref)))) or 1.0
    bound = np.abs(ref) * 2.0 ** -8 + slack * rms
    worst = float(np.max(np.abs(got - ref) - bound))
    assert worst <= 0.0, (ctx, worst)
    # what is stored really is bf16: the low 16 bits of every value are clear
    assert not (got.astype(np.float32).view(np.uint32) & 0xFFFF).any(), ctx


@pytest.mark.parametrize("s", SHAPES, ids=lambda s: s.name)
@pytest.mark.parametrize("op", [ucd.FWD, ucd.BWD_DATA, ucd.BWD_FILTER], ids=["fwd", "bwd_data", "bwd_filter"])
def test_bf16_parity_all_algorithms_and_divisions(s, op):
    bits, (x, w, dy) = bf16_inputs(s, seed=21)
    ref = run_oracle(s, op, x=x, w=w, dy=dy)
    desc = ucd.layer(s, dtype=1)
    ran = 0
    for algo in range(ucd.N_ALGO):
        for parts in DIVISIONS[s.N]:
            if any(ucd.ucd_workspace_size(desc, op, algo, b) == ucd.WS_NA for b in parts):
                continue
            got = run_hip_bf16(s, op, [(algo, b) for b in parts], bits)
            ctx = (s.name, ucd.OP_NAMES[op], ucd.ALGO_NAMES[algo], parts)
            if op == ucd.BWD_FILTER:
                assert rel_l2(got, ref) <= l2_tol([(algo, 0)]), (ctx, rel_l2(got, ref))
            else:
                check_bf16_output(got, ref, ctx, slack=3e-2 if algo == ucd.ALGO_WINOGRAD_FUSED else 1e-5)
            ran += 1
    assert ran >= 2


def test_bf16_workspace_sizes_equal_fp32():
    """Workspace matrices stay fp32, so the workspace need does not depend on the dtype; the one
    exceptions are the mirrored filter copy, which has the tensors' element type, and the 5x5 Winograd
    kernels, which exist for fp32 tensors only."""
    for s in SHAPES:
        for op in range(3):
            for algo in range(ucd.N_ALGO):
                half, full = (ucd.ucd_workspace_size(ucd.layer(s, dtype=dt), op, algo, s.N) for dt in (1, 0))
                if algo == ucd.ALGO_IMPLICIT_MIRROR and full != ucd.WS_NA:
                    n = s.K * s.C * s.R * s.S
                    assert (half, full) == ((2 * n + 15) // 16 * 16, (4 * n + 15) // 16 * 16)
                elif algo == ucd.ALGO_WINOGRAD5_FUSED:
                    assert half == ucd.WS_NA   # written for fp32 tensors only
                else:
                    assert half == full


def test_bf16_bwd_filter_beta_one_accumulates_in_fp32():
    s = SHAPES[3]
    bits, (x, w, dy) = bf16_inputs(s, seed=4)
    dw0 = np.random.default_rng(1).standard_normal(s.w_shape).astype(np.float32)
    ref = run_oracle(s, ucd.BWD_FILTER, x=x, dy=dy, beta=1.0, dw0=dw0)
    got = run_hip_bf16(s, ucd.BWD_FILTER, [(ucd.ALGO_IMPLICIT, 1), (ucd.ALGO_IM2COL, 3)], bits, beta=1.0, dw0=dw0)
    assert rel_l2(got, ref) <= 1e-5


def test_bf16_plan_on_device_and_execute():
    """WR planning on bf16 buffers (the w scratch doubles as the fp32 dw), then execution."""
    import torch
    s = SHAPES[0]
    desc = ucd.layer(s, dtype=1)
    bits, (x, w, dy) = bf16_inputs(s, seed=8)
    xb, wb, dyb = (dev_bf16(b) for b in bits)
    dev = xb.device
    limit = 1 << 20
    ws = torch.empty(limit // 4, dtype=torch.float32, device=dev)
    dw_scratch = torch.empty(s.w_shape, dtype=torch.float32, device=dev)
    for op in (ucd.FWD, ucd.BWD_DATA, ucd.BWD_FILTER):
        scratch_x, scratch_y = xb.clone(), dyb.clone()
        plan = ucd.ucd_plan(desc, op, limit, ucd.POLICY_ALL, scratch_x,
                            dw_scratch if op == ucd.BWD_FILTER else wb.clone(), scratch_y, ws)
        assert sum(b for _, b in plan.micro) == s.N
        ref = run_oracle(s, op, x=x, w=w, dy=dy)
        if op == ucd.FWD:
            out = torch.empty(s.y_shape, dtype=torch.bfloat16, device=dev)
            ucd.ucd_conv_fwd(plan, xb, wb, out, ws)
            check_bf16_output(out.float().cpu().numpy(), ref, "fwd")
        elif op == ucd.BWD_DATA:
            out = torch.empty(s.x_shape, dtype=torch.bfloat16, device=dev)
            ucd.ucd_conv_bwd_data(plan, dyb, wb, out, ws)
            check_bf16_output(out.float().cpu().numpy(), ref, "bwd_data")
        else:
            out = torch.empty(s.w_shape, dtype=torch.float32, device=dev)
            ucd.ucd_conv_bwd_filter(plan, xb, dyb, out, 0.0, ws)
            assert rel_l2(out.cpu().numpy(), ref) <= 1e-5
