"""Shared helpers of the GPU parity tests: run the HIP path through the C-ABI binding on torch
device buffers and return numpy results; run the oracle on the same bits."""
import numpy as np

from oracle import conv as oc
from paper_1804_04806_amd import synth, ucd


def oracle_layer(s):
    return oc.Layer(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.stride, s.pad, s.pad)


def rel_l2(got, ref):
    got = np.asarray(got, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / den) if den > 0 else float(np.linalg.norm(got))


def ws_need(desc, op, micro):
    need = 0
    for a, b in micro:
        n = ucd.ucd_workspace_size(desc, op, a, b)
        assert n != ucd.WS_NA, (op, a, b)
        need = max(need, n)
    return need


# Relative-L2 bounds by what a configuration runs.  The benchmark spec gives 1e-5 for the direct /
# GEMM paths and 1e-3 for Winograd; the Winograd kernels measure 3e-7 (2x2 tiles) to 4e-6 (4x4
# tiles) and the tiled FFT 1e-7 to 2e-7, so Winograd is held to 1e-4 and the FFT to the GEMM bound.
def l2_tol(micro):
    return 1e-4 if any(a in ucd.WINOGRAD_ALGOS for a, _ in micro) else 1e-5


# Elementwise bound, as a multiple of the reference's rms: |got - ref| <= elementwise_tol * rms(ref).
# An fp32 result of rms-sized terms is off by a few 1e-7 rms per element (1e-5 rms for 4x4 Winograd
# tiles): one wrong term (a dropped tap, a neighbour's pixel) is off by about 1/sqrt(reduction
# length) of an rms, i.e. 1e-2 or more.
# With bf16 tensors the fused Winograd kernel multiplies on the bf16 matrix pipe: the transformed filter
# and patches are rounded to bf16 (a relative 2^-9 each, 16 x Ci products per output), which in a numpy
# model of the kernel leaves elements up to 1.8e-2 rms off (4.2e-3 relative L2): 3e-2 there.
def elementwise_tol(micro, bf16=False):
    if bf16 and any(a == ucd.ALGO_WINOGRAD_FUSED for a, _ in micro):
        return 3e-2
    return 1e-3 if any(a in ucd.WINOGRAD_ALGOS for a, _ in micro) else 1e-4


class GuardedWorkspace:
    """A device workspace of exactly `nbytes` usable bytes followed by a guard region; the whole
    buffer is poisoned with NaN and `check_guard` asserts that nothing outside the byte ranges a
    run was entitled to has been written."""
    GUARD = 4096
    PATTERN = 0x7FC00000   # float32 NaN as torch writes it

    def __init__(self, nbytes):
        import torch
        self.nbytes = int(nbytes)
        words = (self.nbytes + 3) // 4
        self.buf = torch.empty(words + self.GUARD // 4, dtype=torch.float32, device="cuda:0")
        self.tensor = self.buf[:max(words, 1)]
        self.ptr = self.buf.data_ptr()
        self.poison()

    def poison(self):
        self.buf.fill_(float("nan"))

    def check_guard(self, used):
        """used: a byte count (the run may have written [0, used)) or a list of (offset, bytes)."""
        import torch
        ranges = [(0, used)] if isinstance(used, int) else list(used)
        dirty = self.buf.view(torch.int32) != self.PATTERN
        for off, n in ranges:
            dirty[off // 4:(off + n + 3) // 4] = False
        bad = torch.nonzero(dirty)
        assert bad.numel() == 0, f"workspace written outside its ranges {ranges}: first at byte {4 * int(bad[0])}"


def run_hip(s, op, micro, x=None, w=None, dy=None, beta=0.0, dw0=None, poison=True):
    """Execute a forced configuration in a workspace of exactly the size the plan reports (a guard
    region behind it must stay untouched); inputs are numpy float32 arrays. Returns numpy float32."""
    import torch
    dev = torch.device("cuda:0")
    desc = ucd.layer(s)
    plan = ucd.ucd_plan_fixed(desc, op, micro)
    need = plan.ws_bytes
    guarded = GuardedWorkspace(need)
    ws = guarded.tensor
    fill = float("nan") if poison else 0.0
    if op == ucd.FWD:
        xd, wd = torch.from_numpy(x).to(dev), torch.from_numpy(w).to(dev)
        out = torch.full(s.y_shape, fill, dtype=torch.float32, device=dev)
        ucd.ucd_conv_fwd(plan, xd, wd, out, ws, need)
    elif op == ucd.BWD_DATA:
        dyd, wd = torch.from_numpy(dy).to(dev), torch.from_numpy(w).to(dev)
        out = torch.full(s.x_shape, fill, dtype=torch.float32, device=dev)
        ucd.ucd_conv_bwd_data(plan, dyd, wd, out, ws, need)
    else:
        xd, dyd = torch.from_numpy(x).to(dev), torch.from_numpy(dy).to(dev)
        if dw0 is not None:
            out = torch.from_numpy(dw0).to(dev).clone()
        else:
            out = torch.full(s.w_shape, fill, dtype=torch.float32, device=dev)
        ucd.ucd_conv_bwd_filter(plan, xd, dyd, out, beta, ws, need)
    torch.cuda.synchronize()
    guarded.check_guard(need)
    return out.cpu().numpy()


def run_oracle(s, op, x=None, w=None, dy=None, beta=0.0, dw0=None):
    L = oracle_layer(s)
    if op == ucd.FWD:
        return oc.conv_fwd(L, x, w)
    if op == ucd.BWD_DATA:
        return oc.conv_bwd_data(L, dy, w)
    return oc.conv_bwd_filter(L, x, dy, beta=beta, dw=dw0)


def inputs(s, seed=0, idx=0):
    return synth.make_x(s, seed, idx), synth.make_w(s, seed, idx), synth.make_dy(s, seed, idx)
