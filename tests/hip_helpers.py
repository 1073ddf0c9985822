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


def run_hip(s, op, micro, x=None, w=None, dy=None, beta=0.0, dw0=None, poison=True):
    """Execute a forced configuration; inputs are numpy float32 arrays. Returns numpy float32."""
    import torch
    dev = torch.device("cuda:0")
    desc = ucd.layer(s)
    plan = ucd.ucd_plan_fixed(desc, op, micro)
    need = plan.ws_bytes
    ws = torch.empty(max(need, 4) // 4 + 64, dtype=torch.float32, device=dev)
    if poison:
        ws.fill_(float("nan"))
    fill = float("nan") if poison else 0.0
    if op == ucd.FWD:
        xd, wd = torch.from_numpy(x).to(dev), torch.from_numpy(w).to(dev)
        out = torch.full(s.y_shape, fill, dtype=torch.float32, device=dev)
        ucd.ucd_conv_fwd(plan, xd, wd, out, ws)
    elif op == ucd.BWD_DATA:
        dyd, wd = torch.from_numpy(dy).to(dev), torch.from_numpy(w).to(dev)
        out = torch.full(s.x_shape, fill, dtype=torch.float32, device=dev)
        ucd.ucd_conv_bwd_data(plan, dyd, wd, out, ws)
    else:
        xd, dyd = torch.from_numpy(x).to(dev), torch.from_numpy(dy).to(dev)
        if dw0 is not None:
            out = torch.from_numpy(dw0).to(dev).clone()
        else:
            out = torch.full(s.w_shape, fill, dtype=torch.float32, device=dev)
        ucd.ucd_conv_bwd_filter(plan, xd, dyd, out, beta, ws)
    torch.cuda.synchronize()
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
