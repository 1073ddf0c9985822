#!/usr/bin/env python3
"""Benchmark of the micro-batched convolution hot path on one MI355X.

Workload: the AlexNet-shaped five-layer convolution stack at mini-batch 256, fp32 NCHW, a
64 MiB workspace limit per layer (WR policy).  One step = Forward + BackwardData +
BackwardFilter of every layer, each executed as the micro-batch configuration the WR planner
chose from on-device benchmarks (planning happens once, before the timed region, as in the
paper where it is amortised over training).  Inputs are seeded synthetic tensors already
resident in HBM.

Prints ONE JSON line: throughput in TFLOP/s of algorithmic convolution flops
(3 * sum 2*N*K*P*Q*C*R*S per step), ms per step, the same for the best undivided
single-algorithm plan, a roofline object for the dominant kernel and a CPU-oracle baseline.

    python bench.py [--gpus 1] [--steps 50] [--warmup 3] [--policy all|pow2|undivided]

Other workloads of the same shape family can be timed with --workload (not the contract line):
small (N=8, 64 KiB), resnet18 (64 MiB/layer, WR), densenet (B=64, 8 MiB/layer, WR),
resnet50-wr (64 MiB/layer) and resnet50-wd (one 512 MiB budget over all 159 kernels, WD).

    python bench.py --micro --net alexnet --layer conv4 --op fwd --algo implicit --b 256

times one (layer, operation, algorithm, micro-batch size) instead (or, with --copy-mib / --mfma-peak,
a plain device copy of known traffic / the register-only MFMA loop): the unit to put under
`rocprofv3 --kernel-trace --stats` or `--pmc` to look at a single kernel.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "conv ms/iter (fwd+bwdData+bwdFilter) @64MB workspace; TFLOP/s, % MFMA peak"
FP32_MFMA_PEAK_TFLOPS = 157.3   # MI355X dense fp32 matrix peak: 256 CU x 2.4 GHz x 256 flop/clk/CU
BF16_MFMA_PEAK_TFLOPS = 2500.0  # dense bf16 matrix peak (16x the fp32 rate); kernels named gemm_kernel_bf16
WS_LIMIT = 64 << 20

# HBM bytes (fetched + written) per matrix flop of the kernels of the default workload's planned
# step, from two rocprofv3 --pmc passes over this script (FETCH_SIZE, then WRITE_SIZE, each scaled by
# what the counter reads for a plain device copy of known size: x2.00 and x1.00): mean bytes per
# dispatch of a run whose benchmark cache came from a file (so that every dispatch has a shape of
# the step), divided by the mean matrix flops per launch of that run's step.
# `traffic` = this figure x the flops per launch of the step being timed: the planner does not
# pick the same micro-batch sizes every run, and a kernel's traffic follows its size.
MEASURED_TRAFFIC_BYTES_PER_FLOP = {
    "wino_fused_kernel": 313.0e6 / 37.52e9,
    "wino5_fused_kernel": 735.6e6 / 87.77e9,
    "wino_fused_filter_kernel": 569.6e6 / 46.04e9,
    "wino5_fused_filter_kernel": 913.4e6 / 90.6e9,
    "wino_fused_kernel<phases>": 475.1e6 / 31.38e9,
    "gemm_kernel<Tile<96x128>,PixelKLane<dy>,PixelKLane<x, no padding>,EpiAtomic>": 545.6e6 / 53.97e9,
    "gemm_kernel<Tile<96x128>,KLane0,GatherNLane<no padding>,EpiNCHW>": 242.9e6 / 26.99e9,
}

ALGO_IDS = {"implicit": 0, "im2col": 1, "winograd": 2, "winograd4": 3, "fft": 4, "winograd-fused": 5,
            "implicit-mirror": 6, "winograd5x5-fused": 7}

# name -> (description, layer table, batch, per-layer limit or total budget, "wr" | "wd", default policy)
WORKLOADS = {
    "alexnet": ("AlexNet-shaped 5-layer conv stack", "config_alexnet", 256, 64 << 20, "wr", "all"),
    "small": ("single small 3x3 layer", "config_small", 8, 64 << 10, "wr", "all"),
    # one budget of 15 kernels x 64 MiB: the WD counterpart of the default workload (Section 4.4 pairs WR at M
    # per kernel with WD at kernels x M in total)
    "alexnet-wd": ("AlexNet-shaped 5-layer conv stack", "config_alexnet", 256, 960 << 20, "wd", "all"),
    "resnet18": ("ResNet-18-shaped conv layers (20 layers)", "config_resnet18", 256, 64 << 20, "wr", "all"),
    "densenet": ("DenseNet-BC-style block (24 layers)", "config_densenet_block", 64, 8 << 20, "wr", "all"),
    "resnet50-wr": ("ResNet-50-shaped conv layers (53 layers)", "config_resnet50", 256, 64 << 20, "wr", "pow2"),
    "resnet50-wd": ("ResNet-50-shaped conv layers (53 layers, 159 kernels)", "config_resnet50", 256, 512 << 20,
                    "wd", "pow2"),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="alexnet", choices=sorted(WORKLOADS))
    ap.add_argument("--policy", default=None, choices=["all", "pow2", "undivided"])
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--ws-mib", type=float, default=None,
                    help="override the workload's workspace limit (per layer for WR, total for WD), in MiB")
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"],
                    help="bf16: x, w, dy, y, dx stored as bfloat16, implicit GEMMs on the bf16 matrix pipe with fp32 "
                         "accumulation (dw and workspaces fp32)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-samples", type=int, default=24)
    ap.add_argument("--bench-db", default=None,
                    help="benchmark database file: loaded before planning if it exists, saved afterwards")
    ap.add_argument("--skip-undivided", action="store_true",
                    help="do not time the undivided baseline (profiling runs: every launch of the process then "
                         "belongs to the planned step)")
    ap.add_argument("--memory-table", action="store_true",
                    help="also print, as markdown on stderr, the per-kernel workspace of the planned configuration "
                         "next to the undivided plan under a 512 MiB limit (the paper's Section 4.3 comparison)")
    # single-kernel mode
    ap.add_argument("--micro", action="store_true", help="time one algorithm on one micro-batch (see the docstring)")
    ap.add_argument("--net", default="alexnet", choices=["small", "alexnet", "resnet18", "densenet", "resnet50"])
    ap.add_argument("--layer", default="conv4")
    ap.add_argument("--op", default="fwd", choices=["fwd", "bwd_data", "bwd_filter"])
    ap.add_argument("--algo", default="implicit", choices=sorted(ALGO_IDS))
    ap.add_argument("--b", default="256", help="micro-batch size, or a comma-separated list (one JSON line each)")
    ap.add_argument("--back-to-back", action="store_true",
                    help="--micro: time --reps launches between one pair of events instead of one launch per pair")
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--copy-mib", type=int, default=0,
                    help="with --micro: a plain device copy of this many MiB (a kernel of known traffic, to "
                         "calibrate the FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--mfma-peak", action="store_true",
                    help="with --micro: the register-only MFMA loop with 0/2/4/8 vector FMAs per MFMA")
    return ap.parse_args()


class Pool:
    """One set of device buffers, sized for the largest layer, that every layer of a big
    workload takes views of (a resident ResNet-50 at batch 256 would need hundreds of GB)."""

    def __init__(self, layers, torch, dev, tdtype, synth):
        nx = max(s.N * s.C * s.H * s.W for s in layers)
        ny = max(s.N * s.K * s.P * s.Q for s in layers)
        nw = max(s.K * s.C * s.R * s.S for s in layers)
        # the same generator and distributions as the per-layer tensors (full-mantissa values: the
        # chip's clock under matrix load depends on the operands' bit patterns)
        self.x = torch.from_numpy(synth.make_flat(nx, "x")).to(dev).to(tdtype)
        self.dy = torch.from_numpy(synth.make_flat(ny, "dy")).to(dev).to(tdtype)
        self.w = torch.from_numpy(synth.make_flat(nw, "w", std=0.03)).to(dev).to(tdtype)
        self.y = torch.empty(ny, dtype=tdtype, device=dev)
        self.dx = torch.empty(nx, dtype=tdtype, device=dev)
        self.dw = torch.empty(nw, dtype=torch.float32, device=dev)


class LayerState:
    """Device tensors and plans of one layer."""

    def __init__(self, s, idx, torch, ucd, synth, dev, pool=None, tdtype=None):
        self.s = s
        self.desc = ucd.layer(s, dtype=1 if tdtype == torch.bfloat16 else 0)
        if pool is None:
            # the seeded fp32 values, rounded to nearest-even when the tensors are bf16
            self.x = torch.from_numpy(synth.make_x(s, 0, idx)).to(dev).to(tdtype)
            self.w = torch.from_numpy(synth.make_w(s, 0, idx)).to(dev).to(tdtype)
            self.dy = torch.from_numpy(synth.make_dy(s, 0, idx)).to(dev).to(tdtype)
            self.y = torch.empty(s.y_shape, dtype=tdtype, device=dev)
            self.dx = torch.empty(s.x_shape, dtype=tdtype, device=dev)
            self.dw = torch.empty(s.w_shape, dtype=torch.float32, device=dev)
        else:
            nx, ny, nw = s.N * s.C * s.H * s.W, s.N * s.K * s.P * s.Q, s.K * s.C * s.R * s.S
            self.x, self.dx = pool.x[:nx], pool.dx[:nx]
            self.dy, self.y = pool.dy[:ny], pool.y[:ny]
            self.w, self.dw = pool.w[:nw], pool.dw[:nw]

    def plan(self, ucd, policy, ws, limit):
        """WR planning for the three operations; each benchmark clobbers only output buffers."""
        p = {}
        p[ucd.FWD] = ucd.ucd_plan(self.desc, ucd.FWD, limit, policy, self.x, self.w, self.y, ws)
        p[ucd.BWD_DATA] = ucd.ucd_plan(self.desc, ucd.BWD_DATA, limit, policy, self.dx, self.w, self.dy, ws)
        p[ucd.BWD_FILTER] = ucd.ucd_plan(self.desc, ucd.BWD_FILTER, limit, policy, self.x, self.dw, self.dy, ws)
        return p

    def run(self, ucd, plans, ws, offsets=None):
        """offsets: byte offsets of the three kernels' workspace segments (WD), else one shared workspace."""
        if offsets is None:
            ucd.ucd_conv_fwd(plans[ucd.FWD], self.x, self.w, self.y, ws)
            ucd.ucd_conv_bwd_data(plans[ucd.BWD_DATA], self.dy, self.w, self.dx, ws)
            ucd.ucd_conv_bwd_filter(plans[ucd.BWD_FILTER], self.x, self.dy, self.dw, 0.0, ws)
        else:
            base, total = ws.data_ptr(), ws.numel() * 4
            f, d, g = offsets
            ucd.ucd_conv_fwd(plans[ucd.FWD], self.x, self.w, self.y, base + f, total - f)
            ucd.ucd_conv_bwd_data(plans[ucd.BWD_DATA], self.dy, self.w, self.dx, base + d, total - d)
            ucd.ucd_conv_bwd_filter(plans[ucd.BWD_FILTER], self.x, self.dy, self.dw, 0.0, base + g, total - g)


def plan_wd(ucd, states, pool, policy, ws, budget):
    """One global budget over all kernels (layers x {fwd, bwdData, bwdFilter}): desirable sets +
    0-1 programme.  Returns per-layer plan dicts and per-layer segment offsets."""
    descs, ops = [], []
    for st in states:
        for op in (ucd.FWD, ucd.BWD_DATA, ucd.BWD_FILTER):
            descs.append(st.desc)
            ops.append(op)
    # Benchmark every kernel first on its proper buffers (inputs read, only outputs clobbered) with
    # the whole budget as the limit, which fills the cache with exactly the timings the WD planner
    # asks for; its own scratch tensors are then never launched on.
    for st in states:
        st.plan(ucd, policy, ws, budget)
    # scratch for the call's capacity checks: the largest output buffers (never launched on)
    sx = max((st.dx for st in states), key=lambda t: t.numel())
    sw = max((st.dw for st in states), key=lambda t: t.numel())
    sy = max((st.y for st in states), key=lambda t: t.numel())
    plans, offs = ucd.ucd_plan_wd(descs, ops, budget, policy, sx, sw, sy, ws)
    per_layer, per_off = [], []
    for i in range(len(states)):
        per_layer.append({ucd.FWD: plans[3 * i], ucd.BWD_DATA: plans[3 * i + 1], ucd.BWD_FILTER: plans[3 * i + 2]})
        per_off.append(tuple(offs[3 * i:3 * i + 3]))
    return per_layer, per_off


def time_steps(torch, fn, steps, warmup):
    """Times exactly `steps` calls of fn between two synchronisations (the contract's figure) and,
    from events recorded on the launch stream between the calls, each step's own duration.
    Returns (ms per step, median step ms, min step ms)."""
    for _ in range(warmup):
        fn()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        ev[i].record()
        fn()
    ev[steps].record()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    each = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
    return ms, each[len(each) // 2], each[0]


def time_interleaved(torch, fn_a, fn_b, rounds, warmup):
    """A/B/A/B timing with events: the two configurations see the same clock and cache history.
    Returns (median ms of a, median ms of b, min of a, min of b)."""
    for _ in range(warmup):
        fn_a()
        fn_b()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2 * rounds + 1)]
    torch.cuda.synchronize()
    for i in range(rounds):
        ev[2 * i].record()
        fn_a()
        ev[2 * i + 1].record()
        fn_b()
    ev[2 * rounds].record()
    torch.cuda.synchronize()
    a = sorted(ev[2 * i].elapsed_time(ev[2 * i + 1]) for i in range(rounds))
    b = sorted(ev[2 * i + 1].elapsed_time(ev[2 * i + 2]) for i in range(rounds))
    return a[len(a) // 2], b[len(b) // 2], a[0], b[0]


def num(v):
    """Rounded for the JSON line; None for a figure that was not measured."""
    return None if v != v else round(v, 4)


def gemm_flops(text):
    """MFMA flops the GEMM launches of a micro-batch description issue: 2*M*N*K*batch each."""
    total = 0.0
    for part in text.split(";"):
        part = part.strip()
        if part.startswith(("wino_fused", "wino5_fused")):
            total += float(part.split("gemm_flops=")[1].split()[0])
        if not part.startswith("gemm_kernel"):
            continue
        f = dict(kv.split("=") for kv in part.split("> ")[-1].split() if "=" in kv)
        total += 2.0 * int(f["M"]) * int(f["N"]) * int(f["K"]) * int(f["batch"])
    return total


def executed_flops(ucd, states, plans):
    """Matrix flops one step really issues (Winograd and FFT issue fewer than the direct count,
    merged-phase BackwardData and padded Winograd tiles more)."""
    total = 0.0
    for st, pl in zip(states, plans):
        for op in (ucd.FWD, ucd.BWD_DATA, ucd.BWD_FILTER):
            for algo, b in pl[op].micro:
                total += gemm_flops(ucd.ucd_describe_micro(st.desc, op, algo, b)[0])
    return total


def kernel_class(ucd, desc, op, algo, b):
    """The dominant kernel a micro-batch run launches, as the library describes it (the names
    rocprofv3 shows are these template instantiations), if the run is that one kernel besides
    helpers of a few microseconds (zero fills, the Winograd filter transform and the final
    16 -> 9 reduction of the fused BackwardFilter); otherwise None (im2col, the unfused Winograd
    variants, FFT and strided BackwardData launch several kernels of comparable weight).
    Returns (name, matrix flops the kernel issues)."""
    text, n = ucd.ucd_describe_micro(desc, op, algo, b)
    parts = [p.strip() for p in text.split(";")]
    helpers = ("fill_zero_kernel", "zero_tiles_kernel", "wino_filter_kernel", "wino_dw_kernel", "mirror_filter_kernel",
               "wino5_filter_kernel", "wino5_dw_kernel", "wino_phase_filter_kernel", "wino_filter_bf16_kernel")
    main = [p for p in parts if p.startswith(("gemm_kernel", "wino_fused", "wino5_fused"))]
    others = [p for p in parts if p not in main and p not in helpers]
    if len(main) != 1 or others:
        return None
    if main[0].startswith(("wino_fused", "wino5_fused")):
        return main[0].split()[0], gemm_flops(main[0])
    name = main[0].split("> tiles=")[0] + ">"
    return name + (" (after " + parts[0] + ")" if len(parts) > 1 else ""), gemm_flops(main[0])


def dominant_kernel_roofline(torch, ucd, states, plans, ws, reps, traffic_table=None):
    """HIP-event timing (events recorded on the launch stream, `reps` launches back to back between
    them, as the launches of a step follow each other) of every single-kernel micro-batch launch of
    the planned step, grouped by kernel instantiation; returns the roofline object of the
    instantiation with the largest total time, and the per-instantiation table.  Flops are the
    matrix flops the kernel issues (2*M*N*K of its GEMM; for the fused Winograd kernels the 16 tile
    products), with the direct-convolution-equivalent rate beside them.
    BackwardFilter launches are timed as the accumulating (beta = 1) call, which is the GEMM
    kernel alone; with beta = 0 a small fill kernel precedes it."""
    groups = {}
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for st, pl in zip(states, plans):
        s = st.s
        x_img, y_img = s.C * s.H * s.W, s.K * s.P * s.Q
        for op in (ucd.FWD, ucd.BWD_DATA, ucd.BWD_FILTER):
            o = 0
            for algo, b in pl[op].micro:
                found = kernel_class(ucd, st.desc, op, algo, b)
                if found is not None:
                    cls, executed = found
                    xo = st.x.view(-1)[o * x_img:]
                    yo = st.y.view(-1)[o * y_img:]
                    dyo = st.dy.view(-1)[o * y_img:]
                    dxo = st.dx.view(-1)[o * x_img:]
                    args = {ucd.FWD: (xo, st.w, yo), ucd.BWD_DATA: (dyo, st.w, dxo),
                            ucd.BWD_FILTER: (xo, dyo, st.dw)}[op]
                    beta = 1.0 if op == ucd.BWD_FILTER else 0.0
                    ucd.ucd_run_micro(st.desc, op, algo, b, *args, beta, ws)
                    e0.record()
                    for _ in range(reps):
                        ucd.ucd_run_micro(st.desc, op, algo, b, *args, beta, ws)
                    e1.record()
                    e1.synchronize()
                    tot = e0.elapsed_time(e1)
                    g = groups.setdefault(cls, {"ms": 0.0, "flops": 0.0, "direct": 0.0, "launches": 0})
                    g["ms"] += tot / reps
                    g["flops"] += executed
                    g["direct"] += s.with_batch(b).flops
                    g["launches"] += 1
                o += b
    if not groups:
        return None, []
    table = [{"kernel": k, "launches_per_step": g["launches"], "ms_per_step": round(g["ms"], 4),
              "avg_launch_ms": round(g["ms"] / g["launches"], 4),
              "tflops": round(g["flops"] / (g["ms"] * 1e-3) / 1e12, 2),
              "direct_equivalent_tflops": round(g["direct"] / (g["ms"] * 1e-3) / 1e12, 2)}
             for k, g in sorted(groups.items(), key=lambda kv: -kv[1]["ms"])]
    name, g = max(groups.items(), key=lambda kv: kv[1]["ms"])
    achieved = g["flops"] / (g["ms"] * 1e-3) / 1e12
    peak = BF16_MFMA_PEAK_TFLOPS if name.startswith("gemm_kernel_bf16") else FP32_MFMA_PEAK_TFLOPS
    roof = {"bound": "mfma", "kernel": name, "achieved": round(achieved, 2), "peak": peak,
            "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
            "traffic": None,
            "launches_per_step": g["launches"], "avg_launch_ms": round(g["ms"] / g["launches"], 4),
            "flops_per_launch": g["flops"] / g["launches"],
            "direct_equivalent_tflops": round(g["direct"] / (g["ms"] * 1e-3) / 1e12, 2)}
    per_flop = (traffic_table or {}).get(name.split(" (after")[0])
    if per_flop is not None:
        roof["traffic"] = round(per_flop * roof["flops_per_launch"])
    return roof, table


def cpu_baseline(layers, n_samples):
    """The fp64 oracle, as it stands, on the first n_samples samples of every layer."""
    from oracle import conv as oc
    from paper_1804_04806_amd import synth
    flops, secs = 0.0, 0.0
    for idx, s in enumerate(layers):
        sb = s.with_batch(n_samples)
        L = oc.Layer(sb.N, sb.C, sb.H, sb.W, sb.K, sb.R, sb.S, sb.stride, sb.stride, sb.pad, sb.pad)
        x, w, dy = synth.make_x(sb, 0, idx), synth.make_w(sb, 0, idx), synth.make_dy(sb, 0, idx)
        t0 = time.perf_counter()
        oc.conv_fwd(L, x, w)
        oc.conv_bwd_data(L, dy, w)
        oc.conv_bwd_filter(L, x, dy)
        secs += time.perf_counter() - t0
        flops += 3 * sb.flops
    return {"value": round(flops / secs / 1e12, 6), "unit": "TFLOP/s", "cores": oc.threads(), "kind": "oracle",
            "sample": f"first {n_samples} samples of each of the {len(layers)} layers, fwd+bwdData+bwdFilter, "
                      f"fp64 direct loops, {secs:.1f} s",
            "ms_per_iter_scaled": round(secs * 1e3 * layers[0].N / n_samples, 1)}


def memory_table(ucd, states, plans, ws, title, batch, limit):
    """Markdown: per kernel, the workspace of the planned configuration under `limit` next to the
    best undivided plan with 512 MiB (what a framework that hands the library a generous workspace
    would hold), with each layer's tensor bytes (Section 4.3's per-layer memory comparison)."""
    import torch
    big = 512 << 20
    ws_big = torch.empty(big // 4, dtype=torch.float32, device=ws.device)
    lines = [f"### {title}, batch {batch}: workspace per kernel, planned at {limit >> 20} MiB vs undivided at 512 MiB", "",
             "| layer | x + y + w MiB | op | planned configuration | planned ws MiB | planned ms | undivided@512MiB | ws MiB | ms |",
             "|---|---|---|---|---|---|---|---|---|"]
    tot = {"data": 0.0, "planned": 0.0, "big": 0.0, "planned_ms": 0.0, "big_ms": 0.0}
    for st, pl in zip(states, plans):
        s = st.s
        u = st.plan(ucd, ucd.POLICY_UNDIVIDED, ws_big, big)
        esz = st.x.element_size()
        data = (s.N * s.C * s.H * s.W + s.N * s.K * s.P * s.Q + s.K * s.C * s.R * s.S) * esz / 2 ** 20
        tot["data"] += data
        peak_p = max(pl[op].ws_bytes for op in pl) / 2 ** 20
        peak_u = max(u[op].ws_bytes for op in u) / 2 ** 20
        tot["planned"] = max(tot["planned"], peak_p)   # WR: one workspace, reused by every kernel
        tot["big"] = max(tot["big"], peak_u)
        for op in (ucd.FWD, ucd.BWD_DATA, ucd.BWD_FILTER):
            micro, cost, need = pl[op].query()
            umicro, ucost, uneed = u[op].query()
            cfg = ", ".join(f"{ucd.ALGO_NAMES[a]}x{b}" for a, b in micro[:4]) + (" ..." if len(micro) > 4 else "")
            lines.append(f"| {s.name} | {data:.1f} | {ucd.OP_NAMES[op]} | {cfg} ({len(micro)} micro-batches) | "
                         f"{need / 2 ** 20:.1f} | {cost / 1e6:.3f} | {ucd.ALGO_NAMES[umicro[0][0]]} | {uneed / 2 ** 20:.1f} | {ucost / 1e6:.3f} |")
            tot["planned_ms"] += cost / 1e6
            tot["big_ms"] += ucost / 1e6
    lines += ["", f"Tensors of all layers: {tot['data']:.1f} MiB.  Workspace held (one buffer, reused by every kernel): "
                  f"{tot['planned']:.1f} MiB planned against {tot['big']:.1f} MiB undivided at 512 MiB; predicted step "
                  f"{tot['planned_ms']:.2f} ms against {tot['big_ms']:.2f} ms.", ""]
    return "\n".join(lines)


def micro_main(args):
    """One (layer, operation, algorithm, micro-batch size) through ucd_run_micro, or a calibration kernel."""
    import torch
    from paper_1804_04806_amd import synth, ucd
    dev = torch.device("cuda:0")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn):
        times = []
        for it in range(args.warmup + args.reps):
            e0.record()
            r = fn()
            e1.record()
            e1.synchronize()
            if it >= args.warmup:
                times.append(e0.elapsed_time(e1))
        return times, r

    if args.mfma_peak:
        blocks, iters = 512, 2000
        scratch = torch.empty(blocks * 256, dtype=torch.float32, device=dev)
        out = {}
        for valu in (0, 2, 4, 8):
            times, flops = timed(lambda: ucd.ucd_mfma_probe(valu, blocks, iters, scratch))
            out[f"tflops_with_{valu}_valu_per_mfma"] = round(flops / min(times) / 1e9, 1)
        # 16 accumulator tiles per wave (256 registers): one wave per SIMD, as in the fused Winograd kernel
        for valu in (0, 2, 4):
            times, flops = timed(lambda: ucd.ucd_mfma_probe(100 + valu, blocks, iters, scratch))
            out[f"one_wave_per_simd_tflops_with_{valu}_valu_per_mfma"] = round(flops / min(times) / 1e9, 1)
        # the same, but every accumulator takes 4 dependent MFMAs in a row
        for valu in (0, 2):
            times, flops = timed(lambda: ucd.ucd_mfma_probe(200 + valu, blocks, iters, scratch))
            out[f"one_wave_per_simd_4_in_a_row_tflops_with_{valu}_valu_per_mfma"] = round(flops / min(times) / 1e9, 1)
        print(json.dumps(out))
        return
    if args.copy_mib:
        n = args.copy_mib * (1 << 20) // 4
        src = torch.rand(n, device=dev)
        dst = torch.empty_like(src)
        times, _ = timed(lambda: dst.copy_(src))
        print(json.dumps({"copy_mib": args.copy_mib, "ms_min": round(min(times), 4),
                          "GBps_read_plus_write": round(2 * n * 4 / min(times) / 1e6, 1)}))
        return
    nets = {"small": synth.config_small, "alexnet": synth.config_alexnet, "resnet18": synth.config_resnet18,
            "densenet": synth.config_densenet_block, "resnet50": synth.config_resnet50}
    op = {"fwd": ucd.FWD, "bwd_data": ucd.BWD_DATA, "bwd_filter": ucd.BWD_FILTER}[args.op]
    algo = ALGO_IDS[args.algo]
    td = torch.bfloat16 if args.dtype == "bf16" else torch.float32
    for b in [int(v) for v in str(args.b).split(",")]:
        s = next(l for l in nets[args.net]() if l.name == args.layer).with_batch(b)
        desc = ucd.layer(s, dtype=1 if args.dtype == "bf16" else 0)
        need = ucd.ucd_workspace_size(desc, op, algo, b)
        if need == ucd.WS_NA:
            raise SystemExit("algorithm does not apply to this layer/operation")
        x = torch.from_numpy(synth.make_x(s)).to(dev).to(td)
        w = torch.from_numpy(synth.make_w(s)).to(dev).to(td)
        y = torch.from_numpy(synth.make_dy(s)).to(dev).to(td)
        if op == ucd.BWD_FILTER:
            w = w.float()   # dw is fp32 for every dtype
        ws = torch.empty(max(need, 4) // 4, dtype=torch.float32, device=dev)
        a, bsrc, out = {ucd.FWD: (x, w, y), ucd.BWD_DATA: (y, w, x), ucd.BWD_FILTER: (x, y, w)}[op]
        beta = 1.0 if op == ucd.BWD_FILTER else 0.0
        run = lambda: ucd.ucd_run_micro(desc, op, algo, b, a, bsrc, out, beta, ws)
        if args.back_to_back:
            for _ in range(max(args.warmup, 1)):
                run()
            e0.record()
            for _ in range(args.reps):
                run()
            e1.record()
            e1.synchronize()
            times = [e0.elapsed_time(e1) / args.reps]
        else:
            times, _ = timed(run)
        ms = min(times)
        text, _ = ucd.ucd_describe_micro(desc, op, algo, b)
        print(json.dumps({"layer": s.name, "op": args.op, "algo": args.algo, "b": b, "dtype": args.dtype,
                          "timing": "back-to-back" if args.back_to_back else "one launch per event pair",
                          "ms_min": round(ms, 4), "ms_avg": round(sum(times) / len(times), 4),
                          "tflops": round(s.flops / ms / 1e9, 2),
                          "executed_mfma_tflops": round(gemm_flops(text) / ms / 1e9, 2), "ws_bytes": need,
                          "launches": text}), flush=True)


def main():
    args = parse()
    if args.micro:
        if args.gpus != 1:
            sys.exit(2)
        micro_main(args)
        return
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_1804_04806_amd import synth, ucd
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(3)
    ucd.lib()  # fails loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    title, table, batch0, limit, mode, policy0 = WORKLOADS[args.workload]
    batch = args.batch or batch0
    if args.ws_mib is not None:
        limit = int(args.ws_mib * (1 << 20))
    policy_name = args.policy or policy0
    policy = {"all": ucd.POLICY_ALL, "pow2": ucd.POLICY_POW2, "undivided": ucd.POLICY_UNDIVIDED}[policy_name]
    layers = getattr(synth, table)() if args.workload == "small" else getattr(synth, table)(batch)
    tdtype = torch.bfloat16 if args.dtype == "bf16" else torch.float32
    pool = None if args.workload in ("alexnet", "alexnet-wd", "small") else Pool(layers, torch, dev, tdtype, synth)
    states = [LayerState(s, i, torch, ucd, synth, dev, pool, tdtype) for i, s in enumerate(layers)]
    ws = torch.empty(max(limit, 4) // 4, dtype=torch.float32, device=dev)
    flops_per_step = 3 * sum(s.flops for s in layers)

    have_db = bool(args.bench_db and os.path.exists(args.bench_db))
    if have_db:
        ucd.ucd_bench_load(args.bench_db)
    offsets = None
    # baseline: the best single algorithm per kernel with no workspace beyond its own layer limit
    # (WR undivided); for the WD workload the same per-kernel share of the budget
    base_limit = limit if mode == "wr" else limit // (3 * len(layers))
    plan_seconds = {}

    def timed_plan(name, pol, lim):
        """WR-plans every layer with one policy from an empty benchmark cache (unless a database
        file supplied it), so that the time is that policy's own benchmarking cost."""
        if not have_db:
            ucd.ucd_bench_clear()
        t0 = time.perf_counter()
        pl = [st.plan(ucd, pol, ws, lim) for st in states]
        plan_seconds[name] = round(time.perf_counter() - t0, 2)
        return pl

    undiv = timed_plan("undivided", ucd.POLICY_UNDIVIDED, base_limit)
    if mode == "wr":
        if policy_name != "pow2" and (policy_name == "all" or not have_db):
            timed_plan("pow2", ucd.POLICY_POW2, limit)   # reported for the comparison of Section 4.2 only
        plans = undiv if policy_name == "undivided" else timed_plan(policy_name, policy, limit)
    else:
        if not have_db:
            ucd.ucd_bench_clear()
        t0 = time.perf_counter()
        plans, offsets = plan_wd(ucd, states, pool, policy, ws, limit)
        plan_seconds[policy_name + "-wd"] = round(time.perf_counter() - t0, 2)

    if args.bench_db:
        ucd.ucd_bench_save(args.bench_db)

    def step(pl, offs=None):
        for i, (st, p) in enumerate(zip(states, pl)):
            st.run(ucd, p, ws, None if offs is None else offs[i])

    # the contract's figure: exactly --steps planned steps between two synchronisations
    ms, ms_median, ms_min = time_steps(torch, lambda: step(plans, offsets), args.steps, args.warmup)
    # planned against undivided, interleaved step by step so that both see the same clock
    if args.skip_undivided:
        u_med = p_med = u_min = p_min = float("nan")
    else:
        u_med, p_med, u_min, p_min = time_interleaved(torch, lambda: step(undiv), lambda: step(plans, offsets),
                                                      args.steps, args.warmup)

    tflops = flops_per_step / (ms * 1e-3) / 1e12
    peak = FP32_MFMA_PEAK_TFLOPS if args.dtype == "f32" else BF16_MFMA_PEAK_TFLOPS
    exec_flops = executed_flops(ucd, states, plans)
    roof, kernel_table = dominant_kernel_roofline(
        torch, ucd, states, plans, ws, reps=5,
        traffic_table=MEASURED_TRAFFIC_BYTES_PER_FLOP if (args.workload, batch, args.dtype) == ("alexnet", 256, "f32") else None)

    plan_report = []
    for st, p, u in zip(states, plans, undiv):
        for op in (ucd.FWD, ucd.BWD_DATA, ucd.BWD_FILTER):
            micro, cost, need = p[op].query()
            umicro, ucost, _ = u[op].query()
            runs, last = [], None
            for a, b in micro:   # run-length encode the configuration
                if last == (a, b):
                    runs[-1][2] += 1
                else:
                    runs.append([ucd.ALGO_NAMES[a], b, 1])
                last = (a, b)
            plan_report.append({"layer": st.s.name, "op": ucd.OP_NAMES[op], "config": runs,
                                "predicted_ms": round(cost / 1e6, 4), "ws_MiB": round(need / 2 ** 20, 2),
                                "undivided": [ucd.ALGO_NAMES[umicro[0][0]], umicro[0][1]],
                                "undivided_predicted_ms": round(ucost / 1e6, 4)})

    out = {
        "metric": METRIC, "value": round(tflops, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if args.dtype == "f32" else "bf16",
        "data": "synthetic",
        "config": {"workload": f"{title}, batch {batch}, "
                               + ("fp32" if args.dtype == "f32" else "bf16 tensors (fp32 dw)") + " NCHW, "
                               + (f"{limit >> 20} MiB workspace per layer (WR)" if mode == "wr" and limit >= 1 << 20
                                  else f"{limit >> 10} KiB workspace per layer (WR)" if mode == "wr"
                                  else f"one {limit >> 20} MiB workspace budget over {3 * len(layers)} kernels (WD)"),
                   "policy": policy_name, "global_batch": batch, "ws_limit_bytes": limit, "mode": mode},
        "ms_per_iter": round(ms, 4), "ms_median": round(ms_median, 4), "ms_min": round(ms_min, 4),
        # algorithmic (direct-convolution) flops over time, as a share of the matrix peak ...
        ("pct_fp32_mfma_peak" if args.dtype == "f32" else "pct_bf16_mfma_peak"): round(100 * tflops / peak, 2),
        # ... and the matrix flops the step's GEMM launches really issue (fewer where Winograd / FFT run)
        "executed_mfma_tflops": round(exec_flops / (ms * 1e-3) / 1e12, 3),
        "pct_mfma_peak_executed": round(100 * exec_flops / (ms * 1e-3) / 1e12 / peak, 2),
        "executed_gflop_per_step": round(exec_flops / 1e9, 1),
        "undivided_ms_per_iter": num(u_med), "planned_ms_interleaved": num(p_med),
        "undivided_ms_min": num(u_min), "planned_ms_min_interleaved": num(p_min),
        "speedup_vs_undivided": num(u_med / p_med),
        "plan_seconds": plan_seconds,
        "gflop_per_step": round(flops_per_step / 1e9, 1),
        "roofline": roof,
        "kernels": kernel_table,
        "cpu_baseline": None if args.no_cpu_baseline else cpu_baseline(layers, min(args.cpu_samples, batch)),
        "peak_ws_MiB": round(max(max(p[op].ws_bytes for op in p) for p in plans) / 2 ** 20, 2),
        "total_ws_MiB": round(sum(p[op].ws_bytes for p in plans for op in p) / 2 ** 20, 2),
        "plans": plan_report,
    }
    if args.memory_table:
        print(memory_table(ucd, states, plans, ws, title, batch, limit), file=sys.stderr)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
