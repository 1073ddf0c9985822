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

# HBM bytes (fetched + written) per algorithmic flop of the GEMM instantiations of the default
# workload's planned step, from two rocprofv3 --pmc passes over this script (FETCH_SIZE, then
# WRITE_SIZE, each scaled by what the counter reads for a plain device copy of known size: x2.00 and
# x1.00): mean bytes per dispatch of a run whose benchmark cache came from a file (so that every
# dispatch has a shape of the step), divided by the mean flops per launch of that run's step.
# `traffic` = this figure x the flops per launch of the step being timed: the planner does not
# pick the same micro-batch sizes every run, and a kernel's traffic follows its size (the ratio
# itself differs by layer: 1.8e-3 to 2.7e-3 bytes per flop over the four BackwardFilter launches).
# Summary: profiles/bench_alexnet_b256_ws64MiB_kernel_stats.md.  A profiler cannot run inside the
# timed script, so these are recorded figures; they apply to the AlexNet workload at batch 256
# only and `traffic` is null for anything else.
MEASURED_TRAFFIC_BYTES_PER_FLOP = {
    "gemm_kernel<Tile<128x128>,PixelTab<dy>,PixelTab<x>,EpiAtomic>": 283.0e6 / 133.56e9,
    "gemm_kernel<Tile<96x128>,PixelKLane<dy>,PixelKLane<x>,EpiAtomic>": 538.3e6 / 53.97e9,
    "gemm_kernel<Tile<128x128>,KLane0,GatherNLane<taps<=31>,EpiNCHW>": 326.3e6 / 229.32e9,
    "gemm_kernel<Tile<96x128>,FilterKLane,GatherNLane<taps<=31>,EpiNCHW>": 322.2e6 / 214.09e9,
    "gemm_kernel<Tile<96x128>,KLane0,GatherNLane<taps>31>,EpiNCHW>": 274.0e6 / 26.98e9,
    "gemm_kernel<Tile<64x128>,PhaseFilterKLane,GatherNLane<taps<=31>,EpiPhases>": 451.9e6 / 52.71e9,
}

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
    return ap.parse_args()


class Pool:
    """One set of device buffers, sized for the largest layer, that every layer of a big
    workload takes views of (a resident ResNet-50 at batch 256 would need hundreds of GB)."""

    def __init__(self, layers, torch, dev, tdtype):
        nx = max(s.N * s.C * s.H * s.W for s in layers)
        ny = max(s.N * s.K * s.P * s.Q for s in layers)
        nw = max(s.K * s.C * s.R * s.S for s in layers)
        g = torch.Generator(device=dev)
        g.manual_seed(1234)
        self.x = (torch.rand(nx, device=dev, generator=g) * 2 - 1).to(tdtype)
        self.dy = (torch.rand(ny, device=dev, generator=g) * 2 - 1).to(tdtype)
        self.w = (torch.randn(nw, device=dev, generator=g) * 0.03).to(tdtype)
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
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def kernel_class(ucd, desc, op, algo, b):
    """The GEMM kernel instantiation a micro-batch run launches, as the library describes it
    (the names rocprofv3 shows are these template instantiations), if the run is that one kernel
    (a zero-fill kernel in front of it is tolerated: a few microseconds); otherwise None
    (im2col, Winograd and strided BackwardData launch several kernels)."""
    text, n = ucd.ucd_describe_micro(desc, op, algo, b)
    parts = [p.strip() for p in text.split(";")]
    gemms = [p for p in parts if p.startswith("gemm_kernel")]
    others = [p for p in parts if not p.startswith("gemm_kernel") and p not in ("fill_zero_kernel", "zero_tiles_kernel")]
    if len(gemms) != 1 or others:
        return None
    name = gemms[0].split("> tiles=")[0] + ">"
    return name + (" (after " + parts[0] + ")" if len(parts) > 1 else "")


def dominant_kernel_roofline(torch, ucd, states, plans, ws, reps, traffic_table=None):
    """HIP-event timing (events recorded on the launch stream) of every single-kernel micro-batch
    launch of the planned step, grouped by kernel instantiation; returns the roofline object of
    the instantiation with the largest total time, and the per-instantiation table.
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
                cls = kernel_class(ucd, st.desc, op, algo, b)
                if cls is not None:
                    xo = st.x.view(-1)[o * x_img:]
                    yo = st.y.view(-1)[o * y_img:]
                    dyo = st.dy.view(-1)[o * y_img:]
                    dxo = st.dx.view(-1)[o * x_img:]
                    args = {ucd.FWD: (xo, st.w, yo), ucd.BWD_DATA: (dyo, st.w, dxo),
                            ucd.BWD_FILTER: (xo, dyo, st.dw)}[op]
                    beta = 1.0 if op == ucd.BWD_FILTER else 0.0
                    tot = 0.0
                    for _ in range(reps):
                        e0.record()
                        ucd.ucd_run_micro(st.desc, op, algo, b, *args, beta, ws)
                        e1.record()
                        e1.synchronize()
                        tot += e0.elapsed_time(e1)
                    g = groups.setdefault(cls, {"ms": 0.0, "flops": 0.0, "launches": 0})
                    g["ms"] += tot / reps
                    g["flops"] += s.with_batch(b).flops
                    g["launches"] += 1
                o += b
    if not groups:
        return None, []
    table = [{"kernel": k, "launches_per_step": g["launches"], "ms_per_step": round(g["ms"], 4),
              "avg_launch_ms": round(g["ms"] / g["launches"], 4),
              "tflops": round(g["flops"] / (g["ms"] * 1e-3) / 1e12, 2)}
             for k, g in sorted(groups.items(), key=lambda kv: -kv[1]["ms"])]
    name, g = max(groups.items(), key=lambda kv: kv[1]["ms"])
    achieved = g["flops"] / (g["ms"] * 1e-3) / 1e12
    peak = BF16_MFMA_PEAK_TFLOPS if name.startswith("gemm_kernel_bf16") else FP32_MFMA_PEAK_TFLOPS
    roof = {"bound": "mfma", "kernel": name, "achieved": round(achieved, 2), "peak": peak,
            "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
            "traffic": None,
            "launches_per_step": g["launches"], "avg_launch_ms": round(g["ms"] / g["launches"], 4),
            "flops_per_launch": g["flops"] / g["launches"]}
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


def main():
    args = parse()
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
    pool = None if args.workload in ("alexnet", "alexnet-wd", "small") else Pool(layers, torch, dev, tdtype)
    states = [LayerState(s, i, torch, ucd, synth, dev, pool, tdtype) for i, s in enumerate(layers)]
    ws = torch.empty(max(limit, 4) // 4, dtype=torch.float32, device=dev)
    flops_per_step = 3 * sum(s.flops for s in layers)

    if args.bench_db and os.path.exists(args.bench_db):
        ucd.ucd_bench_load(args.bench_db)
    offsets = None
    t0 = time.perf_counter()
    # baseline: the best single algorithm per kernel with no workspace beyond its own layer limit
    # (WR undivided); for the WD workload the same per-kernel share of the budget
    base_limit = limit if mode == "wr" else limit // (3 * len(layers))
    undiv = [st.plan(ucd, ucd.POLICY_UNDIVIDED, ws, base_limit) for st in states]
    t_plan_undiv = time.perf_counter() - t0
    t0 = time.perf_counter()
    if mode == "wr":
        plans = [st.plan(ucd, policy, ws, limit) for st in states]
    else:
        plans, offsets = plan_wd(ucd, states, pool, policy, ws, limit)
    t_plan = time.perf_counter() - t0

    if args.bench_db:
        ucd.ucd_bench_save(args.bench_db)

    def step(pl, offs=None):
        for i, (st, p) in enumerate(zip(states, pl)):
            st.run(ucd, p, ws, None if offs is None else offs[i])

    ms_undiv = time_steps(torch, lambda: step(undiv), args.steps, args.warmup)
    ms = time_steps(torch, lambda: step(plans, offsets), args.steps, args.warmup)

    tflops = flops_per_step / (ms * 1e-3) / 1e12
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
        "ms_per_iter": round(ms, 4),
        ("pct_fp32_mfma_peak" if args.dtype == "f32" else "pct_bf16_mfma_peak"):
            round(100 * tflops / (FP32_MFMA_PEAK_TFLOPS if args.dtype == "f32" else BF16_MFMA_PEAK_TFLOPS), 2),
        "undivided_ms_per_iter": round(ms_undiv, 4), "speedup_vs_undivided": round(ms_undiv / ms, 4),
        "plan_seconds": round(t_plan, 2), "plan_seconds_undivided": round(t_plan_undiv, 2),
        "gflop_per_step": round(flops_per_step / 1e9, 1),
        "roofline": roof,
        "kernels": kernel_table,
        "cpu_baseline": None if args.no_cpu_baseline else cpu_baseline(layers, min(args.cpu_samples, batch)),
        "peak_ws_MiB": round(max(max(p[op].ws_bytes for op in p) for p in plans) / 2 ** 20, 2),
        "total_ws_MiB": round(sum(p[op].ws_bytes for p in plans for op in p) / 2 ** 20, 2),
        "plans": plan_report,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
