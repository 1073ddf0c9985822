"""Time one (layer, operation, algorithm, micro-batch size) through the C-ABI.

    python3 -m paper_1804_04806_amd.microbench --net alexnet --layer conv4 --op fwd --algo implicit --b 256

Prints ms, algorithmic TFLOP/s and workspace bytes.  Meant to be run alone or under
``rocprofv3 --kernel-trace --stats`` / ``--pmc`` to look at a single kernel.
"""
import argparse
import json


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--net", default="alexnet", choices=["small", "alexnet", "resnet18", "densenet", "resnet50"])
    ap.add_argument("--layer", default="conv4")
    ap.add_argument("--op", default="fwd", choices=["fwd", "bwd_data", "bwd_filter"])
    ap.add_argument("--algo", default="implicit", choices=["implicit", "im2col", "winograd", "winograd4", "fft"])
    ap.add_argument("--b", type=int, default=256)
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"],
                    help="bf16: x, w, dy, y, dx stored as bfloat16 (dw fp32)")
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--copy-mib", type=int, default=0,
                    help="instead of a convolution, run a plain device copy of this many MiB "
                         "(a kernel of known traffic, to calibrate FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--mfma-peak", action="store_true",
                    help="instead of a convolution, time the register-only MFMA loop with 0/2/4/8 "
                         "vector FMAs per MFMA (on-box fp32 matrix ceiling)")
    args = ap.parse_args()

    import torch
    from . import synth, ucd
    if args.mfma_peak:
        blocks, iters = 512, 2000
        scratch = torch.empty(blocks * 256, dtype=torch.float32, device="cuda:0")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        out = {}
        for valu in (0, 2, 4, 8):
            best = 1e9
            for it in range(args.warmup + args.reps):
                e0.record()
                flops = ucd.ucd_mfma_probe(valu, blocks, iters, scratch)
                e1.record()
                e1.synchronize()
                if it >= args.warmup:
                    best = min(best, e0.elapsed_time(e1))
            out[f"tflops_with_{valu}_valu_per_mfma"] = round(flops / best / 1e9, 1)
        print(json.dumps(out))
        return
    if args.copy_mib:
        n = args.copy_mib * (1 << 20) // 4
        src = torch.rand(n, device="cuda:0")
        dst = torch.empty_like(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        times = []
        for it in range(args.warmup + args.reps):
            e0.record()
            dst.copy_(src)
            e1.record()
            e1.synchronize()
            if it >= args.warmup:
                times.append(e0.elapsed_time(e1))
        ms = min(times)
        print(json.dumps({"copy_mib": args.copy_mib, "ms_min": round(ms, 4),
                          "GBps_read_plus_write": round(2 * n * 4 / ms / 1e6, 1)}))
        return
    nets = {"small": synth.config_small, "alexnet": synth.config_alexnet, "resnet18": synth.config_resnet18,
            "densenet": synth.config_densenet_block, "resnet50": synth.config_resnet50}
    s = next(l for l in nets[args.net]() if l.name == args.layer).with_batch(args.b)
    op = {"fwd": ucd.FWD, "bwd_data": ucd.BWD_DATA, "bwd_filter": ucd.BWD_FILTER}[args.op]
    algo = {"implicit": ucd.ALGO_IMPLICIT, "im2col": ucd.ALGO_IM2COL, "winograd": ucd.ALGO_WINOGRAD,
            "winograd4": ucd.ALGO_WINOGRAD4, "fft": ucd.ALGO_FFT}[args.algo]
    dev = torch.device("cuda:0")
    desc = ucd.layer(s, dtype=1 if args.dtype == "bf16" else 0)
    need = ucd.ucd_workspace_size(desc, op, algo, args.b)
    if need == ucd.WS_NA:
        raise SystemExit("algorithm does not apply to this layer/operation")
    td = torch.bfloat16 if args.dtype == "bf16" else torch.float32
    x = torch.from_numpy(synth.make_x(s)).to(dev).to(td)
    w = torch.from_numpy(synth.make_w(s)).to(dev).to(td)
    y = torch.from_numpy(synth.make_dy(s)).to(dev).to(td)
    if op == ucd.BWD_FILTER:
        w = w.float()   # dw is fp32 for every dtype
    ws = torch.empty(max(need, 4) // 4, dtype=torch.float32, device=dev)
    a, bsrc, out = {ucd.FWD: (x, w, y), ucd.BWD_DATA: (y, w, x), ucd.BWD_FILTER: (x, y, w)}[op]
    beta = 1.0 if op == ucd.BWD_FILTER else 0.0
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    times = []
    for it in range(args.warmup + args.reps):
        e0.record()
        ucd.ucd_run_micro(desc, op, algo, args.b, a, bsrc, out, beta, ws)
        e1.record()
        e1.synchronize()
        if it >= args.warmup:
            times.append(e0.elapsed_time(e1))
    ms = min(times)
    print(json.dumps({"layer": s.name, "op": args.op, "algo": args.algo, "b": args.b, "ms_min": round(ms, 4),
                      "ms_avg": round(sum(times) / len(times), 4), "tflops": round(s.flops / ms / 1e9, 2),
                      "ws_bytes": need}))


if __name__ == "__main__":
    main()
