"""Runs the calls of one benchmark configuration a few times and prints per-call timings.

    python -m paper_1611_07819_amd.run_config <1|2|3|3h|4|5|5h|skinny> [--iters N] [--only CALL]
        [--copy-probe] [--vendor-reference] [--warm-ms T]

Meant as the target of a profiler (`rocprofv3 ... -- python3 -m paper_1611_07819_amd.run_config 3`):
inputs are the seeded synthetic recipes of ``synth.py``; nothing is checked here.
``--copy-probe`` appends three 1 GiB device-to-device copies (a kernel of known traffic that
calibrates the HBM byte counters).  ``skinny`` is the batch-of-64 workload of the benchmark's
side table (fp16 64 x 4096 x 4096 and 64 x 4096 x 9216, fp32 64 x 4096 x 9216).
``--vendor-reference`` also times the vendor GEMM library (through torch.matmul) on the same
shapes and operand orientations: a measuring stick for what this chip gives a tuned kernel at
these sizes, never part of the product path."""
import argparse
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("config")
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--only", default=None)
    ap.add_argument("--copy-probe", action="store_true")
    ap.add_argument("--vendor-reference", action="store_true")
    ap.add_argument("--warm-ms", type=float, default=20.0,
                    help="warm-up per call: at least three calls, and on until this much wall time has passed "
                         "(0 for counter runs, where every dispatch is slow)")
    ap.add_argument("--cycle-probe", action="store_true",
                    help="print the fp16 GEMM kernel's own cycle counts (needs the probe build of the "
                         "library: python -m paper_1611_07819_amd.build --probe, then DMATH_LIBRARY=...)")
    args = ap.parse_args()
    import torch
    import paper_1611_07819_amd as dm
    from paper_1611_07819_amd import synth

    import numpy as np

    def skinny():
        r = np.random.default_rng(16110781)
        mats, calls = {}, []
        for i, (dt, M, N, K) in enumerate((("f16", 64, 4096, 4096), ("f16", 64, 4096, 9216), ("f32", 64, 4096, 9216))):
            npdt = np.float16 if dt == "f16" else np.float32
            mats[f"A{i}"] = r.uniform(0, 1, (M, K)).astype(npdt)
            mats[f"B{i}"] = r.normal(0, 0.01, (K, N)).astype(npdt)
            mats[f"C{i}"] = np.zeros((M, N), np.float32)
            calls.append(synth.GemmCall(f"nn_{dt}_M{M}_N{N}_K{K}", False, False, f"A{i}", f"B{i}", f"C{i}"))
        return synth.Workload("skinny_batch64", "mixed", (1, 1), mats, calls)

    make = {"skinny": skinny, "1": synth.config1, "2": synth.config2, "3": lambda: synth.config3("f32"),
            "3h": lambda: synth.config3("f16"), "4": synth.config4,
            "5": lambda: synth.config5("f32"), "5h": lambda: synth.config5("f16")}[args.config]
    w = make()
    slab = torch.empty(6 << 30, dtype=torch.uint8, device="cuda:0")
    st = torch.cuda.current_stream()
    ctx = dm.Context(slab, stream=st.cuda_stream)
    ctx.set_relayout_reuse(False)     # every call shows all of its kernels in the trace
    dev = {k: ctx.from_host(v, w.grid) for k, v in w.mats.items()}
    calls = []
    for c in w.calls:
        M, N, K = c.mnk(w.mats)
        info = dm.gemm_plan_info(ctx, int(c.transA), int(c.transB), dev[c.a], dev[c.b], dev[c.c])
        desc = f"kernel {info['kernel']} tile {info['tile_m']}x{info['tile_n']} tiles {info['tiles']} split {info['split_k']}"
        calls.append((c.name, 2.0 * M * N * K, desc,
                      lambda c=c: dm.gemm(ctx, int(c.transA), int(c.transB), c.alpha, dev[c.a],
                                          dev[c.b], c.beta, dev[c.c])))
    vendor = {}
    if args.vendor_reference:
        tdev = {k: torch.from_numpy(v).cuda() for k, v in w.mats.items()}
        for c in w.calls:
            a, b = tdev[c.a], tdev[c.b]
            vendor[c.name] = (lambda a=a, b=b, c=c: torch.matmul(a.t() if c.transA else a, b.t() if c.transB else b))
    if w.conv:
        d = dm.ConvDesc(**w.conv)
        g = w.conv
        fl = 2.0 * g["n"] * g["h"] * g["w"] * g["k"] * g["c"] * g["r"] * g["s"]
        calls.append(("conv_fwd", fl, "", lambda: dm.conv_fwd(ctx, d, 1.0, dev["X"], dev["F"], 0.0, dev["Y"])))
        calls.append(("conv_bwd_filter", fl, "",
                      lambda: dm.conv_bwd_filter(ctx, d, 1.0, dev["X"], dev["dY"], 0.0, dev["dF"])))
        dev["dX"] = ctx.matrix(dev["X"].rows, dev["X"].cols, (1, 1), dev["Y"].dtype)
        calls.append(("conv_bwd_data", fl, "",
                      lambda: dm.conv_bwd_data(ctx, d, 1.0, dev["dY"], dev["F"], 0.0, dev["dX"])))
    import time

    def warm_up(fn):
        """At least three calls, and on until --warm-ms have passed (the clocks settle)."""
        t0, n = time.perf_counter(), 0
        while n < 3 or time.perf_counter() - t0 < args.warm_ms * 1e-3:
            fn()
            n += 1
            if n % 8 == 0:
                torch.cuda.synchronize()
        torch.cuda.synchronize()

    for name, fl, desc, f in calls:
        if args.only and args.only != name:
            continue
        warm_up(f)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(args.iters):
            f()
        e1.record(st)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.iters
        print(f"{w.name} {name}: {desc}: {ms * 1e3:.1f} us  {fl / ms / 1e9:.1f} TFLOP/s", flush=True)
        if args.vendor_reference and name in vendor:
            vf = vendor[name]
            warm_up(vf)
            e0.record(st)
            for _ in range(args.iters):
                vf()
            e1.record(st)
            torch.cuda.synchronize()
            vms = e0.elapsed_time(e1) / args.iters
            print(f"    vendor library (torch.matmul), same shape and orientation: {vms * 1e3:.1f} us  "
                  f"{fl / vms / 1e9:.1f} TFLOP/s", flush=True)
        if args.cycle_probe and name.startswith(("fwd", "dW", "dX", "nn")):
            c = ctx.cycle_probe_read()
            cyc = c["prologue"] + c["loop"] + c["epilogue"]
            ghz = cyc / (c["ticks_100mhz"] / 100e6) / 1e9
            print(f"    workgroup of tile (0,0): prologue {c['prologue']} + loop {c['loop']} "
                  f"({c['loop'] / c['ktiles']:.0f} per k-tile) + epilogue {c['epilogue']} cycles, "
                  f"{c['barrier_wait'] / max(c['ktiles'] - 1, 1):.0f} per k-tile waiting at the barrier; "
                  f"{c['ticks_100mhz'] / 100:.1f} us -> {ghz:.2f} GHz in the kernel", flush=True)
    if args.copy_probe:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    ctx.close()


if __name__ == "__main__":
    main()
