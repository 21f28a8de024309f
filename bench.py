"""Benchmark of the hot path on one MI355X.

One step = one pass of configuration 2 (the fp32 fully connected layer of the paper's AlexNet
workload at its batch of 1024): forward Y = X*W (N,N), weight gradient dW = X^T*dY (T,N) and
data gradient dX = dY*W^T (N,T), operands resident in HBM as 4x4 block grids.  The reported
value is TFLOP/s over whole steps; the other configurations are timed per call and listed under
"calls".  The CPU oracle is timed on a bounded sample of the same workload as a reported
baseline.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f16": 2516.6, "f32": 157.3, "f64": 78.6}   # dense MFMA peaks of MI355X
# HBM bytes per GEMM call of cfg2 (mean over the three calls of a step): FETCH_SIZE + WRITE_SIZE of
# two rocprofv3 --pmc runs of this program, scaled by a 1 GiB copy of known size; the runs, their
# command lines and the commit they were made at are in profiles/gemm_f32_cfg2_hbm_traffic.txt.  A
# counter cannot be read from inside this program, so the figure is carried here, not re-measured.
MEASURED_TRAFFIC_BYTES = 585415583


def cpu_model():
    """Model string of the host CPU the oracle is timed on."""
    try:
        seen = {}
        with open("/proc/cpuinfo") as f:
            for line in f:
                key, _, val = line.partition(":")
                key = key.strip().lower()
                if key in ("model name", "cpu family", "model") and key not in seen:
                    seen[key] = val.strip()
        if "model name" in seen:  # virtual machines report a generic name: family / model tell the part
            return "%s (family %s, model %s, %d logical CPUs)" % (
                seen["model name"], seen.get("cpu family", "?"), seen.get("model", "?"), os.cpu_count() or 0)
    except OSError:
        pass
    import platform
    return platform.processor() or platform.machine()


def set_oracle_threads(n):
    """Thread count of the OpenMP runtime the oracle library is linked with (the oracle itself
    is not touched: it is timed as it stands)."""
    import ctypes
    ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only-main", action="store_true", help="skip the per-call side table")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run three 1 GiB device-to-device copies (calibrates HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
                 "use --gpus 1")

    import numpy as np
    import torch
    import paper_1611_07819_amd as dm
    from paper_1611_07819_amd import synth

    dm.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    # one dedicated stream (default priority) for every launch and every timing event; a
    # non-default stream is also what pipeline recording needs
    stream = torch.cuda.Stream()
    torch.cuda.set_stream(stream)
    slab = torch.empty(8 << 30, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    ctx = dm.Context(slab, stream=stream.cuda_stream)

    def time_calls(fns, steps, warmup, warm_ms=20.0, stats=None):
        """ms per pass over fns (mean), HIP events on the stream the kernels are launched on, one
        event between every two passes so that the median and the minimum pass can be reported
        beside the mean (`stats`, a dict, receives them; they come from a second run of the same
        passes, so that the mean is taken without events between the passes).  After `warmup` passes the warm-up goes on
        until warm_ms of wall time have passed: after an idle gap (uploading the next operands) the
        first 10-20 ms of kernels run at lower clocks (fp32 1280x4096x4096: 382 us in the first 25
        calls, 326 us from then on)."""
        t_warm = time.perf_counter()
        for _ in range(warmup):
            for f in fns:
                f()
        while warm_ms and (time.perf_counter() - t_warm) * 1e3 < warm_ms:
            for f in fns:
                f()
            torch.cuda.synchronize()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for _ in range(steps):
            for f in fns:
                f()
        e1.record(stream)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / steps
        if stats is not None:      # a second run of the same passes, one event after each
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
            ev[0].record(stream)
            for i in range(steps):
                for f in fns:
                    f()
                ev[i + 1].record(stream)
            torch.cuda.synchronize()
            per = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
            mid = len(per) // 2
            stats["median_ms"] = round(per[mid] if len(per) % 2 else 0.5 * (per[mid - 1] + per[mid]), 4)
            stats["min_ms"] = round(per[0], 4)
            stats["timed"] = steps
        return e0.elapsed_time(e1) / steps, wall

    def entry(ms, flop, peak_key, stats=None, **more):
        e = {"ms": round(ms, 4), "tflops": round(flop / ms / 1e9, 2),
             "frac_peak": round(flop / ms / 1e9 / PEAK_TFLOPS[peak_key], 4)}
        if stats:
            e.update(stats)
        e.update(more)
        return e

    # ---------------- main workload: configuration 2 ----------------
    w = synth.config2()
    dev = {k: ctx.from_host(v, w.grid) for k, v in w.mats.items()}
    fns, flops = [], []
    for c in w.calls:
        fns.append(lambda c=c: dm.gemm(ctx, int(c.transA), int(c.transB), c.alpha, dev[c.a],
                                       dev[c.b], c.beta, dev[c.c]))
        M, N, K = c.mnk(w.mats)
        flops.append(2.0 * M * N * K)
    main_stats = {}
    ms_step, wall_ms = time_calls(fns, args.steps, args.warmup, stats=main_stats)
    value = sum(flops) / (ms_step * 1e-3) / 1e12
    # dominant kernel = the GEMM main loop; three calls per step, each doing the same
    # 2*M*N*K = 77.31 GFLOP in one launch (dX: two, the second over the tiles left after the
    # last full round of workgroups, in four k-parts, plus the kernel that adds them).
    avg_launch_ms = ms_step / len(fns)
    achieved = (sum(flops) / len(fns)) / (avg_launch_ms * 1e-3) / 1e12
    calls = {}
    if not args.only_main:
        for c, f, fl in zip(w.calls, fns, flops):
            st = {}
            ms, _ = time_calls([f], 50, 3, stats=st)
            calls[f"cfg2.{c.name}"] = entry(ms, fl, "f32", st)
    info = dm.gemm_plan_info(ctx, 0, 0, dev["X"], dev["W"], dev["Y"])
    if not args.only_main:
        # the same step after selection from timing samples (done once, outside the timed region,
        # as plans are); the headline value above stays on the cost model's choices
        tuned = [dm.gemm_tune(ctx, int(c.transA), int(c.transB), dev[c.a], dev[c.b], dev[c.c], 1 << 30, 10)
                 for c in w.calls]
        st = {}
        ms, _ = time_calls(fns, args.steps, 3, stats=st)
        calls["cfg2.step_tuned"] = entry(ms, sum(flops), "f32", st,
                                         tiles=[[t["tile_m"], t["tile_n"], t["split_k"]] for t in tuned])
        ctx.tune_reset()
    for m in dev.values():
        m.destroy()

    # ---------------- side table: the other configurations, per call ----------------
    if not args.only_main:
        def bench_workload(wl, tag, dtype_key):
            d = {k: ctx.from_host(v, wl.grid) for k, v in wl.mats.items()}
            for c in wl.calls:
                M, N, K = c.mnk(wl.mats)
                fl = 2.0 * M * N * K
                f = lambda c=c: dm.gemm(ctx, int(c.transA), int(c.transB), c.alpha, d[c.a], d[c.b],
                                        c.beta, d[c.c])
                st = {}
                ms, _ = time_calls([f], 50 if fl < 5e11 else 10, 3, stats=st)
                calls[f"{tag}.{c.name}"] = entry(ms, fl, dtype_key, st)
            for m in d.values():
                m.destroy()
        def bench_step(wl, tag, dtype_key):
            """Whole forward+backward step of a configuration, issued call by call and as one
            recorded pipeline replay."""
            d = {k: ctx.from_host(v, wl.grid) for k, v in wl.mats.items()}
            fl = sum(2.0 * np.prod(c.mnk(wl.mats)) for c in wl.calls)

            def step():
                for c in wl.calls:
                    dm.gemm(ctx, int(c.transA), int(c.transB), c.alpha, d[c.a], d[c.b], c.beta, d[c.c])
            step()
            ctx.pipeline_begin()
            step()
            pid = ctx.pipeline_end()
            for name, f in (("step_eager", step), ("step_replay", lambda: ctx.pipeline_replay(pid))):
                st = {}
                ms, _ = time_calls([f], 50, 5, stats=st)
                calls[f"{tag}.{name}"] = entry(ms, fl, dtype_key, st)
            ctx.pipeline_destroy(pid)
            for m in d.values():
                m.destroy()
        bench_workload(synth.config1(), "cfg1", "f32")
        bench_step(synth.config1(), "cfg1", "f32")      # its two launches issued and replayed as a recorded pipeline
        bench_step(synth.config3("f32"), "cfg3_f32out", "f16")
        bench_workload(synth.config3("f32"), "cfg3_f32out", "f16")
        bench_workload(synth.config3("f16"), "cfg3_f16out", "f16")
        bench_workload(synth.config4(), "cfg4", "f64")
        # small batch against the configuration-2/3 weight matrices: bound by streaming W from HBM
        # (fp16) or by the matrix instructions on a 64-row tile (fp32, fp64), not by the MFMA peak
        rs = np.random.default_rng(16110781)
        for tag, code, npdt, (M, N, K) in (("f16", dm.F16, np.float16, (64, 4096, 4096)),
                                           ("f16", dm.F16, np.float16, (64, 4096, 9216)),
                                           ("f32", dm.F32, np.float32, (64, 4096, 9216))):
            sa = ctx.from_host(rs.uniform(0, 1, (M, K)).astype(npdt))
            sb = ctx.from_host(rs.normal(0, 0.01, (K, N)).astype(npdt))
            sc = ctx.matrix(M, N, (1, 1), dm.F32)
            st = {}
            ms, _ = time_calls([lambda: dm.gemm(ctx, 0, 0, 1.0, sa, sb, 0.0, sc)], 50, 5, stats=st)
            byt = (M * K + K * N) * npdt().itemsize + M * N * 4
            pinfo = dm.gemm_plan_info(ctx, 0, 0, sa, sb, sc)
            calls[f"skinny_{tag}.M{M}_N{N}_K{K}"] = {
                "ms": round(ms, 4), "tflops": round(2.0 * M * N * K / ms / 1e9, 2),
                "hbm_tb_s": round(byt / ms / 1e9, 3), "frac_hbm_peak": round(byt / ms / 1e9 / 8.0, 4),
                "tile": [pinfo["tile_m"], pinfo["tile_n"], pinfo["split_k"]], **st}
            for m in (sa, sb, sc):
                m.destroy()
        w5 = synth.config5("f32")
        d5 = {k: ctx.from_host(v) for k, v in w5.mats.items()}
        desc = dm.ConvDesc(**w5.conv)
        fl5 = 2.0 * 50176 * 256 * 2304
        d5["dX"] = ctx.matrix(d5["X"].rows, d5["X"].cols, (1, 1), dm.F32)
        # per-call figures: every call re-lays-out its operands (no copy kept from the call
        # before, which would take work out of the timed region)
        ctx.set_relayout_reuse(False)
        for name, f in [("fwd", lambda: dm.conv_fwd(ctx, desc, 1.0, d5["X"], d5["F"], 0.0, d5["Y"])),
                        ("bwd_filter", lambda: dm.conv_bwd_filter(ctx, desc, 1.0, d5["X"], d5["dY"], 0.0, d5["dF"])),
                        ("bwd_data", lambda: dm.conv_bwd_data(ctx, desc, 1.0, d5["dY"], d5["F"], 0.0, d5["dX"]))]:
            st = {}
            ms, _ = time_calls([f], 50, 3, stats=st)
            calls[f"cfg5.{name}"] = entry(ms, fl5, "f16", st)
        # one training step of the layer: new activations, new gradient and an updated filter
        # arrive (declared with touch), then forward + weight gradient + data gradient; with
        # copies kept, X is re-laid-out once for the two calls that read it
        def step5():
            for k in ("X", "dY", "F"):
                d5[k].touch()
            dm.conv_fwd(ctx, desc, 1.0, d5["X"], d5["F"], 0.0, d5["Y"])
            dm.conv_bwd_filter(ctx, desc, 1.0, d5["X"], d5["dY"], 0.0, d5["dF"])
            dm.conv_bwd_data(ctx, desc, 1.0, d5["dY"], d5["F"], 0.0, d5["dX"])
        for name, keep in (("step_rewrite_all", False), ("step_copies_kept", True)):
            ctx.set_relayout_reuse(keep)
            st = {}
            ms, _ = time_calls([step5], 50, 3, stats=st)
            calls[f"cfg5.{name}"] = entry(ms, 3 * fl5, "f16", st)
        ctx.set_relayout_reuse(False)
        # the three calls again with fp16 results (half the bytes stored by each epilogue), as for
        # configuration 3; inputs, kernels and re-layouts are the same
        h5 = {"Y": ctx.matrix(d5["Y"].rows, d5["Y"].cols, (1, 1), dm.F16),
              "dF": ctx.matrix(d5["dF"].rows, d5["dF"].cols, (1, 1), dm.F16),
              "dX": ctx.matrix(d5["X"].rows, d5["X"].cols, (1, 1), dm.F16)}
        for name, f in [("fwd", lambda: dm.conv_fwd(ctx, desc, 1.0, d5["X"], d5["F"], 0.0, h5["Y"])),
                        ("bwd_filter", lambda: dm.conv_bwd_filter(ctx, desc, 1.0, d5["X"], d5["dY"], 0.0, h5["dF"])),
                        ("bwd_data", lambda: dm.conv_bwd_data(ctx, desc, 1.0, d5["dY"], d5["F"], 0.0, h5["dX"]))]:
            st = {}
            ms, _ = time_calls([f], 50, 3, stats=st)
            calls[f"cfg5_f16out.{name}"] = entry(ms, fl5, "f16", st)
        for m in list(d5.values()) + list(h5.values()):
            m.destroy()
        # the same layer in fp32 (fp32 MFMA pipeline), per call, copies rewritten every call
        d5 = {k: ctx.from_host(v.astype(np.float32)) for k, v in w5.mats.items()}
        d5["dX"] = ctx.matrix(d5["X"].rows, d5["X"].cols, (1, 1), dm.F32)
        for name, f in [("fwd", lambda: dm.conv_fwd(ctx, desc, 1.0, d5["X"], d5["F"], 0.0, d5["Y"])),
                        ("bwd_filter", lambda: dm.conv_bwd_filter(ctx, desc, 1.0, d5["X"], d5["dY"], 0.0, d5["dF"])),
                        ("bwd_data", lambda: dm.conv_bwd_data(ctx, desc, 1.0, d5["dY"], d5["F"], 0.0, d5["dX"]))]:
            st = {}
            ms, _ = time_calls([f], 50, 3, stats=st)
            calls[f"cfg5_as_f32.{name}"] = entry(ms, fl5, "f32", st)
        ctx.set_relayout_reuse(True)
        for m in d5.values():
            m.destroy()
        # a 1x1 stride-1 layer (n=64, 256 -> 512 channels, 28x28, fp16): run as a block GEMM on the
        # tensors as they lie, one column block per image, no re-layout copies
        g1 = dict(n=64, c=256, h=28, w=28, k=512, r=1, s=1)
        d1 = dm.ConvDesc(**g1)
        x1 = ctx.from_host(rs.uniform(0, 1, (64, 256 * 784)).astype(np.float16))
        f1 = ctx.from_host(rs.normal(0, 0.06, (512, 256)).astype(np.float16))
        y1 = ctx.from_host(rs.normal(0, 0.1, (64, 512 * 784)).astype(np.float16))
        o1 = {"Y": ctx.matrix(64, 512 * 784, (1, 1), dm.F32), "dF": ctx.matrix(512, 256, (1, 1), dm.F32),
              "dX": ctx.matrix(64, 256 * 784, (1, 1), dm.F32)}
        fl1 = 2.0 * 64 * 784 * 512 * 256
        for name, f in [("fwd", lambda: dm.conv_fwd(ctx, d1, 1.0, x1, f1, 0.0, o1["Y"])),
                        ("bwd_filter", lambda: dm.conv_bwd_filter(ctx, d1, 1.0, x1, y1, 0.0, o1["dF"])),
                        ("bwd_data", lambda: dm.conv_bwd_data(ctx, d1, 1.0, y1, f1, 0.0, o1["dX"]))]:
            st = {}
            ms, _ = time_calls([f], 50, 3, stats=st)
            calls[f"conv1x1_f16.{name}"] = entry(ms, fl1, "f16", st)
        for m in [x1, f1, y1] + list(o1.values()):
            m.destroy()
        # K that is not a multiple of the kernels' k-step: data gradient of a 4096 -> 1000 layer at
        # batch 1024 (K = 1000 goes through zero-padded scratch panels)
        for tag, code, npdt in (("f32", dm.F32, np.float32), ("f16", dm.F16, np.float16)):
            M, N, K = 1024, 4096, 1000
            sa = ctx.from_host(rs.normal(0, 0.1, (M, K)).astype(npdt))
            sb = ctx.from_host(rs.normal(0, 0.02, (N, K)).astype(npdt))
            sc = ctx.matrix(M, N, (1, 1), dm.F32)
            st = {}
            ms, _ = time_calls([lambda: dm.gemm(ctx, 0, 1, 1.0, sa, sb, 0.0, sc)], 50, 5, stats=st)
            pinfo = dm.gemm_plan_info(ctx, 0, 1, sa, sb, sc)
            calls[f"ktail_{tag}.dX_nt_M{M}_N{N}_K{K}"] = entry(
                ms, 2.0 * M * N * K, tag, st, kernel=pinfo["kernel"],
                tile=[pinfo["tile_m"], pinfo["tile_n"], pinfo["split_k"]])
            for m in (sa, sb, sc):
                m.destroy()

        # tile counts that do not fill whole rounds of workgroups (1.25 and 2.125 rounds): the
        # tiles of the last round are split in k
        for tag, code, npdt, (M, N, K) in (("f32", dm.F32, np.float32, (1280, 4096, 4096)),
                                           ("f64", dm.F64, np.float64, (1280, 4096, 4096)),
                                           ("f16", dm.F16, np.float16, (4352, 4096, 4096))):
            sa = ctx.from_host(rs.uniform(0, 1, (M, K)).astype(npdt))
            sb = ctx.from_host(rs.normal(0, 0.02, (K, N)).astype(npdt))
            sc = ctx.matrix(M, N, (1, 1), dm.F32 if code == dm.F16 else code)
            st = {}
            ms, _ = time_calls([lambda: dm.gemm(ctx, 0, 0, 1.0, sa, sb, 0.0, sc)], 50, 5, stats=st)
            pinfo = dm.gemm_plan_info(ctx, 0, 0, sa, sb, sc)
            calls[f"partial_round_{tag}.nn_M{M}_N{N}_K{K}"] = entry(
                ms, 2.0 * M * N * K, tag, st, tile=[pinfo["tile_m"], pinfo["tile_n"], pinfo["split_k"]],
                split_tiles=[pinfo["split_tiles"], pinfo["tiles"]])
            for m in (sa, sb, sc):
                m.destroy()

    # ---------------- MFMA-only probe: what the matrix cores sustain at their clocks under load
    sustained = {}
    for key, code, iters in (("f32", dm.F32, 4000), ("f16", dm.F16, 8000), ("f16_32x32x16", dm.F16, 8000),
                             ("f64", dm.F64, 4000)):
        wide = key == "f16_32x32x16"
        ctx.mfma_peak_probe(code, 200, wide)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        fl = ctx.mfma_peak_probe(code, iters, wide)
        e1.record(stream)
        torch.cuda.synchronize()
        sustained[key] = round(fl / e0.elapsed_time(e1) / 1e9, 1)

    # ---------------- CPU oracle on a bounded sample (reported baseline only) ----------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import cpu_oracle as oracle
        blk = {k: oracle.BlockMatrix(v, w.grid) for k, v in w.mats.items()}
        t0 = time.perf_counter()
        for c in w.calls:       # the whole step, every output row: a few seconds of CPU work
            oracle.gemm(c.transA, c.transB, c.alpha, blk[c.a], blk[c.b], c.beta, blk[c.c])
        t = time.perf_counter() - t0
        cpu = {"value": round(sum(flops) / t / 1e12, 5), "unit": "TFLOP/s",
               "cores": oracle.num_threads(), "kind": "oracle", "cpu_model": cpu_model(),
               "sample": f"one whole cfg2 step (all three GEMMs, all rows, 231.9 GFLOP) in {t:.1f} s "
                         f"including the exact widening of the operands to fp64"}
        # configuration 1 (256^3, 33.6 MFLOP) on one thread: what a single host core does
        w1 = synth.config1()
        b1 = {k: oracle.BlockMatrix(v, w1.grid) for k, v in w1.mats.items()}
        threads = oracle.num_threads()
        set_oracle_threads(1)
        try:
            reps, t0 = 0, time.perf_counter()
            while reps < 3 or time.perf_counter() - t0 < 0.5:
                oracle.gemm(False, False, 1.0, b1["A"], b1["B"], 1.0, b1["C"])
                reps += 1
            t1 = (time.perf_counter() - t0) / reps
        finally:
            set_oracle_threads(threads)
        cpu["cfg1_one_thread"] = {"ms": round(t1 * 1e3, 3), "gflops": round(2.0 * 256 ** 3 / t1 / 1e9, 3),
                                  "threads": 1}

    if args.copy_probe:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    ctx.close()
    out = {
        "metric": "GEMM TFLOP/s per shape/precision and % of MI355X MFMA peak (1 GPU)",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "configs[1]: fp32 FC layer fwd (NN) + dW (TN) + dX (NT), "
                               "X[1024x9216] W[9216x4096], 4x4 block grids, alpha=1 beta=0",
                   "gflop_per_step": round(sum(flops) / 1e9, 2), "kernel": info["kernel"],
                   "tile": [info["tile_m"], info["tile_n"], info["tile_k"]],
                   "wall_ms_per_step": round(wall_ms, 4), "median_ms_per_step": main_stats.get("median_ms"),
                   "min_ms_per_step": main_stats.get("min_ms")},
        "frac_of_peak": round(value / PEAK_TFLOPS["f32"], 4),
        "roofline": {"bound": "mfma", "achieved": round(achieved, 3), "peak": PEAK_TFLOPS["f32"],
                     "unit": "TFLOP/s", "frac": round(achieved / PEAK_TFLOPS["f32"], 4),
                     "traffic": MEASURED_TRAFFIC_BYTES},
        "cpu_baseline": cpu,
        "sustained_mfma_tflops": sustained,
        "frac_of_sustained": round(value / sustained["f32"], 4),
        "calls": calls,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
