#!/usr/bin/env python3
"""Benchmark of the pruned-FFT 3D convolutional layer on one MI355X.

A step is one whole layer call (kernel prep, forward passes, multiply-accumulate, inverse passes) on the seeded
synthetic inputs of the parity tests, already resident in HBM, with a pre-allocated workspace.  The timed steps go through the profiling
entry point, which records a HIP event on the launch stream between stages, so the per-stage durations behind
the roofline figures come from the same timed region as the throughput.  One JSON line is printed.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
MFMA_FP32_PEAK_TFLOPS = 157.3    # dense fp32 matrix, published
# Plain-VALU fp32 without packed instructions (this build switches them off):
# 256 CUs x 4 SIMDs x 16 lanes x 2 flop (FMA) x 2.4 GHz.
VALU_FP32_UNPACKED_TFLOPS = 256 * 4 * 16 * 2 * 2.4e9 / 1e12


TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic_bytes.txt")


def measured_traffic(workload, kernel):
    """HBM bytes per launch (read + written) of `kernel` on `workload`, from the table of calibrated rocprofv3
    FETCH_SIZE / WRITE_SIZE counter runs kept under profiles/ (lines: workload kernel read_bytes written_bytes
    source); None if the table has no such line."""
    try:
        with open(TRAFFIC_FILE) as fh:
            for line in fh:
                t = line.split()
                if len(t) >= 4 and not line.startswith("#") and t[0] == workload and t[1] == kernel:
                    return float(t[2]) + float(t[3])
    except OSError:
        pass
    return None


def check_timed_output(layer, workloads, inp, w, bias, out_gpu):
    """The output tensor the timed steps left, against the oracle on about 1e5 sampled positions (corner blocks
    and face patches of every output image, mid-planes of one, random positions).  Part of the oracle leg."""
    import numpy as np
    import torch
    from oracle import ref
    pts = workloads.sample_points(layer, n_random=100_000, block=4, midplanes=layer.out_voxels < 5e8)
    tp = torch.from_numpy(pts.astype(np.int64)).to(out_gpu.device)
    got = out_gpu[tp[:, 0], tp[:, 1], tp[:, 2], tp[:, 3], tp[:, 4]].cpu().numpy().astype(np.float64)
    exp = ref.conv3d_points(inp, w, bias, pts, relu=layer.relu)
    tol = ref.tolerance(inp, w)[pts[:, 1]]
    return {"sampled_voxels": int(len(pts)), "max_err_over_tol": float(np.max(np.abs(got - exp) / tol))}


def cpu_baseline(layer, workloads):
    """The oracle, as it stands, on a bounded sample: a cubic crop of the layer's input, as many output
    images as there are host threads (the oracle parallelises over (s, j) pairs)."""
    import numpy as np
    from oracle import ref
    threads = ref.max_threads()
    fo_s = min(layer.fo, threads)
    # crop edge so the sample costs roughly 4e11 multiply-adds (tens of seconds on a many-core host)
    budget = 4.0e11
    n_s = layer.n
    while n_s > layer.k and layer.S * fo_s * layer.f * layer.k ** 3 * (n_s - layer.k + 1) ** 3 > budget:
        n_s -= 1
    rng = np.random.default_rng(0)
    inp = rng.uniform(-1, 1, (layer.S, layer.f, n_s, n_s, n_s)).astype(np.float32)
    w = (rng.standard_normal((fo_s, layer.f, layer.k, layer.k, layer.k))
         * (layer.f * layer.k ** 3) ** -0.5).astype(np.float32)
    b = (rng.standard_normal(fo_s) * np.sqrt(0.1)).astype(np.float32)
    t0 = time.perf_counter()
    out = ref.conv3d(inp, w, b, relu=layer.relu)
    dt = time.perf_counter() - t0
    # the same oracle on one thread, on one output image of the same crop (a few seconds)
    t0 = time.perf_counter()
    out1 = ref.conv3d(inp[:1], w[:1], b[:1], relu=layer.relu, nthreads=1)
    dt1 = time.perf_counter() - t0
    return {
        "value": out.size / dt, "unit": "output voxels/s", "cores": min(threads, layer.S * fo_s),
        "kind": "oracle", "value_1_thread": out1.size / dt1,
        "sample": f"fp64 direct convolution of a {n_s}^3 crop, S={layer.S}, f={layer.f}, {fo_s} of {layer.fo} "
                  f"output images, k={layer.k} ({out.size} output voxels in {dt:.1f} s; cost per output voxel "
                  f"is uniform: f*k^3 multiply-adds)",
    }


def _time_ms(torch, fn, reps):
    """Average milliseconds of fn() over reps calls, by events on torch's current stream (where fn launches)."""
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def bench_mpf(torch, B, dev):
    """Max-pooling fragments (Section VI) on 48 images of 255^3 with window 2^3 -> 8 x 48 fragments of 127^3:
    the pooling layer that would follow a layer of the benchmark's size.  Pure data movement: 4 bytes read per
    input voxel, 4 bytes written per fragment voxel."""
    S, f, n, p = 1, 48, 255, 2
    inp = torch.rand((S, f, n, n, n), device=dev) * 2 - 1
    out = torch.empty((S * p ** 3, f) + (n // p,) * 3, device=dev)
    ms = _time_ms(torch, lambda: B.znni_mpf(inp, p, out=out), 10)
    nbytes = 4 * (inp.numel() + out.numel())
    gbs = nbytes / (ms * 1e-3) / 1e9
    return {"workload": f"mpf_S{S}_f{f}_{n}c_p{p}", "ms": ms, "GB": nbytes / 1e9, "GB/s": gbs,
            "frac_hbm": gbs / HBM_PEAK_GBS, "out_voxels_per_s": out.numel() / (ms * 1e-3)}


def bench_direct(torch, B, dev):
    """Direct-convolution primitive against the transform route on two shapes: a first layer (one input image,
    where direct wins) and the wide 3^3 layer of the workload list (where the transform route wins), with the
    library's pick for each."""
    res = []
    for (S, f, fo, n, k) in ((1, 1, 48, 128, 3), (1, 40, 40, 128, 3)):
        inp = torch.rand((S, f, n, n, n), device=dev) * 2 - 1
        w = torch.randn((fo, f, k, k, k), device=dev) * (f * k ** 3) ** -0.5
        b = torch.randn((fo,), device=dev)
        out = torch.empty((S, fo) + (n - k + 1,) * 3, device=dev)
        wsd = torch.empty(B.znni_conv3d_direct_workspace(S, f, fo, n, k), dtype=torch.uint8, device=dev)
        wsf = B.alloc_workspace(S, f, fo, n, k, dev)
        md = _time_ms(torch, lambda: B.znni_conv3d_direct(inp, w, b, relu=True, out=out, workspace=wsd), 10)
        mf = _time_ms(torch, lambda: B.znni_conv3d_fft(inp, w, b, relu=True, out=out, workspace=wsf), 10)
        flops = 2.0 * S * f * fo * k ** 3 * (n - k + 1) ** 3
        pick, est = B.znni_conv3d_choose(S, f, fo, n, k)
        res.append({"workload": f"S{S}_f{f}x{fo}_{n}c_k{k}", "direct_ms": md, "fft_ms": mf,
                    "direct_TFLOP/s": flops / (md * 1e-3) / 1e12,
                    "direct_frac_mfma_fp32": flops / (md * 1e-3) / 1e12 / MFMA_FP32_PEAK_TFLOPS,
                    "direct_out_GB/s": 4.0 * out.numel() / (md * 1e-3) / 1e9,
                    "picked": pick, "estimated_ms": est})
    return res


def bench_sublayers(torch, B, layer, inp, w, bias, out, full_ms):
    """The benchmark layer again with half of its workspace (Section VII-A sub-layers)."""
    S, f, fo, n, k = layer.S, layer.f, layer.fo, layer.n, layer.k
    full = B.znni_conv3d_fft_workspace(S, f, fo, n, k)
    budget = full // 2
    sub, need = B.znni_conv3d_fft_sublayers(S, f, fo, n, k, budget)
    ws = torch.empty(budget, dtype=torch.uint8, device=inp.device)
    ms = _time_ms(torch, lambda: B.znni_conv3d_fft_budget(inp, w, bias, relu=layer.relu, out=out, workspace=ws), 3)
    return {"workload": layer.name, "budget_bytes": budget, "workspace_bytes_used": need,
            "division": {"S_i": sub[0], "f_i": sub[1], "f_out_i": sub[2]}, "ms": ms,
            "out_voxels_per_s": layer.out_voxels / (ms * 1e-3), "slowdown_vs_whole_layer": ms / full_ms}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, help="benchmark layer 1..5 (default: the largest)")
    ap.add_argument("--shape", default=None, metavar="S,f,fo,n,k",
                    help="a layer of the same kind that is not one of the five (cubic images and kernels, bias and "
                         "transfer function on), e.g. 8,80,80,107,5; overrides --config")
    ap.add_argument("--route", choices=("default", "single", "batch", "xdirect", "xblock"), default="default",
                    help="force a form of the multiply-accumulate stage (default: the library picks)")
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="skip the oracle leg: its timing and the check of the timed output against it")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the short measurements of the pooling layer and of the budgeted (sub-layer) run")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import torch
    from paper_1606_05688_amd import binding as B
    from paper_1606_05688_amd import workloads as W

    layer = W.CONFIGS[args.config - 1]
    if args.shape:
        S_, f_, fo_, n_, k_ = (int(v) for v in args.shape.split(","))
        layer = W.Layer(f"S{S_}_{n_}c_f{f_}x{fo_}_k{k_}", S=S_, f=f_, fo=fo_, n=n_, k=k_)
    route = None if args.route == "default" else args.route
    dev = torch.device("cuda:0")
    S, f, fo, n, k = layer.S, layer.f, layer.fo, layer.n, layer.k
    # the seeded synthetic inputs the parity tests use (images U(-1,1), kernels N(0, 1/(f k^3)), bias N(0, 0.1))
    inp_h, w_h, bias_h = W.make_inputs(layer)
    inp, w = torch.from_numpy(inp_h).to(dev), torch.from_numpy(w_h).to(dev)
    bias = torch.from_numpy(bias_h).to(dev) if bias_h is not None else None
    out = torch.empty((S, fo, n - k + 1, n - k + 1, n - k + 1), device=dev)
    ws = B.alloc_workspace(S, f, fo, n, k, dev)
    N = B.znni_fft_size(n)

    for _ in range(args.warmup):
        B.znni_conv3d_fft(inp, w, bias, relu=layer.relu, out=out, workspace=ws, mac_reference=route)
    torch.cuda.synchronize()

    stage_sum = {s: 0.0 for s in B.STAGES}
    t0 = time.perf_counter()
    for _ in range(args.steps):
        _, ms = B.znni_conv3d_fft_profile(inp, w, bias, relu=layer.relu, out=out, workspace=ws, mac_reference=route)
        for s_, v in ms.items():
            stage_sum[s_] += v
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps
    stage_ms = {s_: v / args.steps for s_, v in stage_sum.items()}

    # the same steps through the plain asynchronous entry point, for reference
    t1 = time.perf_counter()
    for _ in range(args.steps):
        B.znni_conv3d_fft(inp, w, bias, relu=layer.relu, out=out, workspace=ws, mac_reference=route)
    torch.cuda.synchronize()
    ms_plain = 1e3 * (time.perf_counter() - t1) / args.steps

    # ... and with the stored kernel transforms of the previous call kept (inference: one kernel bank, many inputs)
    t2 = time.perf_counter()
    for _ in range(args.steps):
        B.znni_conv3d_fft(inp, w, bias, relu=layer.relu, out=out, workspace=ws, mac_reference=route, keep_kernels=True)
    torch.cuda.synchronize()
    ms_kept = 1e3 * (time.perf_counter() - t2) / args.steps

    # what a plain copy kernel reaches on this machine: the achievable line next to the 8 TB/s peak (also the kernel
    # the rocprofv3 traffic counters are calibrated against)
    src = torch.ones(1 << 28, device=dev)               # 1 GiB
    dst = torch.empty_like(src)
    copy_ms = _time_ms(torch, lambda: B.znni_copy_probe(dst, src), 5)
    copy_gbs = 2 * src.numel() * 4 / (copy_ms * 1e-3) / 1e9
    del src, dst

    # the work of the kernels that actually ran (fused kernels and skipped stages priced as such)
    nbytes, nflops = B.znni_conv3d_fft_stage_work(S, f, fo, n, k, relu=layer.relu, mac_reference=route)
    stages = {}
    for s_ in B.STAGES:
        if nbytes[s_] == 0 and nflops[s_] == 0:
            continue                                    # the call has no such stage
        t = stage_ms[s_] * 1e-3
        e = {"ms": stage_ms[s_], "GB": nbytes[s_] / 1e9, "GB/s": nbytes[s_] / t / 1e9,
             "frac_hbm": nbytes[s_] / t / 1e9 / HBM_PEAK_GBS}
        if nflops[s_]:
            e.update({"GFLOP": nflops[s_] / 1e9, "TFLOP/s": nflops[s_] / t / 1e12,
                      "frac_peak": nflops[s_] / t / 1e12 / MFMA_FP32_PEAK_TFLOPS})
        stages[s_] = e
    dom = max(stages, key=lambda s_: stage_ms[s_])
    t = stage_ms[dom] * 1e-3
    if nflops[dom]:
        roof = {"kernel": dom, "bound": "mfma", "achieved": nflops[dom] / t / 1e12, "peak": MFMA_FP32_PEAK_TFLOPS,
                "unit": "TFLOP/s"}
    else:
        roof = {"kernel": dom, "bound": "hbm", "achieved": nbytes[dom] / t / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = measured_traffic(layer.name + ("" if route is None else ":" + route), dom)
    roof["traffic_source"] = os.path.relpath(TRAFFIC_FILE, ROOT)
    roof["avg_launch_ms"] = stage_ms[dom]
    if dom == "mac":
        # `achieved` counts 8 flops per complex multiply-add of the form of the stage that ran (see
        # znni_conv3d_fft_stage_work_v); each is issued as three real matrix-core products (6 flops), so the matrix
        # pipes are busy for 3/4 of that rate
        roof["counting"] = "algorithmic: 8 flops per complex multiply-add; issued_*: the 6 the three-product form issues"
        roof["issued_TFLOP/s"] = 0.75 * roof["achieved"]
        roof["issued_frac"] = 0.75 * roof["frac"]
        # for comparison, the same stage priced as if the x axis were transformed at full length: the per-bin product
        # plus the kernel-tap sum per bin that stands in for a stored kernel-spectrum bank (the form that ran may
        # do less work than that: these two are rates of an equivalent, not of work done)
        full_len = (8.0 * S + 8.0 * (k - 1)) * f * fo * (N // 2 + 1) * N * N
        roof["full_length_equivalent_TFLOP/s"] = full_len / t / 1e12
        mac_only = 8.0 * S * f * fo * (N // 2 + 1) * N * N
        roof["mac_only_TFLOP/s"] = mac_only / t / 1e12
    pass_names = [s_ for s_ in ("fwd_z", "fwd_y", "fwd_x", "inv_x", "inv_y", "inv_z") if s_ in stages]
    fft_bytes = sum(nbytes[s_] for s_ in pass_names)
    fft_ms = sum(stage_ms[s_] for s_ in pass_names)

    rec = {
        "metric": "output voxels/sec per conv layer at 1 GPU",
        "value": layer.out_voxels / (ms_per_step * 1e-3),
        "unit": "output voxels/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "ms_per_step_async_entry": ms_plain, "ms_per_step_kernels_kept": ms_kept,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": layer.name, "S": S, "f": f, "f_out": fo, "n": n, "k": k,
                   "fft_size": N, "out_voxels": layer.out_voxels, "relu": layer.relu, "bias": layer.bias,
                   "route": args.route, "stages_run": list(stages)},
        "roofline": roof,
        "fft_passes": {"kernels": pass_names, "GB": fft_bytes / 1e9, "ms": fft_ms,
                       "GB/s": fft_bytes / (fft_ms * 1e-3) / 1e9,
                       "frac_hbm": fft_bytes / (fft_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "copy_probe": {"GB/s": copy_gbs, "frac_hbm": copy_gbs / HBM_PEAK_GBS,
                       "what": "plain 1 GiB device copy kernel, read + write: the achievable line for the passes"},
        "stages": stages,
    }
    if not args.no_cpu_baseline:
        # the oracle leg, part one: the tensor the timed steps wrote, checked before anything overwrites it
        rec["parity_of_timed_output"] = check_timed_output(layer, W, inp_h, w_h, bias_h, out)
    if not args.no_extras:
        # not part of the timed steps above: the rows built next to the hot path, measured once each
        whole = out.clone() if out.numel() * 4 < 8e9 else None
        rec["next_rows"] = {"sublayers": bench_sublayers(torch, B, layer, inp, w, bias, out, ms_plain)}
        if whole is not None:
            tolj = (1e-4 * float(inp.abs().max()) * w.abs().sum(dim=(1, 2, 3, 4)))[None, :, None, None, None]
            rec["next_rows"]["sublayers"]["max_diff_vs_whole_layer_over_tol"] = float(((out - whole).abs() / tolj).max())
            del whole
        del ws
        torch.cuda.empty_cache()
        rec["next_rows"]["mpf"] = bench_mpf(torch, B, dev)
        rec["next_rows"]["direct"] = bench_direct(torch, B, dev)
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(layer, W)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
