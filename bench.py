#!/usr/bin/env python3
"""Benchmark of the kn2row MCMK convolution on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-table] [--no-cpu] [--vendor]

A step is one call of conv_mcmk_kn2row (the 1x1 GEMMs of all k*k taps with the shift-add fused,
paper section III-A) on one batch of synthetic input that is already resident in HBM; the kernel
re-ordering is done once before timing, as the paper prescribes.  Prints ONE JSON line: conv
GFLOP/s (2 M C k^2 P Q N per call), the roofline of the kernel, the CPU oracle timed on the host's
cores, and -- outside the timed steps -- the same layer through the im2col, two-pass kn2row and
direct variants plus the other benchmark layers, so the kn2row : im2col time and memory ratios are
reported per configuration.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_F32_MFMA_TFLOPS = 157.3      # MI355X dense fp32 matrix peak
PEAK_BF16_MFMA_TFLOPS = 2500.0    # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0
DEFAULT_WORKLOAD = "cfg5a_vgg_deep56"

# The GPU needs some tens of milliseconds under load to reach its steady clock.  Whatever --warmup says, the timed
# plan first runs untimed for at least this long (reported as clock_ramp_ms); --steps and --warmup stay as given.
CLOCK_RAMP_MS = 150.0

# HBM bytes per launch of the fused kernel measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE scaled by a copy
# kernel of known size), from the committed summaries.  A figure belongs to one kernel on one layer, so the key is
# (workload, operand type, the plan the library reports for it, without its time estimate); a launch whose plan is
# not in the table reports no traffic rather than another kernel's.
MEASURED_TRAFFIC_BYTES = {
    # profiles/kn2row_tile_f32_cfg5a_hbm_traffic.txt
    ("cfg5a_vgg_deep56", "f32", "kn2row fused f32: tile 14x28, waves 4x4, row blocks 1, channel groups 1, channel split 1, "
                                "256 workgroups"): 74_316_000,
    # profiles/cfg4_hbm_traffic_all_variants.txt
    ("cfg4_vgg_early", "f32", "kn2row fused f32: tile 14x14, waves 4x2, row blocks 1, channel groups 1, channel split 1, "
                              "256 workgroups"): 27_964_000,
}


def plan_key(plan_text):
    """The plan line without its trailing time estimate."""
    return plan_text.split(", est ")[0]


def measured_traffic(workload, dtype_name, plan_text):
    return MEASURED_TRAFFIC_BYTES.get((workload, dtype_name, plan_key(plan_text)))


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_calls(fn, steps, warmup):
    """Wall-clock around `steps` back-to-back calls (synchronised both sides) and the average
    device time per call from HIP events recorded on the launch stream."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for _ in range(steps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return wall_ms / steps, start.elapsed_time(stop) / steps


def ramp_clocks(fn, min_ms=CLOCK_RAMP_MS):
    """Run `fn` back to back, untimed, until at least `min_ms` of device time have passed.  Returns the ms spent."""
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while True:
        for _ in range(50):
            fn()
        torch.cuda.synchronize()
        spent = (time.perf_counter() - t0) * 1e3
        if spent >= min_ms:
            return spent


def measured_machine_rates(dev):
    """What the device at hand sustains: the matrix-core instructions in a register-only loop (fp32 and bf16) and
    a plain 16-byte copy, through the library's probe kernels.  TFLOP/s, TFLOP/s, GB/s (read + written)."""
    import torch
    from paper_1704_04428_amd import binding as B
    blocks = 2048                                    # 8 workgroups of 4 waves per compute unit
    sink = torch.empty(blocks * 256, dtype=torch.float32, device=dev)
    out = {}
    for name, dtype, iters, flop in (("f32", B.F32, 2000, 2048.0), ("bf16", B.BF16, 4000, 16384.0)):
        run = lambda: B.conv_mcmk_probe_mfma(dtype, blocks, iters, sink)        # noqa: E731
        _, ms = time_calls(run, 10, 10)
        out["mfma_" + name + "_tflops"] = round(blocks * 4 * iters * 16 * flop / (ms * 1e-3) / 1e12, 1)
    nbytes = 256 << 20
    src = torch.ones(nbytes // 4, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    run = lambda: B.conv_mcmk_probe_copy(src, dst, nbytes)                       # noqa: E731
    _, ms = time_calls(run, 20, 10)
    out["copy_gbs"] = round(2 * nbytes / (ms * 1e-3) / 1e9, 1)
    return out


def auto_counts(fn, warm_ms=60.0, timed_ms=120.0):
    """Warm-up and step counts that give about `warm_ms` of warm-up and `timed_ms` of timed work."""
    _, ms = time_calls(fn, 5, 2)
    ms = max(ms, 1e-3)
    return max(20, int(timed_ms / ms)), max(10, int(warm_ms / ms))


def time_in_graph(fn, launches=50, replays=40):
    """Average time per call when `launches` calls are captured into one HIP graph and the graph is
    replayed: what a launch-bound layer costs once the host is out of the loop."""
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()                                   # anything lazy happens outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(launches):
            fn()
    for _ in range(5):
        graph.replay()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(replays):
        graph.replay()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / (replays * launches)


def bench_layer(L, variants, steps, warmup, I_dev=None, K_dev=None, dtype=0):
    import torch
    from paper_1704_04428_amd import binding as B
    from paper_1704_04428_amd import workloads as wl
    dev = torch.device("cuda:0")
    if I_dev is None:
        I_dev = torch.from_numpy(wl.make_input(L)).to(dev)
        K_dev = torch.from_numpy(wl.make_kernel(L)).to(dev)
    if dtype == B.BF16:
        I_bf = torch.empty(I_dev.shape, dtype=torch.bfloat16, device=dev)
        B.conv_mcmk_cvt_f32_bf16(I_dev, I_bf)
        I_dev = I_bf
    d = B.desc(L.n, L.c, L.h, L.w, L.m, L.k, L.pad, L.stride, dtype)
    I_cl = None
    out = {}
    for name in variants:
        # two entry points that are not variants of their own: the fused kernel with the bias /
        # rectifier epilogue, and the 1 x 1 building block called directly
        variant = B.KN2ROW if name in ("kn2row_bias_relu", "1x1") else B.VARIANTS[name]
        if variant in B.CHANNELS_LAST and L.c % (8 if dtype == B.BF16 else 4):
            continue
        plan = B.Plan(d, variant, K_dev)
        I_use = I_dev
        if variant in B.CHANNELS_LAST:       # kn2col and im2row take I[N][H][W][C]
            if I_cl is None:
                I_cl = I_dev.permute(0, 2, 3, 1).contiguous()
            I_use = I_cl
        if name == "kn2row_bias_relu":
            bias = torch.full((L.m,), -0.05, dtype=torch.float32, device=dev)
            run = lambda: B.conv_mcmk_kn2row_bias_relu(d, I_use, plan.kernel, bias, 1, plan.out)   # noqa: E731
        elif name == "1x1":
            run = lambda: B.conv_mcmk_1x1(d, I_use, plan.kernel, plan.out)                         # noqa: E731
        else:
            run = lambda: plan.run(I_use)                                                          # noqa: E731
        torch.cuda.synchronize()
        if steps is None:
            n_steps, n_warm = auto_counts(run)
        else:
            n_steps, n_warm = steps, warmup
        wall_ms, dev_ms = time_calls(run, n_steps, n_warm)
        out[name] = {
            "ms": round(dev_ms, 5),
            "gflops": round(L.flops / (dev_ms * 1e-3) / 1e9, 1),
            "workspace_bytes": B.conv_mcmk_workspace_bytes(d, variant),
        }
        if name == "kn2row" and dev_ms < 0.02:
            # a launch-bound layer: the interval between launches issued from Python is part of "ms";
            # the same calls replayed from a HIP graph show the device's share
            out[name]["ms_in_graph"] = round(time_in_graph(run), 5)
        del plan
    return out


def library_gemm_ms(L, bf16=False):
    """Context for the im2col baseline, not part of the library: the GEMM [M x C k^2].[C k^2 x QP] per image
    (the product im2col hands to a GEMM, section II-B) through torch.bmm, i.e. the vendor BLAS."""
    import torch
    dt = torch.bfloat16 if bf16 else torch.float32
    a = torch.randn(L.m, L.c * L.k * L.k, device="cuda", dtype=dt)
    b = torch.randn(L.n, L.c * L.k * L.k, L.q * L.p, device="cuda", dtype=dt)
    out = torch.empty(L.n, L.m, L.q * L.p, device="cuda", dtype=dt)
    run = lambda: torch.matmul(a, b, out=out)                    # noqa: E731
    n_steps, n_warm = auto_counts(run)
    return time_calls(run, n_steps, n_warm)[1]


def library_conv_ms(L, bf16=False):
    """Context only: the same layer through torch.nn.functional.conv2d, i.e. the vendor's convolution library
    as PyTorch calls it (whatever algorithm it picks; framework overhead included)."""
    import torch
    import torch.nn.functional as F
    dt = torch.bfloat16 if bf16 else torch.float32
    x = torch.rand(L.input_shape(), device="cuda", dtype=dt)
    k = torch.randn(L.kernel_shape(), device="cuda", dtype=dt) * 0.05
    run = lambda: F.conv2d(x, k, padding=L.pad, stride=L.stride)       # noqa: E731
    for _ in range(3):
        run()
    torch.cuda.synchronize()
    n_steps, n_warm = auto_counts(run)
    return time_calls(run, n_steps, n_warm)[1]


SELECTOR_CASES = [          # (n, c, h, w, m, k, pad, stride): layers inside and outside the fused kernels' range
    (1, 3, 227, 227, 96, 11, 0, 4), (1, 64, 30, 30, 64, 9, 4, 1), (1, 32, 28, 28, 96, 5, 2, 1), (2, 128, 28, 28, 128, 3, 1, 1),
    (1, 16, 32, 32, 16, 3, 1, 1), (1, 8, 64, 64, 8, 8, 4, 3), (2, 3, 224, 224, 64, 7, 3, 2), (2, 3, 112, 112, 32, 3, 1, 1),
]


def selector_report():
    """How the per-layer choice among the algorithms (conv_mcmk_select) compares with timing them all: a report, not a
    test -- parity tests never assert on time."""
    import torch
    from paper_1704_04428_amd import binding as B
    names = {v: k for k, v in B.VARIANTS.items()}
    out = []
    for case in SELECTOR_CASES:
        n, c, h, w, m, k, pad, stride = case
        d = B.desc(n, c, h, w, m, k, pad, stride)
        I = torch.rand(n, c, h, w, device="cuda")
        K = torch.randn(m, c, k, k, device="cuda") * 0.05
        chosen, est = B.conv_mcmk_select(d)
        times = {}
        for variant in (B.KN2ROW, B.KN2ROW_2PASS, B.IM2COL, B.DIRECT):
            if B.conv_mcmk_check(d, variant) != B.OK:
                continue
            plan = B.Plan(d, variant, K)
            n_steps, n_warm = auto_counts(lambda: plan.run(I), 10.0, 20.0)
            times[names[variant]] = round(time_calls(lambda: plan.run(I), n_steps, n_warm)[1], 5)
        out.append({"layer": list(case), "chosen": names[chosen], "estimate_us": round(est, 1), "ms": times,
                    "chosen_over_fastest": round(times[names[chosen]] / min(times.values()), 3)})
    return out


def cpu_baseline(L, I, K, budget_s=12.0, max_passes=40):
    """The oracle as it stands, timed on the host cores: whole passes over the workload until about
    `budget_s` seconds of CPU work have been spent."""
    import oracle
    passes, t0 = 0, time.perf_counter()
    while True:
        oracle.mcmk(I, K, L.pad, L.stride)
        passes += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or passes >= max_passes:
            break
    cores = int(os.environ.get("OMP_NUM_THREADS", "0")) or len(os.sched_getaffinity(0))
    return {"value": round(passes * L.flops / dt / 1e9, 3), "unit": "GFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"{passes} pass(es) over the whole {L.name} batch ({L.flops / 1e9:.2f} GFLOP each, "
                      f"fp64 direct loop nest, OpenMP), {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the GPU needs some tens of milliseconds under load to reach its steady clock: 300 warm-up steps
    # of the default workload are about 70 ms, 1000 timed steps about a quarter of a second
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--variant", default="kn2row", choices=["kn2row", "kn2row_2pass", "im2col", "direct", "kn2col", "im2row"],
                    help="which entry point the timed steps call (the headline is kn2row)")
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"], help="operand type of the timed steps")
    ap.add_argument("--no-table", action="store_true", help="skip the other variants and layers")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--vendor", action="store_true",
                    help="context only: also time the vendor libraries (torch.matmul, torch conv2d) on the table's layers")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (one process, one MI355X); use --gpus 1")

    import numpy as np
    import torch
    from paper_1704_04428_amd import binding as B
    from paper_1704_04428_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    B.lib()
    layers = {**wl.LAYERS, **wl.GENERALISED_LAYERS}
    if args.workload not in layers:
        sys.exit("bench.py: unknown workload %r (known: %s)" % (args.workload, ", ".join(layers)))
    L = layers[args.workload]
    dev = torch.device("cuda:0")
    I, K = wl.make_input(L), wl.make_kernel(L)
    I_dev, K_dev = torch.from_numpy(I).to(dev), torch.from_numpy(K).to(dev)
    dtype = B.BF16 if args.dtype == "bf16" else B.F32
    d = B.desc(L.n, L.c, L.h, L.w, L.m, L.k, L.pad, L.stride, dtype)
    plan = B.Plan(d, B.VARIANTS[args.variant], K_dev)   # re-orders the kernel once, outside the timed region
    I_run = I_dev
    if dtype == B.BF16:
        I_run = torch.empty(I_dev.shape, dtype=torch.bfloat16, device=dev)
        B.conv_mcmk_cvt_f32_bf16(I_dev, I_run)
    channels_last = B.VARIANTS[args.variant] in B.CHANNELS_LAST
    if channels_last:
        I_run = I_run.permute(0, 2, 3, 1).contiguous()
    torch.cuda.synchronize()

    ramp_ms = ramp_clocks(lambda: plan.run(I_run))
    wall_ms, dev_ms = time_calls(lambda: plan.run(I_run), args.steps, args.warmup)
    rates = measured_machine_rates(dev)
    gflops = L.flops / (wall_ms * 1e-3) / 1e9
    achieved_tflops = L.flops / (dev_ms * 1e-3) / 1e12

    # sanity: the timed output against the oracle on sampled points
    pts = wl.sample_points(L, 512)
    out_nmqp = plan.out.permute(0, 3, 1, 2) if channels_last else plan.out
    got = out_nmqp.cpu().numpy()[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]].astype(np.float64)
    import oracle
    ref, absref = oracle.mcmk_at(I, K, L.pad, pts, L.stride)
    worst = float(np.max(np.abs(got - ref) / np.maximum(absref, 1e-30)))
    if not worst <= (1e-2 if dtype == B.BF16 else 1e-4):
        sys.exit(f"bench.py: output fails parity (worst error {worst:.3e} of sum|K||I|)")

    peak = PEAK_BF16_MFMA_TFLOPS if dtype == B.BF16 else PEAK_F32_MFMA_TFLOPS
    measured_peak = rates["mfma_bf16_tflops" if dtype == B.BF16 else "mfma_f32_tflops"]
    plan_text = B.conv_mcmk_describe_plan(d, B.VARIANTS[args.variant])
    result = {
        "metric": f"conv GFLOP/s (2*M*C*k^2*P*Q*N / time), {args.variant}",
        "value": round(gflops, 1),
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": args.dtype,
        "data": "synthetic",
        "config": {"workload": L.name, "n": L.n, "c": L.c, "h": L.h, "w": L.w, "m": L.m, "k": L.k,
                   "pad": L.pad, "stride": L.stride, "variant": args.variant + (" (fused shift-add)" if args.variant == "kn2row" else ""),
                   "flops_per_step": L.flops, "plan": plan_text},
        "clock_ramp_ms": round(ramp_ms, 1),
        "roofline": {"bound": "mfma", "achieved": round(achieved_tflops, 3), "peak": peak,
                     "unit": "TFLOP/s", "frac": round(achieved_tflops / peak, 4),
                     "traffic": measured_traffic(L.name, args.dtype, plan_text) if args.variant == "kn2row" else None,
                     "kernel_ms": round(dev_ms, 5),
                     # the same instruction in a register-only loop on this device, measured just now
                     "measured_peak": measured_peak,
                     "frac_of_measured_peak": round(achieved_tflops / measured_peak, 4)},
        "machine": rates,
        "parity_worst_err_over_bound_norm": worst,
    }
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(L, I, K)
    if not args.no_table:
        table = {}
        for name, layer in wl.LAYERS.items():
            variants = ["kn2row", "kn2col", "im2col", "im2row", "kn2row_2pass"] + (["direct"] if layer.flops < 5e9 else [])
            steps = None          # enough launches for ~60 ms of warm-up and ~120 ms of timed work
            same = name == L.name
            table[name] = bench_layer(layer, variants, steps, None, I_dev if same else None, K_dev if same else None)
            r = table[name]
            r["kn2row_over_im2col_time"] = round(r["kn2row"]["ms"] / r["im2col"]["ms"], 4)
            if args.vendor:
                r["library_conv_ms"] = {"f32": round(library_conv_ms(layer), 5)}
                # how the hand-written GEMM of the im2col baseline compares with the vendor BLAS on the same product
                r["library_gemm_ms"] = {"f32": round(library_gemm_ms(layer), 5)}
            r["frac_f32_mfma_peak"] = round(r["kn2row"]["gflops"] / 1e3 / PEAK_F32_MFMA_TFLOPS, 4)
            if name.startswith("cfg5"):          # the deep-layer sweep is also quoted with bf16 operands
                b = bench_layer(layer, ["kn2row", "kn2col", "im2col", "im2row", "kn2row_2pass"], steps, None,
                                I_dev if same else None, K_dev if same else None, dtype=B.BF16)
                b["frac_bf16_mfma_peak"] = round(b["kn2row"]["gflops"] / 1e3 / PEAK_BF16_MFMA_TFLOPS, 4)
                if args.vendor:
                    r["library_gemm_ms"]["bf16"] = round(library_gemm_ms(layer, bf16=True), 5)
                    r["library_conv_ms"]["bf16"] = round(library_conv_ms(layer, bf16=True), 5)
                r["bf16"] = b
            log(name, json.dumps(r))
        result["table"] = table
        # beyond the paper: stride 2, an even kernel side, the 1 x 1 block on its own, the epilogue
        extras = {}
        for name, layer in wl.GENERALISED_LAYERS.items():
            variants = ["kn2row", "kn2col", "im2col"] + (["1x1"] if layer.k == 1 else [])
            extras[name] = bench_layer(layer, variants, None, None)
            extras[name]["bf16"] = bench_layer(layer, variants, None, None, dtype=B.BF16)
            log(name, json.dumps(extras[name]))
        extras["cfg5a_bias_relu"] = bench_layer(L, ["kn2row", "kn2row_bias_relu"], None, None, I_dev, K_dev) \
            if L.name == DEFAULT_WORKLOAD else None
        log("cfg5a_bias_relu", json.dumps(extras["cfg5a_bias_relu"]))
        result["generalisations"] = extras
        result["selector"] = selector_report()
        log("selector", json.dumps(result["selector"]))
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
