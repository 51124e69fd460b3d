#!/usr/bin/env python3
"""Benchmark of the TORQ hot path on one MI355X.

One "step" is one pass of the whole online path over one batch of synthetic
activations: torq_linear = two-level rotation + MXFP4 quantisation of X
(Algorithm 3 steps 1-4) followed by the W4A4 MXFP4 GEMM against weights that
were rotated and quantised offline (Algorithm 3 "Return").  Inputs are resident
in HBM before the timed region starts.

Prints ONE JSON line.  `value` is the whole step's throughput in TFLOP/s
(2 M N d per step); `roofline` describes the dominant kernel (the GEMM, against
the dense fp4 MFMA peak); `roofline_rotate_quant` describes the rotate+quantise
kernel against the HBM peak (2.53125 algorithmic bytes per element);
`cpu_baseline` is the CPU oracle timed on a bounded sample in the same run.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
FP4_PEAK_TFLOPS = 10100.0      # MI355X dense fp4 MFMA, published
BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
RQ_BYTES_PER_ELEMENT = 2.0 + 0.5 + 1.0 / 32.0   # bf16 in, packed nibble + 1/32 scale byte out



def measured_traffic(key):
    """HBM bytes per launch of the headline kernels, from profiles/traffic.json (written by
    `python -m paper_2605_19561_amd.traffic` out of two rocprofv3 --pmc runs of this program), and whether
    the kernel sources have changed since those runs."""
    from paper_2605_19561_amd import traffic
    return traffic.lookup(key)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="llama3_70b_up")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-board-sample", action="store_true",
                    help="skip the two one-second runs that sample board power and shader clock (for kernel "
                         "traces: they add some 20000 launches to the per-kernel averages)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run the library's plain copy kernel on 1 GiB (known traffic) so that a rocprofv3 --pmc "
                         "run of this command carries its own scale for FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--headline-only", action="store_true",
                    help="leave out the `configs` array (the other shapes of the benchmark configurations): for "
                         "kernel traces and counter runs of the headline step")
    ap.add_argument("--ablate", action="store_true",
                    help="also print, for the two headline kernels, the launch time with parts of their work left out "
                         "(torq_diag_gemm_ablation / torq_diag_rotate_ablation): what each part costs on this machine")
    ap.add_argument("--sweep", action="store_true",
                    help="also print one line per rotate+quantise bandwidth-sweep shape ([16384, d])")
    ap.add_argument("--decode-forms", action="store_true",
                    help="instead of the benchmark: torq_linear as the library routes it, as its two launches (rotate + "
                         "quantise, then the GEMM) and as the one launch whose workgroups rotate the rows themselves, on a "
                         "grid of decode shapes with one to four token-groups, weights from HBM; one JSON line per shape")
    ap.add_argument("--plan-sweep", choices=("fit", "check", "decode", "rounds"), default=None,
                    help="instead of the benchmark: time every plan the GEMM's planner can choose from (tile shape x k "
                         "pieces x load pipeline, forced through torq_diag_gemm_plan) on a grid of shapes of up to one "
                         "round of 256x256 tiles, one JSON line per shape with the planner's own choice beside them; "
                         "'fit' and 'check' are two disjoint grids, 'decode' has 8 to 64 rows; 'rounds' is the regime beyond "
                         "one round (one to seven rounds of 256x256 tiles): the planner's choice, two launches included, "
                         "against one launch of each tile shape, plain and persistent")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "re-run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2605_19561_amd import binding as tq, synth
    if args.plan_sweep == "rounds":
        rounds_sweep(tq, torch)
        return
    if args.plan_sweep:
        plan_sweep(tq, torch, args.plan_sweep)
        return
    if args.decode_forms:
        decode_forms(tq, synth, torch)
        return

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    wl = synth.WORKLOADS[args.workload]
    M, d, N = wl["M"], wl["d"], wl["N"]
    G = synth.default_G(d)

    # ---- synthetic inputs, generated on the device, resident before timing ----
    x = synth.workload_activations(args.workload, device=dev)
    Ri, Ra = synth.rotations(G)
    rot = tq.Rotation(d, G, Ri, Ra)
    w = synth.workload_weights(args.workload, device=dev)
    W_q, W_s = tq.torq_rotate_quantize(rot, w)          # offline weight preparation
    del w
    out = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    ws_bytes = tq.torq_linear_workspace_bytes(M, d)
    workspace = torch.empty((ws_bytes,), dtype=torch.uint8, device=dev)
    codes = torch.empty((M, d // 2), dtype=torch.uint8, device=dev)
    scales = torch.empty((M, d // 32), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    def step():
        tq.torq_linear(rot, x, W_q, W_s, out=out, workspace=workspace)

    # W untimed steps, then more of them until 40 ms have passed: after the pause that input generation
    # is, the shader clock needs that long under load to reach the level it then keeps
    settle(torch, step, args.warmup)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    flops = 2.0 * M * N * d
    value = flops / (ms_per_step * 1e-3) / 1e12

    # ---- per-kernel durations: HIP events on the stream the kernels run on (torch's current
    # stream, which is the one handed to the library).  Each kernel is launched `steps` times back
    # to back between two events, so launch gaps are not attributed to it.  rotate+quantise moves
    # only 170 MB per launch, which would fit the 256 MB Infinity Cache: it cycles over five copies
    # of the input (670 MB) so that every launch reads from HBM.
    x_copies = [x, x.clone(), x.clone()]
    e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    x_copies += [x.clone() for _ in range(2)]          # five copies, 670 MB: far beyond the Infinity Cache
    counter = [0]

    def rq_call():
        tq.torq_rotate_quantize(rot, x_copies[counter[0] % len(x_copies)], codes=codes, scales=scales)
        counter[0] += 1
    settle(torch, rq_call, 3)
    e[0].record()
    for i in range(args.steps):
        tq.torq_rotate_quantize(rot, x_copies[i % len(x_copies)], codes=codes, scales=scales)
    e[1].record()
    settle(torch, lambda: tq.mxfp4_gemm(codes, scales, W_q, W_s, out=out), 1)
    e[2].record()
    for i in range(args.steps):
        tq.mxfp4_gemm(codes, scales, W_q, W_s, out=out)
    e[3].record()
    torch.cuda.synchronize()
    rq_ms = e[0].elapsed_time(e[1]) / args.steps
    gemm_ms = e[2].elapsed_time(e[3]) / args.steps

    # ---- board power and shader clock while each kernel runs alone for a second (the driver's
    # sensors, read from sysfs; None where the machine does not expose them)
    gemm_env = rq_env = None
    if not args.no_board_sample:
        gemm_env = sample_board(torch, lambda i: tq.mxfp4_gemm(codes, scales, W_q, W_s, out=out), 1.0)
        rq_env = sample_board(torch, lambda i: tq.torq_rotate_quantize(rot, x_copies[i % len(x_copies)], codes=codes, scales=scales), 1.0)

    # ---- what the matrix cores sustain on this part with nothing else running, on this step's own
    # operands (the weights' packed codes; the bf16 activations): the part lowers its clock under
    # matrix work on non-trivial operands, so the published peaks are not reachable by any kernel
    sink = torch.empty((tq.TORQ_DIAG_SINK_FLOATS,), dtype=torch.float32, device=dev)
    sustained = {}
    for kind, ops, iters in ((tq.TORQ_DIAG_FP4, W_q, 8000), (tq.TORQ_DIAG_BF16, x, 8000)):
        tq.torq_diag_mfma_burn(kind, ops, 500, sink=sink)
        e[0].record()
        burn_flop = tq.torq_diag_mfma_burn(kind, ops, iters, sink=sink)
        e[1].record()
        torch.cuda.synchronize()
        sustained[kind] = burn_flop / (e[0].elapsed_time(e[1]) * 1e-3) / 1e12
    del sink

    gemm_tflops = flops / (gemm_ms * 1e-3) / 1e12
    rq_bytes = M * d * RQ_BYTES_PER_ELEMENT
    rq_gbs = rq_bytes / (rq_ms * 1e-3) / 1e9
    # split-bf16 contraction actually executed: 2 passes over R_inter (2G flop each), 3 over R_intra (64)
    rq_mfma_tflops = M * d * (2 * 2 * G + 3 * 64) / (rq_ms * 1e-3) / 1e12
    # context: what the runtime's own device-to-device copy of 1 GiB reaches on this machine
    copy_gbs = copy_line(torch, dev, 10)["value"]

    gemm_traffic, gemm_stale = measured_traffic(f"mxfp4_gemm/{args.workload}")
    rq_traffic, rq_stale = measured_traffic(f"torq_rotate_quantize/{args.workload}")
    result = {
        "metric": "TORQ W4A4 MXFP4 linear layer (rotate + MXFP4 quantise + fp4 GEMM), whole step",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "fp4 (e2m1 x E8M0) with fp32 accumulation; rotation in split bf16",
        "data": "synthetic",
        "timing": "timed steps start after the warm-up steps and 40 ms more of them (clock settled); per-kernel times "
                  "from HIP events around back-to-back launches; HBM-bound kernels cycle over input copies of more than "
                  "600 MB in all, and the GEMM and torq_linear lines of `configs` over weight copies of as much, so the "
                  "256 MB Infinity Cache serves none of them (weights come from HBM, as a model's do)",
        "config": {"workload": f"{args.workload}: X bf16 [{M}, {d}] Student-t(nu={wl['nu']}) with "
                               f"{wl['outliers']} outlier channels x{wl['outlier_scale']:g}, G={G}, "
                               f"W [{N}, {d}] ~ N(0, {wl['wstd']}^2) rotated+quantised offline, out bf16 [{M}, {N}]",
                   "M": M, "N": N, "d": d, "G": G},
        "roofline": {"kernel": "mxfp4_gemm", "bound": "mfma", "achieved": round(gemm_tflops, 1),
                     "peak": FP4_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(gemm_tflops / FP4_PEAK_TFLOPS, 4),
                     "traffic": gemm_traffic, "traffic_stale": gemm_stale,
                     "avg_kernel_ms": round(gemm_ms, 4),
                     "sustained_mfma_only": round(sustained[tq.TORQ_DIAG_FP4], 1),
                     "board": gemm_env},
        "roofline_rotate_quant": {"kernel": "torq_rotate_quantize", "bound": "hbm", "achieved": round(rq_gbs, 1),
                                  "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(rq_gbs / HBM_PEAK_GBS, 4),
                                  "traffic": rq_traffic, "traffic_stale": rq_stale,
                                  "avg_kernel_ms": round(rq_ms, 4),
                                  "mfma_bf16_tflops": round(rq_mfma_tflops, 1),
                                  "mfma_bf16_frac": round(rq_mfma_tflops / BF16_PEAK_TFLOPS, 4),
                                  "mfma_bf16_sustained_mfma_only": round(sustained[tq.TORQ_DIAG_BF16], 1),
                                  "runtime_copy_1GiB_GBps": copy_gbs,
                                  "board": rq_env},
    }

    if not args.headline_only:
        del x_copies[1:]
        result["configs"] = config_lines(tq, synth, torch, args.steps, args.warmup, result)

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(x, W_q, W_s, Ri, Ra, G, M, N, d)

    print(json.dumps(result), flush=True)

    if args.calibrate_copy:
        src = torch.full((1 << 30,), 7, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            tq.torq_diag_copy(src, dst)
        torch.cuda.synchronize()
        del src, dst

    if args.ablate:
        print(json.dumps(ablation_lines(tq, torch, rot, x, codes, scales, W_q, W_s, out, args.steps)), flush=True)

    if args.sweep:
        # context for the HBM-bound lines below: what the runtime's own device-to-device copy of 1 GiB
        # (read + write, far beyond the 256 MB Infinity Cache) reaches on this machine
        print(json.dumps(copy_line(torch, dev, args.steps)), flush=True)
        for dd in (4096, 8192, 14336, 28672):
            print(json.dumps(sweep_line(tq, synth, dd, args.steps, args.warmup)), flush=True)
        # the Qwen3-32B widths (d/32 = 160 and 800: G = 80, the 16x16x32 MFMA kernel; and G = 160 at d = 5120)
        for dd in (5120, 25600):
            print(json.dumps(sweep_line(tq, synth, dd, args.steps, args.warmup)), flush=True)
        print(json.dumps(sweep_line(tq, synth, 5120, args.steps, args.warmup, G=160)), flush=True)
        # G = d/32: Algorithm 3 as printed (one R_inter over the whole row), a dense contraction
        print(json.dumps(sweep_line(tq, synth, 8192, args.steps, args.warmup, G=256)), flush=True)
        # smaller inter-block rotations (Appendix A.7 counts with B = 32): less contraction per byte,
        # the kernel moves towards the HBM roofline
        for dd, gg in ((4096, 32), (8192, 32), (8192, 64)):
            print(json.dumps(sweep_line(tq, synth, dd, args.steps, args.warmup, G=gg)), flush=True)
        # R_inter as a butterfly of plane rotations (Section 5.1's efficient form): no G x G contraction
        for dd, gg in ((8192, 32), (8192, 64), (8192, 128), (8192, 256), (28672, 128)):
            print(json.dumps(sweep_line(tq, synth, dd, args.steps, args.warmup, G=gg, butterfly=True)), flush=True)
        # the other block formats of Section 6 through the same kernel
        for ff in (1, 2):
            print(json.dumps(sweep_line(tq, synth, 8192, args.steps, args.warmup, fmt=ff)), flush=True)
        # calibration statistic (Section 5.1): block Gram matrix of the benchmark's activations, HBM bound
        print(json.dumps(gram_line(tq, x, G, args.steps, args.warmup)), flush=True)
        xl = torch.cat([x, x, x, x], dim=0)             # a longer calibration sample: [32768, d]
        print(json.dumps(gram_line(tq, xl, G, args.steps, args.warmup)), flush=True)
        del xl
        # calibration statistic (Section 5.2): codeword histogram per in-block position of the step's
        # packed codes, and of a set eight times as long; HBM bound at half a byte per element
        print(json.dumps(hist_line(tq, codes, d, args.steps, args.warmup)), flush=True)
        print(json.dumps(hist_line(tq, torch.cat([codes] * 8, dim=0), d, args.steps, args.warmup)), flush=True)
        # the W4A4 GEMM alone on the other layer shapes of the LLaMA3-8B / Qwen3-32B / LLaMA3-70B configurations
        for (mm, nn, dd) in ((8192, 8192, 28672), (8192, 8192, 8192), (2048, 14336, 4096), (2048, 4096, 14336),
                             (2048, 4096, 4096), (2048, 1024, 4096), (4096, 25600, 5120), (4096, 5120, 25600),
                             (4096, 8192, 5120), (4096, 5120, 5120), (4096, 1024, 5120)):
            print(json.dumps(gemm_line(tq, mm, nn, dd, args.steps, args.warmup)), flush=True)
        # decode-sized linear layers (few activation rows: weight streaming, HBM bound), timed as
        # replays of a HIP graph of 20 calls so that Python's launch overhead is not in the figure
        for (mm, nn, dd) in ((1, 14336, 4096), (16, 14336, 4096), (16, 4096, 14336), (16, 28672, 8192),
                             (64, 28672, 8192), (128, 8192, 28672), (256, 4096, 14336)):
            print(json.dumps(decode_line(tq, synth, mm, nn, dd)), flush=True)
    rot.close()


def cpu_baseline(x, W_q, W_s, Ri, Ra, G, M, N, d):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: rotate+quantise of the
    first rows of X, and the reference GEMM on an output corner, each extrapolated to the full step."""
    import numpy as np
    import oracle
    from paper_2605_19561_amd import synth

    rows = min(M, 8192)
    gm, gn = min(M, 256), min(N, 4096)
    xb = synth.bf16_bits(x[:rows])
    t0 = time.perf_counter()
    A_q, A_s = oracle.rotate_quantize(xb, G, Ri, Ra)
    t_rq = time.perf_counter() - t0
    Wq_h = W_q[:gn].cpu().numpy()
    Ws_h = W_s[:gn].cpu().numpy()
    t0 = time.perf_counter()
    oracle.gemm(A_q[:gm], A_s[:gm], Wq_h, Ws_h)
    t_gemm = time.perf_counter() - t0
    step_s = t_rq * (M / rows) + t_gemm * (M * N / (gm * gn))
    return {"value": round(2.0 * M * N * d / step_s / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.threads(),
            "kind": "oracle",
            "sample": f"oracle rotate_quantize on the first {rows} rows ({t_rq:.2f} s) + oracle GEMM on a "
                      f"{gm}x{gn} output corner ({t_gemm:.2f} s), each extrapolated linearly to the full "
                      f"[{M}, {N}, {d}] step",
            "rotate_quantize_GBps": round(rows * d * RQ_BYTES_PER_ELEMENT / t_rq / 1e9, 4),
            "gemm_GFLOPps": round(2.0 * gm * gn * d / t_gemm / 1e9, 3)}


def sample_board(torch, launch, seconds):
    """Median board power (W), its cap and the median shader clock (MHz) while `launch(i)` runs back to
    back for `seconds`: the amdgpu driver's hwmon power1_input / power1_cap and pp_dpm_sclk."""
    import glob
    import threading
    hw = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input")
    ck = glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")
    if not hw or not ck:
        return None
    samples, stop = [], [False]

    def read():
        try:
            watts = int(open(hw[0]).read()) / 1e6
            cur = [l for l in open(ck[0]).read().splitlines() if "*" in l]
            mhz = int(cur[0].split(":")[1].lower().replace("mhz", "").replace("*", "").strip()) if cur else None
            return watts, mhz
        except (OSError, ValueError, IndexError):
            return None

    def loop():
        while not stop[0]:
            r = read()
            if r:
                samples.append(r)
            time.sleep(0.02)
    t = threading.Thread(target=loop)
    t0 = time.perf_counter()
    i = 0
    t.start()
    while time.perf_counter() - t0 < seconds:
        for _ in range(16):
            launch(i)
            i += 1
        torch.cuda.synchronize()
    stop[0] = True
    t.join()
    samples = samples[len(samples) // 3:]            # the clock settles within the first third
    if not samples:
        return None
    med = lambda v: sorted(v)[len(v) // 2]
    try:
        cap = int(open(hw[0].replace("power1_input", "power1_cap")).read()) / 1e6
    except (OSError, ValueError):
        cap = None
    clocks = [m for _, m in samples if m]
    return {"power_w": round(med([w for w, _ in samples])), "power_cap_w": cap,
            "shader_clock_mhz": med(clocks) if clocks else None, "nominal_clock_mhz": 2400}


def copy_line(torch, dev, steps):
    src = torch.empty((1 << 30,), dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty_like(src)
    settle(torch, lambda: dst.copy_(src), 3)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    gbs = 2.0 * (1 << 30) / (ms * 1e-3) / 1e9
    return {"metric": "device copy bandwidth (runtime's kernel, context)", "value": round(gbs, 1), "unit": "GB/s",
            "config": {"workload": "1 GiB read + 1 GiB written"}, "ms": round(ms, 4),
            "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}


def settle(torch, call, warmup, seconds=0.04):
    """Untimed launches in front of a measurement: `warmup` of them, then more until `seconds` have passed.
    After a pause (input generation is one for the part's power management) the shader clock takes some
    tens of milliseconds of sustained work to reach the level it then keeps: the first few hundred launches
    of a 50 us kernel run up to 20 % slower than the ones that follow."""
    for _ in range(warmup):
        call()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(8):
            call()
        torch.cuda.synchronize()


def timed_median(torch, call, steps, groups=5):
    """Milliseconds per call: `groups` timed groups of `steps` calls each, the median group.  The lines
    that use it time windows of 0.2 to 20 ms, and one interruption of the queue inside a window that short
    (seen in about one default run of three, on a different line each time, gone on the next run) would
    otherwise decide the line."""
    per_call = []
    for _ in range(groups):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            call()
        e1.record()
        torch.cuda.synchronize()
        per_call.append(e0.elapsed_time(e1) / steps)
    return sorted(per_call)[groups // 2]


def sweep_line(tq, synth, d, steps, warmup, G=None, fmt=0, butterfly=False, M=16384, recipe=None):
    """rotate+quantise alone on X [M, d] (the memory-bound sweep); fmt 1 / 2: MXINT4 / NVFP4 output;
    butterfly: R_inter as log2 G rounds of plane rotations instead of a dense G x G matrix.  The launches
    cycle over copies of X of at least 600 MB in all (at least three), so that no launch finds its input
    in the 256 MB Infinity Cache."""
    import torch
    dev = "cuda:0"
    G = G or synth.default_G(d)
    r = dict(nu=3.0, outliers=round(0.005 * d), outlier_scale=50.0, seed=synth.SEED_BASE + 5)
    r.update(recipe or {})
    x = synth.activations(M, d, device=dev, **r)
    n_copies = max(3, int(600e6 // (x.numel() * 2)) + 1)
    xs = [x] + [x.clone() for _ in range(n_copies - 1)]
    Ri, Ra = synth.rotations(G)
    if butterfly:
        import numpy as np
        T = np.random.default_rng(synth.SEED_BASE + 6).uniform(-1, 1, (G.bit_length() - 1, G // 2)).astype(np.float32)
        rot = tq.ButterflyRotation(d, G, T, Ra)
    else:
        rot = tq.Rotation(d, G, Ri, Ra)
    codes = torch.empty((M, d // 2), dtype=torch.uint8, device=dev)
    scales = torch.empty((M, d // (16 if fmt == 2 else 32)), dtype=torch.uint8, device=dev)
    gs = 0.01                                          # NVFP4's tensor-wide scale (unused otherwise)
    turn = [0]

    def call():
        xi = xs[turn[0] % n_copies]
        turn[0] += 1
        if fmt == 0:
            tq.torq_rotate_quantize(rot, xi, codes=codes, scales=scales)
        else:
            tq.torq_rotate_quantize_fmt(rot, xi, fmt, gs, codes=codes, scales=scales)
    settle(torch, call, warmup)
    ms = timed_median(torch, call, steps)
    bytes_per_element = 2.0 + 0.5 + (1.0 / 16 if fmt == 2 else 1.0 / 32)
    gbs = M * d * bytes_per_element / (ms * 1e-3) / 1e9
    rot.close()
    name = ("", " -> MXINT4", " -> NVFP4")[fmt] + (", butterfly R_inter" if butterfly else "")
    mfma_flop = 2 * 64 if butterfly else 2 * 2 * G + 3 * 64      # per element: bf16 passes of the contractions
    return {"metric": "torq_rotate_quantize bandwidth", "value": round(gbs, 1), "unit": "GB/s",
            "config": {"workload": f"sweep: X bf16 [{M}, {d}], G={G}{name}", "input_copies": n_copies}, "ms": round(ms, 4),
            "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
            "mfma_bf16_tflops": round(M * d * mfma_flop / (ms * 1e-3) / 1e12, 1)}


def config_lines(tq, synth, torch, steps, warmup, headline):
    """The other shapes of the benchmark configurations, one compact entry each: the rotate+quantise kernel
    against the HBM peak, the GEMM against the fp4 MFMA peak (prefill) and torq_linear per call with the
    rate at which the weights stream (decode).  `config` is the number of the configuration in the task's
    list: 1 tiny, 2 LLaMA3-8B, 3 Qwen3-32B, 4 LLaMA3-70B, 5 the rotate+quantise bandwidth sweep."""
    out = []

    def rq(cfg, M, d, recipe, G=None, butterfly=False):
        r = sweep_line(tq, synth, d, steps, warmup, M=M, recipe=recipe, G=G, butterfly=butterfly)
        G_ = G or synth.default_G(d)
        out.append({"config": cfg, "kernel": "torq_rotate_quantize" + (" (butterfly R_inter)" if butterfly else ""),
                    "shape": f"X[{M},{d}] G={G_}", "us": round(r["ms"] * 1e3, 2), "value": r["value"], "unit": "GB/s",
                    "bound": "hbm", "frac": r["frac_hbm_peak"], "input_copies": r["config"]["input_copies"]})

    def gemm(cfg, M, N, d):
        r = gemm_line(tq, M, N, d, steps, warmup)
        out.append({"config": cfg, "kernel": "mxfp4_gemm (" + r["config"]["gemm_kernel"] + ")", "shape": f"[{M},{N},{d}]",
                    "us": round(r["ms"] * 1e3, 2), "value": r["value"], "unit": "TFLOP/s", "bound": "mfma",
                    "frac": r["frac_fp4_peak"], "weight_copies": r["config"]["weight_copies"]})

    def decode(cfg, M, N, d):
        r = decode_line(tq, synth, M, N, d, single_launch=False)
        out.append({"config": cfg, "kernel": "torq_linear (" + r["config"]["gemm_kernel"] + ")", "shape": f"X[{M},{d}] -> {N}",
                    "us": r["value"], "value": r["weight_stream_GBps"], "unit": "GB/s of weights", "bound": "hbm",
                    "frac": r["frac_hbm_peak"]})

    t3 = dict(nu=3.0, outlier_scale=50.0)
    # 5: the bandwidth sweep
    for d in (4096, 8192, 14336, 28672):
        rq(5, 16384, d, dict(t3, outliers=round(0.005 * d)))
    # 4: LLaMA3-70B; up / gate is the headline step above, here the down projection's two kernels
    out.append({"config": 4, "kernel": "torq_rotate_quantize", "shape": "X[8192,8192] G=128", "us": round(headline["roofline_rotate_quant"]["avg_kernel_ms"] * 1e3, 2),
                "value": headline["roofline_rotate_quant"]["achieved"], "unit": "GB/s", "bound": "hbm",
                "frac": headline["roofline_rotate_quant"]["frac"], "input_copies": 5})
    out.append({"config": 4, "kernel": "mxfp4_gemm (tiled 256x256)", "shape": "[8192,28672,8192]", "us": round(headline["roofline"]["avg_kernel_ms"] * 1e3, 2),
                "value": headline["roofline"]["achieved"], "unit": "TFLOP/s", "bound": "mfma", "frac": headline["roofline"]["frac"]})
    rq(4, 8192, 28672, dict(nu=2.5, outliers=round(0.01 * 28672), outlier_scale=100.0))
    gemm(4, 8192, 8192, 28672)
    # 3: Qwen3-32B (G = 80), per-token log-normal scale
    for d in (5120, 25600):
        rq(3, 4096, d, dict(t3, outliers=round(0.005 * d), token_lognormal=True))
    for N, d in ((25600, 5120), (5120, 25600), (8192, 5120), (5120, 5120), (1024, 5120)):
        gemm(3, 4096, N, d)
    # 2: LLaMA3-8B, prefill (M = 2048) and decode (M = 1, 16)
    for d in (4096, 14336):
        rq(2, 2048, d, dict(t3, outliers=round(0.005 * d)))
    for N, d in ((14336, 4096), (4096, 4096), (1024, 4096), (4096, 14336)):
        gemm(2, 2048, N, d)
    for M in (1, 16):
        for N, d in ((14336, 4096), (4096, 4096), (1024, 4096), (4096, 14336)):
            decode(2, M, N, d)
    # 1: the tiny layer
    decode(1, 64, 1024, 4096)
    # the calibrated alternative of Section 5.1 at the headline width: R_inter as a butterfly
    rq(4, 8192, 8192, dict(nu=2.5, outliers=82, outlier_scale=100.0), G=128, butterfly=True)
    return out


def ablation_lines(tq, torch, rot, x, codes, scales, W_q, W_s, out, steps):
    """Launch times of the two headline kernels with parts of their work left out (diagnostic builds of the
    same kernels; their outputs are meaningless and go to scratch copies).  Both kernels run at the board's
    power limit, so the cost of a part is the time the launch shortens by without it."""
    M, d = x.shape
    xs = [x.clone() for _ in range(5)]
    c2, s2, o2 = torch.empty_like(codes), torch.empty_like(scales), torch.empty_like(out)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(call, reps):
        turn = [0]

        def f():
            call(turn[0])
            turn[0] += 1
        settle(torch, f, 3)
        e0.record()
        for _ in range(reps):
            f()
        e1.record()
        torch.cuda.synchronize()
        return round(e0.elapsed_time(e1) * 1e3 / reps, 2)

    gemm_names = {0: "product kernel", 1: "no buffer loads in the k loop", 3: "... and no LDS stores",
                  7: "... and no fragment reads (MFMAs + barrier)", 15: "... and no barrier (MFMAs only)",
                  4: "no fragment reads only"}
    rot_names = {0: "product kernel (704 MFMA flop per element)", 6: "no vector-ALU split, no step-4 arithmetic",
                 2: "no vector-ALU split only", 4: "no step-4 arithmetic only", 8: "one R_intra pass (576 flop)",
                 1: "no R_inter low pass (448 flop)", 9: "high parts only (320 flop)", 15: "high parts only, no vector ALU"}
    res = {"metric": "launch time with parts of the kernel's work left out", "unit": "us", "gemm": [], "rotate_quantize": []}
    for rnd in range(2):                               # twice: the second pass is the one on a warm board
        g, r = [], []
        for skip, name in gemm_names.items():
            g.append({"skip": skip, "what": name,
                      "us": timed(lambda i: tq.torq_diag_gemm_ablation(codes, scales, W_q, W_s, o2, skip), steps)})
        for skip, name in rot_names.items():
            r.append({"skip": skip, "what": name,
                      "us": timed(lambda i: tq.torq_diag_rotate_ablation(rot, xs[i % 5], c2, s2, skip), 4 * steps)})
        res["gemm"], res["rotate_quantize"] = g, r
    return res


PLAN_SWEEP_GRIDS = {   # (d, M, N)
    "fit": ((4096, 8192, 14336, 28672), (96, 128, 256, 512, 1024, 2048), (1024, 4096, 8192, 14336, 28672)),
    "check": ((5120, 7168, 12288, 25600), (80, 192, 384, 768, 1536), (2048, 5120, 6144, 11008, 25600)),
    "decode": ((4096, 8192, 14336, 28672), (8, 16, 32, 48, 64), (1024, 4096, 14336, 28672)),
}


def plan_sweep(tq, torch, grid):
    """Every plan of the tiled GEMM kernel on every shape of a grid (up to one round of 256x256 tiles), timed as
    HIP-graph replays over weight copies of at least 600 MB in all, so that weights come from HBM and activations
    from the caches, as in a model.  One JSON line per shape: the planner's choice with and without a workspace and
    its time, then [tile, k_pieces, deep, us] for every candidate (tile 0 ... 3 = 256x256, 256x128, 128x128, 128x64)."""
    dev = "cuda:0"
    tile_m, tile_n = (256, 256, 128, 128), (256, 128, 128, 64)

    def graph_us(fn, n):
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for _ in range(2):
                fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(n):
                fn()
        settle(torch, graph.replay, 1, seconds=0.01)
        return round(timed_median(torch, graph.replay, 3, groups=3) * 1e3 / n, 2)

    ds, Ms, Ns = PLAN_SWEEP_GRIDS[grid]
    for d in ds:
        for M in Ms:
            for N in Ns:
                if ((M + 255) // 256) * ((N + 255) // 256) > 256 or N * d > 28672 * 8192:
                    continue
                gen = torch.Generator(device=dev)
                gen.manual_seed(M + N + d)
                n_copies = max(3, int(600e6 // (N * d * 0.53125)) + 1)
                A_q = torch.randint(0, 256, (M, d // 2), dtype=torch.uint8, device=dev, generator=gen)
                A_s = torch.randint(118, 136, (M, d // 32), dtype=torch.uint8, device=dev, generator=gen)
                W_q = [torch.randint(0, 256, (N, d // 2), dtype=torch.uint8, device=dev, generator=gen)]
                W_s = [torch.randint(110, 126, (N, d // 32), dtype=torch.uint8, device=dev, generator=gen)]
                W_q += [W_q[0].clone() for _ in range(n_copies - 1)]
                W_s += [W_s[0].clone() for _ in range(n_copies - 1)]
                out = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
                need = tq.mxfp4_gemm_workspace_bytes(M, N, d)
                ws = torch.empty((16 * M * N * 4,), dtype=torch.uint8, device=dev)
                calls, turn = max(12, n_copies), [0]

                def cycling(f):
                    def g():
                        i = turn[0] % n_copies
                        turn[0] += 1
                        f(W_q[i], W_s[i])
                    return g
                rec = {"metric": "mxfp4_gemm plans", "unit": "us per launch", "shape": [M, N, d], "weight_copies": n_copies,
                       "planner_with_workspace": list(tq.mxfp4_gemm_plan(M, N, d, need)),
                       "planner_without": list(tq.mxfp4_gemm_plan(M, N, d, 0))}
                rec["us_with_workspace"] = graph_us(cycling(lambda wq, wsc: tq.mxfp4_gemm_ws(
                    A_q, A_s, wq, wsc, out=out, workspace=ws[:max(need, 16)])), calls)
                rec["us_without"] = graph_us(cycling(lambda wq, wsc: tq.mxfp4_gemm(A_q, A_s, wq, wsc, out=out)), calls)
                cands = []
                for tile in range(4):
                    tiles = ((M + tile_m[tile] - 1) // tile_m[tile]) * ((N + tile_n[tile] - 1) // tile_n[tile])
                    if tiles > 1024:
                        continue
                    for pieces in (1, 2, 4, 5, 7, 8, 10, 14, 16):
                        if pieces > 1 and ((d // 512) % pieces or tile == 0 or tiles * pieces > 1024 or N % 8):
                            continue
                        for deep in ((False, True) if (tile >= 2 and pieces == 1) else (False,)):
                            us = graph_us(cycling(lambda wq, wsc: tq.torq_diag_gemm_plan(
                                A_q, A_s, wq, wsc, tile, pieces, deep, out=out, workspace=ws)), calls)
                            cands.append([tile, pieces, int(deep), us])
                rec["candidates"] = cands
                rec["best"] = min(cands, key=lambda c: c[3])
                print(json.dumps(rec), flush=True)
                del A_q, A_s, W_q, W_s, out, ws


def _graph_us(torch, fn, n, groups=5):
    """Microseconds per call of fn from replays of a HIP graph of n calls (no launch overhead of the host)."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(2):
            fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for _ in range(n):
            fn()
    settle(torch, graph.replay, 1, seconds=0.02)
    return round(timed_median(torch, graph.replay, 3, groups=groups) * 1e3 / n, 2)


def _weight_copies(torch, N, d, seed, dev="cuda:0"):
    """Copies of one random packed weight matrix, at least 600 MB in all (at least three)."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    n_copies = max(3, int(600e6 // (N * d * 0.53125)) + 1)
    W_q = [torch.randint(0, 256, (N, d // 2), dtype=torch.uint8, device=dev, generator=gen)]
    W_s = [torch.randint(110, 126, (N, d // 32), dtype=torch.uint8, device=dev, generator=gen)]
    W_q += [W_q[0].clone() for _ in range(n_copies - 1)]
    W_s += [W_s[0].clone() for _ in range(n_copies - 1)]
    return W_q, W_s, n_copies


def rounds_sweep(tq, torch):
    """Beyond one round of 256x256 tiles: mxfp4_gemm_ws as planned (whole rounds first where the planner takes two
    launches, the persistent form where it pays) against ONE launch of each tile shape, plain (torq_diag_gemm_plan)
    and persistent (torq_diag_gemm_persistent); launches cycle over weight copies of at least 600 MB in all."""
    dev = "cuda:0"
    for d in (4096, 8192):
        for M in (2048, 4096, 8192):
            for N in (4096, 5120, 8192, 11008, 14336):
                tiles = ((M + 255) // 256) * ((N + 255) // 256)
                if tiles <= 256 or tiles > 2048:
                    continue
                gen = torch.Generator(device=dev)
                gen.manual_seed(M + N + d)
                A_q = torch.randint(0, 256, (M, d // 2), dtype=torch.uint8, device=dev, generator=gen)
                A_s = torch.randint(118, 136, (M, d // 32), dtype=torch.uint8, device=dev, generator=gen)
                W_q, W_s, n_copies = _weight_copies(torch, N, d, M + N + d + 1)
                out = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
                ws = torch.empty((max(tq.mxfp4_gemm_workspace_bytes(M, N, d), 16),), dtype=torch.uint8, device=dev)
                turn = [0]

                def form(kind, tile=0):
                    def f():
                        i = turn[0] % n_copies
                        turn[0] += 1
                        if kind == "planned":
                            tq.mxfp4_gemm_ws(A_q, A_s, W_q[i], W_s[i], out=out, workspace=ws)
                        elif kind == "plain":
                            tq.torq_diag_gemm_plan(A_q, A_s, W_q[i], W_s[i], tile, 1, False, out=out)
                        else:
                            tq.torq_diag_gemm_persistent(A_q, A_s, W_q[i], W_s[i], tile=tile, workgroups=256, out=out)
                    return f
                rec = {"metric": "mxfp4_gemm beyond one round", "unit": "us per launch", "shape": [M, N, d],
                       "tiles_256x256": tiles, "weight_copies": n_copies,
                       "planned": gemm_kernel_name(tq, M, N, d, ws.numel())}
                for name, f in (("us_planned", form("planned")), ("us_256x256", form("plain", 0)),
                                ("us_256x128", form("plain", 1)), ("us_128x128", form("plain", 2)),
                                ("us_256x256_persistent", form("persistent", 0)),
                                ("us_256x128_persistent", form("persistent", 1))):
                    settle(torch, f, 3)
                    rec[name] = round(timed_median(torch, f, 20) * 1e3, 1)
                print(json.dumps(rec), flush=True)
                del W_q, W_s


def decode_forms(tq, synth, torch):
    """torq_linear with one to four token-groups as the library routes it, as two launches and as the one launch
    whose workgroups rotate the rows themselves; HIP-graph replays over weight copies of at least 600 MB in all."""
    dev = "cuda:0"
    shapes = [(M, N, 4096) for M in (1, 2, 4) for N in (1024, 2048, 4096, 6144, 8192, 11008, 14336)]
    shapes += [(M, N, 8192) for M in (1, 2) for N in (1024, 2048, 4096, 8192)]
    shapes += [(1, N, 14336) for N in (1024, 2048, 4096)]
    for M, N, d in shapes:
        G = synth.default_G(d)
        x = synth.activations(M, d, nu=3.0, outliers=round(0.005 * d), outlier_scale=50.0, seed=synth.SEED_BASE + 7,
                              device=dev)
        Ri, Ra = synth.rotations(G)
        rot = tq.Rotation(d, G, Ri, Ra)
        W_q, W_s, n_copies = _weight_copies(torch, N, d, N + d)
        out = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        ws = torch.empty((tq.torq_linear_workspace_bytes_n(M, N, d),), dtype=torch.uint8, device=dev)
        codes = torch.empty((M, d // 2), dtype=torch.uint8, device=dev)
        scales = torch.empty((M, d // 32), dtype=torch.uint8, device=dev)
        gws = torch.empty((max(tq.mxfp4_gemm_workspace_bytes(M, N, d), 16),), dtype=torch.uint8, device=dev)
        turn = [0]

        def routed():
            i = turn[0] % n_copies
            turn[0] += 1
            tq.torq_linear(rot, x, W_q[i], W_s[i], out=out, workspace=ws)

        def two():
            i = turn[0] % n_copies
            turn[0] += 1
            tq.torq_rotate_quantize(rot, x, codes=codes, scales=scales)
            tq.mxfp4_gemm_ws(codes, scales, W_q[i], W_s[i], out=out, workspace=gws)

        def one():
            i = turn[0] % n_copies
            turn[0] += 1
            tq.torq_linear_single_launch(rot, x, W_q[i], W_s[i], out=out, workspace=ws)
        calls = max(24, n_copies)
        print(json.dumps({"metric": "torq_linear, decode forms", "unit": "us per call", "shape": [M, N, d], "G": G,
                          "token_groups": M * (d // 32 // G), "weights_MB": round(N * d * 0.53125 / 1e6, 1),
                          "weight_copies": n_copies, "us_torq_linear": _graph_us(torch, routed, calls),
                          "us_two_launches": _graph_us(torch, two, calls),
                          "us_one_launch": _graph_us(torch, one, calls)}), flush=True)
        rot.close()
        del W_q, W_s


def gemm_kernel_name(tq, M, N, d, workspace_bytes):
    """Which kernel(s) mxfp4_gemm_ws runs a product on, for the lines' labels."""
    def one(n):
        streaming, tile_m, tile_n, pieces = tq.mxfp4_gemm_plan(M, n, d, workspace_bytes)
        return "weight-streaming" if streaming else f"tiled {tile_m}x{tile_n}" + (f", k cut in {pieces}" if pieces > 1 else "")
    main = tq.mxfp4_gemm_main_columns(M, N, d, workspace_bytes)
    if main < N:
        return f"{one(N)} on {main} columns (whole rounds), then {one(N - main)} on {N - main}"
    return one(N)


def gemm_line(tq, M, N, d, steps, warmup):
    """mxfp4_gemm alone on random codes and scale bytes of one layer shape (with the workspace the planner asks
    for).  The launches cycle over weight copies of at least 600 MB in all (at least three), so that the weights
    come from HBM, as a model's do; the activations stay where the kernel before left them."""
    import torch
    dev = "cuda:0"
    gen = torch.Generator(device=dev)
    gen.manual_seed(M + N + d)
    n_copies = max(3, int(600e6 // (N * d * 0.53125)) + 1)
    A_q = torch.randint(0, 256, (M, d // 2), dtype=torch.uint8, device=dev, generator=gen)
    A_s = torch.randint(118, 136, (M, d // 32), dtype=torch.uint8, device=dev, generator=gen)
    W_q = [torch.randint(0, 256, (N, d // 2), dtype=torch.uint8, device=dev, generator=gen)]
    W_s = [torch.randint(110, 126, (N, d // 32), dtype=torch.uint8, device=dev, generator=gen)]
    W_q += [W_q[0].clone() for _ in range(n_copies - 1)]
    W_s += [W_s[0].clone() for _ in range(n_copies - 1)]
    out = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    ws = torch.empty((max(tq.mxfp4_gemm_workspace_bytes(M, N, d), 16),), dtype=torch.uint8, device=dev)
    turn = [0]

    def call():
        i = turn[0] % n_copies
        turn[0] += 1
        tq.mxfp4_gemm_ws(A_q, A_s, W_q[i], W_s[i], out=out, workspace=ws)
    settle(torch, call, warmup)
    ms = timed_median(torch, call, steps)
    tf = 2.0 * M * N * d / (ms * 1e-3) / 1e12
    kernel = gemm_kernel_name(tq, M, N, d, ws.numel())
    return {"metric": "mxfp4_gemm", "value": round(tf, 1), "unit": "TFLOP/s",
            "config": {"workload": f"A [{M}, {d}] x W [{N}, {d}] packed MXFP4 -> bf16 [{M}, {N}]", "gemm_kernel": kernel,
                       "weight_copies": n_copies},
            "ms": round(ms, 4), "frac_fp4_peak": round(tf / 10100.0, 4)}


def gram_line(tq, x, G, steps, warmup):
    """torq_block_gram on the step's activations: 2 bytes per element read once."""
    import torch
    M, d = x.shape
    xs = [x, x.clone(), x.clone()]                   # 3 x 134 MB: more than the Infinity Cache holds
    Sigma = torch.empty((G, G), dtype=torch.float64, device=x.device)
    ws = torch.empty((tq.torq_block_gram_workspace_bytes(G),), dtype=torch.uint8, device=x.device)
    settle(torch, lambda: tq.torq_block_gram(xs[0], G, Sigma=Sigma, workspace=ws), warmup)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        tq.torq_block_gram(xs[i % 3], G, Sigma=Sigma, workspace=ws)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    gbs = M * d * 2.0 / (ms * 1e-3) / 1e9
    # the per-position matrices Sigma_k: 32 passes of the same kernel over x
    Sp = torch.empty((32, G, G), dtype=torch.float64, device=x.device)
    tq.torq_block_gram_positions(xs[0], G, Sigma_pos=Sp, workspace=ws)
    e0.record()
    for i in range(3):
        tq.torq_block_gram_positions(xs[i % 3], G, Sigma_pos=Sp, workspace=ws)
    e1.record()
    torch.cuda.synchronize()
    pos_ms = e0.elapsed_time(e1) / 3
    return {"metric": "torq_block_gram bandwidth", "value": round(gbs, 1), "unit": "GB/s",
            "config": {"workload": f"calibration statistic: X bf16 [{M}, {d}], G={G}"}, "ms": round(ms, 4),
            "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4), "positions_ms": round(pos_ms, 3)}


def hist_line(tq, codes, d, steps, warmup):
    """torq_code_histogram on packed codes: half a byte per element read once."""
    import torch
    M = codes.shape[0]
    copies = max(3, int(600e6 // codes.numel()) + 1)   # rotate through more than the Infinity Cache holds
    cs = [codes] + [codes.clone() for _ in range(copies - 1)]
    counts = torch.empty((32, 8), dtype=torch.int64, device=codes.device)
    ws = torch.empty((tq.torq_code_histogram_workspace_bytes(),), dtype=torch.uint8, device=codes.device)
    settle(torch, lambda: tq.torq_code_histogram(cs[0], d, counts=counts, workspace=ws), warmup)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        tq.torq_code_histogram(cs[i % copies], d, counts=counts, workspace=ws)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    gbs = M * d * 0.5 / (ms * 1e-3) / 1e9
    return {"metric": "torq_code_histogram bandwidth", "value": round(gbs, 1), "unit": "GB/s",
            "config": {"workload": f"calibration statistic: packed codes [{M}, {d}/2]"}, "ms": round(ms, 4),
            "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}


def decode_line(tq, synth, M, N, d, single_launch=True):
    """torq_linear (rotate + quantise + GEMM) on M activation rows: microseconds per call and the rate at
    which the packed weights stream through.  The calls cycle over weight copies of at least 600 MB in all (at
    least six), so that the 256 MB Infinity Cache holds none of them: weights come from HBM, as in a model."""
    import torch
    dev = "cuda:0"
    G = synth.default_G(d)
    x = synth.activations(M, d, nu=3.0, outliers=round(0.005 * d), outlier_scale=50.0, seed=synth.SEED_BASE + 7,
                          device=dev)
    Ri, Ra = synth.rotations(G)
    rot = tq.Rotation(d, G, Ri, Ra)
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.SEED_BASE + N + d)
    n_copies = max(6, int(600e6 // (N * d * 0.53125)) + 1)
    W_q = [torch.randint(0, 256, (N, d // 2), dtype=torch.uint8, device=dev, generator=gen) for _ in range(n_copies)]
    W_s = [torch.randint(110, 126, (N, d // 32), dtype=torch.uint8, device=dev, generator=gen) for _ in range(n_copies)]
    out = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    ws = torch.empty((tq.torq_linear_workspace_bytes_n(M, N, d),), dtype=torch.uint8, device=dev)
    calls = max(24, n_copies)

    def replayed(fn):
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for i in range(n_copies):
                fn(rot, x, W_q[i], W_s[i], out=out, workspace=ws)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for i in range(calls):
                fn(rot, x, W_q[i % n_copies], W_s[i % n_copies], out=out, workspace=ws)
        settle(torch, graph.replay, 1)
        return timed_median(torch, graph.replay, 4) * 1e3 / calls

    us = replayed(tq.torq_linear)
    # the one-launch form of the same layer, where it applies (G = 128, at most 64 rows)
    local = G in (112, 128) and M * (d // 32 // G) <= 4
    us_single = round(replayed(tq.torq_linear_single_launch), 2) if (single_launch and ((G == 128 and M <= 64) or local)) else None
    wbytes = N * d * 0.53125
    rot.close()
    kernel = gemm_kernel_name(tq, M, N, d, tq.mxfp4_gemm_workspace_bytes(M, N, d))
    return {"metric": "torq_linear, decode", "value": round(us, 2), "unit": "us per call", "higher_is_better": False,
            "config": {"workload": f"decode: X bf16 [{M}, {d}], G={G}, W [{N}, {d}] packed MXFP4 ({wbytes / 1e6:.1f} MB)",
                       "gemm_kernel": kernel},
            "single_launch_us": us_single, "weight_stream_GBps": round(wbytes / us / 1e3, 1), "frac_hbm_peak": round(wbytes / us / 1e3 / HBM_PEAK_GBS, 4)}


if __name__ == "__main__":
    main()
