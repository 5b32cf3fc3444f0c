#!/usr/bin/env python3
"""Throughput of the reassembled W4A4 linear layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]

A "step" is one pass of the whole hot path -- qllm_reassembled_linear: fused norm + channel
disassembly + channel assembly + per-token quantization, then the matrix-core GEMM on the codes with its
dequantising epilogue -- over one batch of synthetic activations that is already resident in HBM.
The default workload is the LLaMA-2-70B down-projection shape (N=2048, C=28672, O=8192, W4A4).
With 4-bit codes on both sides and more than 32 tokens the GEMM runs on the FP6 matrix cores (the codes
are exact FP6 numbers, the fp32 sums exact integers / 64: same accumulators bit for bit, `config.gemm_path`);
--int8 keeps it on the int8 matrix cores.

Prints one JSON line.  `value` is 2*N*K*O integer operations per second of the whole step;
`roofline` prices the dominant kernel (the GEMM) against the dense matrix-core peak of the operations it
issues (FP6 10.1 POP/s, int8 5.0 POP/s; against HBM bandwidth for decode-sized batches, where the weights
stream once), and `roofline_fused` the fused kernel
against HBM bandwidth; both use the kernel's own average duration, taken with HIP events on the launch
stream in a second, instrumented pass: the same K launches of that kernel back to back with one event pair
around them (`avg_launch_us`; an event pair around a single launch also spans the few microseconds before the
kernel starts, which a kernel trace does not count: those readings are kept as `single_launch_event_us`,
mean, median and minimum).
Before anything is timed the GPU runs the step for at least 100 ms, whatever --warmup says (the clocks
settle over the first tens of milliseconds).  `cpu_baseline` times the CPU oracle, as it stands, on a
bounded sample of the same workload, from its own calibration and weights; `parity_checked` compares
what the TIMED launches wrote with that oracle run.
`traffic` (HBM bytes per launch) cannot be measured from inside the process: it is read from the
committed counter summary profiles/<workload>_hbm_traffic.md if that exists, else null.
--calibration-copy adds one plain device-to-device copy of 256 MiB before the timed region, so that a
counter run of this script also holds the reading for a kernel whose traffic is known.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
INT8_PEAK_TOPS = 5000.0      # MI355X dense int8 matrix-core peak, published
FP6_PEAK_TOPS = 10100.0      # MI355X dense FP6 / FP4 matrix-core peak, published
MIN_WARMUP_MS = 100.0        # GPU time spent on the step before anything is timed, whatever --warmup says
N_ROTATE = 4                 # distinct activation / output buffers cycled through, so that no step
#                              finds its inputs in the 256 MB last-level cache


def read_traffic(workload):
    """HBM bytes per launch, by kernel, from the committed counter summary of this workload: table rows
    `| kernel | FETCH_SIZE KiB | WRITE_SIZE KiB | scale | HBM bytes per launch |`."""
    path = os.path.join(ROOT, "profiles", workload + "_hbm_traffic.md")
    out = {}
    if os.path.exists(path):
        for line in open(path):
            cells = [c.strip().strip("`") for c in line.strip().strip("|").split("|")]
            if len(cells) == 5 and cells[4].replace(".", "", 1).isdigit():
                out[cells[0].split("<")[0].replace("_kernel", "").replace("_big", "").replace("_w4a4", "")] = float(cells[4])
    return out


def bench_swiglu(args, w, dev):
    """The producer of a down projection's input: x = silu(gate) * up at the workload's N x C, bfloat16.
    A step = one qllm_swiglu call; 6 bytes per element against HBM."""
    import numpy as np
    import torch

    from paper_2310_08041_amd import binding as b

    g = torch.Generator(device=dev).manual_seed(w.seed)
    sets = 3                                                                       # 3 x 352 MB at the 70B shape: past the last-level cache
    gate = [(torch.randn((w.N, w.C), device=dev, generator=g) * 3).to(torch.bfloat16) for _ in range(sets)]
    up = [torch.randn((w.N, w.C), device=dev, generator=g).to(torch.bfloat16) for _ in range(sets)]
    x = [torch.empty((w.N, w.C), dtype=torch.bfloat16, device=dev) for _ in range(sets)]
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    warm_ms, warm_steps = 0.0, 0
    while warm_steps < args.warmup or warm_ms < MIN_WARMUP_MS:
        ev[0].record()
        for i in range(16):
            b.qllm_swiglu(gate[i % sets], up[i % sets], x[i % sets])
        ev[1].record()
        torch.cuda.synchronize()
        warm_steps += 16
        warm_ms += ev[0].elapsed_time(ev[1])
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(args.steps):
        b.qllm_swiglu(gate[i % sets], up[i % sets], x[i % sets])
    ev[1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    t_kernel = ev[0].elapsed_time(ev[1]) * 1e-3 / args.steps
    nbytes = 6.0 * w.N * w.C
    result = {
        "metric": "silu(gate)*up producer of the reassembled linear layer's input, GB/s", "value": nbytes / (wall / args.steps) / 1e9,
        "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 (fixed sequence of fp32 operations, bf16 in and out)", "data": "synthetic",
        "config": {"workload": w.name + " (producer of its input)", "N": w.N, "C": w.C, "warmup_done": {"steps": warm_steps, "gpu_ms": warm_ms}},
        "roofline": {"kernel": "swiglu_kernel", "bound": "hbm", "achieved": nbytes / t_kernel / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": nbytes / t_kernel / 1e9 / HBM_PEAK_GBS, "avg_launch_us": t_kernel * 1e6, "algorithmic_bytes": nbytes,
                     "traffic": None},
    }
    if not args.no_cpu_baseline:
        from oracle import api as oracle
        rows = np.sort(np.random.default_rng(w.seed).choice(w.N, min(256, w.N), replace=False))
        idx = torch.from_numpy(rows).to(dev)
        bits = lambda t: t[idx].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        gb, ub = bits(gate[(args.steps - 1) % sets]), bits(up[(args.steps - 1) % sets])
        t1 = time.perf_counter()
        ref = oracle.swiglu(gb, ub)
        cpu_s = time.perf_counter() - t1
        result["cpu_baseline"] = {"value": 6.0 * rows.size * w.C / cpu_s / 1e9, "unit": "GB/s", "cores": oracle.max_threads(), "kind": "oracle",
                                  "sample": f"{rows.size} sampled rows of {w.N}, {cpu_s:.1f} s"}
        result["parity_checked"] = {"rows": int(rows.size), "bit_exact": bool(np.array_equal(bits(x[(args.steps - 1) % sets]), ref))}
        result["parity_checked"]["ok"] = result["parity_checked"]["bit_exact"]
    print(json.dumps(result))
    return 0 if result.get("parity_checked", {"ok": True})["ok"] else 1


def bench_matching(args, w, norm, dev):
    """The step before the path: Appendix A steps 1-2 with the distance of Eq. (5) for the workload's
    layer, 256 calibration tokens.  A step = one qllm_match_nearest call (norms + nearest-member search)."""
    import numpy as np
    import torch

    from paper_2310_08041_amd import binding as b
    from paper_2310_08041_amd import calibrate, workloads as wl

    n_match = min(256, w.N)
    x_host, _, _ = wl.draw_activations(w)
    gamma_h, beta_h = wl.draw_norm_params(w)
    x0 = (torch.from_numpy(x_host.view(np.int16)).to(dev).view(torch.bfloat16) if x_host.dtype == np.uint16
          else torch.from_numpy(x_host).to(dev))
    gamma = torch.from_numpy(gamma_h).to(dev)
    beta = None if beta_h is None else torch.from_numpy(beta_h).to(dev)
    absmax = torch.zeros(w.C, dtype=torch.float32, device=dev)
    y = torch.empty((n_match, w.C), dtype=torch.float32, device=dev)
    b.qllm_norm_channel_absmax(x0, norm, gamma, beta, w.eps, absmax, y)
    m = absmax.cpu().numpy()
    theta = calibrate.choose_theta(m, w.theta_rule)
    T = b.qllm_build_map_host(m, theta, [], [], with_plan=False)["num_split"]
    W_host = wl.draw_weight(w)
    W = torch.from_numpy(W_host).to(dev)
    sets = b.qllm_matching_sets_host(T)
    chan_a, chan_b = torch.from_numpy(sets["chan_a"]).to(dev), torch.from_numpy(sets["chan_b"]).to(dev)
    nA, nB = chan_a.numel(), chan_b.numel()
    best_j = torch.empty(nA, dtype=torch.int32, device=dev)
    best_d = torch.empty(nA, dtype=torch.float64, device=dev)
    ws = torch.empty(b.qllm_match_workspace_bytes(nA, nB), dtype=torch.uint8, device=dev)
    if args.calibration_copy:      # a device copy of known size, for scaling the HBM counters of a profiler run
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    steps, warmup = min(args.steps, 20), min(args.warmup, 3)
    for _ in range(warmup):
        b.qllm_match_nearest(y, W, chan_a, chan_b, best_j, best_d, ws)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    t_start = time.perf_counter()
    ev[0].record()
    for _ in range(steps):
        b.qllm_match_nearest(y, W, chan_a, chan_b, best_j, best_d, ws)
    ev[1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    t_kernel = ev[0].elapsed_time(ev[1]) * 1e-3 / steps
    flops = 2.0 * nA * nB * (n_match + w.O)             # two Gram matrices, one multiply-add per pair and index
    result = {
        "metric": "channel matching (Eq. 5, Appendix A steps 1-2): fp64 TFLOP/s of the two Gram contractions",
        "value": flops / (wall / steps) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": wall * 1e3 / steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64 (fp64 matrix cores; fp32 inputs widened exactly)", "data": "synthetic",
        "config": {"workload": w.name + " / offline matching", "C": w.C, "O": w.O, "calibration_tokens": n_match,
                   "set_A": nA, "set_B": nB, "split_channels": int((T > 1).sum()), "pairs": nA * nB},
        "roofline": {"kernel": "match_nearest_kernel (+ match_norms_kernel)", "bound": "mfma", "achieved": flops / t_kernel / 1e12,
                     "peak": 78.6, "unit": "TFLOP/s", "frac": flops / t_kernel / 1e12 / 78.6,
                     "avg_launch_us": t_kernel * 1e6, "traffic": read_traffic(w.name + "_match").get("match_nearest")},
    }
    if not args.no_cpu_baseline:
        from oracle import calibrate as ocal
        from oracle import api as oracle
        rows = np.arange(0, nA, max(1, nA // 8))[:8]
        y_h = y.cpu().numpy()
        t0 = time.perf_counter()
        ref_j, ref_d, _, _ = ocal.nearest_by_eq5(y_h, W_host, T, n_match_tokens=n_match, rows=rows)
        dt = time.perf_counter() - t0
        got_j = best_j.cpu().numpy()[rows]
        same = int((got_j == ref_j).sum())
        result["cpu_baseline"] = {"value": 2.0 * rows.size * nB * (n_match + w.O) / dt / 1e12, "unit": "TFLOP/s",
                                  "cores": oracle.max_threads(), "kind": "oracle",
                                  "sample": f"{rows.size} of {nA} members of set A against all {nB} members of set B, {dt:.1f} s "
                                            f"(setup included); nearest member agrees for {same} of {rows.size}"}
    print(json.dumps(result))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100)   # ~50 ms: the clocks settle over the first tens of ms
    ap.add_argument("--workload", default="llama70b_down")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--int8", action="store_true",
                    help="4-bit codes: keep the GEMM on the int8 matrix cores (no FP6-path copy of the weight)")
    ap.add_argument("--bits", default=None,
                    help="A,W: activation and weight bits instead of the workload's own (6,6 / 8,8 / 8,4: the other "
                         "settings of Sec. 5), same shapes and inputs")
    ap.add_argument("--norm", default=None, choices=["none", "rms", "layer"],
                    help="the norm in front of the layer instead of the workload's own (none: a layer whose producer is not "
                         "a norm, e.g. a down projection after the gated activation)")
    ap.add_argument("--packed", action="store_true",
                    help="6- and 8-bit activations: no one-byte-per-code copy of the weight, so that the GEMM expands "
                         "the packed codes itself")
    ap.add_argument("--cpu-sample-tokens", type=int, default=2048)
    ap.add_argument("--calibration-copy", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of a HIP graph holding one step per rotating buffer set (launch-bound shapes)")
    ap.add_argument("--assemble-more", type=float, default=0.0,
                    help="merge this fraction of C more channel pairs than disassembly added (C^ < C: the paper's "
                         "speed-up variant); 0 keeps C^ = C as in the paper's experiments")
    ap.add_argument("--expand", type=float, default=None,
                    help="expansion ratio that fixes theta (Sec. 5.2 varies it up to 0.1); default: the workload's own")
    ap.add_argument("--allow-map-walk", action="store_true",
                    help="do not stop when the fused kernel would fall back to walking the map's CSR rows")
    ap.add_argument("--stage", default="layer", choices=["layer", "match", "swiglu"],
                    help="layer: the hot path (the default, the line the contract asks for); match: the offline "
                         "channel matching of Eq. (5) / Appendix A at the workload's channel count; swiglu: the "
                         "producer of a down projection's input, silu(gate) * up, at the workload's N x C")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path shards over tokens with no "
                 "communication between GPUs). Run with --gpus 1.")

    import numpy as np
    import torch

    from paper_2310_08041_amd import binding as b
    from paper_2310_08041_amd import calibrate, workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = torch.device("cuda:0")
    w = wl.WORKLOADS[args.workload]
    if args.bits:
        import dataclasses
        a_bits, w_bits = (int(v) for v in args.bits.split(","))
        w = dataclasses.replace(w, a_bits=a_bits, w_bits=w_bits)
    if args.norm:
        import dataclasses
        w = dataclasses.replace(w, norm=args.norm)
    norm = {"none": b.NORM_NONE, "layer": b.NORM_LAYER, "rms": b.NORM_RMS}[w.norm]
    if args.stage == "match":
        return bench_matching(args, w, norm, dev)
    if args.stage == "swiglu":
        return bench_swiglu(args, w, dev)

    # ---- synthetic inputs, resident in HBM before anything is timed
    t0 = time.time()
    x_host, _, _ = wl.draw_activations(w)
    gamma_h, beta_h = wl.draw_norm_params(w)
    if x_host.dtype == np.uint16:
        x0 = torch.from_numpy(x_host.view(np.int16)).to(dev).view(torch.bfloat16)
    else:
        x0 = torch.from_numpy(x_host).to(dev)
    gamma = torch.from_numpy(gamma_h).to(dev)
    beta = None if beta_h is None else torch.from_numpy(beta_h).to(dev)

    # ---- offline: calibration -> map; weight reassembly + quantization (library host helpers)
    theta_rule = w.theta_rule if args.expand is None else ("expand", args.expand)
    cal = calibrate.calibrate(x0, norm, gamma, beta, w.eps, theta_rule, assemble_more=args.assemble_more)
    dmap = b.DeviceMap(cal["row_ptr"], cal["src"], cal["scale"], w.C, cal["plan"])
    K = dmap.C_out
    form = b.qllm_fused_kernel_choice(dmap, x0.dtype, w.N, w.C, norm, beta is not None, w.a_bits)
    if form == b.FUSED_WALKS_MAP and not args.allow_map_walk:
        sys.exit("bench.py: this map does not fit the planned fused kernel; the timed kernel would be the one that "
                 "walks the CSR rows (--allow-map-walk to time that)")
    W = wl.draw_weight(w)
    q = b.qllm_quantize_weight_host(W, cal["row_ptr"], cal["src"], w.w_bits)
    del W
    # what was measured on: digests of the seeded inputs as the kernels get them, and the machine
    import hashlib
    digest = lambda *arrays: hashlib.sha256(b"".join(np.ascontiguousarray(v).tobytes() for v in arrays)).hexdigest()
    inputs_sha256 = {"x": digest(x_host), "map": digest(cal["row_ptr"], cal["src"], cal["scale"]),
                     "packed_weights": digest(q["codes"], q["scale"], q["zero"], q["colsum"])}
    prop = torch.cuda.get_device_properties(0)
    cpu_model = next((line.split(":", 1)[1].strip() for line in open("/proc/cpuinfo") if line.startswith("model name")), "unknown")
    machine = {"gpu": prop.name, "compute_units": prop.multi_processor_count, "gpu_memory_GiB": round(prop.total_memory / 2 ** 30, 1),
               "arch": getattr(prop, "gcnArchName", ""), "cpu": cpu_model, "host_cpus": os.cpu_count()}
    dw = b.DeviceWeight(q["codes"], q["scale"], q["zero"], q["colsum"], K, w.w_bits, tiles6=not args.int8 and w.a_bits == 4,
                        tiles8=not args.packed and (w.a_bits, w.w_bits) != (4, 4))
    # 4-bit codes, more than 64 tokens: the GEMM runs on the FP6 matrix cores
    streams_weights = w.N <= 32 or ((w.a_bits, w.w_bits) == (4, 4) and w.N <= 64)   # the decode kernel: weights read once
    fp6_path = dw.tiles6 is not None and w.a_bits == 4 and not streams_weights
    xs = [x0] + [x0.roll(i, dims=0).contiguous() for i in range(1, N_ROTATE)]   # same rows, other addresses
    ys = [torch.empty((w.N, w.O), dtype=torch.bfloat16, device=dev) for _ in range(N_ROTATE)]
    ws = torch.empty(b.qllm_workspace_bytes(w.N, K, w.O, w.a_bits), dtype=torch.uint8, device=dev)
    qa = b.DeviceQAct(w.N, K, w.a_bits)
    gws = torch.empty(max(b.qllm_gemm_workspace_bytes(w.N, K, w.O, w.a_bits), 16), dtype=torch.uint8, device=dev)
    setup_s = time.time() - t0

    if args.calibration_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def step(i):
        b.qllm_reassembled_linear(xs[i % N_ROTATE], norm, gamma, beta, w.eps, dmap, w.a_bits, dw, ys[i % N_ROTATE], ws)

    # ---- warm-up: at least --warmup steps AND at least 100 ms of GPU time
    warm_ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    warm_steps, warm_ms = 0, 0.0
    while warm_steps < args.warmup or warm_ms < MIN_WARMUP_MS:
        n = max(N_ROTATE, min(64, args.warmup - warm_steps))
        warm_ev[0].record()
        for i in range(n):
            step(warm_steps + i)
        warm_ev[1].record()
        torch.cuda.synchronize()
        warm_steps += n
        warm_ms += warm_ev[0].elapsed_time(warm_ev[1])
    if args.graph:
        if args.steps % N_ROTATE:
            sys.exit(f"bench.py: --graph needs --steps to be a multiple of {N_ROTATE}")
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(N_ROTATE):
                step(i)
        graph.replay()
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for _ in range(args.steps // N_ROTATE):
            graph.replay()
    else:
        t_start = time.perf_counter()
        for i in range(args.steps):
            step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    ms_per_step = wall * 1e3 / args.steps
    # what the timed launches wrote, kept for the parity check below (the instrumented pass writes ys again)
    ys_timed = [y.cpu() for y in ys[:min(N_ROTATE, args.steps)]]
    ws_codes_timed = ws[:w.N * b.qllm_packed_row_bytes(K, w.a_bits)].cpu()      # activation codes of the last timed step
    last_buf = (args.steps - 1) % N_ROTATE

    # ---- instrumented pass: the same K steps as two calls with HIP events (recorded on the launch
    # stream, torch's current stream) around each kernel
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    for i in range(args.steps):
        ev[i][0].record()
        b.qllm_norm_reassemble_quant(xs[i % N_ROTATE], norm, gamma, beta, w.eps, dmap, w.a_bits, qa)
        ev[i][1].record()
        b.qllm_int_gemm(qa, dw, ys[i % N_ROTATE], workspace=gws)
        ev[i][2].record()
    torch.cuda.synchronize()
    fused_us = np.array([e[0].elapsed_time(e[1]) for e in ev]) * 1e3
    gemm_us = np.array([e[1].elapsed_time(e[2]) for e in ev]) * 1e3
    spread = lambda v: {"mean": float(v.mean()), "median": float(np.median(v)), "min": float(v.min())}
    # An event pair around ONE launch also spans the few microseconds between the first event and the kernel's
    # start, which a kernel trace does not count.  The average duration therefore comes from the same K launches
    # of each kernel back to back (rotating buffers), one event pair around all of them; the per-launch pairs
    # above give the spread (median, minimum).
    bev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    qas = [qa] + [b.DeviceQAct(w.N, K, w.a_bits) for _ in range(N_ROTATE - 1)]

    def settle(launch, ms=30.0):
        """The GPU sat idle while the host copied results back, and its clocks fell: the kernel about to be timed runs
        untimed first, for at least `ms` of GPU time (and at least once per buffer set), whatever --steps is."""
        done, n = 0.0, 0
        while done < ms or n < N_ROTATE:
            sev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            sev[0].record()
            for i in range(4 * N_ROTATE):
                launch(n + i)
            sev[1].record()
            torch.cuda.synchronize()
            done += sev[0].elapsed_time(sev[1])
            n += 4 * N_ROTATE

    def launch_fused(i):
        b.qllm_norm_reassemble_quant(xs[i % N_ROTATE], norm, gamma, beta, w.eps, dmap, w.a_bits, qas[i % N_ROTATE])

    def launch_gemm(i):
        b.qllm_int_gemm(qas[i % N_ROTATE], dw, ys[i % N_ROTATE], workspace=gws)

    settle(launch_fused)
    bev[0].record()
    for i in range(args.steps):
        launch_fused(i)
    bev[1].record()
    torch.cuda.synchronize()
    settle(launch_gemm)
    bev[2].record()
    for i in range(args.steps):
        launch_gemm(i)
    bev[3].record()
    torch.cuda.synchronize()
    t_fused, t_gemm = bev[0].elapsed_time(bev[1]) * 1e-3 / args.steps, bev[2].elapsed_time(bev[3]) * 1e-3 / args.steps
    t_pack = 0.0
    if fp6_path:
        # the GEMM call is two kernels on this path: the activations re-laid for the FP6 matrix cores, then the
        # product; the first one alone, back to back in the same way, gives the split
        tiles = torch.empty(b.qllm_tiles6_bytes(w.N, K), dtype=torch.uint8, device=dev)
        settle(lambda i: b.qllm_pack_tiles6(qas[i % N_ROTATE].codes, w.N, K, tiles), ms=10.0)
        bev[0].record()
        for i in range(args.steps):
            b.qllm_pack_tiles6(qas[i % N_ROTATE].codes, w.N, K, tiles)
        bev[1].record()
        torch.cuda.synchronize()
        t_pack = bev[0].elapsed_time(bev[1]) * 1e-3 / args.steps
        del tiles
    # the roofline below prices the whole GEMM call (on the FP6 path both of its kernels): the sum a kernel trace shows
    t_gemm_kernel = t_gemm

    ops = 2.0 * w.N * K * w.O
    x_bytes = w.N * w.C * x0.element_size()
    code_bytes = w.N * K * w.a_bits // 8
    fused_bytes = x_bytes + code_bytes + 12 * w.N            # read X once, write codes + (alpha, beta, rowsum)
    gemm_tops = ops / t_gemm_kernel / 1e12
    fused_gbs = fused_bytes / t_fused / 1e9

    # ---- what the machine delivers on the two resources, with none of the path's work in the way
    # (same process, same clocks): a loop of nothing but int8 matrix-core operations, and a plain
    # stream with the fused kernel's 4 : 1 read : write mix over a buffer larger than the last-level cache
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    probe_iters = 4096
    pe = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for _ in range(3):
        b.qllm_probe_mfma(cus, probe_iters, sink)
    pe[0].record()
    for _ in range(10):
        b.qllm_probe_mfma(cus, probe_iters, sink)
    pe[1].record()
    torch.cuda.synchronize()
    mfma_probe_tops = 10 * cus * 8 * probe_iters * 32 * 2.0 * 16 * 16 * 64 / (pe[0].elapsed_time(pe[1]) * 1e-3) / 1e12
    if fp6_path:
        fsink = torch.zeros(1, dtype=torch.float32, device=dev)
        for _ in range(3):
            b.qllm_probe_mfma_fp6(cus, probe_iters, fsink)
        pe[0].record()
        for _ in range(10):
            b.qllm_probe_mfma_fp6(cus, probe_iters, fsink)
        pe[1].record()
        torch.cuda.synchronize()
        fp6_probe_tops = 10 * cus * 8 * probe_iters * 32 * 2.0 * 16 * 16 * 128 / (pe[0].elapsed_time(pe[1]) * 1e-3) / 1e12
    sbytes = 1 << 30
    ssrc = torch.empty(sbytes, dtype=torch.uint8, device=dev).fill_(3)
    sdst = torch.empty(sbytes // 4, dtype=torch.uint8, device=dev)
    for _ in range(2):
        b.qllm_probe_stream(ssrc, sdst, cus * 8)
    pe[0].record()
    for _ in range(10):
        b.qllm_probe_stream(ssrc, sdst, cus * 8)
    pe[1].record()
    torch.cuda.synchronize()
    stream_probe_gbs = 10 * (sbytes + sbytes // 4) / (pe[0].elapsed_time(pe[1]) * 1e-3) / 1e9
    del ssrc, sdst

    bytes_path = dw.tiles8 is not None and not streams_weights
    if fp6_path:
        gemm_kernel = "gemm_w4a4_fp6_kernel<bf16>"
    elif bytes_path:
        gemm_kernel = "gemm_tiles8_kernel<%d,%d,bf16> after tiles8_kernel" % (w.a_bits, w.w_bits)
    elif w.N > 128:
        gemm_kernel = ("int_gemm_w4a4_kernel<bf16>" if (w.a_bits, w.w_bits) == (4, 4) else
                       "int_gemm_big_kernel<%d,%d,bf16>" % (w.a_bits, w.w_bits))
    else:
        gemm_kernel = "int_gemm_skinny_kernel" if streams_weights else "int_gemm_kernel"
    traffic = read_traffic(w.name + ("_w%da%d" % (w.w_bits, w.a_bits) if args.bits else ""))
    if streams_weights:
        # decode-sized batch: the GEMM streams the packed weights once and does little arithmetic per byte
        gemm_bytes = (w.O * b.qllm_packed_row_bytes(K, w.w_bits) + w.N * b.qllm_packed_row_bytes(K, w.a_bits)
                      + w.N * w.O * 2 + 12 * (w.N + w.O))
        gemm_gbs = gemm_bytes / t_gemm / 1e9
        roofline = {"kernel": gemm_kernel, "bound": "hbm", "achieved": gemm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": gemm_gbs / HBM_PEAK_GBS, "avg_launch_us": t_gemm * 1e6, "single_launch_event_us": spread(gemm_us),
                    "algorithmic_bytes": gemm_bytes, "traffic": traffic.get("int_gemm"), "int8_TOPs": gemm_tops,
                    "probe": {"what": "plain stream, 16 bytes read : 4 written, 1.25 GB per pass",
                              "achieved": stream_probe_gbs, "frac_of_probe": gemm_gbs / stream_probe_gbs}}
    elif fp6_path:
        # the operations are those of Eq. (1) on the codes (2 N K O), done by FP6 matrix-core operations: priced
        # against the FP6 peak
        roofline = {"kernel": gemm_kernel + " after tiles6_kernel", "bound": "mfma", "achieved": gemm_tops,
                    "peak": FP6_PEAK_TOPS, "unit": "TOP/s", "frac": gemm_tops / FP6_PEAK_TOPS,
                    "avg_launch_us": t_gemm * 1e6, "single_launch_event_us": spread(gemm_us),
                    "note": "durations are those of the GEMM call, i.e. of both its kernels (the activation codes re-laid, then "
                            "the product): in a kernel trace the sum of the two averages; tiles6_kernel_us is the first one "
                            "alone, launched back to back (launch-bound when it is only a few microseconds long)",
                    "tiles6_kernel_us": t_pack * 1e6,
                    "traffic": (traffic.get("gemm_fp6", 0) + traffic.get("tiles6", 0)) or None,
                    "frac_of_int8_peak": gemm_tops / INT8_PEAK_TOPS,
                    "probe": {"what": "loop of FP6 matrix-core operations on register operands that hold 4-bit codes, all CUs",
                              "achieved": fp6_probe_tops, "frac_of_probe": gemm_tops / fp6_probe_tops,
                              "int8_loop": mfma_probe_tops}}
    else:
        roofline = {"kernel": gemm_kernel, "bound": "mfma", "achieved": gemm_tops,
                    "peak": INT8_PEAK_TOPS, "unit": "TOP/s", "frac": gemm_tops / INT8_PEAK_TOPS,
                    "avg_launch_us": t_gemm * 1e6, "single_launch_event_us": spread(gemm_us),
                    "traffic": ((traffic.get("gemm_tiles8", 0) + traffic.get("tiles8", 0)) or None) if bytes_path
                    else traffic.get("int_gemm"),
                    "probe": {"what": "loop of int8 matrix-core operations on register operands, all CUs",
                              "achieved": mfma_probe_tops, "frac_of_probe": gemm_tops / mfma_probe_tops}}
    result = {
        "metric": "reassembled W%dA%d linear TOPS at 70B shapes; fused norm+reassembly+quant GB/s" % (w.w_bits, w.a_bits)
                  if args.bits else "reassembled W4A4 linear TOPS at 70B shapes; fused norm+reassembly+quant GB/s",
        "value": ops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("fp6 E2M3 (4-bit codes as FP6 numbers on the FP6 matrix cores, fp32 sums that are exact integers / 64); "
                  "fp32 norm/quantizer" if fp6_path else
                  "int8 (%d-bit activation and %d-bit weight codes on the int8 matrix cores, int32 accumulate); "
                  "fp32 norm/quantizer" % (w.a_bits, w.w_bits)),
        "data": "synthetic",
        "config": {"workload": w.name, "N": w.N, "C": w.C, "C_hat": K, "O": w.O, "a_bits": w.a_bits,
                   "w_bits": w.w_bits, "in_dtype": w.in_dtype, "out_dtype": "bf16", "norm": w.norm,
                   "theta": cal["theta"], "theta_rule": list(theta_rule), "assemble_more": args.assemble_more,
                   "fused_kernel_form": {b.FUSED_WALKS_MAP: "walks the map", b.FUSED_LISTS_IN_LDS: "planned, lists in LDS",
                                         b.FUSED_LISTS_STREAMED: "planned, lists streamed"}[form],
                   "extra_channels": int(cal["nnz"] - w.C),
                   "merged_pairs": int(cal["src_idx"].size), "T_max": int(cal["num_split"].max()),
                   "gemm_path": "fp6 matrix cores" if fp6_path else "int8 matrix cores", "rotating_buffers": N_ROTATE, "launch": "hip graph replay" if args.graph else "eager",
                   "warmup_done": {"steps": warm_steps, "gpu_ms": warm_ms}},
        "fused_GBps": fused_gbs,
        "roofline": roofline,
        "roofline_fused": {"kernel": "fused_planned_kernel", "bound": "hbm", "achieved": fused_gbs,
                           "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": fused_gbs / HBM_PEAK_GBS,
                           "avg_launch_us": t_fused * 1e6, "single_launch_event_us": spread(fused_us), "algorithmic_bytes": fused_bytes,
                           "traffic": traffic.get("fused_planned"),
                           "probe": {"what": "plain stream, 16 bytes read : 4 written, 1.25 GB per pass",
                                     "achieved": stream_probe_gbs, "frac_of_probe": fused_gbs / stream_probe_gbs}},
        "setup_s": setup_s,
        "inputs_sha256": inputs_sha256,
        "machine": machine,
    }

    if not args.no_cpu_baseline:
        # cpu_baseline leg only: the oracle as it stands, fed from the seeded generators, with its OWN calibration
        # (over all tokens, as the device's) and its own reassembled and quantized weights: nothing computed by the
        # HIP path enters it.  The timed part is the whole path on the first `ns` tokens.
        from oracle import api as oracle
        from oracle import calibrate as oracle_cal
        ns = min(args.cpu_sample_tokens, w.N)
        t1 = time.perf_counter()
        ocal = oracle_cal.calibrate(oracle.norm(x_host, norm, gamma_h, beta_h, w.eps), theta_rule,
                                    assemble_more=args.assemble_more)
        W = wl.draw_weight(w)
        wq = oracle.quantize_weight(oracle.reassemble_weight(W, ocal["T"], ocal["src_idx"], ocal["dst_idx"]), w.w_bits)
        del W
        prep_s = time.perf_counter() - t1
        xs_host = np.ascontiguousarray(x_host[:ns])
        t1 = time.perf_counter()
        ref = oracle.reassembled_linear(xs_host, norm, gamma_h, beta_h, w.eps, ocal["T"], ocal["src_idx"], ocal["dst_idx"],
                                        w.a_bits, wq, want_acc=False)
        cpu_s = time.perf_counter() - t1
        Ko = ref["codes"].shape[1]
        result["cpu_baseline"] = {"value": 2.0 * ns * Ko * w.O / cpu_s / 1e12, "unit": "TOP/s",
                                  "cores": oracle.max_threads(), "kind": "oracle",
                                  "sample": f"first {ns} of {w.N} tokens through the whole path (all {Ko} channels, "
                                            f"all {w.O} output features), {cpu_s:.1f} s; its own calibration and "
                                            f"weight quantization before that, {prep_s:.1f} s, are not in the rate"}
        # ---- parity of what the TIMED launches wrote: buffer i holds the rows of the batch rotated by i
        same_map = (np.array_equal(ocal["T"], cal["num_split"]) and np.array_equal(ocal["src_idx"], cal["src_idx"])
                    and np.array_equal(ocal["dst_idx"], cal["dst_idx"]) and float(ocal["theta"]) == float(cal["theta"]))
        ref_y = oracle.widen_bf16(oracle.round_to_bf16(ref["y"]))
        rows_checked, y_exact, y_max_rel = 0, True, 0.0
        for i, yt in enumerate(ys_timed):
            rows = (np.arange(ns) + i) % w.N                       # row r of the batch sits at row r + i of buffer i
            got = oracle.widen_bf16(yt.view(torch.int16).numpy().view(np.uint16)[rows])
            y_exact = y_exact and bool(np.array_equal(got, ref_y))
            den = np.maximum(np.abs(ref["y"]), 1e-3 * np.sqrt((ref["y"].astype(np.float64) ** 2).mean()))
            y_max_rel = max(y_max_rel, float((np.abs(got - ref["y"]) / den).max()))
            rows_checked += ns
        rows = (np.arange(ns) + last_buf) % w.N
        got_codes = ws_codes_timed.numpy().reshape(w.N, -1)[rows]
        codes_exact = bool(Ko == K and np.array_equal(got_codes, oracle.pack_codes(ref["codes"], w.a_bits, got_codes.shape[1])))
        result["parity_checked"] = {"against": "the cpu_baseline oracle run (its own map and weights)",
                                    "maps_identical": bool(same_map), "timed_buffers": len(ys_timed),
                                    "token_rows_x_all_features": rows_checked, "y_bit_exact_bf16": bool(y_exact),
                                    "y_max_rel_err": y_max_rel, "y_tolerance": 2e-2,
                                    "activation_codes_rows": int(ns), "activation_codes_exact": codes_exact,
                                    "ok": bool(same_map and codes_exact and y_max_rel <= 2e-2)}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
