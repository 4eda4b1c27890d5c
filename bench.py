#!/usr/bin/env python3
"""Benchmark of the arbitrary-precision bit-plane hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-extra] [--no-cpu]

A step is one pass of the hot path on the headline workload (benchmark
configuration 1: w1a2 GEMM, M = N = K = 4096, +-1 weights, unsigned 2-bit
activations): bit-decompose and pack the activations, then the bit-plane GEMM
to int32 (by default the FP4 matrix-core form of the plane-pair product; the
literal AND + popcount form is timed as well).  Weights are packed once before
timing (they are quantised at initialisation, Sec. 5.1).  All inputs are
resident in HBM when the timed region starts.

Prints ONE JSON line: effective TOPS (2 M N K / time), the roofline of the
dominant kernel (FP4 matrix peak) measured with events around its launches
inside the timed region, the same for the AND + popcount kernel (VALU
bitwise+popcount issue rate), and the CPU oracle timed on a bounded row sample.
The other benchmark configurations and the paper's own layer shapes are
reported under "extra" (device time per launch via HIP-graph replay), each with
the oracle's time for the same work and a bit-exact comparison.

Modes for profiling and for the evidence tables under profiles/ (each prints
its own JSON and exits):
    --gemm M,N,K,p,q[,encW,encX] [--force NAME=V,...] [--reps R] [--zeros]
        R eager launches of one GEMM (operands from the seeded generator, or
        all-zero planes), for rocprofv3 kernel traces and counters
    --evidence
        K-scaling and zero-against-random-operand timings of the two headline
        kernels and the register-only vector instruction rate
    --network-only N [--network-batch B]
        N eager passes of the ResNet-18-shaped network
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

VALU_PEAK_LANE_OPS = 256 * 64 * 2.4e9      # 256 CUs x 64 lanes/clk x 2.4 GHz (32-bit integer vector ops)
HBM_PEAK = 8.0e12
MFMA_FP4_PEAK = 10.1e15                    # dense FP4 matrix peak, FLOP/s
MFMA_INT8_PEAK = 5.0e15                    # dense int8 matrix peak, OP/s
VALU_FLOOR_CONFIG4_US = 62.0               # AND+popcount lane-operations of the network at the VALU peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def graph_time(fn, reps=20, replays=5):
    """Device seconds per call of fn, from replays of a HIP graph holding `reps` calls."""
    import torch
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        fn()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(reps):
            fn()
    g.replay()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(replays):
        g.replay()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e-3 / (reps * replays)


def profile_traffic(name):
    """HBM bytes per launch that a tracked rocprofv3 counter summary recorded ("traffic_bytes_per_launch = N")."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        m = re.search(r"^traffic_bytes_per_launch\s*=\s*(\d+)", open(path).read(), re.M)
        return (int(m.group(1)), "profiles/" + name) if m else (None, None)
    except OSError:
        return None, None


def stats_us(seconds):
    import numpy as np
    a = np.asarray(seconds) * 1e6
    return {"median_us": round(float(np.median(a)), 2), "mean_us": round(float(a.mean()), 2),
            "min_us": round(float(a.min()), 2), "samples": int(a.size)}


def parse_force(text):
    out = []
    for item in filter(None, (text or "").split(",")):
        k, v = item.split("=")
        out.append((k.strip(), int(v)))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)      # the paper averages 200 executions (Sec. 6)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-extra", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--network-only", type=int, default=0, metavar="N",
                    help="run only N eager forward passes of the ResNet-18-shaped network (for rocprofv3 kernel traces)")
    ap.add_argument("--network-batch", type=int, default=8, metavar="B", help="batch size of --network-only")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch one 256 MiB apnn_probe_copy (reference for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--gemm", default=None, metavar="M,N,K,p,q[,encW,encX]", help="profiling mode: eager launches of one GEMM")
    ap.add_argument("--force", default="", metavar="NAME=V,...", help="kernel-choice overrides (include/apnn_debug.h)")
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--zeros", action="store_true", help="--gemm with all-zero operand planes")
    ap.add_argument("--evidence", action="store_true")
    ap.add_argument("--phases", action="store_true",
                    help="phase time stamps of mfma_big_kernel on config 1; needs the library built with -DAPNN_BIG_TIMING "
                         "(python -c \"from paper_2106_12169_amd import build; build.build(True, ['-DAPNN_BIG_TIMING=1'])\")")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import numpy as np
    import torch
    if args.phases:                               # (the instrumented library reads the address when apnn_gemm is called)
        phase_buf = torch.zeros(256 * 4 * 8, dtype=torch.int64, device="cuda")
        os.environ["APNN_DBG_PTR"] = str(phase_buf.data_ptr())
    from paper_2106_12169_amd import binding as B
    from paper_2106_12169_amd import workloads as wl

    B.lib()                                       # fails loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    if args.network_only > 0:
        from paper_2106_12169_amd.network import PackedNet
        layers = wl.resnet18_layers()
        net = PackedNet(layers, wl.network_params(layers), args.network_batch)
        img = dev(wl.image_batch(2004, args.network_batch, 224))
        for _ in range(args.network_only):
            net.forward(img)
        torch.cuda.synchronize()
        return
    if args.gemm:
        return gemm_mode(args, B, wl, dev)
    if args.evidence:
        return evidence_mode(B, wl, dev)
    if args.phases:
        return phases_mode(B, wl, dev, phase_buf)

    wk = wl.CONFIG1
    Wv, Xv = wk.weights(), wk.activations()
    Wd, Xd = dev(Wv), dev(Xv)
    Wp = B.apnn_pack(Wd, wk.p, wk.encW)           # init-time weight packing
    Xp = torch.empty(B.apnn_packed_words(wk.N, wk.K, wk.q), dtype=torch.int32, device="cuda")
    Y = torch.empty((wk.M, wk.N), dtype=torch.int32, device="cuda")

    def step(ev=None):
        B.apnn_pack(Xd, wk.q, wk.encX, out=Xp)
        if ev is not None:
            ev[0].record()
        B.apnn_gemm(Wp, Xp, wk.M, wk.N, wk.K, wk.p, wk.q, wk.encW, wk.encX, out=Y)
        if ev is not None:
            ev[1].record()

    if args.copy_probe:
        from paper_2106_12169_amd import bench_probes
        src = torch.zeros(1 << 28, dtype=torch.uint8, device="cuda")
        bench_probes.apnn_probe_copy(src, torch.empty_like(src))

    def timed(steps, warmup, stride):
        """Wall time per step over `steps` steps, and the event-bracketed durations of the GEMM launch of every
        stride-th step (each event record is a command of its own on the stream the kernels are launched on)."""
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) if i % stride == 0 else None
               for i in range(steps)]
        t0 = time.perf_counter()
        for i in range(steps):
            step(evs[i])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        kern = np.array([e[0].elapsed_time(e[1]) for e in evs if e is not None]) * 1e-3
        return (t1 - t0) / steps, kern

    # headline: the library's own dispatch (FP4 matrix-core kernel for <= 2-bit operands); at least 20 event samples
    sec_per_step, gemm_samples = timed(args.steps, args.warmup, max(1, args.steps // 50))
    gemm_s = float(gemm_samples.mean())
    flops = wk.effective_ops                                       # 2 M N K multiply-adds on the matrix cores
    # the AND + popcount kernel on the same workload (the VALU bitwise+popcount roofline): 24 samples whatever --steps is
    B.apnn_debug_force("MFMA", 0)
    _, pop_samples = timed(24, 4, 1)
    pop_s = float(pop_samples.mean())
    B.apnn_debug_reset()
    step()                                                         # leave the default path's result in Y
    torch.cuda.synchronize()
    lane_ops = 2.0 * wk.M * wk.N * wk.K * wk.p * wk.q / 32.0     # AND + popcount-accumulate per 32 bit-products

    # cheap self-check on the timed output (full parity lives in tests/)
    colsum = Y.sum(dim=0, dtype=torch.int64).cpu().numpy()
    want = Xv.astype(np.int64) @ Wv.astype(np.int64).sum(0)
    assert np.array_equal(colsum, want), "timed output failed its column-sum check"

    # the same step (both launches) replayed as a HIP graph: what the launch gaps of the eager loop cost (not `value`)
    step_graph_s = graph_time(step, reps=10, replays=5)
    traffic, traffic_src = profile_traffic("mfma_big_kernel_gemm_w1a2_4096_hbm_counters.txt")
    pop_traffic, pop_traffic_src = profile_traffic("tile_kernel_gemm_w1a2_4096_hbm_counters.txt")
    out = {
        "metric": "effective TOPS, w1a2 4096^3 bit-GEMM (2*M*N*K / time)",
        "value": round(wk.effective_ops / sec_per_step / 1e12, 2),
        "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp4 e2m1 products of packed bit planes, fp32 accumulate (exact: K max|w| max|x| = 12288 < 2^24), int32 out",
        "data": "synthetic",
        "config": {"workload": "config1: w1a2 GEMM M=N=K=4096, +-1 weights x unsigned 2-bit activations, int32 out",
                   "step": "apnn_pack(activations) + apnn_gemm", "seeds": [wk.seedW, wk.seedX],
                   "launch": "eager, one library call per kernel; the same step replayed as a HIP graph takes step_graph_replay_ms"},
        "step_graph_replay_ms": round(step_graph_s * 1e3, 5),
        "roofline": {
            "bound": "mfma", "kernel": "mfma_big_kernel<PM1,U2> (v_mfma_scale_f32_32x32x64_f8f6f4, FP4 E2M1)",
            "achieved": round(flops / gemm_s / 1e12, 1), "peak": MFMA_FP4_PEAK / 1e12, "unit": "TFLOP/s",
            "frac": round(flops / gemm_s / MFMA_FP4_PEAK, 4),
            "kernel_us": round(gemm_s * 1e6, 2), "kernel_time": stats_us(gemm_samples),
            # HBM bytes per launch as measured with rocprofv3 FETCH_SIZE / WRITE_SIZE in the named summary (not in
            # this run); algorithmic: 6 MiB in + 64 MiB out
            "traffic": traffic, "traffic_source": traffic_src,
            "algorithmic_bytes": (wk.M * wk.p + wk.N * wk.q) * (wk.K // 8) + 4 * wk.M * wk.N,
        },
        "roofline_popcount_kernel": {
            "bound": "alu", "kernel": "tile_kernel<4,4,16,4,4,false,false> (64x64 tile, v_and + v_bcnt), MFMA override 0",
            "achieved": round(lane_ops / pop_s / 1e12, 3), "peak": round(VALU_PEAK_LANE_OPS / 1e12, 3),
            "unit": "T lane-op/s (32-bit VALU, 2 lane-ops per 32 bit-products per plane pair)",
            "frac": round(lane_ops / pop_s / VALU_PEAK_LANE_OPS, 4),
            "kernel_us": round(pop_s * 1e6, 2), "kernel_time": stats_us(pop_samples),
            "eff_tops": round(wk.effective_ops / pop_s / 1e12, 1),
            "traffic": pop_traffic, "traffic_source": pop_traffic_src,
        },
    }

    # the pack kernel of the step (HBM bound): 16 MiB of codes in, 4 MiB of planes out
    t_pack = graph_time(lambda: B.apnn_pack(Xd, wk.q, wk.encX, out=Xp))
    pack_bytes = wk.N * wk.K + wk.N * wk.K * wk.q // 8
    out["roofline_pack_kernel"] = {"bound": "hbm", "kernel": "pack_rows_kernel (activations of the step)",
                                   "achieved": round(pack_bytes / t_pack / 1e9, 1), "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                                   "frac": round(pack_bytes / t_pack / HBM_PEAK, 4), "kernel_us": round(t_pack * 1e6, 2),
                                   "algorithmic_bytes": pack_bytes,
                                   "what": "device time per launch by graph replay, of which about 1.9 us is the launch itself "
                                           "(bench.py --evidence, launch_of_16_bytes_us): 20 MiB in what remains is the HBM rate"}

    if not args.no_cpu:
        import oracle
        rows = 32
        t = time.perf_counter()
        oracle.gemm_rows(Wv, wk.encW, wk.p, Xv, wk.encX, wk.q, 0, rows)
        dt = time.perf_counter() - t
        rows = int(min(wk.M, max(rows, rows * 15.0 / max(dt, 1e-3))))      # aim at ~15 s of CPU work
        rows -= rows % oracle.threads() or 0
        t = time.perf_counter()
        ref = oracle.gemm_rows(Wv, wk.encW, wk.p, Xv, wk.encX, wk.q, 0, rows)
        dt = time.perf_counter() - t
        assert np.array_equal(Y[:rows].cpu().numpy(), ref), "GPU result differs from the oracle on the sampled rows"
        out["cpu_baseline"] = {"value": round(2.0 * rows * wk.N * wk.K / dt / 1e12, 5), "unit": "TOPS",
                               "cores": oracle.threads(), "kind": "oracle",
                               "sample": f"rows 0..{rows - 1} of the same 4096^3 product ({dt:.1f} s), also compared bit-exactly"}

    if not args.no_extra:
        out["extra"] = extra_configs(B, wl, dev, graph_time, with_cpu=not args.no_cpu)

    print(json.dumps(out), flush=True)


def gemm_mode(args, B, wl, dev):
    """--gemm: eager launches of one product, for kernel traces and counter runs."""
    import torch
    f = [int(x) for x in args.gemm.split(",")]
    M, N, K, p, q = f[:5]
    encW, encX = (f[5], f[6]) if len(f) >= 7 else (wl.ENC_UNSIGNED, wl.ENC_UNSIGNED)
    if args.zeros:
        Wp = torch.zeros(B.apnn_packed_words(M, K, p), dtype=torch.int32, device="cuda")
        Xp = torch.zeros(B.apnn_packed_words(N, K, q), dtype=torch.int32, device="cuda")
    else:
        Wp = B.apnn_pack(dev(wl.operand(1000 + 16 * p + q, M, K, p, encW)), p, encW)
        Xp = B.apnn_pack(dev(wl.operand(2000 + 16 * p + q, N, K, q, encX)), q, encX)
    Y = torch.empty((M, N), dtype=torch.int32, device="cuda")
    for name, v in parse_force(args.force):
        B.apnn_debug_force(name, v)
    call = lambda: B.apnn_gemm(Wp, Xp, M, N, K, p, q, encW, encX, out=Y)
    for _ in range(args.reps):
        call()
    torch.cuda.synchronize()
    t = graph_time(call, reps=10, replays=3)
    print(json.dumps({"mode": "gemm", "shape": [M, N, K], "bits": [p, q], "enc": [encW, encX], "force": args.force,
                      "zeros": bool(args.zeros), "graph_replay_us": round(t * 1e6, 2)}), flush=True)


def phases_mode(B, wl, dev, buf):
    """Where the time of mfma_big_kernel goes on config 1 and on the same outputs with K = 256: per-wave time stamps
    (100 MHz clock) of an instrumented build, relative to the first wave's entry; min / mean / max over the 1024 waves."""
    import numpy as np
    import torch
    out = {"mode": "phases", "unit": "us", "clock": "wall_clock64, 100 MHz"}
    for K in (256, 4096):
        W, X = wl.operand(1, 4096, K, 1, wl.ENC_PM1), wl.operand(2, 4096, K, 2, wl.ENC_UNSIGNED)
        Wp, Xp = B.apnn_pack(dev(W), 1, wl.ENC_PM1), B.apnn_pack(dev(X), 2, wl.ENC_UNSIGNED)
        Y = torch.empty((4096, 4096), dtype=torch.int32, device="cuda")
        for _ in range(3):
            B.apnn_gemm(Wp, Xp, 4096, 4096, K, 1, 2, wl.ENC_PM1, wl.ENC_UNSIGNED, out=Y)
        torch.cuda.synchronize()
        d = buf.cpu().numpy().reshape(256, 4, 8).astype(np.float64) * 0.01
        if not d[:, :, 0].any():
            sys.exit("bench.py --phases: no time stamps; build the library with -DAPNN_BIG_TIMING first")
        base = d[:, :, 0].min()
        st = lambda x: {"min": round(float(x.min()), 2), "mean": round(float(x.mean()), 2), "max": round(float(x.max()), 2)}
        out[f"K{K}"] = {"entry": st(d[:, :, 0] - base), "entry_to_loop": st(d[:, :, 1] - d[:, :, 0]),
                        "loop": st(d[:, :, 2] - d[:, :, 1]), "last_store_issued_after_loop": st(d[:, :, 3] - d[:, :, 2]),
                        "stores_acknowledged_after_that": st(d[:, :, 4] - d[:, :, 3]),
                        "loop_end_since_first_entry": st(d[:, :, 2] - base), "done_since_first_entry": st(d[:, :, 4] - base)}
    print(json.dumps(out), flush=True)


def evidence_mode(B, wl, dev):
    """K-scaling and zero-against-random-operand timings of the two headline kernels (4096 x 4096 outputs, w1a2),
    and the register-only rate of the vector AND+popcount chain; HIP-graph replays."""
    import torch
    from paper_2106_12169_amd import bench_probes
    M = N = 4096
    Y = torch.empty((M, N), dtype=torch.int32, device="cuda")
    rows = []
    for K in (256, 1024, 2048, 4096, 8192):
        W, X = wl.operand(1, M, K, 1, wl.ENC_PM1), wl.operand(2, N, K, 2, wl.ENC_UNSIGNED)
        Wp, Xp = B.apnn_pack(dev(W), 1, wl.ENC_PM1), B.apnn_pack(dev(X), 2, wl.ENC_UNSIGNED)
        Wz, Xz = torch.zeros_like(Wp), torch.zeros_like(Xp)
        r = {"K": K}
        for kernel, force in (("mfma_big_kernel", []), ("tile_kernel", [("MFMA", 0)])):
            if kernel == "tile_kernel" and K > 4096:
                continue
            for name, v in force:
                B.apnn_debug_force(name, v)
            for label, (a, b) in (("random", (Wp, Xp)), ("zeros", (Wz, Xz))):
                t = graph_time(lambda: B.apnn_gemm(a, b, M, N, K, 1, 2, wl.ENC_PM1, wl.ENC_UNSIGNED, out=Y), reps=5, replays=3)
                r[f"{kernel}_{label}_us"] = round(t * 1e6, 2)
            B.apnn_debug_reset()
        rows.append(r)
    outw = torch.empty(1024 * 256, dtype=torch.int32, device="cuda")
    ops = bench_probes.apnn_probe_valu(1024, 2000, outw)
    t = graph_time(lambda: bench_probes.apnn_probe_valu(1024, 2000, outw), reps=2, replays=3)
    # the two kernels of the 8-bit integer matrix form over K (2048 x 2048 outputs, 4 x 4 bits)
    i8_rows = []
    Y2 = torch.empty((2048, 2048), dtype=torch.int32, device="cuda")
    for K in (256, 1024, 2048, 4096, 8192):
        Wp = B.apnn_pack(dev(wl.uniform_codes(3, (2048, K), 4)), 4, wl.ENC_UNSIGNED)
        Xp = B.apnn_pack(dev(wl.uniform_codes(4, (2048, K), 4)), 4, wl.ENC_UNSIGNED)
        r = {"K": K}
        for kernel, force in (("mfma_i8_kernel", 2), ("mfma_i8_wide_kernel", 3)):
            B.apnn_debug_force("INT8", force)
            r[f"{kernel}_us"] = round(graph_time(lambda: B.apnn_gemm(Wp, Xp, 2048, 2048, K, 4, 4, wl.ENC_UNSIGNED, wl.ENC_UNSIGNED, out=Y2),
                                                 reps=5, replays=3) * 1e6, 2)
        B.apnn_debug_reset()
        i8_rows.append(r)
    # time per slot (matrix instruction + n vector instructions) of a SIMD with one and two waves, in cycles of the
    # nominal 2.4 GHz clock
    issue = []
    iters = 4000
    for waves in (1, 2):
        for with_matrix, nv in ((True, 0), (False, 8), (False, 16), (True, 4), (True, 8), (True, 16)):
            ts = graph_time(lambda: bench_probes.apnn_probe_issue(nv, with_matrix, waves, iters, outw), reps=1, replays=3)
            issue.append({"waves_per_simd": waves, "matrix": with_matrix, "vector": nv,
                          "nominal_cycles_per_slot": round(ts / (4 * iters * waves) * 2.4e9, 1)})
    # a launch that does (almost) nothing, and a plain 256 MiB copy: the fixed cost of a launch and the HBM rate
    tiny_s, tiny_d = torch.zeros(16, dtype=torch.uint8, device="cuda"), torch.zeros(16, dtype=torch.uint8, device="cuda")
    t_empty = graph_time(lambda: bench_probes.apnn_probe_copy(tiny_s, tiny_d), reps=20, replays=5)
    big_s = torch.zeros(1 << 28, dtype=torch.uint8, device="cuda")
    big_d = torch.empty_like(big_s)
    t_copy = graph_time(lambda: bench_probes.apnn_probe_copy(big_s, big_d), reps=2, replays=3)
    fill = torch.empty(1 << 26, dtype=torch.uint8, device="cuda")
    t_fill = graph_time(lambda: fill.zero_(), reps=5, replays=3)
    print(json.dumps({"mode": "evidence", "outputs": [M, N], "k_scaling": rows,
                      "launch_of_16_bytes_us": round(t_empty * 1e6, 2),
                      "copy_256MiB": {"us": round(t_copy * 1e6, 1), "read_plus_write_TBps": round(2 * (1 << 28) / t_copy / 1e12, 2)},
                      "fill_64MiB_us": round(t_fill * 1e6, 2),
                      "valu_and_popcount_chain": {"lane_ops_per_s": ops / t, "frac_of_nominal_peak": ops / t / VALU_PEAK_LANE_OPS},
                      "int8_k_scaling_2048x2048_w4a4": i8_rows, "issue_probe": issue}),
          flush=True)


def extra_configs(B, wl, dev, graph_time, with_cpu=True):
    """Device time of the other benchmark configurations (HIP-graph replays), each checked bit-exactly against the
    oracle, whose time for the same work on the host cores is reported beside it."""
    import numpy as np
    import torch
    from paper_2106_12169_amd.network import PackedNet
    from tests import helpers as hp
    if with_cpu:
        import oracle
        from oracle import network as onet
    ex = {}

    def gemm_case(wk, check):
        Wv, Xv = wk.weights(), wk.activations()
        Wp = B.apnn_pack(dev(Wv), wk.p, wk.encW)
        Xp = B.apnn_pack(dev(Xv), wk.q, wk.encX)
        Y = torch.empty((wk.M, wk.N), dtype=torch.int32, device="cuda")
        call = lambda: B.apnn_gemm(Wp, Xp, wk.M, wk.N, wk.K, wk.p, wk.q, wk.encW, wk.encX, out=Y)
        t = graph_time(call)
        # the FP4 matrix-core form runs ceil(p/2)*ceil(q/2) base-4 digit passes of 2*M*N*K flops each; the 8-bit
        # integer form, taken for wide operands, runs one pass of 2*M*N*K integer operations
        passes = ((wk.p + 1) // 2) * ((wk.q + 1) // 2)
        tiles128 = -(-wk.M // 128) * -(-wk.N // 128)
        int8 = passes >= 5 or (passes == 4 and ((wk.p > 2 and wk.q > 2) or tiles128 <= 256))        # the library's rule
        r = {"us": round(t * 1e6, 2), "eff_tops": round(wk.effective_ops / t / 1e12, 2)}
        if int8 and wk.M * wk.N >= 64 * 128 * 128:
            r.update(form="int8 matrix instruction, one pass", int8_mfma_frac=round(wk.effective_ops / t / MFMA_INT8_PEAK, 4))
        else:
            r.update(form=f"fp4 matrix instruction, {passes} digit pass(es)", digit_passes=passes,
                     fp4_mfma_frac=round(wk.effective_ops * passes / t / MFMA_FP4_PEAK, 4))
        # memory view of the same launch: packed planes in, int32 out
        nbytes = (wk.M * wk.p + wk.N * wk.q) * B.apnn_row_words(wk.K) * 4 + 4 * wk.M * wk.N
        r.update(algorithmic_bytes=nbytes, achieved_GBps=round(nbytes / t / 1e9, 1), hbm_frac=round(nbytes / t / HBM_PEAK, 4))
        if check and with_cpu:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            want = oracle.gemm(Wv, wk.encW, wk.p, Xv, wk.encX, wk.q)
            r["cpu_oracle_s"] = round(time.perf_counter() - t0, 4)
            call()
            torch.cuda.synchronize()
            assert np.array_equal(Y.cpu().numpy(), want), f"{wk.name}: GPU result differs from the oracle"
            r["bit_exact_vs_oracle"] = True
        return r

    ex["config0_gemm_w1a2_128"] = gemm_case(wl.CONFIG0, True)
    ex["config0_gemm_w1a2_128"]["what"] = "latency bound: one launch (an empty launch takes about 2.5 us)"
    ex["config2_sweep_2048"] = {f"w{wk.p}a{wk.q}": gemm_case(wk, True) for wk in wl.CONFIG2}

    c = wl.CONFIG3
    d = B.Conv(c.BS, c.H, c.W, c.Cin, c.Cout, c.R, c.S, c.stride, c.pad, c.p, c.q, c.encW, c.encX)
    Wv3, Xv3 = c.weights_oihw(), c.features_nchw()
    Wp = B.apnn_pack_conv_weights(dev(Wv3), c.p, c.encW)
    Xp = B.apnn_pack_fmap(dev(Xv3), B.LAYOUT_NCHW, c.q, c.encX)
    sc, bi = dev(c.scale()), dev(c.bias())
    outp = torch.empty(B.apnn_fmap_words(d.N * d.Ho * d.Wo, c.Cout, c.q_out), dtype=torch.int32, device="cuda")
    t = graph_time(lambda: B.apnn_layer(d, Wp, Xp, q_out=c.q_out, scale=sc, bias=bi, out=outp))
    in_bytes = 4 * (B.apnn_fmap_words(c.BS * c.H * c.W, c.Cin, c.q) + c.Cout * c.p * c.R * c.S * (c.Cin // 32)) + 8 * c.Cout
    out_bytes = 4 * B.apnn_fmap_words(d.N * d.Ho * d.Wo, c.Cout, c.q_out)
    ex["config3_conv_layer"] = {"us": round(t * 1e6, 2), "eff_tops": round(c.effective_ops / t / 1e12, 2),
                                "fp4_mfma_frac": round(c.effective_ops / t / MFMA_FP4_PEAK, 4),
                                "algorithmic_bytes": in_bytes + out_bytes,
                                "achieved_GBps": round((in_bytes + out_bytes) / t / 1e9, 1),
                                "hbm_frac": round((in_bytes + out_bytes) / t / HBM_PEAK, 5),
                                "what": "fused conv + scale/bias + requantise + repack, packed in/out (latency bound)"}
    if with_cpu:
        t0 = time.perf_counter()
        acc = oracle.conv2d(Wv3, c.encW, c.p, Xv3, c.encX, c.q, c.stride, c.pad)
        want_codes, _ = oracle.epilogue(acc, c.scale(), c.bias(), c.q_out)
        ex["config3_conv_layer"]["cpu_oracle_s"] = round(time.perf_counter() - t0, 4)
        B.apnn_layer(d, Wp, Xp, q_out=c.q_out, scale=sc, bias=bi, out=outp)
        torch.cuda.synchronize()
        codes, pad_bits = hp.unpack_fmap(hp.words_u32(outp), c.BS, d.Ho, d.Wo, c.Cout, c.q_out)
        assert np.array_equal(codes, want_codes) and pad_bits == 0, "config 3: packed codes differ from the oracle"
        ex["config3_conv_layer"]["bit_exact_vs_oracle"] = True

    # Fusion of pooling (Sec. 5.2; the paper's fusion experiment uses APConv-w1a2 + 2 x 2 pooling + 2-bit
    # quantisation): one kernel against conv+requantise followed by the pooling kernel on packed codes.
    pooled = torch.empty(B.apnn_fmap_words(d.N * (d.Ho // 2) * (d.Wo // 2), c.Cout, c.q_out), dtype=torch.int32, device="cuda")
    t_f = graph_time(lambda: B.apnn_layer(d, Wp, Xp, q_out=c.q_out, scale=sc, bias=bi, out=pooled, pool=B.POOL_MAX2))

    def two_kernels():
        B.apnn_layer(d, Wp, Xp, q_out=c.q_out, scale=sc, bias=bi, out=outp)
        B.apnn_maxpool(outp, d.N, d.Ho, d.Wo, c.Cout, c.q_out, 2, 2, 0, out=pooled)
    t_u = graph_time(two_kernels)
    ex["config3_conv_maxpool2_requant"] = {"fused_us": round(t_f * 1e6, 2), "two_kernels_us": round(t_u * 1e6, 2),
                                           "what": "conv + 2x2 max pooling + 2-bit requantise: one kernel vs conv+requantise then pooling on codes"}

    # Layer shapes of the paper's own APMM / APConv evaluation (Sec. 6.1): device time per launch.
    # Its raw-latency table (64 x 1024 x 1024, RTX 3090) reads 6.67 / 6.81 / 7.06 / 7.15 us for
    # w1a2 / w1a3 / w1a4 / w2a2 -- another machine, quoted as context only.
    fc = {}
    for (w, a) in wl.PAPER_FC_BITS:
        fc[f"w{w}a{a}"] = {str(dim): gemm_case(wl.paper_fc_workload(w, a, dim), False)["us"] for dim in wl.PAPER_FC_DIMS}
    ex["paper_fc_batch64_us_by_dim"] = fc
    cv = {}
    for ch in wl.PAPER_CONV_CHANNELS:
        cc = wl.paper_conv_workload(ch)
        dd = B.Conv(cc.BS, cc.H, cc.W, cc.Cin, cc.Cout, cc.R, cc.S, cc.stride, cc.pad, cc.p, cc.q, cc.encW, cc.encX)
        Wpc = B.apnn_pack_conv_weights(dev(cc.weights_oihw()), cc.p, cc.encW)
        Xpc = B.apnn_pack_fmap(dev(cc.features_nchw()), B.LAYOUT_NCHW, cc.q, cc.encX)
        scc, bic = dev(cc.scale()), dev(cc.bias())
        outc = torch.empty(B.apnn_fmap_words(dd.N * dd.Ho * dd.Wo, cc.Cout, cc.q_out), dtype=torch.int32, device="cuda")
        t = graph_time(lambda: B.apnn_layer(dd, Wpc, Xpc, q_out=cc.q_out, scale=scc, bias=bic, out=outc))
        cv[str(ch)] = round(t * 1e6, 2)
    ex["paper_conv_w1a2_16x16_batch1_us_by_channels"] = cv

    layers = wl.resnet18_layers()
    params = wl.network_params(layers)
    net = PackedNet(layers, params, 8)
    img_np = wl.image_batch(2004, 8, 224)
    img = dev(img_np)
    t = graph_time(lambda: net.forward(img), reps=1, replays=50)
    macs = sum(8 * L.Ho * L.Wo * L.Cout * L.Cin * L.R * L.S for L in layers if L.kind in ("conv", "fc"))
    ex["config4_resnet18_w1a2_batch8"] = {"ms": round(t * 1e3, 4), "library_calls": net.launches,
                                          "eff_tops": round(2.0 * macs / t / 1e12, 2),
                                          "matrix_frac_vs_fp4_peak": round(2.0 * macs / t / MFMA_FP4_PEAK, 4),
                                          "valu_floor_us": VALU_FLOOR_CONFIG4_US,
                                          "valu_floor_over_time": round(VALU_FLOOR_CONFIG4_US * 1e-6 / t, 3),
                                          "what": "HIP-graph replay, 8-bit image in, int32 logits out (launch and latency bound)"}
    if with_cpu:
        t0 = time.perf_counter()
        want = onet.run(layers, params, img_np)["fc"]
        ex["config4_resnet18_w1a2_batch8"]["cpu_oracle_s"] = round(time.perf_counter() - t0, 3)
        logits = net.forward(img)
        torch.cuda.synchronize()
        assert np.array_equal(logits.cpu().numpy(), want), "config 4: logits differ from the oracle"
        ex["config4_resnet18_w1a2_batch8"]["bit_exact_vs_oracle"] = True

    # Throughput at batch 128, the batch of the paper's throughput column (1.70e4 images/s on an RTX 3090: context).
    net128 = PackedNet(layers, params, 128)
    img128 = dev(wl.image_batch(2004, 128, 224))
    t128 = graph_time(lambda: net128.forward(img128), reps=1, replays=20)
    ex["config4_resnet18_w1a2_batch128"] = {"ms": round(t128 * 1e3, 4), "images_per_s": round(128 / t128),
                                            "library_calls": net128.launches}
    del net128, img128

    # AlexNet- and VGG-16-shaped chains (the paper's other two models, Sec. 6.2; layer shapes are this build's, the
    # paper prints none), batch 8, w1a2 after the 8-bit input layer; oracle check on the first images of the batch.
    for name, make, ncheck in (("alexnet_shaped_w1a2_batch8", wl.alexnet_layers, 8), ("vgg16_shaped_w1a2_batch8", wl.vgg16_layers, 2)):
        ls = make()
        ps = wl.network_params(ls)
        netx = PackedNet(ls, ps, 8)
        imgx_np = wl.image_batch(2006, 8, 224)
        imgx = dev(imgx_np)
        tx = graph_time(lambda: netx.forward(imgx), reps=1, replays=20)
        mx = sum(8 * L.Ho * L.Wo * L.Cout * L.Cin * L.R * L.S for L in ls if L.kind in ("conv", "fc"))
        ex[name] = {"ms": round(tx * 1e3, 4), "library_calls": netx.launches, "images_per_s": round(8 / tx),
                    "eff_tops": round(2.0 * mx / tx / 1e12, 2), "matrix_frac_vs_fp4_peak": round(2.0 * mx / tx / MFMA_FP4_PEAK, 4)}
        if with_cpu:
            t0 = time.perf_counter()
            wantx = onet.run(ls, ps, imgx_np[:ncheck])[ls[-1].name]
            ex[name]["cpu_oracle_s"] = round(time.perf_counter() - t0, 3)
            ex[name]["cpu_oracle_images"] = ncheck
            lx = netx.forward(imgx)
            torch.cuda.synchronize()
            assert np.array_equal(lx.cpu().numpy()[:ncheck], wantx), f"{name}: logits differ from the oracle"
            ex[name]["bit_exact_vs_oracle"] = True
        del netx, imgx

    # The network's input layer (8-bit image x 1-bit weights, 7 x 7 stride 2) in its three forms: the 8-bit integer
    # matrix instruction straight from the image, and receptive-field planes multiplied by the FP4 matrix-core
    # kernel (4 digit passes) or by the AND+popcount kernel (8 plane passes).
    L = layers[0]
    wv, sc1, bi1 = params[L.name]
    sc1, bi1 = dev(sc1), dev(bi1)
    d1 = B.Conv(8, L.H, L.W, L.Cin, L.Cout, L.R, L.S, L.stride, L.pad, L.p, L.q)
    out1 = torch.empty(B.apnn_fmap_words(8 * L.Ho * L.Wo, L.Cout, L.q_out), dtype=torch.int32, device="cuda")
    Wi = B.apnn_pack_input_weights(dev(wv), L.p, B.ENC_PM1)
    t_i8 = graph_time(lambda: B.apnn_input_layer(d1, Wi, img, q_out=L.q_out, scale=sc1, bias=bi1, out=out1))
    Wpp = B.apnn_pack_patch_weights(dev(wv), L.p, B.ENC_PM1)
    patches = torch.empty(B.apnn_packed_words(8 * L.Ho * L.Wo, 32 * L.R, L.q), dtype=torch.int32, device="cuda")
    dg = B.Conv(8 * L.Ho * L.Wo, 1, 1, 32 * L.R, L.Cout, 1, 1, 1, 0, L.p, L.q)

    def planes_form():
        B.apnn_pack_patches(img, L.R, L.S, L.stride, L.pad, L.q, out=patches)
        B.apnn_layer(dg, Wpp, patches, is_gemm=True, q_out=L.q_out, scale=sc1, bias=bi1, out=out1)
    B.apnn_debug_force("INT8", 0)
    t_fp4 = graph_time(planes_form)
    B.apnn_debug_force("MFMA", 0)
    t_pop = graph_time(planes_form)
    B.apnn_debug_reset()
    ex["config4_input_layer_us"] = {"int8_matrix_instruction_from_image": round(t_i8 * 1e6, 2),
                                    "patch_planes_fp4_matrix_kernel": round(t_fp4 * 1e6, 2),
                                    "patch_planes_and_popcount_kernel": round(t_pop * 1e6, 2)}
    return ex


if __name__ == "__main__":
    main()
