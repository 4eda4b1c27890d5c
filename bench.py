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
dominant kernel (FP4 matrix peak) measured with events around each of its
launches inside the timed region, the same for the AND + popcount kernel (VALU
bitwise+popcount issue rate), and the CPU oracle timed on a bounded row sample.
The other benchmark configurations and the paper's own layer shapes are
reported under "extra" (device time per launch via HIP-graph replay).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

VALU_PEAK_LANE_OPS = 256 * 64 * 2.4e9      # 256 CUs x 64 lanes/clk x 2.4 GHz (32-bit integer vector ops)
HBM_PEAK = 8.0e12
MFMA_FP4_PEAK = 10.1e15                    # dense FP4 matrix peak, FLOP/s


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
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import numpy as np
    import torch
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
        src = torch.zeros(1 << 28, dtype=torch.uint8, device="cuda")
        from paper_2106_12169_amd import bench_probes
        bench_probes.apnn_probe_copy(src, torch.empty_like(src))
    def timed(steps, warmup):
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        # events around the GEMM launch of every 4th step (each record is a command of its own on the stream)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) if i % 4 == 0 else None
               for i in range(steps)]
        t0 = time.perf_counter()
        for i in range(steps):
            step(evs[i])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        kern = np.array([e[0].elapsed_time(e[1]) for e in evs if e is not None]) * 1e-3
        return (t1 - t0) / steps, float(kern.mean())

    # headline: the library's own dispatch (FP4 matrix-core kernel for <= 2-bit operands)
    sec_per_step, gemm_s = timed(args.steps, args.warmup)
    flops = wk.effective_ops                                       # 2 M N K multiply-adds on the matrix cores
    # the AND + popcount kernel on the same workload (the VALU bitwise+popcount roofline)
    B.apnn_debug_force("MFMA", 0)
    _, pop_s = timed(max(args.steps // 4, 5), max(args.warmup // 4, 2))
    B.apnn_debug_reset()
    step()                                                         # leave the default path's result in Y
    torch.cuda.synchronize()
    lane_ops = 2.0 * wk.M * wk.N * wk.K * wk.p * wk.q / 32.0     # AND + popcount-accumulate per 32 bit-products

    # cheap self-check on the timed output (full parity lives in tests/)
    colsum = Y.sum(dim=0, dtype=torch.int64).cpu().numpy()
    want = Xv.astype(np.int64) @ Wv.astype(np.int64).sum(0)
    assert np.array_equal(colsum, want), "timed output failed its column-sum check"

    out = {
        "metric": "effective TOPS, w1a2 4096^3 bit-GEMM (2*M*N*K / time)",
        "value": round(wk.effective_ops / sec_per_step / 1e12, 2),
        "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 bit planes -> int32", "data": "synthetic",
        "config": {"workload": "config1: w1a2 GEMM M=N=K=4096, +-1 weights x unsigned 2-bit activations, int32 out",
                   "step": "apnn_pack(activations) + apnn_gemm", "seeds": [wk.seedW, wk.seedX]},
        "roofline": {
            "bound": "mfma", "kernel": "mfma_big_kernel<PM1,U2> (v_mfma_scale_f32_32x32x64_f8f6f4, FP4 E2M1)",
            "achieved": round(flops / gemm_s / 1e12, 1), "peak": MFMA_FP4_PEAK / 1e12, "unit": "TFLOP/s",
            "frac": round(flops / gemm_s / MFMA_FP4_PEAK, 4),
            "kernel_us": round(gemm_s * 1e6, 2),
            # HBM bytes per launch from rocprofv3 FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000 (KiB), see
            # profiles/mfma_big_kernel_gemm_w1a2_4096_hbm_counters.txt; algorithmic: 6 MiB in + 64 MiB out
            "traffic": 8355.1 * 2.0 * 1024 + 65536.0 * 1024,
            "algorithmic_bytes": (wk.M * wk.p + wk.N * wk.q) * (wk.K // 8) + 4 * wk.M * wk.N,
        },
        "roofline_popcount_kernel": {
            "bound": "alu", "kernel": "tile_kernel<4,4,16,4,4,false,false> (64x64 tile, v_and + v_bcnt), APNN_MFMA=0",
            "achieved": round(lane_ops / pop_s / 1e12, 3), "peak": round(VALU_PEAK_LANE_OPS / 1e12, 3),
            "unit": "T lane-op/s (32-bit VALU, 2 lane-ops per 32 bit-products per plane pair)",
            "frac": round(lane_ops / pop_s / VALU_PEAK_LANE_OPS, 4),
            "kernel_us": round(pop_s * 1e6, 2), "eff_tops": round(wk.effective_ops / pop_s / 1e12, 1),
            "traffic": 8300.7 * 2.0 * 1024 + 65536.0 * 1024,
        },
    }

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
        out["extra"] = extra_configs(B, wl, dev, graph_time)

    print(json.dumps(out), flush=True)


def extra_configs(B, wl, dev, graph_time):
    """Device time of the other benchmark configurations (HIP-graph replays)."""
    import torch
    from paper_2106_12169_amd.network import PackedNet
    ex = {}

    def gemm_case(wk):
        Wp = B.apnn_pack(dev(wk.weights()), wk.p, wk.encW)
        Xp = B.apnn_pack(dev(wk.activations()), wk.q, wk.encX)
        Y = torch.empty((wk.M, wk.N), dtype=torch.int32, device="cuda")
        t = graph_time(lambda: B.apnn_gemm(Wp, Xp, wk.M, wk.N, wk.K, wk.p, wk.q, wk.encW, wk.encX, out=Y))
        # the FP4 matrix-core kernel runs ceil(p/2)*ceil(q/2) base-4 digit passes of 2*M*N*K flops each
        passes = ((wk.p + 1) // 2) * ((wk.q + 1) // 2)
        return {"us": round(t * 1e6, 2), "eff_tops": round(wk.effective_ops / t / 1e12, 2),
                "digit_passes": passes, "fp4_mfma_frac": round(wk.effective_ops * passes / t / MFMA_FP4_PEAK, 4)}

    ex["config0_gemm_w1a2_128"] = gemm_case(wl.CONFIG0)
    ex["config2_sweep_2048"] = {f"w{wk.p}a{wk.q}": gemm_case(wk) for wk in wl.CONFIG2}

    c = wl.CONFIG3
    d = B.Conv(c.BS, c.H, c.W, c.Cin, c.Cout, c.R, c.S, c.stride, c.pad, c.p, c.q, c.encW, c.encX)
    Wp = B.apnn_pack_conv_weights(dev(c.weights_oihw()), c.p, c.encW)
    Xp = B.apnn_pack_fmap(dev(c.features_nchw()), B.LAYOUT_NCHW, c.q, c.encX)
    sc, bi = dev(c.scale()), dev(c.bias())
    outp = torch.empty(B.apnn_fmap_words(d.N * d.Ho * d.Wo, c.Cout, c.q_out), dtype=torch.int32, device="cuda")
    t = graph_time(lambda: B.apnn_layer(d, Wp, Xp, q_out=c.q_out, scale=sc, bias=bi, out=outp))
    ex["config3_conv_layer"] = {"us": round(t * 1e6, 2), "eff_tops": round(c.effective_ops / t / 1e12, 2),
                                "fp4_mfma_frac": round(c.effective_ops / t / MFMA_FP4_PEAK, 4),
                                "what": "fused conv + scale/bias + requantise + repack, packed in/out (latency bound)"}

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
        fc[f"w{w}a{a}"] = {str(dim): gemm_case(wl.paper_fc_workload(w, a, dim))["us"] for dim in wl.PAPER_FC_DIMS}
    ex["paper_fc_batch64_us_by_dim"] = fc
    cv = {}
    for ch in wl.PAPER_CONV_CHANNELS:
        c = wl.paper_conv_workload(ch)
        d = B.Conv(c.BS, c.H, c.W, c.Cin, c.Cout, c.R, c.S, c.stride, c.pad, c.p, c.q, c.encW, c.encX)
        Wp = B.apnn_pack_conv_weights(dev(c.weights_oihw()), c.p, c.encW)
        Xp = B.apnn_pack_fmap(dev(c.features_nchw()), B.LAYOUT_NCHW, c.q, c.encX)
        sc, bi = dev(c.scale()), dev(c.bias())
        outp = torch.empty(B.apnn_fmap_words(d.N * d.Ho * d.Wo, c.Cout, c.q_out), dtype=torch.int32, device="cuda")
        t = graph_time(lambda: B.apnn_layer(d, Wp, Xp, q_out=c.q_out, scale=sc, bias=bi, out=outp))
        cv[str(ch)] = round(t * 1e6, 2)
    ex["paper_conv_w1a2_16x16_batch1_us_by_channels"] = cv

    layers = wl.resnet18_layers()
    net = PackedNet(layers, wl.network_params(layers), 8)
    img = dev(wl.image_batch(2004, 8, 224))
    t = graph_time(lambda: net.forward(img), reps=1, replays=50)
    ex["config4_resnet18_w1a2_batch8"] = {"ms": round(t * 1e3, 4), "library_calls": net.launches,
                                          "what": "HIP-graph replay, 8-bit image in, int32 logits out"}

    # Throughput at batch 128, the batch of the paper's throughput column (1.70e4 images/s on an RTX 3090: context).
    net128 = PackedNet(layers, wl.network_params(layers), 128)
    img128 = dev(wl.image_batch(2004, 128, 224))
    t128 = graph_time(lambda: net128.forward(img128), reps=1, replays=20)
    ex["config4_resnet18_w1a2_batch128"] = {"ms": round(t128 * 1e3, 4), "images_per_s": round(128 / t128),
                                            "library_calls": net128.launches}
    del net128, img128

    # The network's input layer (8-bit image x 1-bit weights, 7 x 7 stride 2) in its three forms: the 8-bit integer
    # matrix instruction straight from the image, and receptive-field planes multiplied by the FP4 matrix-core
    # kernel (4 digit passes) or by the AND+popcount kernel (8 plane passes).
    L = layers[0]
    wv, sc1, bi1 = wl.network_params(layers)[L.name]
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
