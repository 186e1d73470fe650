#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: the sixteen binary 3x3 convolutions of a
Bi-Real-Net-18 body at 224x224 input, batch 256, each preceded by the bit-pack of its fp32
activation.  One step = 16 x (dabnn_bitpack + dabnn_bconv2d) over inputs resident in HBM.

Prints ONE JSON line.

  value            binary-convolution GOPS: 2*K*Cout*Ho*Wo*N summed over the 16 layers, divided by
                   the wall time of a whole step (bit-packing included), from a loop of exactly
                   --steps steps that carries no instrumentation.
  roofline         from a separate SAMPLING PASS after the headline loop: every launch of a step
                   is bracketed by HIP events on the launch stream, --samples times (default 24,
                   whatever --steps is); per layer the median and the minimum are kept.
                   achieved = sum of the layers' ops / sum of the layers' median intervals.
  configs          the other four benchmark configurations (single 14x14x64 convolution, the
                   stride-1 sweep at batch 1 and 64, the bit-pack shapes incl. C = 80 / 200, the
                   stride-2 layers at batch 128): microseconds, GOPS or GB/s, roofline fraction
                   and the oracle's time on the same tensors.  Never part of `value`.
  fused_bnsign, bireal_block_chain, batch1_chain_latency, int8_mfma_comparison,
  mfma_from_packed_bits_comparison
                   widened entry points on the same layers, timed after everything above.
  cpu_baseline     the CPU oracle on the same 16 layers, all host threads.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Peak of the plain-VALU path on MI355X, derived from the chip's unit counts and clock:
# 256 CUs x 64 lanes/clk x 2.4 GHz = 39.32 T lane-ops/s; one v_xor_b32 + one v_bcnt_u32_b32
# (popcount with fused accumulate) process 32 bits of one output, i.e. 64 counted binary ops per
# 2 lane-ops => 32 ops per lane-op => 1258.29 TOP/s.
VALU_PEAK_TOPS = 256 * 64 * 2.4e9 * 32 / 1e12
HBM_PEAK_GBPS = 8000.0
INFINITY_CACHE_BYTES = 256e6
# HBM bytes per step (16 launches each) at batch 256, from two rocprofv3 --pmc runs (FETCH_SIZE,
# then WRITE_SIZE) scaled by a plain 1 GiB copy; see profiles/bireal18_b256_hbm_traffic.md.
# Algorithmic: conv 1.597e9 (56 MB read + 1541 MB written), bit-pack 1.775e9.
MEASURED_TRAFFIC_B256 = {"bconv": 1.904e9, "bitpack": 1.775e9}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--samples", type=int, default=24,
                    help="event-bracketed samples per launch in the sampling pass (roofline)")
    ap.add_argument("--batch", type=int, default=None, help="override the batch (default 256)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip the other configs and the widened entry points (profiling runs)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device tensor copy (a kernel of known "
                         "HBM traffic) so that counter runs under rocprofv3 --pmc can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path would shard by batch: every image is "
              "independent and the packed weights are replicated). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1908_05858_amd import binding, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    binding.load()
    torch.cuda.set_device(0)
    N = args.batch or wl.CFG5_BATCH
    layers = wl.BIREAL18_BODY
    want_oracle = not args.no_cpu_baseline
    if want_oracle:
        import oracle
        oracle.build()

    def event():
        return torch.cuda.Event(enable_timing=True)

    def launch_us(fn, reps=20, inner=1):
        """Median and minimum, in microseconds per launch, of `reps` HIP-event intervals around
        `inner` back-to-back calls of fn() on the launch stream."""
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        evs = [(event(), event()) for _ in range(reps)]
        for e0, e1 in evs:
            e0.record()
            for _ in range(inner):
                fn()
            e1.record()
        torch.cuda.synchronize()
        us = sorted(e0.elapsed_time(e1) * 1e3 / inner for e0, e1 in evs)
        return us[len(us) // 2], us[0]

    def graph_us(fn, inner=20, reps=20):
        """Microseconds per launch (median, minimum) of `inner` calls of fn() captured into a HIP
        graph and replayed `reps` times between HIP events: what the launches take on the device
        when the host's launch rate (about 8 us per call from Python) is out of the way."""
        fn()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(inner):
                fn()
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        evs = [(event(), event()) for _ in range(reps)]
        for e0, e1 in evs:
            e0.record()
            graph.replay()
            e1.record()
        torch.cuda.synchronize()
        del graph
        us = sorted(e0.elapsed_time(e1) * 1e3 / inner for e0, e1 in evs)
        return us[len(us) // 2], us[0]

    def wall_ms(fn, reps):
        fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / reps

    # ---- inputs: seeded, synthetic, resident in HBM before any timing ---------------------
    xs, wps, acts, ys = [], [], [], []
    for li, L in enumerate(layers):
        x = wl.activations((N, L.H, L.W, L.Cin), wl.seed_for(5, 100 + li))
        xs.append(torch.from_numpy(x).cuda())
        wf = wl.weights((L.Cout, 3, 3, L.Cin), wl.seed_for(5, li))
        wps.append(binding.pack_weights(torch.from_numpy(wf).cuda()))
        acts.append(torch.empty((N, L.H, L.W, (L.Cin + 63) // 64), dtype=torch.int64, device="cuda"))
        ys.append(torch.empty((N, L.Ho, L.Wo, L.Cout), dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()

    def step():
        """One pass of the hot path."""
        for li, L in enumerate(layers):
            binding.bitpack(xs[li], out=acts[li])
            binding.bconv2d(acts[li], wps[li], L.Cin, L.stride, 1, out=ys[li])

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")  # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- headline: exactly K steps, nothing but the 32 launches of each step ---------------
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # ---- sampling pass: every launch of a step between HIP events, `samples` times ---------
    # The events sit on the stream the kernels are launched on.  An interval holds one kernel
    # plus the gap the command processor leaves between two dependent dispatches (about 3 us).
    S = max(1, args.samples)
    ev = [[[event() for _ in range(3)] for _ in layers] for _ in range(S)]
    torch.cuda.synchronize()
    for s in range(S):
        for li, L in enumerate(layers):
            ev[s][li][0].record()
            binding.bitpack(xs[li], out=acts[li])
            ev[s][li][1].record()
            binding.bconv2d(acts[li], wps[li], L.Cin, L.stride, 1, out=ys[li])
            ev[s][li][2].record()
    torch.cuda.synchronize()
    pack_us = np.array([[ev[s][li][0].elapsed_time(ev[s][li][1]) * 1e3 for li in range(len(layers))]
                        for s in range(S)])
    conv_us = np.array([[ev[s][li][1].elapsed_time(ev[s][li][2]) * 1e3 for li in range(len(layers))]
                        for s in range(S)])
    del ev
    pack_med, pack_min = np.median(pack_us, axis=0), pack_us.min(axis=0)
    conv_med, conv_min = np.median(conv_us, axis=0), conv_us.min(axis=0)

    # ---- the same launches without an event between them: the 16 bit-packs of a step back to
    # back, S times, between one pair of events; then the 16 convolutions likewise.  An event
    # interval of the sampling pass contains the event's own dispatch (1-2 us per launch); these
    # two figures do not, and are what the kernel durations of a rocprofv3 trace add up to.
    def pass_us(launch_all):
        launch_all()
        torch.cuda.synchronize()
        e0, e1 = event(), event()
        e0.record()
        for _ in range(S):
            launch_all()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / S

    def all_packs():
        for li in range(len(layers)):
            binding.bitpack(xs[li], out=acts[li])

    def all_convs():
        for li, L in enumerate(layers):
            binding.bconv2d(acts[li], wps[li], L.Cin, L.stride, 1, out=ys[li])
    pack_pass = pass_us(all_packs)
    conv_pass = pass_us(all_convs)

    ops = [L.ops(N) for L in layers]
    total_ops = float(sum(ops))
    pack_bytes = [xs[li].numel() * 4 + acts[li].numel() * 8 for li in range(len(layers))]
    conv_tops = total_ops / (conv_med.sum() * 1e-6) / 1e12       # conv launches only
    pack_gbps = sum(pack_bytes) / (pack_med.sum() * 1e-6) / 1e9  # bit-pack launches only
    per_layer = []
    for li, L in enumerate(layers):
        per_layer.append({
            "layer": f"{L.H}x{L.W}x{L.Cin}->{L.Cout}s{L.stride}",
            "bconv_us_median": round(float(conv_med[li]), 2), "bconv_us_min": round(float(conv_min[li]), 2),
            "bconv_TOPs": round(ops[li] / (conv_med[li] * 1e-6) / 1e12, 1),
            "bconv_frac_of_valu_peak": round(ops[li] / (conv_med[li] * 1e-6) / 1e12 / VALU_PEAK_TOPS, 4),
            "bitpack_us_median": round(float(pack_med[li]), 2), "bitpack_us_min": round(float(pack_min[li]), 2),
            "bitpack_GBps": round(pack_bytes[li] / (pack_med[li] * 1e-6) / 1e9, 1),
        })

    result = {
        "metric": "binary conv GOPS (2*K*Cout*Hout*Wout*N / s) + bitpack GB/s, % of roofline",
        "value": round(total_ops / (ms_per_step * 1e-3) / 1e9, 1),
        "unit": "GOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u64 packed bits, int32 accumulate",
        "data": "synthetic",
        "config": {
            "workload": f"Bi-Real-Net-18 binary body, 224x224 input, batch {N}: 16 x (bitpack fp32 NHWC "
                        "+ binary 3x3 conv), BASELINE.json configs[4]",
            "batch": N,
            "layers": len(layers),
            "binary_ops_per_step": total_ops,
        },
        "event_samples_per_layer": S,
        "bconv_only_GOPS": round(conv_tops * 1e3, 1),
        "bconv_frac_of_valu_peak": round(conv_tops / VALU_PEAK_TOPS, 4),
        "bitpack_GBps": round(pack_gbps, 1),
        "bitpack_frac_of_hbm_peak": round(pack_gbps / HBM_PEAK_GBPS, 4),
        "roofline": {
            "kernel": "bconv (all 16 launches of dabnn_bconv2d in a step)",
            "bound": "alu",
            "achieved": round(conv_tops, 2),
            "peak": round(VALU_PEAK_TOPS, 2),
            "unit": "TOP/s",
            "frac": round(conv_tops / VALU_PEAK_TOPS, 4),
            "frac_from_minimum_intervals": round(total_ops / (conv_min.sum() * 1e-6) / 1e12 / VALU_PEAK_TOPS, 4),
            "samples_per_launch": S,
            "back_to_back": {"what": f"the 16 conv launches of a step with no event between them, {S} times",
                             "us_per_step": round(conv_pass, 1),
                             "achieved": round(total_ops / (conv_pass * 1e-6) / 1e12, 2),
                             "frac": round(total_ops / (conv_pass * 1e-6) / 1e12 / VALU_PEAK_TOPS, 4)},
            "traffic": MEASURED_TRAFFIC_B256["bconv"] if N == 256 else None,
            "traffic_note": "HBM bytes per step over the 16 conv launches (algorithmic 1.597e9)",
        },
        "roofline_bitpack": {
            "kernel": "bitpack (all 16 launches of dabnn_bitpack in a step)",
            "bound": "hbm",
            "achieved": round(pack_gbps, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(pack_gbps / HBM_PEAK_GBPS, 4),
            "samples_per_launch": S,
            "back_to_back": {"what": f"the 16 bit-pack launches of a step with no event between them, {S} times",
                             "us_per_step": round(pack_pass, 1),
                             "achieved": round(sum(pack_bytes) / (pack_pass * 1e-6) / 1e9, 1),
                             "frac": round(sum(pack_bytes) / (pack_pass * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)},
            "traffic": MEASURED_TRAFFIC_B256["bitpack"] if N == 256 else None,
            "traffic_note": "HBM bytes per step over the 16 bit-pack launches (algorithmic 1.775e9)",
        },
        "per_layer": per_layer,
    }

    # The largest bit-pack shape of the parity configs (256x56x56x256, 822 MB of fp32), far beyond
    # the 256 MB Infinity Cache: the launch the HBM fraction of the bit-pack kernel is claimed on.
    if N == wl.CFG5_BATCH:
        shape = wl.CFG3_SHAPES[2]
        xb = torch.empty(shape, dtype=torch.float32, device="cuda").normal_()
        ob = torch.empty(shape[:-1] + ((shape[-1] + 63) // 64,), dtype=torch.int64, device="cuda")
        med, mn = launch_us(lambda: binding.bitpack(xb, out=ob), reps=max(10, S))
        moved = xb.numel() * 4 + ob.numel() * 8
        result["roofline_bitpack"]["largest_launch"] = {
            "shape": "x".join(map(str, shape)), "MB_moved": round(moved / 1e6, 1),
            "median_us": round(med, 2), "min_us": round(mn, 2),
            "GBps_median": round(moved / med / 1e3, 1),
            "frac_of_hbm_peak": round(moved / med / 1e3 / HBM_PEAK_GBPS, 4)}
        del xb, ob

    # The sections below are reported beside the headline; a failure in one of them is recorded in
    # the line instead of losing the headline that is already measured.
    if not args.headline_only:
        try:
            result["configs"] = other_configs(binding, wl, np, torch, launch_us, graph_us, want_oracle)
        except Exception as e:  # noqa: BLE001
            result["configs_error"] = repr(e)
        try:
            widened_rows(result, args, binding, wl, np, torch, layers, N, xs, acts, wps, ys, total_ops, wall_ms,
                         launch_us)
        except Exception as e:  # noqa: BLE001
            result["widened_rows_error"] = repr(e)

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same workload ----
    if want_oracle:
        n_img = N
        cpu_x = [x.cpu().numpy() for x in xs]
        cpu_w = [wl.weights((L.Cout, 3, 3, L.Cin), wl.seed_for(5, li)) for li, L in enumerate(layers)]
        oracle.sign(cpu_x[0][:1])  # load the library and start the thread pool outside the timing
        c0 = time.perf_counter()
        passes = 0
        while passes == 0 or (time.perf_counter() - c0 < 10.0 and passes < 8):
            for li, L in enumerate(layers):
                oracle.bitpack(cpu_x[li])
                oracle.bconv2d_signed(oracle.sign(cpu_x[li]), oracle.sign(cpu_w[li]), L.stride, 1)
            passes += 1
        c1 = time.perf_counter()
        cpu_ops = float(sum(L.ops(n_img) for L in layers)) * passes
        threads = int(os.environ.get("OMP_NUM_THREADS", 0)) or len(os.sched_getaffinity(0))
        result["cpu_baseline"] = {
            "value": round(cpu_ops / (c1 - c0) / 1e9, 2),
            "unit": "GOPS",
            "cores": threads,
            "kind": "oracle",
            "sample": f"the same 16 layers (sign + bit-pack + float +-1 conv) on all {n_img} images, "
                      f"{passes} pass(es), {c1 - c0:.1f} s",
        }

    print(json.dumps(result))


def other_configs(binding, wl, np, torch, launch_us, graph_us, want_oracle):
    """The other four benchmark configurations (single conv, stride-1 sweep, bit-pack shapes,
    stride-2 layers): per launch microseconds (median of 20 HIP-event intervals),
    throughput, roofline fraction, and the oracle's wall time for the same tensors on the host.
    A short launch (below 40 us) is of the order of what the host takes to issue it from Python
    and of what an event pair adds, so it is timed as 20 launches replayed from a HIP graph (the
    device's time per launch, `us`), with the eager host-issued figure beside it (`eager_us`)."""

    def timed(fn):
        med, _ = launch_us(fn)
        if med >= 40.0:
            return med, None
        eager, _ = launch_us(fn, inner=20)
        med, _ = graph_us(fn)
        return med, eager

    if want_oracle:
        import oracle
    out = {}

    def conv_row(L, n, seed, p_plus=0.5):
        x = wl.activations((n, L.H, L.W, L.Cin), seed)
        wf = wl.weights((L.Cout, 3, 3, L.Cin), seed + 1, p_plus)
        xg = torch.from_numpy(x).cuda()
        wp = binding.pack_weights(torch.from_numpy(wf).cuda())
        a = binding.bitpack(xg)
        y = torch.empty((n, L.Ho, L.Wo, L.Cout), dtype=torch.int32, device="cuda")
        conv = lambda: binding.bconv2d(a, wp, L.Cin, L.stride, 1, out=y)
        pack = lambda: binding.bitpack(xg, out=a)
        med, eager = timed(conv)
        pmed, peager = timed(pack)
        ops = L.ops(n)
        moved = x.size * 4 + a.numel() * 8
        row = {"layer": f"{L.H}x{L.W}x{L.Cin}->{L.Cout}s{L.stride}", "batch": n,
               "bconv_us": round(med, 2), "bconv_GOPS": round(ops / med / 1e3, 1),
               "bconv_frac_of_valu_peak": round(ops / med / 1e6 / VALU_PEAK_TOPS, 4),
               "bitpack_us": round(pmed, 2), "bitpack_GBps": round(moved / pmed / 1e3, 1)}
        if eager is not None:
            row["bconv_eager_us"] = round(eager, 2)
        if peager is not None:
            row["bitpack_eager_us"] = round(peager, 2)
        # fewer outputs than the chip has lanes in flight: the launch is latency-bound
        if n * L.Ho * L.Wo * L.Cout < 256 * 4 * 64 * 16:
            row["note"] = "latency-bound: fewer outputs than resident lanes x 16 channels"
        if want_oracle:
            t = time.perf_counter()
            oracle.bconv2d(x, wf, L.stride, 1)
            dt = time.perf_counter() - t
            row["oracle_ms"] = round(dt * 1e3, 2)
            row["oracle_GOPS"] = round(ops / dt / 1e9, 1)
        return row

    def word_count_row(Cin, n=64, hw=14, Cout=256):
        """A channel count outside the benchmark configs (3, 5, 6, 7 or 16 words per pixel): the
        tuned family against the one-thread-per-output reference kernel."""
        x = torch.randn((n, hw, hw, Cin), device="cuda")
        wp = binding.pack_weights(torch.randn((Cout, 3, 3, Cin), device="cuda"))
        a = binding.bitpack(x)
        y = torch.empty((n, hw, hw, Cout), dtype=torch.int32, device="cuda")
        tuned, _ = launch_us(lambda: binding.bconv2d(a, wp, Cin, 1, 1, out=y))
        ref, _ = launch_us(lambda: binding.bconv2d(a, wp, Cin, 1, 1, out=y, algo=binding.ALGO_REFERENCE), reps=5)
        ops = 2.0 * 9 * Cin * Cout * hw * hw * n
        return {"layer": f"{hw}x{hw}x{Cin}->{Cout}s1", "batch": n, "words_per_pixel": (Cin + 63) // 64,
                "algo": binding.pick_algo(n, hw, hw, Cin, Cout, 3, 3, 1, 1),
                "bconv_us": round(tuned, 2), "bconv_GOPS": round(ops / tuned / 1e3, 1),
                "bconv_frac_of_valu_peak": round(ops / tuned / 1e6 / VALU_PEAK_TOPS, 4),
                "reference_kernel_us": round(ref, 2)}

    out["cfg1_single_conv"] = conv_row(wl.CFG1_LAYER, 1, wl.seed_for(1))
    out["cfg2_stride1_sweep"] = [conv_row(L, n, wl.seed_for(2, li))
                                 for li, L in enumerate(wl.CFG2_LAYERS) for n in wl.CFG2_BATCHES]
    out["cfg4_stride2_batch128"] = [conv_row(L, wl.CFG4_BATCH, wl.seed_for(4, li), wl.CFG4_P_PLUS)
                                    for li, L in enumerate(wl.CFG4_LAYERS)]
    rows = []
    for shape in wl.CFG3_SHAPES:
        x = wl.inject_zeros(wl.activations(shape, wl.seed_for(3, shape[-1] + shape[0])), wl.seed_for(3, 1))
        xg = torch.from_numpy(x).cuda()
        o = torch.empty(shape[:-1] + ((shape[-1] + 63) // 64,), dtype=torch.int64, device="cuda")
        f = lambda: binding.bitpack(xg, out=o)
        med, eager = timed(f)
        moved = x.size * 4 + o.numel() * 8
        row = {"shape": "x".join(map(str, shape)), "MB_moved": round(moved / 1e6, 3), "us": round(med, 2),
               "GBps": round(moved / med / 1e3, 1),
               "frac_of_hbm_peak": round(moved / med / 1e3 / HBM_PEAK_GBPS, 4)}
        if eager is not None:
            row["eager_us"] = round(eager, 2)
        if moved < INFINITY_CACHE_BYTES:
            row["note"] = ("latency-bound" if med < 5.0 else "cache-resident") + \
                          ": the tensor fits the 256 MB Infinity Cache, not an HBM figure"
        if want_oracle:
            t = time.perf_counter()
            oracle.bitpack(x)
            dt = time.perf_counter() - t
            row["oracle_ms"] = round(dt * 1e3, 3)
            row["oracle_GBps"] = round(moved / dt / 1e9, 2)
        rows.append(row)
        del xg, o
    out["cfg3_bitpack"] = rows
    # The same ragged channel counts on tensors far beyond the Infinity Cache: the HBM figure of
    # the bit-pack kernel for channel counts that are no multiple of 64 (device-generated input).
    rows = []
    for shape in ((256, 56, 56, 80), (256, 56, 56, 200), (256, 56, 56, 65)):
        xg = torch.empty(shape, dtype=torch.float32, device="cuda").normal_()
        o = torch.empty(shape[:-1] + ((shape[-1] + 63) // 64,), dtype=torch.int64, device="cuda")
        med, _ = launch_us(lambda: binding.bitpack(xg, out=o))
        moved = xg.numel() * 4 + o.numel() * 8
        rows.append({"shape": "x".join(map(str, shape)), "MB_moved": round(moved / 1e6, 1), "us": round(med, 2),
                     "GBps": round(moved / med / 1e3, 1),
                     "frac_of_hbm_peak": round(moved / med / 1e3 / HBM_PEAK_GBPS, 4)})
        del xg, o
    out["bitpack_ragged_channels_large"] = rows
    out["other_word_counts"] = [word_count_row(c) for c in (160, 320, 384, 448, 1024)]
    return out


def widened_rows(result, args, binding, wl, np, torch, layers, N, xs, acts, wps, ys, total_ops, wall_ms, launch_us):
    """Widened entry points on the same 16 layers; reported beside the headline, never in it."""
    reps = max(4, args.steps // 4)
    # conv + BN threshold + bit-pack of the result in one kernel: packed words in, packed words out
    if all(L.Cout % 64 == 0 for L in layers):
        rng = np.random.default_rng(wl.seed_for(5, 999))
        fused_args = []
        for li, L in enumerate(layers):
            thr, flip = binding.bn_thresholds(rng.uniform(0.5, 1.5, L.Cout), rng.normal(0, 0.3, L.Cout),
                                              rng.normal(0, 5, L.Cout), rng.uniform(1, 30, L.Cout),
                                              1e-5, L.K)
            out = torch.empty((N, L.Ho, L.Wo, L.Cout // 64), dtype=torch.int64, device="cuda")
            fused_args.append((thr, flip, out))

        def fused_step():
            for li, L in enumerate(layers):
                thr, flip, out = fused_args[li]
                binding.bconv2d_bnsign(acts[li], wps[li], thr, flip, L.Cin, L.stride, 1, out=out)
        fused_ms = wall_ms(fused_step, reps)
        result["fused_bnsign"] = {
            "what": "16 x dabnn_bconv2d_bnsign (conv + BN threshold + bit-pack of the result in one "
                    "kernel), packed input resident",
            "ms_per_step": round(fused_ms, 4),
            "GOPS": round(total_ops / (fused_ms * 1e-3) / 1e9, 1),
            "frac_of_valu_peak": round(total_ops / (fused_ms * 1e-3) / 1e12 / VALU_PEAK_TOPS, 4),
        }
        # the same fused layer on the matrix-core comparison route (dabnn_bconv2d_bnsign_mfma)
        if all(binding.mfma_weights_bytes(L.Cin, L.Cout) > 0 for L in layers):
            for name, fmt in (("int8", binding.MFMA_INT8), ("fp4", binding.MFMA_FP4)):
                wqs = [binding.prepare_weights_mfma(wps[li], L.Cin, fmt=fmt) for li, L in enumerate(layers)]

                def fused_mfma_step():
                    for li, L in enumerate(layers):
                        thr, flip, out = fused_args[li]
                        binding.bconv2d_bnsign_mfma(acts[li], wqs[li], thr, flip, L.Cin, L.Cout, L.stride, 1,
                                                    out=out, fmt=fmt)
                ms = wall_ms(fused_mfma_step, reps)
                result["fused_bnsign"][f"mfma_{name}_comparison_ms_per_step"] = round(ms, 4)
                del wqs
        del fused_args

        # The body with its real data dependencies (Sec. 2.3's network): each convolution reads the
        # bits the previous block produced, and the BN + shortcut + sign + pack layer turns its
        # output, plus the real-valued shortcut, into the next block's bits and shortcut.  Where
        # the shape changes (stride 2) a resident synthetic tensor stands in for the float
        # downsampling shortcut.
        scales = [torch.full((L.Cout,), 1.0 / (L.K ** 0.5), dtype=torch.float32, device="cuda") for L in layers]
        shifts = [torch.from_numpy(wl.affine(L.Cout, wl.seed_for(5, 200 + li))[1]).cuda() for li, L in enumerate(layers)]
        zs = [torch.empty((N, L.Ho, L.Wo, L.Cout), dtype=torch.float32, device="cuda") for L in layers]
        bits_out = [torch.empty((N, L.Ho, L.Wo, L.Cout // 64), dtype=torch.int64, device="cuda") for L in layers]
        down = {li: torch.randn((N, L.Ho, L.Wo, L.Cout), device="cuda") for li, L in enumerate(layers)
                if li == 0 or L.stride != 1}

        def chain_step(fused):
            a_in = acts[0]
            for li, L in enumerate(layers):
                r = down[li] if li in down else zs[li - 1]
                if fused:
                    binding.bconv2d_bn_residual(a_in, wps[li], scales[li], shifts[li], r, L.Cin, L.stride, 1,
                                                x_out=zs[li], out=bits_out[li])
                else:
                    binding.bconv2d(a_in, wps[li], L.Cin, L.stride, 1, out=ys[li])
                    binding.bn_sign_pack(ys[li], scales[li], shifts[li], r, x_out=zs[li], out=bits_out[li])
                a_in = bits_out[li]
        chain_ms = [wall_ms(lambda: chain_step(f), reps) for f in (False, True)]
        result["bireal_block_chain"] = {
            "what": "16 dependent blocks: binary conv on the previous block's bits, then BN + real-valued "
                    "shortcut + sign + bit-pack producing the next block's bits and shortcut; as two "
                    "calls per block (dabnn_bconv2d, dabnn_bn_sign_pack) and as one "
                    "(dabnn_bconv2d_bn_residual)",
            "two_calls_per_block_ms_per_step": round(chain_ms[0], 4),
            "two_calls_per_block_GOPS": round(total_ops / (chain_ms[0] * 1e-3) / 1e9, 1),
            "one_call_per_block_ms_per_step": round(chain_ms[1], 4),
            "one_call_per_block_GOPS": round(total_ops / (chain_ms[1] * 1e-3) / 1e9, 1),
        }
        del zs, bits_out, down

        # Batch-1 latency of the dependent 16-block chain (the paper's deployment case is one image
        # at a time): launch-bound, so it is also replayed from a HIP graph.
        a1 = torch.zeros((1, layers[0].H, layers[0].W, layers[0].Cin // 64), dtype=torch.int64, device="cuda")
        z1 = [torch.empty((1, L.Ho, L.Wo, L.Cout), dtype=torch.float32, device="cuda") for L in layers]
        b1 = [torch.empty((1, L.Ho, L.Wo, L.Cout // 64), dtype=torch.int64, device="cuda") for L in layers]
        d1 = {li: torch.randn((1, L.Ho, L.Wo, L.Cout), device="cuda") for li, L in enumerate(layers)
              if li == 0 or L.stride != 1}
        sh1 = [torch.zeros((L.Cout,), dtype=torch.float32, device="cuda") for L in layers]

        def one_image():
            a_in = a1
            for li, L in enumerate(layers):
                r = d1[li] if li in d1 else z1[li - 1]
                binding.bconv2d_bn_residual(a_in, wps[li], scales[li], sh1[li], r, L.Cin, L.stride, 1,
                                            x_out=z1[li], out=b1[li])
                a_in = b1[li]
        # Small launches take the call's two-kernel route (less device time, one launch more):
        # both routes, issued eagerly from this process (bound by the host's launch cost) and
        # replayed from a HIP graph (device time).
        lat = {}
        for name, route in (("", 0), ("_one_kernel_route", 1)):
            binding.set_option(binding.OPT_RES_FUSED, route)
            lat["eager_us" + name] = round(wall_ms(one_image, 200) * 1e3, 1)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                one_image()
            lat["hip_graph_replay_us" + name] = round(wall_ms(graph.replay, 200) * 1e3, 1)
            del graph
        binding.set_option(binding.OPT_RES_FUSED, 0)
        result["batch1_chain_latency"] = {
            "what": "16 dependent blocks (dabnn_bconv2d_bn_residual) on one 224x224 image's feature maps; the "
                    "library's choice for launches this small (convolution + layer kernel) and, forced, the "
                    "one-kernel route of the larger batches", **lat}

    # Comparison row: the same convolutions on the int8 matrix cores with every bit expanded to a
    # +-1 byte (dabnn_expand_int8 + dabnn_bconv2d_int8).  One step = 16 x (expand the packed
    # activations, convolve); filters are expanded ahead of time like they are packed ahead of time.
    if all(L.Cin % 64 == 0 and L.Cout % 64 == 0 for L in layers):
        w8s = [binding.expand_int8(wps[li], L.Cin) for li, L in enumerate(layers)]
        a8s = [torch.empty((N, L.H, L.W, L.Cin), dtype=torch.int8, device="cuda") for L in layers]

        def mfma_step(expand=True):
            for li, L in enumerate(layers):
                if expand:
                    binding.expand_int8(acts[li], L.Cin, out=a8s[li])
                binding.bconv2d_int8(a8s[li], w8s[li], L.stride, 1, out=ys[li])
        mfma_ms = wall_ms(mfma_step, reps)
        mfma_conv_ms = wall_ms(lambda: mfma_step(expand=False), reps)
        result["int8_mfma_comparison"] = {
            "what": "16 x (dabnn_expand_int8 of the packed activations + dabnn_bconv2d_int8 on "
                    "v_mfma_i32_32x32x32_i8), same outputs.  A measured data point of an UNTUNED "
                    "implicit GEMM (LDS-bandwidth-bound 64x64 wavefront tiles), not a verdict on "
                    "the matrix-core route",
            "ms_per_step": round(mfma_ms, 4),
            "GOPS": round(total_ops / (mfma_ms * 1e-3) / 1e9, 1),
            "conv_only_ms_per_step": round(mfma_conv_ms, 4),
            "conv_only_GOPS": round(total_ops / (mfma_conv_ms * 1e-3) / 1e9, 1),
            "conv_only_frac_of_int8_mfma_peak": round(total_ops / (mfma_conv_ms * 1e-3) / 5.0e15, 4),
        }
        del w8s, a8s

    # Second comparison row: the matrix cores fed from the PACKED activations
    # (dabnn_bconv2d_mfma; only the filters are expanded, ahead of time like they are packed ahead
    # of time), with int8 and with FP4 operands.  The step is the headline step with dabnn_bconv2d
    # replaced by it; per layer, HIP event intervals of the same launches beside those of the
    # XOR/popcount kernel.
    if all(binding.mfma_weights_bytes(L.Cin, L.Cout) > 0 for L in layers):
        peaks = {"int8": 5.0e15, "fp4": 10.1e15}
        per_format = {}
        for name, fmt in (("int8", binding.MFMA_INT8), ("fp4", binding.MFMA_FP4)):
            wqs = [binding.prepare_weights_mfma(wps[li], L.Cin, fmt=fmt) for li, L in enumerate(layers)]

            def bits_step(conv_only=False):
                for li, L in enumerate(layers):
                    if not conv_only:
                        binding.bitpack(xs[li], out=acts[li])
                    binding.bconv2d_mfma(acts[li], wqs[li], L.Cin, L.Cout, L.stride, 1, out=ys[li], fmt=fmt)
            bits_ms = wall_ms(bits_step, reps)
            bits_conv_ms = wall_ms(lambda: bits_step(conv_only=True), reps)
            rows, seen = [], set()
            for li, L in enumerate(layers):
                key = (L.H, L.Cin, L.Cout, L.stride)
                if key in seen:
                    continue
                seen.add(key)
                t_mfma, _ = launch_us(lambda: binding.bconv2d_mfma(acts[li], wqs[li], L.Cin, L.Cout, L.stride, 1,
                                                                    out=ys[li], fmt=fmt))
                t_valu, _ = launch_us(lambda: binding.bconv2d(acts[li], wps[li], L.Cin, L.stride, 1, out=ys[li]))
                rows.append({"layer": f"{L.H}x{L.W}x{L.Cin}->{L.Cout}s{L.stride}", "mfma_us": round(t_mfma, 2),
                             "mfma_frac_of_peak": round(L.ops(N) / (t_mfma * 1e-6) / peaks[name], 4),
                             "xor_popcount_us": round(t_valu, 2)})
            per_format[name] = {
                "ms_per_step": round(bits_ms, 4),
                "GOPS": round(total_ops / (bits_ms * 1e-3) / 1e9, 1),
                "conv_only_ms_per_step": round(bits_conv_ms, 4),
                "conv_only_GOPS": round(total_ops / (bits_conv_ms * 1e-3) / 1e9, 1),
                "conv_only_frac_of_mfma_peak": round(total_ops / (bits_conv_ms * 1e-3) / peaks[name], 4),
                "mfma_peak_TOPs": peaks[name] / 1e12,
                "per_layer": rows,
            }
            del wqs
        result["mfma_from_packed_bits_comparison"] = {
            "what": "the headline step with dabnn_bconv2d replaced by dabnn_bconv2d_mfma: matrix "
                    "instructions (int8 v_mfma_i32_32x32x32_i8, or FP4 v_mfma_scale_f32_32x32x64_f8f6f4) "
                    "whose activation operand is expanded from the packed words inside the kernel "
                    "(one AND per operand register) and whose filters are prepared once per model; "
                    "same int32 outputs.  A comparison, not the method's path: the headline stays "
                    "XOR + popcount",
            **per_format,
        }


if __name__ == "__main__":
    main()
