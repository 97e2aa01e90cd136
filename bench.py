#!/usr/bin/env python3
"""Benchmark of the TernGrad hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic
gradients: tg_clip_stats -> tg_share_scalers -> tg_ternarize_pack ->
tg_unpack_average for all W simulated workers (W gradient buffers on the one
device).  Inputs are resident in HBM before the timed region.  Prints ONE JSON
line; `value` is fp32 gradient bytes consumed per second (W * n * 4 B / step).

The default run times the largest single-GPU configuration (C5: one flat layer of 10^9 elements, W = 8)
as the headline and, in the same JSON line under "other_configs", the AlexNet-shaped (C2) and
VGG-A-shaped (C4) ones.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload flat] [--also alexnet,vgg_a]
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="flat",
                    choices=["lenet", "alexnet", "googlenet_like", "vgg_a", "flat"])
    ap.add_argument("--also", default="alexnet,vgg_a",
                    help="comma-separated workloads timed after the headline one and reported under "
                         "other_configs ('' for none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--ceilings", action="store_true",
                    help="instead of the step: what the memory system sustains for the kernels' access "
                         "patterns with the arithmetic taken out (libbench_probe.so), on 4 GB buffers")
    ap.add_argument("--ceilings-elements", type=int, default=1 << 30,
                    help="floats per buffer for --ceilings (a multiple of 1024)")
    return ap.parse_args()


def traffic_profile_path(kernel: str, workload: str) -> str:
    return os.path.join("profiles", "%s_%s_pmc.txt" % (kernel, workload))


def traffic_from_profile(kernel: str, workload: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE, each scaled by a plain copy of known size), or None.  The counters need two profiler
    runs of their own, so the figure is read from that summary, never measured in the timed run."""
    path = os.path.join(ROOT, traffic_profile_path(kernel, workload))
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch="):
            return float(line.split("=", 1)[1])
    return None


def pattern_ceiling():
    """GB/s the bare traffic pattern of ternarize_pack reaches (committed probe run), or None"""
    path = os.path.join(ROOT, "profiles", "hbm_ceilings_probe.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if f and f[0] == "read_nt_with_thin_write" and "GB/s" in f:
            return float(f[f.index("GB/s") - 1])
    return None


def cpu_baseline(wl, grads_host, sample_note):
    """The oracle as it stands, all host cores, same four calls over the W workers."""
    import numpy as np
    import oracle
    cores = len(os.sched_getaffinity(0))
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
    used = oracle.set_threads(cores)
    try:
        off = wl.offsets
        reps, t0 = 0, time.perf_counter()
        # repeat the step until about 15 core-seconds of oracle work have been timed (at most 8 times)
        while reps < 8 and (reps == 0 or (time.perf_counter() - t0) * used < 15.0):
            st = [oracle.clip_stats(g, off, wl.clip_c) for g in grads_host]
            tau = [s[0] for s in st]
            s_shared = oracle.share_scalers(np.stack([s[1] for s in st]))
            codes = [oracle.ternarize_pack(g, off, tau[w], s_shared, wl.seed, wl.step + reps, w)
                     for w, g in enumerate(grads_host)]
            oracle.unpack_average(codes, off, s_shared)
            reps += 1
        dt = (time.perf_counter() - t0) / reps
    finally:
        oracle.set_threads(1)
    in_bytes = sum(g.size for g in grads_host) * 4.0
    res = {"value": in_bytes / dt / 1e9, "unit": "GB/s", "cores": used, "kind": "oracle",
           "sample": "%s, mean of %d repetitions" % (sample_note, reps), "seconds": dt}
    # the same oracle on ONE thread, on a smaller sample: worker 0's clip_stats + ternarize_pack and
    # its share of unpack_average (the decode of its own code buffer)
    g0 = grads_host[0]
    t0 = time.perf_counter()
    tau0, s0 = oracle.clip_stats(g0, off, wl.clip_c)
    c0 = oracle.ternarize_pack(g0, off, tau0, s0, wl.seed, wl.step, 0)
    oracle.unpack_average([c0], off, s0)
    dt1 = time.perf_counter() - t0
    res["single_thread"] = {"value": round(g0.size * 4.0 / dt1 / 1e9, 3), "unit": "GB/s", "cores": 1,
                            "sample": "worker 0 only: clip_stats, ternarize_pack, decode of its codes",
                            "seconds": round(dt1, 2)}
    return res


_PROBE = None


def probe_lib():
    """libbench_probe.so (bench_probe.hip, built by __graft_entry__.build()): the kernels' access
    patterns without arithmetic.  A measurement instrument of this file, not part of the library."""
    global _PROBE
    if _PROBE is None:
        path = os.path.join(ROOT, "libbench_probe.so")
        if not os.path.exists(path):
            from paper_1705_07878_amd import build
            build.build_probe(force=True, verbose=False)
        _PROBE = ctypes.CDLL(path)
        _PROBE.bench_probe.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_int64, ctypes.c_void_p]
        _PROBE.bench_probe.restype = ctypes.c_int
    return _PROBE


def bench_probe(torch, kind, src, dst, thin, n):
    ptr = lambda t: None if t is None else ctypes.c_void_p(t.data_ptr())
    rc = probe_lib().bench_probe(int(kind), ptr(src), ptr(dst), ptr(thin), int(n),
                                 ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    if rc != 0:
        raise RuntimeError("bench_probe(kind=%d) failed: %d" % (kind, rc))


def ceilings(torch, n=1 << 30, reps=10):
    """GB/s of the probe kernels over n floats: same launch shape as the real kernels, no arithmetic"""
    src = torch.empty((n,), dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty((n,), dtype=torch.float32, device="cuda")
    thin = torch.empty((n // 16,), dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    kinds = [(0, "read", 4.0), (1, "read_nt", 4.0), (2, "write_nt", 4.0), (5, "write_nt_cooperative", 4.0),
             (6, "write_one_store_per_wave", 4.0), (3, "copy_nt", 8.0), (7, "copy_one_access_per_wave", 8.0),
             (4, "read_nt_with_thin_write", 4.25), (8, "read_nt_with_thin_write_kept_in_L2", 4.0),
             (9, "read_nt_one_shot_1024_threads_xcd_order", 4.0), (10, "read_nt_wave_per_KiB_xcd_order", 4.0)]
    out = {}
    for kind, name, bytes_per_elem in kinds:
        for _ in range(3):
            bench_probe(torch, kind, src, dst, thin, n)
        e0.record(stream)
        for _ in range(reps):
            bench_probe(torch, kind, src, dst, thin, n)
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        gbs = n * bytes_per_elem / (ms * 1e-3) / 1e9
        out[name] = {"ms": round(ms, 4), "GBps": round(gbs, 1), "pct_hbm_peak": round(100 * gbs / HBM_PEAK_GBS, 1)}
    # the footprint of the flat 1e9 workload: 8 n floats in ONE launch, as the kernels take all eight workers
    del src, thin
    big = torch.empty((8 * n,), dtype=torch.float32, device="cuda")
    for i in range(8):
        big[i * n:(i + 1) * n].normal_()
    big_thin = torch.empty((8 * n // 16,), dtype=torch.int32, device="cuda")
    for name, kind, bpe in (("read_nt_32GiB", 1, 4.0), ("read_nt_with_thin_write_32GiB", 4, 4.25),
                            ("read_nt_with_thin_write_kept_in_L2_32GiB", 8, 4.0),
                            ("read_nt_one_shot_1024_threads_xcd_order_32GiB", 9, 4.0),
                            ("read_nt_wave_per_KiB_xcd_order_32GiB", 10, 4.0)):
        for _ in range(2):
            bench_probe(torch, kind, big, dst, big_thin, 8 * n)
        e0.record(stream)
        for _ in range(4):
            bench_probe(torch, kind, big, dst, big_thin, 8 * n)
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 4
        gbs = 8 * n * bpe / (ms * 1e-3) / 1e9
        out[name] = {"ms": round(ms, 4), "GBps": round(gbs, 1), "pct_hbm_peak": round(100 * gbs / HBM_PEAK_GBS, 1)}
    return {"ceilings": out, "elements": n, "peak_GBps": HBM_PEAK_GBS,
            "note": "bench_probe kinds 0-10: the kernels' access patterns without arithmetic (see bench_probe.hip)"}


def _timed(torch, stream, fn, reps, warm=2):
    """ms per call of fn: the mean over reps back-to-back calls, or - when something other than the calls
    sat in the timed region (a stall of the allocator or the driver after large buffers were released has
    been seen to add tens of ms once) - the median of the per-call times"""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    for _ in range(warm):
        fn()
    ev[0].record(stream)
    for i in range(reps):
        fn()
        ev[i + 1].record(stream)
    torch.cuda.synchronize()
    mean = ev[0].elapsed_time(ev[reps]) / reps
    per_call = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(reps))
    median = per_call[reps // 2] if reps % 2 else 0.5 * (per_call[reps // 2 - 1] + per_call[reps // 2])
    return median if mean > 1.2 * median else mean


def _rate(nbytes, ms):
    gbs = nbytes / (ms * 1e-3) / 1e9
    return {"ms": round(ms, 4), "algorithmic_GBps": round(gbs, 1), "pct_hbm_peak": round(100 * gbs / HBM_PEAK_GBS, 1)}


def roofline_of(kernel_symbol, short, workload_key, alg_bytes, ms):
    """the roofline object of one HBM-bound kernel: algorithmic bytes per launch over its mean launch
    duration (HIP events on the launch stream, this run) against the published 8 TB/s"""
    achieved = alg_bytes / (ms * 1e-3) / 1e9
    traffic = traffic_from_profile(short, workload_key)
    return {"bound": "hbm", "kernel": kernel_symbol, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
            "traffic_source": (traffic_profile_path(short, workload_key) + " (committed rocprofv3 --pmc "
                               "FETCH_SIZE / WRITE_SIZE summary; not measured in this run)") if traffic else None,
            "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_ms": round(ms, 4)}


def measure(torch, np, binding, workloads, key, steps, warmup, extras):
    """One workload: K timed steps of the four calls, the same step replayed from a HIP graph, per-call
    timings with events, and (extras) the calls beyond the step.  Returns (result dict, state for the
    CPU baseline)."""
    wl = workloads.BY_NAME[key]()
    W, n, L = wl.n_workers, wl.n, wl.n_layers
    grads = [workloads.make_gradient(wl, w, "cuda") for w in range(W)]
    plan = binding.Plan(wl.offsets, W)
    tau = torch.empty((W, L), dtype=torch.float32, device="cuda")
    s_local = torch.empty((W, L), dtype=torch.float32, device="cuda")
    s_shared = torch.empty((L,), dtype=torch.float32, device="cuda")
    codes = [torch.empty((plan.packed_bytes,), dtype=torch.uint8, device="cuda") for _ in range(W)]
    avg = torch.empty((n,), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def step(t, ev=None):
        if ev: ev[0].record(stream)
        plan.tg_clip_stats(grads, wl.clip_c, tau, s_local)
        if ev: ev[1].record(stream)
        plan.tg_share_scalers(W, s_local, s_shared)
        if ev: ev[2].record(stream)
        plan.tg_ternarize_pack(grads, tau, s_shared, wl.seed, wl.step + t, codes)
        if ev: ev[3].record(stream)
        plan.tg_unpack_average(codes, s_shared, avg)
        if ev: ev[4].record(stream)

    for t in range(warmup):
        step(t)
    torch.cuda.synchronize()

    # whole-step timing: exactly K steps between two synchronisations
    t0 = time.perf_counter()
    for t in range(steps):
        step(t)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps

    # per-call timing with events on the launch stream, over K more steps (before the graph below is
    # captured: host-side work around a capture has been seen to stall a later launch for milliseconds,
    # which an event pair around a 20 us kernel would count)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps)]
    for t in range(steps):
        step(t, evs[t])
    torch.cuda.synchronize()
    names = ["clip_stats", "share_scalers", "ternarize_pack", "unpack_average"]
    samples = {nm: np.array([e[i].elapsed_time(e[i + 1]) for e in evs]) for i, nm in enumerate(names)}
    call_ms = {nm: float(samples[nm].mean()) for nm in names}
    # an event pair also counts any time the host took to issue the call behind it: the median is shown
    # beside the mean so that one stalled launch among K (seen after large frees) is recognisable
    call_median_ms = {nm: float(np.median(samples[nm])) for nm in names}

    # the same step recorded once into a HIP graph and replayed (the iteration counter lives in device
    # memory and is advanced by the graph's last node): what a launch-bound caller would do
    step_dev = torch.zeros((1,), dtype=torch.int32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(stream)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        plan.tg_clip_stats(grads, wl.clip_c, tau, s_local)
        plan.tg_share_scalers(W, s_local, s_shared)
        plan.tg_ternarize_pack_devstep(grads, tau, s_shared, wl.seed, step_dev, codes)
        plan.tg_unpack_average(codes, s_shared, avg)
        binding.tg_step_advance(step_dev, 1)
    for _ in range(warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    ms_per_step_graph = (time.perf_counter() - t0) * 1e3 / steps
    del graph

    in_bytes = W * n * 4.0
    alg_bytes = {"clip_stats": W * n * 4.0, "ternarize_pack": W * n * 4.25,
                 "unpack_average": n * (4.0 + 0.25 * W)}
    kern = {nm: _rate(alg_bytes[nm], call_ms[nm]) for nm in ("clip_stats", "ternarize_pack", "unpack_average")}
    for nm in kern:
        kern[nm]["median_ms"] = round(call_median_ms[nm], 4)
    kern["ternarize_pack"]["fp32_in_GBps"] = round(in_bytes / (call_ms["ternarize_pack"] * 1e-3) / 1e9, 1)
    kern["share_scalers"] = {"ms": round(call_ms["share_scalers"], 4)}
    rooflines = {
        "ternarize_pack": roofline_of("tg::ternarize_pack_kernel", "ternarize_pack", key,
                                      alg_bytes["ternarize_pack"], call_ms["ternarize_pack"]),
        "unpack_average": roofline_of("tg::unpack_average_kernel<codes -> average>", "unpack_average", key,
                                      alg_bytes["unpack_average"], call_ms["unpack_average"]),
    }

    if extras:
        reps = max(5, steps // 2)
        # next line of Algorithm 1 (not part of the timed step): decode fused with the parameter update
        weights = torch.zeros((n,), dtype=torch.float32, device="cuda")
        ms = _timed(torch, stream, lambda: plan.tg_unpack_update(codes, s_shared, 1e-3, weights), reps, 3)
        kern["unpack_update (not in step)"] = _rate(n * (8.0 + 0.25 * W), ms)
        velocity = torch.zeros((n,), dtype=torch.float32, device="cuda")
        ms = _timed(torch, stream, lambda: plan.tg_unpack_update_momentum(codes, s_shared, 1e-3, 0.9, velocity, weights), reps)
        kern["unpack_update_momentum (not in step)"] = _rate(n * (16.0 + 0.25 * W), ms)
        del weights, velocity

        # Section 3.1 server-to-worker pull (not part of the timed step): the average as k in narrow fields;
        # both the byte-aligned width (4 or 8 bits) and, where it differs, the narrowest one, ceil(log2(2W+1))
        for bits in sorted({4 if W <= 7 else 8, binding.tg_sum_bits(W)}, reverse=True):
            ksum = torch.empty((plan.tg_sum_bytes(bits),), dtype=torch.uint8, device="cuda")
            ms = _timed(torch, stream, lambda: plan.tg_unpack_sum_pack(codes, bits, ksum), reps)
            kern["unpack_sum_pack %d-bit (not in step)" % bits] = _rate(n * (0.25 * W + bits / 8.0), ms)
            ms = _timed(torch, stream, lambda: plan.tg_decode_sum(W, ksum, bits, s_shared, avg), reps)
            kern["decode_sum %d-bit (not in step)" % bits] = _rate(n * (bits / 8.0 + 4.0), ms)
            del ksum

        # Section 3.1, toward 32/log2(3): the base-3 container, five ternary values per byte (not in the step)
        codes3 = [torch.empty((plan.packed_bytes_base3,), dtype=torch.uint8, device="cuda") for _ in range(W)]
        ms = _timed(torch, stream, lambda: plan.tg_ternarize_pack_base3(grads, tau, s_shared, wl.seed, wl.step, codes3), reps)
        kern["ternarize_pack_base3 (not in step)"] = _rate(n * W * 4.2, ms)
        ms = _timed(torch, stream, lambda: plan.tg_unpack_average_base3(codes3, s_shared, avg), reps)
        kern["unpack_average_base3 (not in step)"] = _rate(n * (0.2 * W + 4.0), ms)
        del codes3

        # Algorithm 1's server line without scaler sharing (not part of the timed step)
        ms = _timed(torch, stream, lambda: plan.tg_unpack_average_scalers(codes, s_local, avg), reps)
        kern["unpack_average_scalers (not in step)"] = _rate(n * (4.0 + 0.25 * W), ms)

        # Section 4.2 variant (not part of the timed step): plain fp32 average, as used for a layer that is
        # kept in floating point; timed here over the whole flat buffer to get a bandwidth figure
        favg = torch.empty((n,), dtype=torch.float32, device="cuda")
        ms = _timed(torch, stream, lambda: binding.tg_average_float(grads, n, favg), reps)
        kern["average_float (not in step)"] = _rate(n * (4.0 * W + 4.0), ms)
        del favg

    res = {"workload": "%s gradients, fp32, W=%d simulated workers on one GPU, n=%d, L=%d, c=%.1f"
                       % (wl.name, W, n, L, wl.clip_c),
           "value": round(in_bytes / (ms_per_step * 1e-3) / 1e9, 2), "unit": "GB/s",
           "ms_per_step": round(ms_per_step, 4), "ms_per_step_graph_replay": round(ms_per_step_graph, 4),
           "kernels": kern, "rooflines": rooflines}
    plan.close()
    return res, (wl, grads)


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the W workers are W gradient buffers on one "
              "device; no collectives). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1705_07878_amd import binding, workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.ceilings:
        print(json.dumps(ceilings(torch, n=args.ceilings_elements)))
        return

    head, (wl, grads) = measure(torch, np, binding, workloads, args.workload, args.steps, args.warmup, extras=True)
    W = wl.n_workers
    out = {
        "metric": "ternarize+pack and unpack-average GB/s (fp32 in) and % HBM peak; ms/step",
        "value": head["value"], "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": head["workload"]},
        "ms_per_step_graph_replay": head["ms_per_step_graph_replay"],
        "kernels": head["kernels"],
        # the dominant kernel of the step; the second kernel the metric names follows under its own key
        "roofline": head["rooflines"]["ternarize_pack"],
        "roofline_unpack_average": head["rooflines"]["unpack_average"],
    }

    if not args.no_cpu_baseline:
        # bounded sample: the whole workload if W*n <= 2.6e8 element passes, else its first layers
        cap = 260_000_000 // W
        if wl.n <= cap:
            sub, note = wl, "the whole step (4 calls, all %d workers) of this workload" % W
            host = [g.cpu().numpy() for g in grads]
        else:
            sizes, tot = [], 0
            for s in wl.layer_sizes:
                take = min(s, cap - tot)
                if take <= 0:
                    break
                sizes.append(take)
                tot += take
            sub = workloads.custom(sizes, W, name=wl.name + " (truncated)", clip_c=wl.clip_c, seed=wl.seed,
                                   step=wl.step)
            note = "the whole step on the first %d elements of each of the %d workers" % (tot, W)
            host = [g[:tot].cpu().numpy() for g in grads]
        del grads
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(sub, host, note)
        out["cpu_baseline"]["value"] = round(out["cpu_baseline"]["value"], 3)
        out["cpu_baseline"]["seconds"] = round(out["cpu_baseline"]["seconds"], 2)
        del host
    else:
        del grads
        torch.cuda.empty_cache()

    # the other target configurations, same run, same measurement (the four calls only)
    others = {}
    for key in [k for k in args.also.split(",") if k and k != args.workload]:
        # let the driver finish releasing the previous workload's memory before anything is timed
        torch.cuda.synchronize()
        time.sleep(0.5)
        res, state = measure(torch, np, binding, workloads, key, args.steps, args.warmup, extras=False)
        del state
        torch.cuda.empty_cache()
        others[key] = res
    if others:
        out["other_configs"] = others

    # a plain copy of known size, outside the timed region: the calibration kernel for --pmc runs
    cal_src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()

    print(json.dumps(out))


if __name__ == "__main__":
    main()
