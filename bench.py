#!/usr/bin/env python3
"""Benchmark of the TernGrad hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic
gradients: tg_clip_stats -> tg_share_scalers -> tg_ternarize_pack ->
tg_unpack_average for all W simulated workers (W gradient buffers on the one
device).  Inputs are resident in HBM before the timed region.  Prints ONE JSON
line; `value` is fp32 gradient bytes consumed per second (W * n * 4 B / step).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload alexnet]
"""
import argparse
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
    ap.add_argument("--workload", default="alexnet",
                    choices=["lenet", "alexnet", "googlenet_like", "vgg_a", "flat"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--ceilings", action="store_true",
                    help="instead of the step: what the memory system sustains for the kernels' access "
                         "patterns with the arithmetic taken out (tg_probe), on 4 GB buffers")
    ap.add_argument("--ceilings-elements", type=int, default=1 << 30,
                    help="floats per buffer for --ceilings (a multiple of 1024)")
    return ap.parse_args()


def traffic_from_profile(kernel: str, workload: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary, or None."""
    path = os.path.join(ROOT, "profiles", "%s_%s_pmc.txt" % (kernel, workload))
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


def ceilings(torch, binding, n=1 << 30, reps=10):
    """GB/s of the probe kernels over n floats: same launch shape as the real kernels, no arithmetic"""
    src = torch.empty((n,), dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty((n,), dtype=torch.float32, device="cuda")
    thin = torch.empty((n // 16,), dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    kinds = [(0, "read", 4.0), (1, "read_nt", 4.0), (2, "write_nt", 4.0), (3, "copy_nt", 8.0),
             (4, "read_nt_with_thin_write", 4.25)]
    out = {}
    for kind, name, bytes_per_elem in kinds:
        for _ in range(3):
            binding.tg_probe(kind, src, dst, thin, n)
        e0.record(stream)
        for _ in range(reps):
            binding.tg_probe(kind, src, dst, thin, n)
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        gbs = n * bytes_per_elem / (ms * 1e-3) / 1e9
        out[name] = {"ms": round(ms, 4), "GBps": round(gbs, 1), "pct_hbm_peak": round(100 * gbs / HBM_PEAK_GBS, 1)}
    # the footprint of the flat 1e9 workload: eight 4 GB sources read one after the other
    srcs = [src] + [torch.empty((n,), dtype=torch.float32, device="cuda").normal_() for _ in range(7)]
    thins = [thin] + [torch.empty((n // 16,), dtype=torch.int32, device="cuda") for _ in range(7)]
    for name, kind, bpe in (("read_nt_8x4GB", 1, 4.0), ("read_nt_with_thin_write_8x4GB", 4, 4.25)):
        for i in range(8):
            binding.tg_probe(kind, srcs[i], dst, thins[i], n)
        e0.record(stream)
        for _ in range(3):
            for i in range(8):
                binding.tg_probe(kind, srcs[i], dst, thins[i], n)
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 3
        gbs = 8 * n * bpe / (ms * 1e-3) / 1e9
        out[name] = {"ms": round(ms, 4), "GBps": round(gbs, 1), "pct_hbm_peak": round(100 * gbs / HBM_PEAK_GBS, 1)}
    return {"ceilings": out, "elements": n, "peak_GBps": HBM_PEAK_GBS,
            "note": "tg_probe kinds 0-4: the kernels' access patterns without arithmetic, one wave per 1024 floats"}


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
        print(json.dumps(ceilings(torch, binding, n=args.ceilings_elements)))
        return
    wl = workloads.BY_NAME[args.workload]()
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

    for t in range(args.warmup):
        step(t)
    torch.cuda.synchronize()

    # whole-step timing: exactly K steps between two synchronisations
    t0 = time.perf_counter()
    for t in range(args.steps):
        step(t)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

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
    for _ in range(args.warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    ms_per_step_graph = (time.perf_counter() - t0) * 1e3 / args.steps

    # per-call timing with events on the launch stream, over K more steps
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    for t in range(args.steps):
        step(t, evs[t])
    torch.cuda.synchronize()
    names = ["clip_stats", "share_scalers", "ternarize_pack", "unpack_average"]
    call_ms = {nm: float(np.mean([e[i].elapsed_time(e[i + 1]) for e in evs])) for i, nm in enumerate(names)}

    in_bytes = W * n * 4.0
    alg_bytes = {"clip_stats": W * n * 4.0, "ternarize_pack": W * n * 4.25,
                 "unpack_average": n * (4.0 + 0.25 * W)}
    kern = {}
    for nm in ("clip_stats", "ternarize_pack", "unpack_average"):
        gbs = alg_bytes[nm] / (call_ms[nm] * 1e-3) / 1e9
        kern[nm] = {"ms": round(call_ms[nm], 4), "algorithmic_GBps": round(gbs, 1),
                    "pct_hbm_peak": round(100 * gbs / HBM_PEAK_GBS, 1)}
    kern["ternarize_pack"]["fp32_in_GBps"] = round(in_bytes / (call_ms["ternarize_pack"] * 1e-3) / 1e9, 1)
    kern["share_scalers"] = {"ms": round(call_ms["share_scalers"], 4)}

    # next line of Algorithm 1 (not part of the timed step): decode fused with the parameter update
    weights = torch.zeros((n,), dtype=torch.float32, device="cuda")
    for _ in range(3):
        plan.tg_unpack_update(codes, s_shared, 1e-3, weights)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = max(5, args.steps // 2)
    e0.record(stream)
    for _ in range(reps):
        plan.tg_unpack_update(codes, s_shared, 1e-3, weights)
    e1.record(stream)
    torch.cuda.synchronize()
    upd_ms = e0.elapsed_time(e1) / reps
    upd_gbs = n * (8.0 + 0.25 * W) / (upd_ms * 1e-3) / 1e9
    kern["unpack_update (not in step)"] = {"ms": round(upd_ms, 4), "algorithmic_GBps": round(upd_gbs, 1),
                                           "pct_hbm_peak": round(100 * upd_gbs / HBM_PEAK_GBS, 1)}
    velocity = torch.zeros((n,), dtype=torch.float32, device="cuda")
    for _ in range(2):
        plan.tg_unpack_update_momentum(codes, s_shared, 1e-3, 0.9, velocity, weights)
    e0.record(stream)
    for _ in range(reps):
        plan.tg_unpack_update_momentum(codes, s_shared, 1e-3, 0.9, velocity, weights)
    e1.record(stream)
    torch.cuda.synchronize()
    mom_ms = e0.elapsed_time(e1) / reps
    mom_gbs = n * (16.0 + 0.25 * W) / (mom_ms * 1e-3) / 1e9
    kern["unpack_update_momentum (not in step)"] = {"ms": round(mom_ms, 4), "algorithmic_GBps": round(mom_gbs, 1),
                                                    "pct_hbm_peak": round(100 * mom_gbs / HBM_PEAK_GBS, 1)}
    del weights, velocity

    # Section 3.1 server-to-worker pull (not part of the timed step): the average as k in narrow fields
    # both the byte-aligned width (4 or 8 bits) and, where it differs, the narrowest one, ceil(log2(2W+1))
    for bits in sorted({4 if W <= 7 else 8, binding.tg_sum_bits(W)}, reverse=True):
        ksum = torch.empty((plan.tg_sum_bytes(bits),), dtype=torch.uint8, device="cuda")
        for nm, fn, nbytes in (("unpack_sum_pack", lambda: plan.tg_unpack_sum_pack(codes, bits, ksum), 0.25 * W + bits / 8.0),
                               ("decode_sum", lambda: plan.tg_decode_sum(W, ksum, bits, s_shared, avg), bits / 8.0 + 4.0)):
            for _ in range(2):
                fn()
            e0.record(stream)
            for _ in range(reps):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / reps
            gbs = n * nbytes / (ms * 1e-3) / 1e9
            kern["%s %d-bit (not in step)" % (nm, bits)] = {"ms": round(ms, 4), "algorithmic_GBps": round(gbs, 1),
                                                            "pct_hbm_peak": round(100 * gbs / HBM_PEAK_GBS, 1)}
    del ksum

    # Section 3.1, toward 32/log2(3): the base-3 container, five ternary values per byte (not in the step)
    codes3 = [torch.empty((plan.packed_bytes_base3,), dtype=torch.uint8, device="cuda") for _ in range(W)]
    for nm, fn, nbytes in (("ternarize_pack_base3", lambda: plan.tg_ternarize_pack_base3(grads, tau, s_shared, wl.seed, wl.step, codes3), W * 4.2),
                           ("unpack_average_base3", lambda: plan.tg_unpack_average_base3(codes3, s_shared, avg), 0.2 * W + 4.0)):
        for _ in range(2):
            fn()
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        gbs = n * nbytes / (ms * 1e-3) / 1e9
        kern["%s (not in step)" % nm] = {"ms": round(ms, 4), "algorithmic_GBps": round(gbs, 1),
                                         "pct_hbm_peak": round(100 * gbs / HBM_PEAK_GBS, 1)}
    del codes3

    # Algorithm 1's server line without scaler sharing (not part of the timed step): every worker's own scaler
    for _ in range(2):
        plan.tg_unpack_average_scalers(codes, s_local, avg)
    e0.record(stream)
    for _ in range(reps):
        plan.tg_unpack_average_scalers(codes, s_local, avg)
    e1.record(stream)
    torch.cuda.synchronize()
    us_ms = e0.elapsed_time(e1) / reps
    us_gbs = n * (4.0 + 0.25 * W) / (us_ms * 1e-3) / 1e9
    kern["unpack_average_scalers (not in step)"] = {"ms": round(us_ms, 4), "algorithmic_GBps": round(us_gbs, 1),
                                                    "pct_hbm_peak": round(100 * us_gbs / HBM_PEAK_GBS, 1)}

    # Section 4.2 variant (not part of the timed step): plain fp32 average, as used for a layer that is
    # kept in floating point; timed here over the whole flat buffer to get a bandwidth figure
    favg = torch.empty((n,), dtype=torch.float32, device="cuda")
    for _ in range(2):
        binding.tg_average_float(grads, n, favg)
    e0.record(stream)
    for _ in range(reps):
        binding.tg_average_float(grads, n, favg)
    e1.record(stream)
    torch.cuda.synchronize()
    fa_ms = e0.elapsed_time(e1) / reps
    fa_gbs = n * (4.0 * W + 4.0) / (fa_ms * 1e-3) / 1e9
    kern["average_float (not in step)"] = {"ms": round(fa_ms, 4), "algorithmic_GBps": round(fa_gbs, 1),
                                           "pct_hbm_peak": round(100 * fa_gbs / HBM_PEAK_GBS, 1)}
    del favg

    dom = "ternarize_pack"
    achieved = alg_bytes[dom] / (call_ms[dom] * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "tg::ternarize_pack_kernel", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic_from_profile(dom, args.workload),
                "algorithmic_bytes_per_launch": alg_bytes[dom], "avg_launch_ms": round(call_ms[dom], 4),
                # what the same traffic (4 B read + 1/4 B written per element) reaches with no arithmetic at all,
                # 4 GiB per launch, from the committed `bench.py --ceilings` run: context for `frac`
                "pattern_ceiling_GBps": pattern_ceiling()}

    out = {
        "metric": "ternarize+pack and unpack-average GB/s (fp32 in) and % HBM peak; ms/step",
        "value": round(in_bytes / (ms_per_step * 1e-3) / 1e9, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "%s gradients, fp32, W=%d simulated workers on one GPU, n=%d, L=%d, c=%.1f"
                               % (wl.name, W, n, L, wl.clip_c)},
        "ms_per_step_graph_replay": round(ms_per_step_graph, 4),
        "kernels": kern, "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        # bounded sample: the whole workload if W*n <= 2.6e8 element passes, else its first layers
        cap = 260_000_000 // W
        if n <= cap:
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
        out["cpu_baseline"] = cpu_baseline(sub, host, note)
        out["cpu_baseline"]["value"] = round(out["cpu_baseline"]["value"], 3)
        out["cpu_baseline"]["seconds"] = round(out["cpu_baseline"]["seconds"], 2)

    # a plain copy of known size, outside the timed region: the calibration kernel for --pmc runs
    cal_src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()

    print(json.dumps(out))
    plan.close()


if __name__ == "__main__":
    main()
