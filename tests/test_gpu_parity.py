"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle."""
import numpy as np
import pytest
import torch

from parity_util import (assert_avg_close, assert_stats_close, assert_update_close, dev, full_parity, gpu_clip_stats,
                         gpu_share, gpu_ternarize, gpu_unpack_average, gpu_unpack_update)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    from paper_1705_07878_amd import binding as b
    return b


def _grads(rng, off, W, sig=None, mean=0.0):
    n = int(off[-1])
    L = len(off) - 1
    sig = 10.0 ** rng.uniform(-4, -2, size=L) if sig is None else sig
    out = []
    for _ in range(W):
        g = np.concatenate([rng.normal(size=off[l + 1] - off[l]) * sig[l] + mean for l in range(L)])
        k = max(1, n // 1000)
        g[rng.integers(0, n, size=k)] *= 12.0
        out.append(g.astype(np.float32))
    return out


def _off(sizes):
    return np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)


@pytest.mark.parametrize("sizes,W", [
    ([1], 1), ([2], 2), ([3], 1), ([4], 1), ([5], 3), ([15], 1), ([16], 2), ([17], 1),
    ([1023], 1), ([1024], 2), ([1025], 1), ([4096], 1), ([4097], 2), ([16384], 1), ([16385], 1),
    ([1, 2, 3, 4, 5, 15, 16, 17], 2),
    ([1000, 24, 0, 0, 3000, 1, 72, 5000, 16384, 7], 3),
    ([20000, 1, 20000], 4),
    ([500, 20, 25000, 50, 400000, 500, 5000, 10], 2),           # LeNet shapes
    ([70001, 33333], 5), ([9000] * 7, 6), ([12345], 8), ([4099, 4093], 11),
])
def test_all_four_calls_small(oracle, binding, sizes, W):
    rng = np.random.default_rng(abs(hash((tuple(sizes), W))) % (2 ** 32))
    off = _off(sizes)
    full_parity(oracle, binding, off, _grads(rng, off, W), c=2.5, seed=1234567, step=3)


def test_random_models(oracle, binding):
    """40 seeded random models: layer sizes from a mixture of empty, tiny, around one tile and several
    chunks; any number of workers up to 9; clip constants incl. no clipping; any seed, step, first worker"""
    rng = np.random.default_rng(2024)
    for case in range(40):
        L = int(rng.integers(1, 13))
        kinds = rng.integers(0, 5, size=L)
        sizes = [int([0, rng.integers(1, 12), rng.integers(1000, 1050), rng.integers(3000, 9000),
                      rng.integers(15000, 70000)][k]) for k in kinds]
        if sum(sizes) == 0:
            sizes[0] = 7
        off = _off(sizes)
        W = int(rng.integers(1, 10))
        c = float(rng.choice([2.5, 2.5, 1.0, 0.3, 0.0]))
        full_parity(oracle, binding, off, _grads(rng, off, W, mean=float(rng.choice([0.0, 1e-3]))), c=c,
                    seed=int(rng.integers(0, 2 ** 63)), step=int(rng.integers(0, 2 ** 32)),
                    worker_base=int(rng.integers(0, 1000)))


def test_finer_buckets_than_a_layer(oracle, binding):
    """Section 3.3: gradients split into buckets that are ternarized independently (as in QSGD): a finer
    offset table through the same kernels; many boundaries per tile, small statistics segments"""
    rng = np.random.default_rng(33)
    for sizes in ([512] * 64 + [256] * 8 + [64] * 16 + [16] * 9, [1024] * 33, [2048, 2049, 2047] * 5, [100] * 333):
        off = _off(sizes)
        full_parity(oracle, binding, off, _grads(rng, off, 2), seed=77, step=5)


def test_many_tiny_layers(oracle, binding):
    """hundreds of boundaries per tile, empty and one-element layers in runs, more than 1024 layers (the
    thread-per-layer fold of the statistics) and two long layers in between, one with few partials and
    one with many"""
    rng = np.random.default_rng(34)
    sizes = (list(rng.integers(0, 10, size=100)) + [300_001] + list(rng.integers(0, 10, size=15_000)) + [70_001] +
             list(rng.integers(0, 4, size=5_000)))
    off = _off(sizes)
    full_parity(oracle, binding, off, _grads(rng, off, 3), seed=9, step=1)


def test_every_statistics_shape(oracle, binding):
    """the shape of the statistics pass follows n * max_workers: workgroups that loop over chunks of 8192 or
    16384 elements, and from 2^28 elements on chunks of 16384 read in one shot by workgroups of 1024 threads
    in the XCD-aware order (32768 or 65536 in a loop when layers begin in too many chunks); here with two
    workers of a plan made for more, and layer sizes that leave ragged segments in every shape"""
    rng = np.random.default_rng(35)
    off = _off([3, 3_000_001, 70_000, 5_400_001, 11])                    # n = 8,470,016
    grads = _grads(rng, off, 2)
    oracle.set_threads(8)
    try:
        chunks = []
        for mw in (2, 16, 31, 32, 64):                                   # 31: the last looping size, 32: one shot
            chunks.append(int(binding.tg_describe_tables(off, mw)["chunk_elems"]))
            full_parity(oracle, binding, off, grads, max_workers=mw)
        assert chunks == [8192, 16384, 16384, 16384, 16384]
        assert 31 * 8_470_016 < 2 ** 28 <= 32 * 8_470_016
        # many layers at the same size: chunks of 32768 and 65536 in the looping shape
        off2 = _off([4099] * 2066 + [1520])
        assert int(off2[-1]) == 8_470_054
        for mw, chunk in ((32, 32768), (64, 65536)):
            assert int(binding.tg_describe_tables(off2, mw)["chunk_elems"]) == chunk
            full_parity(oracle, binding, off2, _grads(rng, off2, 2), max_workers=mw)
    finally:
        oracle.set_threads(1)


def test_random_tables_in_the_one_shot_statistics_shape(oracle, binding):
    """12 seeded random layer tables over 8.4 - 9.5 M elements in a plan for 64 workers (the one-shot shape
    wherever few chunks hold a layer boundary): boundaries anywhere, close together, on chunk borders,
    empty layers; small, zero and large means"""
    rng = np.random.default_rng(99)
    oracle.set_threads(8)
    try:
        shapes = []
        for case in range(12):
            n = int(rng.integers(8_400_000, 9_500_000))
            k = int(rng.integers(0, 9))
            cuts = np.sort(rng.integers(1, n, size=k)) if k else np.array([], np.int64)
            extra = []
            for cpos in cuts[:3]:
                extra += [int(cpos) + int(rng.integers(0, 5))]
            if rng.random() < 0.5:
                extra += [16384 * int(rng.integers(1, n // 16384))]
            off = np.unique(np.concatenate([[0], cuts, np.array(extra, np.int64), [n]])).astype(np.int64)
            off = off[off <= n]
            if rng.random() < 0.3:
                i = int(rng.integers(1, len(off)))
                off = np.insert(off, i, off[i])                 # an empty layer
            shapes.append(int(binding.tg_describe_tables(off, 64)["chunk_elems"]))
            W = int(rng.integers(1, 3))
            grads = _grads(rng, off, W, mean=float(rng.choice([0.0, 1e-3, 0.5])))
            plan = binding.Plan(off, 64)
            try:
                tau, s_local = gpu_clip_stats(plan, [dev(g) for g in grads], 2.5)
            finally:
                plan.close()
            st = [oracle.clip_stats(g, off, 2.5) for g in grads]
            wt, ws = np.stack([a for a, _ in st]), np.stack([b for _, b in st])
            assert_stats_close(tau, wt, grads, off, "one-shot tau", 2.5)
            assert_stats_close(s_local, ws, grads, off, "one-shot s_local", 2.5, want_tau=wt)
        assert shapes.count(16384) >= 8
    finally:
        oracle.set_threads(1)


def test_w64_and_worker_base(oracle, binding):
    rng = np.random.default_rng(64)
    off = _off([3000, 17, 5000])
    full_parity(oracle, binding, off, _grads(rng, off, 64), seed=2 ** 63 + 5, step=2 ** 31 + 1, worker_base=1000)


def test_noclip_and_zero_and_constant_layers(oracle, binding):
    rng = np.random.default_rng(7)
    off = _off([5000, 300, 4096, 100])
    grads = _grads(rng, off, 2)
    for g in grads:
        g[5000:5300] = 0.0                 # an all-zero layer: sigma = 0, s = 0, all codes 0
        g[5300:5300 + 4096] = 0.25         # a constant layer: sigma exactly 0
    for c in (2.5, 0.0, float("inf"), 1.0):
        res = full_parity(oracle, binding, off, grads, c=c)
        assert np.all(res["avg"][5000:5300] == 0)


def test_large_mean_layer(oracle, binding):
    rng = np.random.default_rng(8)
    off = _off([40000, 777])
    grads = _grads(rng, off, 2, sig=np.array([1e-3, 1e-3]), mean=0.5)
    full_parity(oracle, binding, off, grads)


def test_lenet_config(oracle, binding):
    from paper_1705_07878_amd import workloads
    wl = workloads.lenet()
    grads = [g.numpy() for g in workloads.make_gradients(wl, "cpu")]
    res = full_parity(oracle, binding, wl.offsets, grads, c=wl.clip_c, seed=wl.seed, step=wl.step)
    nz = np.mean(res["codes"][0] != 0)
    assert 0.3 < nz < 0.95


def test_googlenet_like_config(oracle, binding):
    from paper_1705_07878_amd import workloads
    wl = workloads.googlenet_like()
    oracle.set_threads(8)
    try:
        grads = [g.numpy() for g in workloads.make_gradients(wl, "cpu")]
        full_parity(oracle, binding, wl.offsets, grads, c=wl.clip_c, seed=wl.seed, step=wl.step)
    finally:
        oracle.set_threads(1)


def test_unpack_average_arbitrary_bytes(oracle, binding):
    """every byte value, including the never-produced code 10 (decodes as -2)"""
    rng = np.random.default_rng(9)
    off = _off([3000, 1, 6000, 1241])
    n = int(off[-1])
    for W in (1, 2, 3, 5, 6, 8, 10, 11, 16, 64):
        codes = [rng.integers(0, 256, size=(n + 3) // 4, dtype=np.uint8) for _ in range(W)]
        s = (np.abs(rng.normal(size=4)) + 0.01).astype(np.float32)
        plan = binding.Plan(off, W)
        try:
            assert_avg_close(gpu_unpack_average(plan, codes, s), oracle.unpack_average(codes, off, s))
        finally:
            plan.close()


def test_unpack_average_with_each_workers_own_scaler(oracle, binding):
    """Algorithm 1's server line without scaler sharing: every worker ternarizes with its own s_local
    (one call per worker, its row in place of the shared scaler) and the decoder weighs each worker's
    ternary values with that worker's scaler"""
    rng = np.random.default_rng(41)
    for sizes, W in (([37], 1), ([1024], 2), ([5000, 3, 4096, 2001, 0, 20000], 4), ([100] * 50 + [3000], 3),
                     ([70001, 33333], 8), ([1500], 64), ([9000] * 3, 11)):
        off = _off(sizes)
        n, L = int(off[-1]), len(sizes)
        grads = _grads(rng, off, W)
        st = [oracle.clip_stats(g, off, 2.5) for g in grads]
        sw = np.stack([x[1] for x in st])                                  # [W][L]: no sharing
        o_codes = [oracle.ternarize_pack(g, off, st[w][0], sw[w], 11, 2, w) for w, g in enumerate(grads)]
        plan = binding.Plan(off, W)
        try:
            nb = (n + 3) // 4
            for w, g in enumerate(grads):                                  # encoder: one worker per call
                gc = gpu_ternarize(plan, [dev(g)], st[w][0][None, :], sw[w], 11, 2, worker_base=w)[0]
                assert np.array_equal(gc[:nb], o_codes[w]) and not gc[nb:].any()
            cd = []
            for c in o_codes:
                buf = np.zeros(plan.packed_bytes, np.uint8)
                buf[:c.size] = c
                cd.append(dev(buf))
            avg = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
            plan.tg_unpack_average_scalers(cd, dev(sw), avg)
            torch.cuda.synchronize()
            got = avg.cpu().numpy()
            want = oracle.unpack_average_scalers(o_codes, off, sw)
            lay = np.repeat(np.arange(L), np.diff(off))
            # tolerance relative to the mean magnitude of the terms (a sum of signed terms has no relative
            # accuracy of its own); zeros exact
            mag = np.zeros(n)
            allzero = np.ones(n, bool)
            for w, c in enumerate(o_codes):
                f = (c[:, None] >> np.array([0, 2, 4, 6], np.uint8)) & 3
                nz = (f.reshape(-1)[:n] != 0)
                mag += nz * sw[w][lay].astype(np.float64)
                allzero &= ~nz
            assert np.all(np.abs(got.astype(np.float64) - want.astype(np.float64)) <= 1e-6 * mag / W)
            assert np.all(got[allzero] == 0)
            # equal rows: the shared-scaler decoder's values
            s = sw.max(axis=0)
            plan.tg_unpack_average_scalers(cd, dev(np.tile(s, (W, 1))), avg)
            torch.cuda.synchronize()
            assert_avg_close(avg.cpu().numpy(), oracle.unpack_average(o_codes, off, s))
        finally:
            plan.close()


def test_unpack_update_arbitrary_bytes_and_rates(oracle, binding):
    rng = np.random.default_rng(19)
    off = _off([5000, 3, 4096, 2001])
    n = int(off[-1])
    for W, eta in ((1, 1.0), (4, 0.1), (7, 1e-3), (8, 0.0), (64, 2.5)):
        codes = [rng.integers(0, 256, size=(n + 3) // 4, dtype=np.uint8) for _ in range(W)]
        s = (np.abs(rng.normal(size=4)) * 1e-2 + 1e-4).astype(np.float32)
        w0 = rng.normal(size=n).astype(np.float32)
        plan = binding.Plan(off, W)
        try:
            for kernel in (0, 1, 2):
                got = gpu_unpack_update(plan, codes, s, eta, w0, kernel=kernel)
                assert_update_close(got, oracle.unpack_update(codes, off, s, eta, w0), w0,
                                    oracle.unpack_average(codes, off, s))
                if eta == 0.0:
                    assert np.array_equal(got, w0)
        finally:
            plan.close()


def test_average_float_layers(oracle, binding):
    """Section 4.2: a layer kept in fp32 is averaged as floats; bit-exact (fp64 sum, one rounding)"""
    rng = np.random.default_rng(21)
    for W, n in ((1, 5), (2, 1024), (3, 4099), (4, 4_096_000), (8, 100_003), (64, 2050)):
        grads = [(rng.normal(size=n) * 10.0 ** rng.uniform(-5, 1)).astype(np.float32) for _ in range(W)]
        out = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        binding.tg_average_float([dev(g) for g in grads], n, out)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), oracle.average_float(grads))
    with pytest.raises(binding.TgError):
        binding.tg_average_float([out[1:]], 4, out)          # not congruent modulo 16 bytes


def test_average_float_on_slices_of_flat_buffers(oracle, binding):
    """a float layer is a slice of each worker's flat buffer: any float offset, the same in all"""
    rng = np.random.default_rng(22)
    for W, shift, n in ((2, 1, 1), (2, 1, 2), (3, 2, 3), (3, 3, 3), (2, 1, 4), (4, 3, 2051), (8, 2, 70_001), (2, 1, 1_000_003)):
        flat = [(rng.normal(size=shift + n + 5) * 0.1).astype(np.float32) for _ in range(W)]
        fd = [dev(f) for f in flat]
        out = torch.full((shift + n + 5,), float("nan"), dtype=torch.float32, device="cuda")
        binding.tg_average_float([f[shift:] for f in fd], n, out[shift:])
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert np.array_equal(got[shift:shift + n], oracle.average_float([f[shift:shift + n] for f in flat]))
        assert np.isnan(got[:shift]).all() and np.isnan(got[shift + n:]).all()      # nothing outside the slice


def test_last_layer_in_float(oracle, binding):
    """Section 4.2 deployment: every layer ternarized except the last classification layer (weight and
    bias), which travels and is averaged as fp32.  One flat gradient per worker; the plan covers the
    ternarized prefix, the float call the rest of the same buffers."""
    rng = np.random.default_rng(23)
    sizes = [2400, 96, 51_203, 256, 100_001, 10, 4097 * 10, 10]      # ..., fc weight, fc bias
    off = _off(sizes)
    W, n, n_t = 4, int(off[-1]), int(off[-3])
    grads = _grads(rng, off, W)
    gd = [dev(g) for g in grads]
    off_t = off[:-2]
    r = full_parity(oracle, binding, off_t, [g[:n_t] for g in grads], step=5)
    plan = binding.Plan(off_t, W)
    # the ternarized prefix of the full buffers, fed the oracle's tau and s: the oracle's codes
    codes = gpu_ternarize(plan, gd, r["tau"], r["s_shared"], 0, 5)
    nb = (n_t + 3) // 4
    for w in range(W):
        assert np.array_equal(codes[w][:nb], r["codes"][w])
    avg = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    binding.tg_average_float([g[n_t:] for g in gd], n - n_t, avg[n_t:])          # first, so that a decoder
    cd = []                                                                       # writing past n_t would show
    for c in r["codes"]:
        buf = np.zeros(plan.packed_bytes, np.uint8)
        buf[:c.size] = c
        cd.append(dev(buf))
    plan.tg_unpack_average(cd, dev(r["s_shared"]), avg)
    torch.cuda.synchronize()
    got = avg.cpu().numpy()
    assert np.array_equal(got[n_t:], oracle.average_float([g[n_t:] for g in grads]))
    assert_avg_close(got[:n_t], r["avg"])
    plan.close()


def test_layers_kept_in_float_as_a_mode_of_one_plan(oracle, binding):
    """Section 4.2 as a per-layer flag: float layers first, in the middle and last, next to each other and
    alone, beginning and ending at any alignment, one of them empty, one holding NaN and Inf.  The statistics
    give tau = s = 0 there, the codes are 00 (bit-exact with the oracle fed those scalers), the ternarized
    layers come out as without the flag, the float layers as the plain mean."""
    rng = np.random.default_rng(77)
    sizes = [1001, 3, 5000, 0, 4099, 2048, 7, 30001, 513]
    flags = np.array([1, 0, 0, 1, 1, 0, 1, 0, 1], np.uint8)
    off = _off(sizes)
    L = len(sizes)
    for W in (1, 3, 8):
        grads = _grads(rng, off, W)
        grads[0][off[4] + 5] = np.nan
        grads[W - 1][off[4] + 6] = np.inf
        plan = binding.Plan(off, W)
        dg = [dev(g) for g in grads]
        try:
            base = gpu_clip_stats(plan, dg, 2.5)
            plan.tg_plan_set_layer_modes(flags)
            tau, s_local = gpu_clip_stats(plan, dg, 2.5)
            fl = flags.astype(bool)
            assert np.all(tau[:, fl] == 0) and np.all(s_local[:, fl] == 0)
            assert np.array_equal(tau[:, ~fl], base[0][:, ~fl]) and np.array_equal(s_local[:, ~fl], base[1][:, ~fl])
            for w in range(W):
                want_tau, want_s = oracle.clip_stats(grads[w], off, 2.5)
                assert np.allclose(tau[w, ~fl], want_tau[~fl], rtol=1e-6, atol=0)
                assert np.allclose(s_local[w, ~fl], want_s[~fl], rtol=1e-6, atol=0)
            s_shared = gpu_share(plan, s_local)
            assert np.all(s_shared[fl] == 0)
            codes = gpu_ternarize(plan, dg, tau, s_shared, seed=11, step=4)
            nb = (int(off[-1]) + 3) // 4
            ocodes = [oracle.ternarize_pack(grads[w], off, tau[w], s_shared, 11, 4, w) for w in range(W)]
            for w in range(W):
                assert np.array_equal(codes[w][:nb], ocodes[w]) and not codes[w][nb:].any()
            got = np.full(int(off[-1]), 9.0, np.float32)
            dc = [dev(c) for c in codes]
            d_s, d_avg = dev(s_shared), dev(got)
            plan.tg_unpack_average_mixed(dc, dg, d_s, d_avg)
            torch.cuda.synchronize()
            got = d_avg.cpu().numpy()
            want = oracle.unpack_average(ocodes, off, s_shared)
            for l in range(L):
                b, e = int(off[l]), int(off[l + 1])
                if not flags[l]:
                    assert_avg_close(got[b:e], want[b:e])
                elif e > b:
                    wf = oracle.average_float([g[b:e] for g in grads])
                    fin = np.isfinite(wf)
                    assert np.array_equal(np.isnan(got[b:e]), np.isnan(wf)) and np.array_equal(got[b:e][~fin & ~np.isnan(wf)], wf[~fin & ~np.isnan(wf)])
                    assert np.allclose(got[b:e][fin], wf[fin], rtol=1e-6, atol=0)
                    assert np.all(codes[0][(b + 3) // 4:e // 4] == 0)
            # without float layers the call is tg_unpack_average, gradients not needed
            plan.tg_plan_set_layer_modes(None)
            t2, s2 = gpu_clip_stats(plan, dg, 2.5)
            assert np.array_equal(t2, base[0]) and np.array_equal(s2, base[1])
            plan.tg_unpack_average_mixed(dc, None, d_s, d_avg)
            torch.cuda.synchronize()
            assert_avg_close(d_avg.cpu().numpy(), want)
            plan.tg_plan_set_layer_modes(flags)
            with pytest.raises(binding.TgError):
                plan.tg_unpack_average_mixed(dc, None, d_s, d_avg)
            with pytest.raises(binding.TgError):
                plan.tg_plan_set_layer_modes(np.array([2] + [0] * (L - 1), np.uint8))
        finally:
            plan.close()
    # the only flagged layer is empty, no clipping: its tau is 0 all the same, the others are +inf
    off = _off([100, 0, 50])
    g = [dev(x) for x in _grads(rng, off, 2)]
    plan = binding.Plan(off, 2)
    try:
        plan.tg_plan_set_layer_modes(np.array([0, 1, 0], np.uint8))
        tau, s_local = gpu_clip_stats(plan, g, 0.0)
        assert np.all(tau[:, 1] == 0) and np.all(s_local[:, 1] == 0) and np.all(np.isinf(tau[:, [0, 2]]))
    finally:
        plan.close()


def test_random_layer_modes(oracle, binding):
    """40 seeded random models with random float flags (layers of every size class, empty ones too; with
    and without clipping): flagged layers get tau = s = 0 and zero codes, come out as the exact fp32 mean;
    the others as without flags"""
    rng = np.random.default_rng(4242)
    for case in range(40):
        L = int(rng.integers(1, 14))
        kinds = rng.integers(0, 5, size=L)
        sizes = [int([0, rng.integers(1, 12), rng.integers(1000, 1050), rng.integers(3000, 9000),
                      rng.integers(15000, 70000)][k]) for k in kinds]
        if sum(sizes) == 0:
            sizes[0] = 7
        off = _off(sizes)
        n = int(off[-1])
        flags = (rng.random(L) < 0.4).astype(np.uint8)
        W = int(rng.integers(1, 10))
        c = float(rng.choice([2.5, 1.0, 0.0]))
        grads = _grads(rng, off, W)
        plan = binding.Plan(off, W)
        try:
            plan.tg_plan_set_layer_modes(flags)
            dg = [dev(g) for g in grads]
            tau, s_local = gpu_clip_stats(plan, dg, c)
            fl = flags.astype(bool)
            assert np.all(tau[:, fl] == 0) and np.all(s_local[:, fl] == 0), case
            s_shared = gpu_share(plan, s_local)
            seed, step = int(rng.integers(0, 2 ** 63)), int(rng.integers(0, 2 ** 32))
            codes = gpu_ternarize(plan, dg, tau, s_shared, seed=seed, step=step)
            nb = (n + 3) // 4
            oc = [oracle.ternarize_pack(grads[w], off, tau[w], s_shared, seed, step, w) for w in range(W)]
            for w in range(W):
                assert np.array_equal(codes[w][:nb], oc[w]) and not codes[w][nb:].any(), (case, w)
            d_avg = torch.full((n,), 9.0, device="cuda")
            plan.tg_unpack_average_mixed([dev(x) for x in codes], dg, dev(s_shared), d_avg)
            torch.cuda.synchronize()
            got = d_avg.cpu().numpy()
            want = oracle.unpack_average(oc, off, s_shared)
            for l in range(L):
                b, e = int(off[l]), int(off[l + 1])
                if e == b:
                    continue
                if flags[l]:
                    assert np.array_equal(got[b:e], oracle.average_float([g[b:e] for g in grads])), (case, l)
                else:
                    assert_avg_close(got[b:e], want[b:e])
        finally:
            plan.close()


def test_float_layer_in_the_middle(oracle, binding):
    """A layer kept in fp32 anywhere in the flat buffer (Section 4.2 generalised): a plan over the
    layers before it, a plan over the layers after it (on the same buffers, offset), and the float call
    on the slice in between.  The only condition is the ABI's alignment: the slice begins and ends at a
    multiple of four elements.  Every element of the average is written by exactly one of the three."""
    rng = np.random.default_rng(29)
    sizes = [2400, 96, 51_204, 40_000, 100_001, 10, 4097]            # layer 3 stays in fp32
    off = _off(sizes)
    W, n, a, b = 3, int(off[-1]), int(off[3]), int(off[4])
    assert a % 4 == 0 and b % 4 == 0
    grads = _grads(rng, off, W)
    gd = [dev(g) for g in grads]
    avg = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    parts = ((0, a, off[:4]), (b, n, off[4:] - b))
    want = np.empty(n, np.float32)
    for lo, hi, off_p in parts:
        r = full_parity(oracle, binding, off_p, [g[lo:hi] for g in grads], step=7, worker_base=2)
        want[lo:hi] = r["avg"]
        plan = binding.Plan(off_p, W)
        try:
            sl = [g[lo:hi] for g in gd]
            tau, s_local = gpu_clip_stats(plan, sl, 2.5)
            s_shared = gpu_share(plan, s_local)
            assert np.array_equal(s_shared, r["s_shared"]) and np.array_equal(tau, r["tau"])
            codes = gpu_ternarize(plan, sl, tau, s_shared, 0, 7, worker_base=2)
            cd = [dev(c) for c in codes]
            plan.tg_unpack_average(cd, dev(s_shared), avg[lo:hi])
        finally:
            plan.close()
    binding.tg_average_float([g[a:b] for g in gd], b - a, avg[a:b])
    torch.cuda.synchronize()
    want[a:b] = oracle.average_float([g[a:b] for g in grads])
    got = avg.cpu().numpy()
    assert np.array_equal(got[a:b], want[a:b])
    assert_avg_close(np.concatenate([got[:a], got[b:]]), np.concatenate([want[:a], want[b:]]))


@pytest.mark.parametrize("W,bits", [(1, 4), (2, 4), (4, 4), (7, 4), (4, 8), (8, 8), (11, 8), (64, 8),
                                    (1, 2), (2, 3), (3, 3), (8, 5), (15, 5), (16, 6), (31, 6), (33, 7), (63, 7), (3, 5), (2, 6)])
def test_sum_pack_and_decode_sum(oracle, binding, W, bits):
    """Section 3.1 server-to-worker pull: k in narrow fields; bit-exact both ways, and the decoded
    average is bit-identical to tg_unpack_average on the same codes"""
    rng = np.random.default_rng(100 * W + bits)
    for sizes in ([37], [4096, 1, 3000, 5], [20000, 1029], [16384 * 2]):
        off = _off(sizes)
        n = int(off[-1])
        L = len(sizes)
        grads = _grads(rng, off, W)
        st = [oracle.clip_stats(g, off, 2.5) for g in grads]
        s = oracle.share_scalers(np.stack([x[1] for x in st]))
        codes = [oracle.ternarize_pack(g, off, st[w][0], s, 3, 4, w) for w, g in enumerate(grads)]
        plan = binding.Plan(off, W)
        try:
            cd = []
            for c in codes:
                buf = np.zeros(plan.packed_bytes, np.uint8)
                buf[:c.size] = c
                cd.append(dev(buf))
            nbytes = plan.tg_sum_bytes(bits)
            assert nbytes == ((n * bits + 7) // 8 + 15) // 16 * 16
            ksum = torch.full((nbytes,), 0xEE, dtype=torch.uint8, device="cuda")
            plan.tg_unpack_sum_pack(cd, bits, ksum)
            torch.cuda.synchronize()
            want = oracle.sum_pack(codes, n, bits)
            got = ksum.cpu().numpy()
            assert np.array_equal(got[:want.size], want) and not got[want.size:].any()
            avg = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
            plan.tg_decode_sum(W, dev(np.concatenate([want, np.zeros(nbytes - want.size, np.uint8)])), bits, dev(s), avg)
            torch.cuda.synchronize()
            assert_avg_close(avg.cpu().numpy(), oracle.decode_sum(want, bits, W, off, s))
            assert np.array_equal(avg.cpu().numpy(), gpu_unpack_average(plan, codes, s))
        finally:
            plan.close()


def test_sum_pack_rejects_fields_that_cannot_hold_the_sum(binding):
    off = _off([100])
    plan = binding.Plan(off, 8)
    try:
        c = [torch.zeros(plan.packed_bytes, dtype=torch.uint8, device="cuda")] * 8
        k = torch.zeros(plan.tg_sum_bytes(8), dtype=torch.uint8, device="cuda")
        with pytest.raises(binding.TgError) as e:
            plan.tg_unpack_sum_pack(c, 4, k)              # 17 levels do not fit 4 bits
        assert e.value.status == binding.TG_ERR_INVALID_ARG
        for bad in (1, 9, 0, -3):
            with pytest.raises(binding.TgError):
                plan.tg_unpack_sum_pack(c, bad, k)
            assert plan.tg_sum_bytes(bad) == -1
        plan.tg_unpack_sum_pack(c, 5, k)                   # 17 levels fit 5 bits
        torch.cuda.synchronize()
        with pytest.raises(binding.TgError):
            plan.tg_decode_sum(16, k, 5, torch.zeros(1, device="cuda"), torch.zeros(100, device="cuda"))   # 33 levels do not
        assert [binding.tg_sum_bits(N) for N in (1, 2, 3, 4, 7, 8, 16, 64)] == [2, 3, 3, 4, 4, 5, 6, 8]
        assert binding.tg_sum_bits(0) == -1 and binding.tg_sum_bits(65) == -1
    finally:
        plan.close()


def test_momentum_update(oracle, binding):
    rng = np.random.default_rng(23)
    off = _off([5000, 3, 4096, 2001, 20000])
    n = int(off[-1])
    for W, eta, mu in ((1, 0.1, 0.9), (4, 0.01, 0.9), (8, 0.5, 0.0), (5, 0.0, 0.5)):
        grads = _grads(rng, off, W)
        st = [oracle.clip_stats(g, off, 2.5) for g in grads]
        s = oracle.share_scalers(np.stack([x[1] for x in st]))
        codes = [oracle.ternarize_pack(g, off, st[w][0], s, 9, 1, w) for w, g in enumerate(grads)]
        v0 = (rng.normal(size=n) * float(s.max())).astype(np.float32)
        w0 = rng.normal(size=n).astype(np.float32)
        plan = binding.Plan(off, W)
        try:
            cd = []
            for c in codes:
                buf = np.zeros(plan.packed_bytes, np.uint8)
                buf[:c.size] = c
                cd.append(dev(buf))
            v_want, w_want = oracle.unpack_update_momentum(codes, off, s, eta, mu, v0, w0)
            avg = oracle.unpack_average(codes, off, s)
            both = []
            for kernel in (2, 1):                      # a wave per quarter tile, then the cooperative kernel
                v, w = dev(v0), dev(w0)
                plan.tg_plan_set_update_kernel(kernel)
                plan.tg_unpack_update_momentum(cd, dev(s), eta, mu, v, w)
                torch.cuda.synchronize()
                plan.tg_plan_set_update_kernel(0)
                both.append((v.cpu().numpy(), w.cpu().numpy()))
            assert np.array_equal(both[0][0], both[1][0]) and np.array_equal(both[0][1], both[1][1])
            vg, wg = both[1]
            # v' = mu v + avg: within 1e-6 of the larger term; w' = w - eta v': likewise
            v64 = v_want.astype(np.float64)
            sc_v = np.maximum(np.abs(mu * v0.astype(np.float64)), np.abs(avg.astype(np.float64)))
            assert np.all(np.abs(vg - v64) <= 1e-6 * sc_v + 1e-45)
            sc_w = np.maximum(np.abs(w0.astype(np.float64)), np.abs(eta * v64))
            assert np.all(np.abs(wg - w_want.astype(np.float64)) <= 1e-6 * sc_w)
            if mu == 0.0:
                assert np.array_equal(vg, gpu_unpack_average(plan, codes, s))
                assert np.array_equal(wg, gpu_unpack_update(plan, codes, s, eta, w0))
            with pytest.raises(binding.TgError):
                plan.tg_unpack_update_momentum(cd, dev(s), eta, mu, w, w)
        finally:
            plan.close()


@pytest.mark.parametrize("sizes,W", [([1], 1), ([4], 2), ([5], 1), ([6], 1), ([1023], 1), ([1024], 2), ([5119], 1),
                                     ([5120], 3), ([5121], 1), ([10240, 7, 0, 3000], 4), ([500, 20, 25000, 50, 400000, 500, 5000, 10], 2),
                                     ([70001, 33333], 5), ([9000] * 7, 8), ([4099, 4093], 11)])
def test_base3_container(oracle, binding, sizes, W):
    """five ternary values per byte: encoder bit-exact (incl. padding), decoder within 1e-6 and
    bit-identical to the 2-bit path on the same ternary values"""
    rng = np.random.default_rng(abs(hash((tuple(sizes), W, 3))) % (2 ** 32))
    off = _off(sizes)
    n = int(off[-1])
    grads = _grads(rng, off, W)
    st = [oracle.clip_stats(g, off, 2.5) for g in grads]
    tau = np.stack([x[0] for x in st])
    s = oracle.share_scalers(np.stack([x[1] for x in st]))
    want = [oracle.ternarize_pack_base3(g, off, tau[w], s, 31, 7, 2 + w) for w, g in enumerate(grads)]
    plan = binding.Plan(off, W)
    try:
        pb = plan.packed_bytes_base3
        assert pb == ((n + 4) // 5 + 15) // 16 * 16
        codes = [torch.full((pb,), 0xCD, dtype=torch.uint8, device="cuda") for _ in range(W)]
        plan.tg_ternarize_pack_base3([dev(g) for g in grads], dev(tau), dev(s), 31, 7, codes, worker_base=2)
        torch.cuda.synchronize()
        nb = (n + 4) // 5
        for w in range(W):
            got = codes[w].cpu().numpy()
            assert np.array_equal(got[:nb], want[w]), (w, int(np.flatnonzero(got[:nb] != want[w])[0]))
            assert not got[nb:].any()
        cd = []
        for c in want:
            buf = np.zeros(pb, np.uint8)
            buf[:c.size] = c
            cd.append(dev(buf))
        avg = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        plan.tg_unpack_average_base3(cd, dev(s), avg)
        torch.cuda.synchronize()
        assert_avg_close(avg.cpu().numpy(), oracle.unpack_average_base3(want, off, s))
        c2 = [oracle.ternarize_pack(g, off, tau[w], s, 31, 7, 2 + w) for w, g in enumerate(grads)]
        assert np.array_equal(avg.cpu().numpy(), gpu_unpack_average(plan, c2, s))
    finally:
        plan.close()


def test_base3_decoder_arbitrary_bytes(oracle, binding):
    rng = np.random.default_rng(29)
    off = _off([3000, 1, 6000, 1241])
    n = int(off[-1])
    for W in (1, 4, 5, 6, 11, 64):
        codes = [rng.integers(0, 256, size=(n + 4) // 5, dtype=np.uint8) for _ in range(W)]
        s = (np.abs(rng.normal(size=4)) + 0.01).astype(np.float32)
        plan = binding.Plan(off, W)
        try:
            cd = []
            for c in codes:
                buf = np.zeros(plan.packed_bytes_base3, np.uint8)
                buf[:c.size] = c
                cd.append(dev(buf))
            avg = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
            plan.tg_unpack_average_base3(cd, dev(s), avg)
            torch.cuda.synchronize()
            assert_avg_close(avg.cpu().numpy(), oracle.unpack_average_base3(codes, off, s))
        finally:
            plan.close()


def test_extreme_scalers(oracle, binding):
    """tiny (subnormal threshold products), huge and zero scalers: same decisions on both sides"""
    rng = np.random.default_rng(10)
    off = _off([2048, 2048, 2048, 2048])
    n = int(off[-1])
    scales = np.array([1e-37, 1e30, 1.0, 1e-3])
    g = np.concatenate([rng.normal(size=2048) * sc for sc in scales]).astype(np.float32)
    tau = np.array([[3e-37, 2e30, np.inf, 0.0]], np.float32)
    s = np.array([3e-37, 2.5e30, 0.0, 1e-3], np.float32)
    plan = binding.Plan(off, 1)
    try:
        got = gpu_ternarize(plan, [dev(g)], tau, s, 5, 6)[0]
        want = oracle.ternarize_pack(g, off, tau[0], s, 5, 6, 0)
        assert np.array_equal(got[:want.size], want)
    finally:
        plan.close()


def test_run_to_run_identical_statistics(binding):
    """no atomics, fixed order of the additions: the same bits from every run, in the looping shape of the
    statistics pass and in the one-shot shape (a plan for 64 workers of 8.4 M elements)"""
    rng = np.random.default_rng(11)
    for sizes, mw in (([100000, 50, 300000], 3), ([5_000_001, 3, 3_400_000], 64)):
        off = _off(sizes)
        grads = [dev(g) for g in _grads(rng, off, 3)]
        plan = binding.Plan(off, mw)
        try:
            a = gpu_clip_stats(plan, grads, 2.5)
            for _ in range(3):
                b = gpu_clip_stats(plan, grads, 2.5)
                assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
        finally:
            plan.close()


def test_side_stream_and_one_worker_per_call(oracle, binding):
    """calls are asynchronous on the caller's stream; n_workers = 1 with worker_base = rank (the
    one-worker-per-GPU deployment) gives the same codes as the batched launch"""
    rng = np.random.default_rng(41)
    off = _off([30000, 17, 70000])
    W = 3
    grads = _grads(rng, off, W)
    st = [oracle.clip_stats(g, off, 2.5) for g in grads]
    tau = np.stack([x[0] for x in st])
    s = oracle.share_scalers(np.stack([x[1] for x in st]))
    want = [oracle.ternarize_pack(g, off, tau[w], s, 11, 2, 5 + w) for w, g in enumerate(grads)]
    plan = binding.Plan(off, W)
    side = torch.cuda.Stream()
    try:
        gd = [dev(g) for g in grads]
        s_d = dev(s)
        torch.cuda.synchronize()
        nb = want[0].size
        with torch.cuda.stream(side):
            for w in range(W):
                codes = torch.full((plan.packed_bytes,), 0xCD, dtype=torch.uint8, device="cuda")
                plan.tg_ternarize_pack([gd[w]], dev(tau[w:w + 1]), s_d, 11, 2, [codes], worker_base=5 + w, stream=side)
                side.synchronize()
                assert np.array_equal(codes.cpu().numpy()[:nb], want[w])
    finally:
        plan.close()


def test_whole_step_replayed_from_a_hip_graph(oracle, binding):
    """the four calls (+ the step counter advance) captured once, replayed with eager work and
    synchronisations in between; every replay equals the eager step with the same counter, and the
    first one equals the oracle"""
    from paper_1705_07878_amd import workloads
    wl = workloads.lenet()
    W, n, L, off = wl.n_workers, wl.n, wl.n_layers, wl.offsets
    grads_np = [g.numpy() for g in workloads.make_gradients(wl, "cpu")]
    plan = binding.Plan(off, W)
    try:
        gd = [dev(g) for g in grads_np]
        tau = torch.empty((W, L), device="cuda")
        sl = torch.empty((W, L), device="cuda")
        ss = torch.empty((L,), device="cuda")
        codes = [torch.zeros(plan.packed_bytes, dtype=torch.uint8, device="cuda") for _ in range(W)]
        avg = torch.empty(n, device="cuda")
        step0 = 40
        step_dev = torch.tensor([step0], dtype=torch.int32, device="cuda")

        def eager(step):
            c = [torch.zeros(plan.packed_bytes, dtype=torch.uint8, device="cuda") for _ in range(W)]
            a = torch.empty(n, device="cuda")
            t2, s2, sh2 = torch.empty_like(tau), torch.empty_like(sl), torch.empty_like(ss)
            plan.tg_clip_stats(gd, wl.clip_c, t2, s2)
            plan.tg_share_scalers(W, s2, sh2)
            plan.tg_ternarize_pack(gd, t2, sh2, 123, step, c)
            plan.tg_unpack_average(c, sh2, a)
            torch.cuda.synchronize()
            return [x.cpu().numpy() for x in c], a.cpu().numpy(), t2.cpu().numpy(), sh2.cpu().numpy()

        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):                      # warm-up on the capture stream
            plan.tg_clip_stats(gd, wl.clip_c, tau, sl, stream=side)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            plan.tg_clip_stats(gd, wl.clip_c, tau, sl)
            plan.tg_share_scalers(W, sl, ss)
            plan.tg_ternarize_pack_devstep(gd, tau, ss, 123, step_dev, codes)
            plan.tg_unpack_average(codes, ss, avg)
            binding.tg_step_advance(step_dev, 1)
        for i in range(4):
            graph.replay()
            torch.cuda.synchronize()
            got_codes = [c.cpu().numpy() for c in codes]
            got_avg = avg.cpu().numpy()
            e_codes, e_avg, e_tau, e_s = eager(step0 + i)          # eager work between replays
            for w in range(W):
                assert np.array_equal(got_codes[w], e_codes[w]), (i, w)
            assert np.array_equal(got_avg, e_avg), i
            assert int(step_dev.item()) == step0 + i + 1
            if i == 0:
                nb = (n + 3) // 4
                for w in range(W):
                    want = oracle.ternarize_pack(grads_np[w], off, e_tau[w], e_s, 123, step0, w)
                    assert np.array_equal(got_codes[w][:nb], want)
    finally:
        plan.close()


def test_non_finite_and_subnormal_gradients_complete(oracle, binding):
    """NaN / Inf gradients give unspecified values but never a fault: the four calls complete with
    TG_OK, and a layer whose own inputs are finite is untouched by its neighbours: statistics and
    codes equal the oracle's, only valid codes (00, 01, 11) appear.  Subnormal gradients are ordinary inputs."""
    rng = np.random.default_rng(99)
    off = _off([3000, 5000, 1029, 4096])
    n = int(off[-1])
    grads = _grads(rng, off, 2)
    for g in grads:
        g[7] = np.nan; g[100] = np.inf; g[2999] = -np.inf                   # layer 0: non-finite
        g[8000:9029] = (rng.integers(-200, 200, size=1029) * 1.4e-45).astype(np.float32)   # layer 2: subnormals only
    plan = binding.Plan(off, 2)
    try:
        gd = [dev(g) for g in grads]
        tau, s_local = gpu_clip_stats(plan, gd, 2.5)
        s_shared = gpu_share(plan, s_local)
        codes = gpu_ternarize(plan, gd, tau, s_shared, 5, 6)
        avg = gpu_unpack_average(plan, codes, s_shared)
        torch.cuda.synchronize()
        assert avg.shape == (n,)
        # the finite layers (1, 2, 3) against the oracle, fed the same tau and s
        fin = slice(3000, n)
        off_f = off[1:] - 3000
        for w, g in enumerate(grads):
            o_tau, o_sl = oracle.clip_stats(g[fin], off_f, 2.5)
            assert np.allclose(tau[w, 1:], o_tau, rtol=1e-6, atol=0) and np.allclose(s_local[w, 1:], o_sl, rtol=1e-6, atol=0)
            c = codes[w][:(n + 3) // 4]
            assert not ((c >> 1) & ~c & 0x55).any(), "code 10 produced"
            # elements 3000.. start at a byte boundary (3000 = 4 * 750): the finite layers' bytes
            # equal the oracle's when it is fed what the GPU was fed
            tau_in = np.where(np.isfinite(tau[w]), tau[w], 0).astype(np.float32)
            s_in = np.where(np.isfinite(s_shared), s_shared, 0).astype(np.float32)
            g0 = np.where(np.isfinite(g), g, 0).astype(np.float32)
            want = oracle.ternarize_pack(g0, off, tau_in, s_in, 5, 6, w)
            assert np.array_equal(c[750:], want[750:])
        assert np.isfinite(avg[3000:]).all()
    finally:
        plan.close()


def test_argument_errors_on_device(binding):
    off = _off([100, 28])
    plan = binding.Plan(off, 2)
    try:
        g = torch.zeros(132, device="cuda")
        t = torch.zeros(4, device="cuda")
        codes = torch.zeros(plan.packed_bytes, dtype=torch.uint8, device="cuda")
        with pytest.raises(binding.TgError) as e:
            plan.tg_clip_stats([g, g, g], 2.5, t, t)
        assert e.value.status == binding.TG_ERR_TOO_MANY_WORKERS
        with pytest.raises(binding.TgError) as e:
            plan.tg_clip_stats([g[1:]], 2.5, t, t)
        assert e.value.status == binding.TG_ERR_ALIGNMENT
        with pytest.raises(binding.TgError) as e:
            plan.tg_ternarize_pack([g], t, t, 0, 0, [None])
        assert e.value.status == binding.TG_ERR_INVALID_ARG
        with pytest.raises(binding.TgError) as e:
            plan.tg_unpack_average([codes], t, g[1:])
        assert e.value.status == binding.TG_ERR_ALIGNMENT
        with pytest.raises(binding.TgError) as e:
            plan.tg_clip_stats([g], float("nan"), t, t)
        assert e.value.status == binding.TG_ERR_INVALID_ARG
        with pytest.raises(binding.TgError) as e:
            plan.tg_unpack_update([codes], t, float("inf"), g)
        assert e.value.status == binding.TG_ERR_INVALID_ARG
        with pytest.raises(binding.TgError) as e:
            plan.tg_unpack_update([codes], t, 0.1, g[1:])
        assert e.value.status == binding.TG_ERR_ALIGNMENT
    finally:
        plan.close()
