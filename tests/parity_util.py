"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI
and compare it with the CPU oracle on the same inputs.

Protocol: (i) tau / s_local within 1e-6 relative, s_shared exact (see
stats_tolerance for the one regime where a relative bound cannot hold);
(ii) the ORACLE's tau and s_shared are fed to both sides, then code buffers are
compared byte for byte; (iii) the same codes and scaler go to both decoders,
averages within 1e-6 relative and zeros exact.
"""
import numpy as np
import torch

REL = 1e-6


def dev(a, dtype=None):
    t = torch.as_tensor(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def gpu_clip_stats(plan, grads_dev, c):
    W, L = len(grads_dev), plan.n_layers
    tau = torch.full((W, L), float("nan"), dtype=torch.float32, device="cuda")
    s_local = torch.full((W, L), float("nan"), dtype=torch.float32, device="cuda")
    plan.tg_clip_stats(grads_dev, c, tau, s_local)
    torch.cuda.synchronize()
    return tau.cpu().numpy(), s_local.cpu().numpy()


def gpu_share(plan, s_local):
    W, L = s_local.shape
    out = torch.full((L,), float("nan"), dtype=torch.float32, device="cuda")
    plan.tg_share_scalers(W, dev(s_local), out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def gpu_ternarize(plan, grads_dev, tau, s_shared, seed, step, worker_base=0):
    W = len(grads_dev)
    codes = [torch.full((plan.packed_bytes,), 0xCD, dtype=torch.uint8, device="cuda") for _ in range(W)]
    plan.tg_ternarize_pack(grads_dev, dev(tau), dev(s_shared), seed, step, codes, worker_base=worker_base)
    torch.cuda.synchronize()
    return [c.cpu().numpy() for c in codes]


def gpu_unpack_average(plan, codes_np, s_shared):
    pb = plan.packed_bytes
    cd = []
    for c in codes_np:
        buf = np.zeros(pb, np.uint8)
        buf[:c.size] = c
        cd.append(dev(buf))
    avg = torch.full((plan.n,), float("nan"), dtype=torch.float32, device="cuda")
    plan.tg_unpack_average(cd, dev(s_shared), avg)
    torch.cuda.synchronize()
    return avg.cpu().numpy()


def gpu_unpack_update(plan, codes_np, s_shared, eta, w0, kernel=0):
    """kernel: 0 = the library's own choice by size, 1 / 2 = force one of the two update kernels"""
    pb = plan.packed_bytes
    cd = []
    for c in codes_np:
        buf = np.zeros(pb, np.uint8)
        buf[:c.size] = c
        cd.append(dev(buf))
    w = dev(w0)
    plan.tg_plan_set_update_kernel(kernel)
    try:
        plan.tg_unpack_update(cd, dev(s_shared), eta, w)
        torch.cuda.synchronize()
    finally:
        plan.tg_plan_set_update_kernel(0)
    return w.cpu().numpy()


def assert_update_close(got, want, w0, avg):
    """w' = w - eta*avg within 1e-6 of the larger of |w| and |eta*avg| (a difference has no
    relative accuracy of its own when the two nearly cancel); where the average is 0 the weight
    is untouched, bit for bit"""
    assert np.array_equal(got[avg == 0], w0[avg == 0])
    w64, want64 = w0.astype(np.float64), want.astype(np.float64)
    err = np.abs(got.astype(np.float64) - want64)
    scale = np.maximum(np.abs(w64), np.abs(want64 - w64))
    assert np.all(err <= REL * scale), float((err / np.maximum(scale, 1e-300)).max())


# worst relative error seen per quantity, over the layers held to the relative bound; printed at
# the end of a test session (tests/conftest.py) and by smoke()
WORST = {}


def note_worst(what, value):
    WORST[what] = max(WORST.get(what, 0.0), float(value))


def layer_mean_minus_first(g, off):
    """|mean - first element| of every layer (0 for an empty one), in fp64"""
    off = np.asarray(off, np.int64)
    out = np.zeros(off.size - 1, np.float64)
    full = np.flatnonzero(off[1:] > off[:-1])
    if full.size:
        # consecutive non-empty layers tile [0, n)
        sums = np.add.reduceat(g, off[full], dtype=np.float64)
        out[full] = np.abs(sums / (off[full + 1] - off[full]) - g[off[full]].astype(np.float64))
    return out


def stats_tolerance(want, g, off, c):
    """Allowed |got - want| per layer for tau and s_local of one worker, and the layers held to the
    pure relative bound.

    The statistics pass takes sum(g - K) and sum((g - K)^2) in fp64 about the pivot K = first element
    of the layer, in one read.  With gamma <= 3e-14 the relative error of each sum (at most 256 serial
    additions per thread, then a tree), the variance sigma^2 = S2/n - (S1/n)^2 carries an absolute error
    of at most 3 gamma (sigma^2 + d^2), d = mean - K, so
        |d sigma| / sigma <= 1.5 gamma (1 + d^2 / sigma^2)      and always      |d sigma| <= sqrt(3 gamma) (sigma + |d|).
    Hence: wherever sigma >= 1e-3 |d| (every layer whose first element is not a million-sigma outlier)
    the error is below 5e-8 relative and the test demands 1e-6 RELATIVE, nothing else.  Only for a
    layer with sigma < 1e-3 |d| is the bound absolute: c * 1e-6 * |d|  (sqrt(3 gamma) = 3e-7).  Since the
    first element alone contributes d^2 / n to the variance, sigma >= |d| / sqrt(n): that regime needs a
    layer of more than 10^6 elements whose first element carries nearly all of its variance.
    """
    want = np.asarray(want, np.float64)
    d = layer_mean_minus_first(g, off)
    finite = np.isfinite(want)
    sigma = np.where(finite, want, 0.0) / c if (c > 0 and np.isfinite(c)) else np.zeros_like(want)
    relative = finite & (sigma >= 1e-3 * d)
    tol = np.where(relative, REL * np.abs(np.where(finite, want, 0.0)), REL * abs(c) * d)
    return tol, relative


def assert_stats_close(got, want, grads_np, off, what, c, want_tau=None):
    """tau or s_local [W][L] against the oracle's.  want_tau: the oracle's tau when `want` is s_local
    (the regime of a layer is decided by its sigma = tau / c)."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape
    noclip = not (c > 0 and np.isfinite(c))
    for w in range(want.shape[0]):
        a, b = got[w], want[w]
        if noclip:
            # tau = +inf and s_local = max|g|: exact on both sides
            assert np.array_equal(a, b), (what, w)
            continue
        tol, relative = stats_tolerance(b if want_tau is None else want_tau[w], grads_np[w], off, c)
        err = np.abs(a - b)
        bad = ~(err <= tol)                                              # a NaN is bad too
        assert not bad.any(), (what, w, int(np.flatnonzero(bad)[0]), a[bad][0], b[bad][0])
        nz = relative & (b != 0)
        if nz.any():
            note_worst(what + " rel.err", (err[nz] / np.abs(b[nz])).max())


def assert_avg_close(got, want):
    assert got.shape == want.shape
    zero = want == 0
    assert np.all(got[zero] == 0), "zeros of the average must be exact"
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    assert np.all(err <= REL * np.abs(want.astype(np.float64))), float((err / np.maximum(np.abs(want), 1e-300)).max())


def full_parity(oracle, binding, off, grads_np, c=2.5, seed=0, step=0, worker_base=0, max_workers=None):
    """All four calls against the oracle on one input set. Returns what the oracle computed."""
    off = np.asarray(off, np.int64)
    W = len(grads_np)
    n = int(off[-1])
    plan = binding.Plan(off, W if max_workers is None else max_workers)
    try:
        assert plan.n == n and plan.n_layers == off.size - 1
        assert plan.packed_bytes == ((n + 3) // 4 + 15) // 16 * 16
        gd = [dev(g) for g in grads_np]
        # (i) statistics
        o_tau, o_sloc = zip(*[oracle.clip_stats(g, off, c) for g in grads_np])
        o_tau, o_sloc = np.stack(o_tau), np.stack(o_sloc)
        g_tau, g_sloc = gpu_clip_stats(plan, gd, c)
        assert_stats_close(g_tau, o_tau, grads_np, off, "tau", c)
        assert_stats_close(g_sloc, o_sloc, grads_np, off, "s_local", c, want_tau=o_tau)
        # Eq. 4 is exact
        o_s = oracle.share_scalers(o_sloc)
        assert np.array_equal(gpu_share(plan, o_sloc), o_s)
        # (ii) codes, fed the oracle's tau and s
        o_codes = [oracle.ternarize_pack(g, off, o_tau[w], o_s, seed, step, worker_base + w)
                   for w, g in enumerate(grads_np)]
        g_codes = gpu_ternarize(plan, gd, o_tau, o_s, seed, step, worker_base)
        nb = (n + 3) // 4
        for w in range(W):
            assert np.array_equal(g_codes[w][:nb], o_codes[w]), ("codes differ", w,
                                                                   int(np.flatnonzero(g_codes[w][:nb] != o_codes[w])[0]))
            assert not g_codes[w][nb:].any(), "padding bytes must be 0"
        # (iii) averages from the same codes and scaler
        o_avg = oracle.unpack_average(o_codes, off, o_s)
        g_avg = gpu_unpack_average(plan, o_codes, o_s)
        assert_avg_close(g_avg, o_avg)
        # the fused update line of Algorithm 1 from the same codes
        w0 = (np.random.default_rng(n + W).normal(size=n) * 0.05).astype(np.float32)
        eta = 0.125 if n % 2 else 0.01
        o_upd = oracle.unpack_update(o_codes, off, o_s, eta, w0)
        upd = [gpu_unpack_update(plan, o_codes, o_s, eta, w0, kernel=k) for k in (1, 2)]
        assert_update_close(upd[0], o_upd, w0, o_avg)
        assert np.array_equal(upd[0], upd[1]), "the two update kernels must agree bit for bit"
        return dict(tau=o_tau, s_local=o_sloc, s_shared=o_s, codes=o_codes, avg=o_avg)
    finally:
        plan.close()
