"""GPU parity at the full sizes of the AlexNet-, VGG-A-shaped and flat 1e9 configurations, in the
batched launch configuration bench.py times (all W workers per launch).

Gradients are generated on the device; the host copy of the same bytes goes to the oracle, one
worker at a time.  Oracle inputs never come from the HIP path: tau, s and the code buffers that feed
the GPU decode are the oracle's own.
"""
import os

import numpy as np
import pytest
import torch

from parity_util import REL, assert_stats_close, assert_update_close, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    from paper_1705_07878_amd import binding as b
    return b


def _threads():
    n = len(os.sched_getaffinity(0))
    return max(1, min(n, int(os.environ.get("OMP_NUM_THREADS", n)), 16))


def _avg_close_chunked(got_dev, want, chunk=1 << 26):
    n = want.size
    for a in range(0, n, chunk):
        b = min(n, a + chunk)
        g = got_dev[a:b].cpu().numpy()
        w = want[a:b]
        zero = w == 0
        assert np.all(g[zero] == 0)
        err = np.abs(g.astype(np.float64) - w.astype(np.float64))
        assert np.all(err <= REL * np.abs(w.astype(np.float64))), (a, float(err.max()))


def _momentum_close_chunked(v_dev, w_dev, v_want, w_want, v0, w0, avg, eta, mu, chunk=1 << 26):
    """v' = mu v + avg within 1e-6 of the larger term, w' = w - eta v' within 1e-6 of the larger of |w|, |eta v'|"""
    for a in range(0, v_want.size, chunk):
        b = min(v_want.size, a + chunk)
        v64 = v_want[a:b].astype(np.float64)
        sc_v = np.maximum(np.abs(mu * v0[a:b].astype(np.float64)), np.abs(avg[a:b].astype(np.float64)))
        assert np.all(np.abs(v_dev[a:b].cpu().numpy() - v64) <= REL * sc_v + 1e-45), ("velocity", a)
        sc_w = np.maximum(np.abs(w0[a:b].astype(np.float64)), np.abs(eta * v64))
        assert np.all(np.abs(w_dev[a:b].cpu().numpy() - w_want[a:b].astype(np.float64)) <= REL * sc_w), ("weights", a)


def _full_config(oracle, binding, wl):
    from paper_1705_07878_amd import workloads
    W, n, L, off = wl.n_workers, wl.n, wl.n_layers, wl.offsets
    oracle.set_threads(_threads())
    try:
        grads = [workloads.make_gradient(wl, w, "cuda") for w in range(W)]
        plan = binding.Plan(off, W)
        nb = (n + 3) // 4
        # ---- GPU statistics, batched over the W workers ----
        tau_g = torch.empty((W, L), dtype=torch.float32, device="cuda")
        sl_g = torch.empty((W, L), dtype=torch.float32, device="cuda")
        plan.tg_clip_stats(grads, wl.clip_c, tau_g, sl_g)
        torch.cuda.synchronize()
        # ---- oracle statistics, one worker at a time; tolerance: 1e-6 relative (parity_util.stats_tolerance) ----
        o_tau = np.empty((W, L), np.float32)
        o_sl = np.empty((W, L), np.float32)
        tau_h, sl_h = tau_g.cpu().numpy(), sl_g.cpu().numpy()
        for w in range(W):
            g = grads[w].cpu().numpy()
            o_tau[w], o_sl[w] = oracle.clip_stats(g, off, wl.clip_c)
            assert_stats_close(tau_h[w:w + 1], o_tau[w:w + 1], [g], off, wl.name + " tau", wl.clip_c)
            assert_stats_close(sl_h[w:w + 1], o_sl[w:w + 1], [g], off, wl.name + " s_local", wl.clip_c,
                               want_tau=o_tau[w:w + 1])
            del g
        o_s = oracle.share_scalers(o_sl)
        s_g = torch.empty((L,), dtype=torch.float32, device="cuda")
        plan.tg_share_scalers(W, dev(o_sl), s_g)
        torch.cuda.synchronize()
        assert np.array_equal(s_g.cpu().numpy(), o_s)
        # ---- codes: both sides fed the oracle's tau and s; batched GPU launch ----
        codes_g = [torch.full((plan.packed_bytes,), 0xCD, dtype=torch.uint8, device="cuda") for _ in range(W)]
        plan.tg_ternarize_pack(grads, dev(o_tau), dev(o_s), wl.seed, wl.step, codes_g)
        torch.cuda.synchronize()
        o_codes = []
        for w in range(W):
            g = grads[w].cpu().numpy()
            oc = oracle.ternarize_pack(g, off, o_tau[w], o_s, wl.seed, wl.step, w)
            del g
            gc = codes_g[w].cpu().numpy()
            assert np.array_equal(gc[:nb], oc), ("codes differ", w, int(np.flatnonzero(gc[:nb] != oc)[0]))
            assert not gc[nb:].any()
            o_codes.append(oc)
        # ---- the rows beyond the four calls run on the first Wf workers: all of them, except on the
        # largest workload, where two keep the oracle's share of the run time bounded (the element,
        # byte and block indices they reach are the same)
        Wf = W if n * W <= 1_200_000_000 else min(W, 2)
        # ---- base-3 container at full size ----
        c3 = [torch.full((plan.packed_bytes_base3,), 0xCD, dtype=torch.uint8, device="cuda") for _ in range(Wf)]
        plan.tg_ternarize_pack_base3(grads[:Wf], dev(o_tau[:Wf]), dev(o_s), wl.seed, wl.step, c3)
        torch.cuda.synchronize()
        nb3 = (n + 4) // 5
        o_c3 = []
        for w in range(Wf):
            oc = oracle.ternarize_pack_base3(grads[w].cpu().numpy(), off, o_tau[w], o_s, wl.seed, wl.step, w)
            gc = c3[w].cpu().numpy()
            assert np.array_equal(gc[:nb3], oc) and not gc[nb3:].any(), ("base-3 codes differ", w)
            o_c3.append(oc)
            del gc
        a3 = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        plan.tg_unpack_average_base3(c3, dev(o_s), a3)      # c3 equals the oracle's bytes (just checked)
        torch.cuda.synchronize()
        _avg_close_chunked(a3, oracle.unpack_average_base3(o_c3, off, o_s))
        del c3, a3, o_c3
        # second moment at full size (Appendix A): non-zero codes ~ sum a/s, here just a sanity band
        nz = float(np.mean(np.unpackbits(o_codes[0][: 1 << 22]).reshape(-1, 2)[:, 1]))
        assert 0.05 < nz < 0.6
        del grads
        # ---- decode + average of the oracle's codes ----
        cd = []
        for oc in o_codes:
            t = torch.zeros(plan.packed_bytes, dtype=torch.uint8, device="cuda")
            t[:nb] = torch.from_numpy(oc).cuda()
            cd.append(t)
        avg_g = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        plan.tg_unpack_average(cd, dev(o_s), avg_g)
        torch.cuda.synchronize()
        o_avg = oracle.unpack_average(o_codes, off, o_s)
        _avg_close_chunked(avg_g, o_avg)
        del avg_g
        # ---- fused decode + update from the same codes ----
        w0 = torch.randn(n, dtype=torch.float32, device="cuda", generator=torch.Generator("cuda").manual_seed(5)) * 0.05
        w0_host = w0.cpu().numpy()
        plan.tg_unpack_update(cd, dev(o_s), 0.01, w0)
        torch.cuda.synchronize()
        o_w = oracle.unpack_update(o_codes, off, o_s, 0.01, w0_host)
        assert_update_close(w0.cpu().numpy(), o_w, w0_host, o_avg)
        del w0, w0_host, o_w
        # ---- the integer sum k in the narrowest field that holds it, and its decoder; momentum update
        # (on the first Wf workers, see above) ----
        del o_avg
        cdf, o_codes_f = cd[:Wf], o_codes[:Wf]
        o_avg_f = oracle.unpack_average(o_codes_f, off, o_s)
        bits = binding.tg_sum_bits(Wf)          # ceil(log2(2W+1)): 2, 3, 4, 5 bits for 1, 2, 4, 8 workers
        nbytes = plan.tg_sum_bytes(bits)
        ksum = torch.full((nbytes,), 0xEE, dtype=torch.uint8, device="cuda")
        plan.tg_unpack_sum_pack(cdf, bits, ksum)
        torch.cuda.synchronize()
        want = oracle.sum_pack(o_codes_f, n, bits)
        got = ksum.cpu().numpy()
        assert np.array_equal(got[:want.size], want) and not got[want.size:].any(), "k fields differ"
        kd = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
        kd[:want.size] = torch.from_numpy(want).cuda()
        avg2 = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        plan.tg_decode_sum(Wf, kd, bits, dev(o_s), avg2)
        torch.cuda.synchronize()
        _avg_close_chunked(avg2, o_avg_f)
        del ksum, kd, avg2, want, got
        gen = torch.Generator("cuda").manual_seed(6)
        v0 = torch.randn(n, dtype=torch.float32, device="cuda", generator=gen) * float(o_s.max())
        w1 = torch.randn(n, dtype=torch.float32, device="cuda", generator=gen)
        v0_host, w1_host = v0.cpu().numpy(), w1.cpu().numpy()
        eta, mu = 0.01, 0.9
        plan.tg_unpack_update_momentum(cdf, dev(o_s), eta, mu, v0, w1)
        torch.cuda.synchronize()
        v_want, w_want = oracle.unpack_update_momentum(o_codes_f, off, o_s, eta, mu, v0_host, w1_host)
        _momentum_close_chunked(v0, w1, v_want, w_want, v0_host, w1_host, o_avg_f, eta, mu)
        plan.close()
    finally:
        oracle.set_threads(1)


def test_alexnet_full(oracle, binding):
    from paper_1705_07878_amd import workloads
    _full_config(oracle, binding, workloads.alexnet())


def test_vgg_a_full(oracle, binding):
    from paper_1705_07878_amd import workloads
    _full_config(oracle, binding, workloads.vgg_a())


def test_flat_1e9_full(oracle, binding):
    from paper_1705_07878_amd import workloads
    _full_config(oracle, binding, workloads.flat())


def test_indices_beyond_2_31(oracle, binding):
    """one worker, two layers, n = 2^31 + 70001: element, byte and Philox-block indices past 32 bits"""
    from paper_1705_07878_amd import workloads
    wl = workloads.custom([(1 << 31) - 12345, 12345 + 70001], 1, name="beyond 2^31", sigma_fixed=2e-3)
    _full_config(oracle, binding, wl)
