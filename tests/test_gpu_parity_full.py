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
        # ---- oracle statistics, one worker at a time ----
        o_tau = np.empty((W, L), np.float32)
        o_sl = np.empty((W, L), np.float32)
        maxabs = np.empty((W, L), np.float32)
        for w in range(W):
            g = grads[w].cpu().numpy()
            o_tau[w], o_sl[w] = oracle.clip_stats(g, off, wl.clip_c)
            maxabs[w] = [np.abs(g[off[l]:off[l + 1]]).max() if off[l + 1] > off[l] else 0 for l in range(L)]
            del g
        for name, got, want in (("tau", tau_g.cpu().numpy(), o_tau), ("s_local", sl_g.cpu().numpy(), o_sl)):
            err = np.abs(got.astype(np.float64) - want.astype(np.float64))
            assert np.all(err <= np.maximum(REL * np.abs(want), REL * maxabs)), (name, float(err.max()))
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
        # ---- base-3 container at full size (skipped for the largest workload to bound the run time) ----
        if n * W <= 1_200_000_000:
            c3 = [torch.full((plan.packed_bytes_base3,), 0xCD, dtype=torch.uint8, device="cuda") for _ in range(W)]
            plan.tg_ternarize_pack_base3(grads, dev(o_tau), dev(o_s), wl.seed, wl.step, c3)
            torch.cuda.synchronize()
            nb3 = (n + 4) // 5
            o_c3 = []
            for w in range(W):
                oc = oracle.ternarize_pack_base3(grads[w].cpu().numpy(), off, o_tau[w], o_s, wl.seed, wl.step, w)
                gc = c3[w].cpu().numpy()
                assert np.array_equal(gc[:nb3], oc) and not gc[nb3:].any(), ("base-3 codes differ", w)
                o_c3.append(oc)
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
        # ---- the integer sum k in narrow fields and its decoder; momentum update (not for the largest
        # workload, to bound the run time) ----
        if n * W <= 1_200_000_000:
            bits = binding.tg_sum_bits(W)          # 4 bits for 4 workers, 5 for 8: ceil(log2(2W+1))
            nbytes = plan.tg_sum_bytes(bits)
            ksum = torch.full((nbytes,), 0xEE, dtype=torch.uint8, device="cuda")
            plan.tg_unpack_sum_pack(cd, bits, ksum)
            torch.cuda.synchronize()
            want = oracle.sum_pack(o_codes, n, bits)
            got = ksum.cpu().numpy()
            assert np.array_equal(got[:want.size], want) and not got[want.size:].any(), "k fields differ"
            kd = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
            kd[:want.size] = torch.from_numpy(want).cuda()
            avg2 = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
            plan.tg_decode_sum(W, kd, bits, dev(o_s), avg2)
            torch.cuda.synchronize()
            _avg_close_chunked(avg2, o_avg)
            del ksum, kd, avg2, want, got
            gen = torch.Generator("cuda").manual_seed(6)
            v0 = torch.randn(n, dtype=torch.float32, device="cuda", generator=gen) * float(o_s.max())
            w1 = torch.randn(n, dtype=torch.float32, device="cuda", generator=gen)
            v0_host, w1_host = v0.cpu().numpy(), w1.cpu().numpy()
            eta, mu = 0.01, 0.9
            plan.tg_unpack_update_momentum(cd, dev(o_s), eta, mu, v0, w1)
            torch.cuda.synchronize()
            v_want, w_want = oracle.unpack_update_momentum(o_codes, off, o_s, eta, mu, v0_host, w1_host)
            v64 = v_want.astype(np.float64)
            sc_v = np.maximum(np.abs(mu * v0_host.astype(np.float64)), np.abs(o_avg.astype(np.float64)))
            assert np.all(np.abs(v0.cpu().numpy() - v64) <= REL * sc_v + 1e-45)
            sc_w = np.maximum(np.abs(w1_host.astype(np.float64)), np.abs(eta * v64))
            assert np.all(np.abs(w1.cpu().numpy() - w_want.astype(np.float64)) <= REL * sc_w)
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
