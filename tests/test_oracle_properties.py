"""Property tests of the CPU oracle on random small models (hypothesis): the relations between its
functions that the paper's definitions fix, checked with numpy written out here.

  Eq. 5, Eq. 2   tau = c * population std, s_local = min(max|g|, tau)      (numpy)
  Eq. 4          s = max over workers
  Eq. 1, Eq. 3   ternary values in {-1, 0, +1}; the sign of g where non-zero; an element whose clipped
                 magnitude equals s is never dropped; a zero is never kept; never kept where Eq. 3 says
                 the probability is 0 (a = 0) and always where it is 1 (a = s)
  Section 3.1    the 2-bit buffer, the base-3 buffer and the k fields hold the same integers
  Algorithm 1    average = s/N * sum of the workers' ternary values, to the last bit of an fp64 product
"""
import numpy as np
import pytest
from hypothesis import HealthCheck, given, settings
from hypothesis import strategies as st


def _decode2(codes, n):
    f = (codes[:, None] >> np.array([0, 2, 4, 6], np.uint8)) & 3
    f = f.reshape(-1)[:n].astype(np.int64)
    return np.where(f >= 2, f - 4, f)


def _decode3(codes3, n):
    v = codes3.astype(np.int64)
    d = np.stack([(v // 3 ** m) % 3 for m in range(5)], axis=1).reshape(-1)[:n]
    return np.where(d == 2, -1, d)


models = st.lists(st.integers(0, 70), min_size=1, max_size=7).filter(lambda s: sum(s) > 0)


@settings(max_examples=60, deadline=None, derandomize=True, database=None,
          suppress_health_check=[HealthCheck.function_scoped_fixture, HealthCheck.too_slow])
@given(sizes=models, W=st.integers(1, 9), seed=st.integers(0, 2 ** 64 - 1), step=st.integers(0, 2 ** 32 - 1),
       c=st.sampled_from([0.5, 1.0, 2.5, 0.0]), data=st.integers(0, 2 ** 31))
def test_relations_between_the_oracle_functions(oracle, sizes, W, seed, step, c, data):
    rng = np.random.default_rng(data)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    n, L = int(off[-1]), len(sizes)
    grads = [(rng.normal(size=n) * 10.0 ** rng.uniform(-4, 1) + rng.normal() * 1e-3).astype(np.float32) for _ in range(W)]
    for g in grads:
        g[rng.integers(0, n, size=max(1, n // 8))] = 0.0
    taus, sloc = [], []
    for g in grads:
        tau, s = oracle.clip_stats(g, off, c)
        for l in range(L):
            seg = g[off[l]:off[l + 1]].astype(np.float64)
            if seg.size == 0:
                want_tau = np.float32(np.inf) if c <= 0 else np.float32(0)
                assert tau[l] == want_tau and s[l] == 0
                continue
            want_tau = np.float32(np.inf) if c <= 0 else np.float32(np.float64(np.float32(c)) * seg.std())
            assert tau[l] == want_tau
            assert s[l] == min(np.float32(np.abs(seg).max()), tau[l])
        taus.append(tau)
        sloc.append(s)
    s = oracle.share_scalers(np.stack(sloc))
    assert np.array_equal(s, np.max(np.stack(sloc), axis=0))
    lay = np.repeat(np.arange(L), np.diff(off))
    ts = []
    for w, g in enumerate(grads):
        codes = oracle.ternarize_pack(g, off, taus[w], s, seed, step, w)
        assert codes.size == (n + 3) // 4
        t = _decode2(codes, n)
        assert set(np.unique(t)) <= {-1, 0, 1}
        a = np.minimum(np.abs(g), taus[w][lay])
        assert not t[a == 0].any()                                   # P = 0
        assert np.all(t[a == s[lay]][a[a == s[lay]] > 0] != 0)       # P = 1
        nz = t != 0
        assert np.array_equal(t[nz], np.where(np.signbit(g[nz]), -1, 1))
        pad = (4 - n % 4) % 4
        assert (codes[-1] >> (8 - 2 * pad)) == 0 if pad else True
        c3 = oracle.ternarize_pack_base3(g, off, taus[w], s, seed, step, w)
        assert c3.size == (n + 4) // 5 and np.array_equal(_decode3(c3, n), t)
        ts.append((codes, c3, t))
    k = np.sum([t for _, _, t in ts], axis=0)
    want = (k.astype(np.float64) * s[lay].astype(np.float64) / W).astype(np.float32)
    avg = oracle.unpack_average([x[0] for x in ts], off, s)
    assert np.array_equal(avg, want)
    assert np.array_equal(oracle.unpack_average_base3([x[1] for x in ts], off, s), want)
    bits = oracle.sum_bits(W)
    assert 2 ** (bits - 1) < 2 * W + 1 <= 2 ** bits
    ks = oracle.sum_pack([x[0] for x in ts], n, bits)
    stream = np.unpackbits(ks, bitorder="little")
    f = stream[:n * bits].reshape(n, bits).astype(np.int64) @ (1 << np.arange(bits))
    fields = np.where(f >= 2 ** (bits - 1), f - 2 ** bits, f)
    assert np.array_equal(fields, k)
    assert np.array_equal(oracle.decode_sum(ks, bits, W, off, s), want)
    # update lines of Algorithm 1 on top of the same average
    w0 = rng.normal(size=n).astype(np.float32)
    eta = np.float32(0.03)
    got = oracle.unpack_update([x[0] for x in ts], off, s, eta, w0)
    ref = (w0.astype(np.float64) - np.float64(eta) * (k.astype(np.float64) * s[lay].astype(np.float64) / W)).astype(np.float32)
    assert np.array_equal(got, ref)
