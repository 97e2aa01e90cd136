"""bench.py's bandwidth probes (bench_probe.hip -> libbench_probe.so): a measurement instrument, not
part of the library; checked here for moving exactly the bytes they claim to move."""
import importlib.util
import os

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def bench():
    spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
    b = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(b)
    return b


def test_probe_kernels_move_what_they_claim(bench):
    """copy reproduces the source, the two write probes fill the destination, the thin stream holds
    the XOR of every 16 consecutive words, the read probes leave the destination alone"""
    n = 4096 * 80
    src = torch.randn(n, device="cuda")
    dst = torch.full((n,), -7.0, device="cuda")
    thin = torch.zeros(n // 16, dtype=torch.int32, device="cuda")
    for kind in (0, 1, 9, 10):
        bench.bench_probe(torch, kind, src, dst, thin, n)
    torch.cuda.synchronize()
    assert bool((dst == -7.0).all())
    bench.bench_probe(torch, 3, src, dst, thin, n)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    for kind in (2, 5, 6):
        dst.fill_(-7.0)
        bench.bench_probe(torch, kind, src, dst, thin, n)
        torch.cuda.synchronize()
        assert dst.view(-1, 4)[:, :3].eq(torch.tensor([1.0, 2.0, 3.0], device="cuda")).all()
        assert bool((dst.view(-1, 4)[:, 3] >= 0).all())
    dst.fill_(-7.0)
    bench.bench_probe(torch, 7, src, dst, thin, n)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    thin.zero_()
    bench.bench_probe(torch, 8, src, dst, thin, n)
    torch.cuda.synchronize()
    assert not bool(thin[256 * 64:].any()) and bool(thin[:256 * 64].any())     # only the first 64 KiB is written
    bench.bench_probe(torch, 4, src, dst, thin, n)
    torch.cuda.synchronize()
    want = np.bitwise_xor.reduce(src.cpu().numpy().view(np.uint32).reshape(-1, 16), axis=1)
    assert np.array_equal(thin.cpu().numpy().view(np.uint32), want)
    for bad in (lambda: bench.bench_probe(torch, 11, src, dst, thin, n),
                lambda: bench.bench_probe(torch, 9, src, dst, thin, 4096 * 3),
                lambda: bench.bench_probe(torch, 0, src, dst, thin, 1024),
                lambda: bench.bench_probe(torch, 4, src, dst, None, n),
                lambda: bench.bench_probe(torch, 1, src[1:], dst, thin, 4096)):
        with pytest.raises(RuntimeError):
            bad()
