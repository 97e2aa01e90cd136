"""bench.py without a GPU: the parts of its contract that need none."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    for extra, env in ((["--gpus", "2"], {}), ([], {"WORLD_SIZE": "2"})):
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + extra, capture_output=True, text=True,
                           env={**os.environ, **env})
        assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_figure_comes_from_the_committed_profile():
    sys.path.insert(0, ROOT)
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
    b = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(b)
    for wl, lo, hi in (("alexnet", 1.0364e9, 1.05e9), ("flat", 3.4e10, 3.45e10)):
        t = b.traffic_from_profile("ternarize_pack", wl)
        assert t is not None and lo <= t <= hi          # at least the algorithmic bytes, at most 1.5 % more
    for wl, alg in (("alexnet", 304_826_120), ("flat", 6_000_000_000)):
        t = b.traffic_from_profile("unpack_average", wl)
        assert t is not None and alg <= t <= 1.015 * alg
    assert b.traffic_from_profile("ternarize_pack", "lenet") is None


def test_default_workload_is_the_largest_single_gpu_configuration():
    import re
    src = open(os.path.join(ROOT, "bench.py")).read()
    assert re.search(r'"--workload", default="flat"', src)
    assert re.search(r'"--also", default="alexnet,vgg_a"', src)
