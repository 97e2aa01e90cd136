"""AddressSanitizer + UndefinedBehaviorSanitizer over the HOST code: the whole oracle, and the
library's table builder and argument checks (no GPU, no kernel runs: device code cannot be
sanitized on this machine)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)


def _run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, "%s\n%s" % (" ".join(cmd), r.stdout[-4000:])
    return r.stdout


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_driver")
    _run(["gcc", "-std=c11", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
          "-fno-omit-frame-pointer", "-ffp-contract=off", "-fopenmp", "-I", os.path.join(ROOT, "oracle"),
          os.path.join(SAN, "oracle_driver.c"), os.path.join(ROOT, "oracle", "tg_oracle.c"), "-lm", "-o", exe])
    out = _run([exe], env=ENV)
    assert out.startswith("ok") and "runtime error" not in out and "AddressSanitizer" not in out


def test_abi_host_code_under_asan_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc) and shutil.which("hipcc") is None:
        pytest.skip("hipcc not available")
    exe = str(tmp_path / "abi_driver")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-omit-frame-pointer"]
    out = _run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-ffp-contract=off",
                "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"] + san +
               ["-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "paper_1705_07878_amd", "csrc", "terngrad.hip"),
                os.path.join(SAN, "abi_driver.cpp"), "-o", exe])
    out = _run([exe], env=ENV)
    assert "ok tiles=" in out and "runtime error" not in out and "AddressSanitizer" not in out
