"""No-GPU checks of the C ABI: the library loads, exports every symbol the
header declares, rejects bad arguments before touching a device, and derives
the right tables from an offset table."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_1705_07878_amd import build
    build.build(force=False, verbose=False)
    from paper_1705_07878_amd import binding as b
    return b


def test_every_declared_symbol_is_exported(binding):
    hdr = open(os.path.join(ROOT, "include", "terngrad.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(tg_[a-z_0-9]+)\s*\(", hdr))
    assert {"tg_clip_stats", "tg_share_scalers", "tg_ternarize_pack", "tg_unpack_average",
            "tg_plan_create", "tg_plan_destroy"} <= names
    for name in names:
        assert hasattr(binding.lib, name), name


def test_strerror_and_status_values(binding):
    assert binding.tg_strerror(0) == "ok"
    for st in (-1, -2, -3, -4, -5, -6):
        assert binding.tg_strerror(st) not in ("ok", "unknown status")
    assert binding.tg_strerror(-99) == "unknown status"
    hdr = open(os.path.join(ROOT, "include", "terngrad.h")).read()
    assert int(re.search(r"#define TG_MAX_WORKERS (\d+)", hdr).group(1)) == binding.TG_MAX_WORKERS


def _create(binding, off, max_workers=2):
    off = np.asarray(off, np.int64)
    h = ctypes.c_void_p()
    st = binding.lib.tg_plan_create(off.size - 1, off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                    max_workers, ctypes.byref(h))
    return st, h


def test_plan_create_rejects_bad_tables_before_any_device_call(binding):
    assert _create(binding, [1, 5])[0] == binding.TG_ERR_INVALID_ARG          # off[0] != 0
    assert _create(binding, [0, 5, 3])[0] == binding.TG_ERR_INVALID_ARG       # not monotone
    assert _create(binding, [0, 0])[0] == binding.TG_ERR_INVALID_ARG          # n = 0
    assert _create(binding, [0, (1 << 35) + 1])[0] == binding.TG_ERR_INVALID_ARG   # beyond TG_MAX_ELEMENTS
    assert _create(binding, [0, 8], 0)[0] == binding.TG_ERR_INVALID_ARG
    assert _create(binding, [0, 8], 65)[0] == binding.TG_ERR_TOO_MANY_WORKERS
    st = binding.lib.tg_plan_create(1, None, 1, ctypes.byref(ctypes.c_void_p()))
    assert st == binding.TG_ERR_INVALID_ARG
    st = binding.lib.tg_plan_create(1, (ctypes.c_int64 * 2)(0, 8), 1, None)
    assert st == binding.TG_ERR_INVALID_ARG


def test_null_plan_is_rejected(binding):
    assert binding.lib.tg_plan_destroy(None) == binding.TG_OK
    assert binding.lib.tg_num_elements(None) == -1
    assert binding.lib.tg_packed_bytes(None) == -1
    assert binding.lib.tg_clip_stats(None, 1, None, 2.5, None, None, None) == binding.TG_ERR_INVALID_ARG
    assert binding.lib.tg_clip_stats_static(None, 1, None, 2.5, None, None, None) == binding.TG_ERR_INVALID_ARG
    assert binding.lib.tg_static_scratch_needed(None, 1) == -1
    assert binding.lib.tg_plan_set_update_kernel(None, 0) == binding.TG_ERR_INVALID_ARG
    assert binding.lib.tg_plan_set_layer_modes(None, None) == binding.TG_ERR_INVALID_ARG
    assert binding.lib.tg_unpack_average_mixed(None, 1, None, None, None, None, None) == binding.TG_ERR_INVALID_ARG
    assert binding.lib.tg_share_scalers(None, 1, None, None, None) == binding.TG_ERR_INVALID_ARG
    assert binding.lib.tg_ternarize_pack(None, 1, 0, None, None, None, 0, 0, None, None) == binding.TG_ERR_INVALID_ARG
    assert binding.lib.tg_unpack_average(None, 1, None, None, None, None) == binding.TG_ERR_INVALID_ARG
    assert binding.lib.tg_unpack_update(None, 1, None, None, 0.1, None, None) == binding.TG_ERR_INVALID_ARG
    assert binding.lib.tg_unpack_update_momentum(None, 1, None, None, 0.1, 0.9, None, None, None) == binding.TG_ERR_INVALID_ARG
    assert binding.lib.tg_ternarize_pack_devstep(None, 1, 0, None, None, None, 0, None, None, None) == binding.TG_ERR_INVALID_ARG
    assert binding.lib.tg_step_advance(None, 1, None) == binding.TG_ERR_INVALID_ARG
    assert binding.lib.tg_packed_bytes_base3(None) == -1
    assert binding.lib.tg_ternarize_pack_base3(None, 1, 0, None, None, None, 0, 0, None, None) == binding.TG_ERR_INVALID_ARG
    assert binding.lib.tg_unpack_average_base3(None, 1, None, None, None, None) == binding.TG_ERR_INVALID_ARG
    assert binding.lib.tg_sum_bytes(None, 4) == -1
    assert [binding.lib.tg_sum_bits(N) for N in (0, 1, 2, 4, 8, 64, 65)] == [-1, 2, 3, 4, 5, 8, -1]
    assert binding.lib.tg_unpack_sum_pack(None, 1, None, 4, None, None) == binding.TG_ERR_INVALID_ARG
    assert binding.lib.tg_decode_sum(None, 1, None, 4, None, None, None) == binding.TG_ERR_INVALID_ARG
    assert binding.lib.tg_average_float(1, 16, None, None, None) == binding.TG_ERR_INVALID_ARG
    assert binding.lib.tg_average_float(65, 16, None, None, None) == binding.TG_ERR_INVALID_ARG


def _brute_tables(off, tile, chunk):
    off = np.asarray(off, np.int64)
    n = int(off[-1])
    lay = np.repeat(np.arange(off.size - 1), np.diff(off))
    tile_layer = lay[np.arange(0, n, tile)]
    tile_whole = np.array([len(set(lay[e:e + tile])) == 1 for e in range(0, n, tile)], np.uint8)
    segs = []
    for cb in range(0, n, chunk):
        ce = min(n, cb + chunk)
        e = cb
        while e < ce:
            l = lay[e]
            end = min(int(off[l + 1]), ce)
            segs.append((l, e, end))
            e = end
    return tile_layer, tile_whole, np.array(segs, np.int64).reshape(-1, 3)


@pytest.mark.parametrize("sizes", [[1], [4096], [4097], [16384, 16384], [5, 0, 0, 20000, 1, 40000, 3],
                                   [500, 20, 25000, 50, 400000, 500, 5000, 10], [0, 0, 7], [100000]])
def test_tables_match_brute_force(binding, sizes):
    off = np.concatenate([[0], np.cumsum(sizes)])
    d = binding.tg_describe_tables(off, 3)
    tl, tw, segs = _brute_tables(off, d["tile_elems"], d["chunk_elems"])
    assert np.array_equal(d["tile_layer"], tl)
    assert np.array_equal(d["tile_whole"], tw)
    assert np.array_equal(d["segments"], segs)
    # segments tile [0, n) exactly, in order, each inside one layer and one chunk
    s = d["segments"]
    assert s[0, 1] == 0 and s[-1, 2] == off[-1] and np.all(s[1:, 1] == s[:-1, 2]) and np.all(s[:, 2] > s[:, 1])


def test_statistics_chunk_follows_the_size_of_the_job(binding):
    # looping shape: chunk = 8192 / 16384 elements for n * max_workers below 2^26 / 2^28; from 2^28 on the one-shot
    # shape with chunks of 16384, unless layers begin in too many chunks (then 32768 below 2^29, 65536 beyond)
    for n, W, chunk in ((1000, 1, 8192), (2 ** 26 - 1, 1, 8192), (2 ** 26, 1, 16384), (2 ** 24, 4, 16384),
                        (2 ** 24, 16, 16384), (60_965_224, 4, 16384), (2 ** 29 - 1, 1, 16384), (2 ** 29, 1, 16384),
                        (132_863_336, 8, 16384), (6_296_176, 4, 8192)):
        d = binding.tg_describe_tables(np.array([0, n]), W)
        assert d["chunk_elems"] == chunk, (n, W, d["chunk_elems"])
        s = d["segments"]
        assert s.shape[0] == -(-n // chunk) and s[0, 1] == 0 and s[-1, 2] == n and np.all(s[:, 2] - s[:, 1] <= chunk)
    # 2^23 elements in layers of 4096, four segments in every chunk of 16384 -> the looping shape: 32 workers
    # (2^28 elements per call) chunks of 32768, 64 workers 65536
    assert binding.tg_describe_tables(np.arange(0, 2 ** 23 + 1, 4096, dtype=np.int64), 32)["chunk_elems"] == 32768
    # 2^23 elements x 64 workers in layers of 4096: four segments in every chunk of 16384 -> the looping shape
    off = np.arange(0, 2 ** 23 + 1, 4096, dtype=np.int64)
    assert binding.tg_describe_tables(off, 64)["chunk_elems"] == 65536
    # the same size with a layer boundary in one chunk out of 64 (and a ragged last chunk): still one-shot ...
    off = np.concatenate([np.arange(0, 2 ** 23, 64 * 16384, dtype=np.int64) + 5, [2 ** 23 + 100]])
    off[0] = 0
    d = binding.tg_describe_tables(off, 64)
    assert d["chunk_elems"] == 16384 and d["segments"].shape[0] == 2 ** 23 // 16384 + 1 + 7
    # ... and with twice as many boundaries not
    off = np.concatenate([np.arange(0, 2 ** 23, 32 * 16384, dtype=np.int64) + 5, [2 ** 23 + 100]])
    off[0] = 0
    assert binding.tg_describe_tables(off, 64)["chunk_elems"] == 65536
    with pytest.raises(binding.TgError):
        binding.tg_describe_tables(np.array([0, 10]), 0)
    with pytest.raises(binding.TgError):
        binding.tg_describe_tables(np.array([0, 10]), 65)


def test_tables_at_the_layer_limit(binding):
    # TG_MAX_LAYERS one-element layers: every layer its own segment, every tile full of boundaries
    L = 1 << 22
    off = np.arange(L + 1, dtype=np.int64)
    d = binding.tg_describe_tables(off)
    assert d["tile_elems"] == 1024 and d["tile_layer"].size == L // 1024
    assert np.array_equal(d["tile_layer"], np.arange(0, L, 1024)) and not d["tile_whole"].any()
    s = d["segments"]
    assert s.shape == (L, 3) and np.array_equal(s[:, 0], off[:-1]) and np.array_equal(s[:, 1], off[:-1])
    assert np.array_equal(s[:, 2], off[1:])
    with pytest.raises(binding.TgError):
        binding.tg_describe_tables(np.arange(L + 2, dtype=np.int64))        # one layer too many


def test_binding_refuses_to_import_without_the_library(tmp_path):
    import subprocess
    import sys
    code = ("import importlib.util, sys\n"
            "spec = importlib.util.spec_from_file_location('b', sys.argv[1])\n"
            "m = importlib.util.module_from_spec(spec)\n"
            "try:\n    spec.loader.exec_module(m)\nexcept ImportError as e:\n    print('IMPORTERROR', e)\n")
    src = open(os.path.join(ROOT, "paper_1705_07878_amd", "binding.py")).read()
    p = tmp_path / "binding.py"
    p.write_text(src)
    out = subprocess.run([sys.executable, "-c", code, str(p)], capture_output=True, text=True).stdout
    assert "IMPORTERROR" in out and "not built" in out
