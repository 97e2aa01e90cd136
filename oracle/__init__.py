"""CPU oracle for the TernGrad hot path -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

ctypes front end of ``tg_oracle.c`` (see ``tg_oracle.h`` for what each function
computes and which passage of the paper it follows).  Only ``tests/``, the
smoke check and the benchmark's ``cpu_baseline`` leg may import this package.
It imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libtg_oracle.so")
_SRC = os.path.join(_HERE, "tg_oracle.c")
_HDR = os.path.join(_HERE, "tg_oracle.h")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp32 operations rounded separately)."""
    stale = (not os.path.exists(_SO)
             or os.path.getmtime(_SO) < max(os.path.getmtime(_SRC), os.path.getmtime(_HDR)))
    if force or stale:
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-Wall", "-Wextra", "-shared", "-fPIC", _SRC, "-o", _SO, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_SO)
        c_f = ctypes.POINTER(ctypes.c_float)
        c_i64 = ctypes.POINTER(ctypes.c_int64)
        c_u8 = ctypes.POINTER(ctypes.c_uint8)
        c_u32 = ctypes.POINTER(ctypes.c_uint32)
        L.tgo_set_threads.argtypes = [ctypes.c_int]
        L.tgo_set_threads.restype = ctypes.c_int
        L.tgo_philox4x32_10.argtypes = [c_u32, c_u32, c_u32]
        L.tgo_philox4x32_10.restype = None
        L.tgo_random_field.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint64]
        L.tgo_random_field.restype = ctypes.c_uint32
        L.tgo_bernoulli.argtypes = [ctypes.c_uint32, ctypes.c_float, ctypes.c_float]
        L.tgo_bernoulli.restype = ctypes.c_int
        L.tgo_clip_stats.argtypes = [c_f, ctypes.c_int64, c_i64, ctypes.c_float, c_f, c_f]
        L.tgo_clip_stats.restype = None
        L.tgo_share_scalers.argtypes = [c_f, ctypes.c_int, ctypes.c_int64, c_f]
        L.tgo_share_scalers.restype = None
        L.tgo_ternarize_pack.argtypes = [c_f, ctypes.c_int64, c_i64, c_f, c_f, ctypes.c_uint64,
                                         ctypes.c_uint32, ctypes.c_uint32, c_u8]
        L.tgo_ternarize_pack.restype = None
        L.tgo_code_at.argtypes = [c_u8, ctypes.c_int64]
        L.tgo_code_at.restype = ctypes.c_int
        L.tgo_unpack_average.argtypes = [ctypes.POINTER(c_u8), ctypes.c_int, ctypes.c_int64, c_i64, c_f, c_f]
        L.tgo_unpack_average.restype = None
        L.tgo_unpack_update.argtypes = [ctypes.POINTER(c_u8), ctypes.c_int, ctypes.c_int64, c_i64, c_f,
                                        ctypes.c_float, c_f]
        L.tgo_unpack_update.restype = None
        L.tgo_average_float.argtypes = [ctypes.POINTER(c_f), ctypes.c_int, ctypes.c_int64, c_f]
        L.tgo_average_float.restype = None
        L.tgo_unpack_average_scalers.argtypes = [ctypes.POINTER(c_u8), ctypes.c_int, ctypes.c_int64, c_i64, c_f, c_f]
        L.tgo_unpack_average_scalers.restype = None
        L.tgo_sum_pack.argtypes = [ctypes.POINTER(c_u8), ctypes.c_int, ctypes.c_int64, ctypes.c_int, c_u8]
        L.tgo_sum_pack.restype = None
        L.tgo_sum_bits.argtypes = [ctypes.c_int]
        L.tgo_sum_bits.restype = ctypes.c_int
        L.tgo_decode_sum.argtypes = [c_u8, ctypes.c_int, ctypes.c_int, ctypes.c_int64, c_i64, c_f, c_f]
        L.tgo_decode_sum.restype = None
        L.tgo_unpack_update_momentum.argtypes = [ctypes.POINTER(c_u8), ctypes.c_int, ctypes.c_int64, c_i64, c_f,
                                                 ctypes.c_float, ctypes.c_float, c_f, c_f]
        L.tgo_unpack_update_momentum.restype = None
        L.tgo_ternarize_pack_base3.argtypes = L.tgo_ternarize_pack.argtypes
        L.tgo_ternarize_pack_base3.restype = None
        L.tgo_trit_at.argtypes = [c_u8, ctypes.c_int64]
        L.tgo_trit_at.restype = ctypes.c_int
        L.tgo_unpack_average_base3.argtypes = L.tgo_unpack_average.argtypes
        L.tgo_unpack_average_base3.restype = None
        _lib = L
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _i64(a):
    a = np.ascontiguousarray(a, dtype=np.int64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def _check_offsets(off, n=None):
    off = np.ascontiguousarray(off, dtype=np.int64)
    assert off.ndim == 1 and off.size >= 2 and off[0] == 0 and np.all(np.diff(off) >= 0)
    if n is not None:
        assert int(off[-1]) == int(n), (int(off[-1]), int(n))
    return off


def set_threads(n: int) -> int:
    return lib().tgo_set_threads(int(n))


def philox4x32_10(ctr, key):
    c = (ctypes.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    o = (ctypes.c_uint32 * 4)()
    lib().tgo_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def random_field(seed: int, step: int, worker: int, e: int) -> int:
    return int(lib().tgo_random_field(seed, step, worker, e))


def bernoulli(r: int, s: float, a: float) -> int:
    return int(lib().tgo_bernoulli(r, np.float32(s), np.float32(a)))


def clip_stats(g, off, c):
    """-> (tau[L], s_local[L]) for one worker's flat gradient g."""
    g, gp = _f32(g)
    off = _check_offsets(off, g.size)
    _, op = _i64(off)
    L = off.size - 1
    tau = np.empty(L, np.float32)
    s = np.empty(L, np.float32)
    lib().tgo_clip_stats(gp, L, op, np.float32(c), _f32(tau)[1], _f32(s)[1])
    return tau, s


def share_scalers(s_local):
    """s_local: [W, L] -> s_shared [L]."""
    s_local = np.ascontiguousarray(s_local, dtype=np.float32)
    W, L = s_local.shape
    out = np.empty(L, np.float32)
    lib().tgo_share_scalers(_f32(s_local)[1], W, L, _f32(out)[1])
    return out


def ternarize_pack(g, off, tau, s_shared, seed, step, worker):
    """-> uint8 codes [ceil(n/4)] for one worker."""
    g, gp = _f32(g)
    off = _check_offsets(off, g.size)
    _, op = _i64(off)
    L = off.size - 1
    tau, tp = _f32(tau)
    s_shared, sp = _f32(s_shared)
    assert tau.size == L and s_shared.size == L
    codes = np.zeros((g.size + 3) // 4, np.uint8)
    lib().tgo_ternarize_pack(gp, L, op, tp, sp, int(seed), int(step), int(worker),
                             codes.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)))
    return codes


def code_at(codes, e: int) -> int:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    return int(lib().tgo_code_at(codes.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), int(e)))


def unpack_average(codes_list, off, s_shared):
    """codes_list: W uint8 arrays [ceil(n/4)] -> float32 average [n]."""
    off = _check_offsets(off)
    _, op = _i64(off)
    L = off.size - 1
    n = int(off[-1])
    keep = [np.ascontiguousarray(c, dtype=np.uint8) for c in codes_list]
    for c in keep:
        assert c.size >= (n + 3) // 4
    W = len(keep)
    u8p = ctypes.POINTER(ctypes.c_uint8)
    arr = (u8p * W)(*[c.ctypes.data_as(u8p) for c in keep])
    s_shared, sp = _f32(s_shared)
    assert s_shared.size == L
    avg = np.empty(n, np.float32)
    lib().tgo_unpack_average(arr, W, L, op, sp, _f32(avg)[1])
    return avg


def unpack_average_scalers(codes_list, off, s_workers):
    """per-worker scalers s_workers [W][L] (no scaler sharing) -> float32 average [n]"""
    off = _check_offsets(off)
    _, op = _i64(off)
    L = off.size - 1
    n = int(off[-1])
    keep = [np.ascontiguousarray(c, dtype=np.uint8) for c in codes_list]
    for c in keep:
        assert c.size >= (n + 3) // 4
    W = len(keep)
    u8p = ctypes.POINTER(ctypes.c_uint8)
    arr = (u8p * W)(*[c.ctypes.data_as(u8p) for c in keep])
    s_workers, sp = _f32(s_workers)
    assert s_workers.shape == (W, L)
    avg = np.empty(n, np.float32)
    lib().tgo_unpack_average_scalers(arr, W, L, op, sp, _f32(avg)[1])
    return avg


def unpack_update(codes_list, off, s_shared, eta, weights):
    """-> new float32 weights [n] = w - eta * average of the decoded codes (input not modified)."""
    off = _check_offsets(off)
    _, op = _i64(off)
    L = off.size - 1
    n = int(off[-1])
    keep = [np.ascontiguousarray(c, dtype=np.uint8) for c in codes_list]
    for c in keep:
        assert c.size >= (n + 3) // 4
    W = len(keep)
    u8p = ctypes.POINTER(ctypes.c_uint8)
    arr = (u8p * W)(*[c.ctypes.data_as(u8p) for c in keep])
    s_shared, sp = _f32(s_shared)
    assert s_shared.size == L
    w = np.array(weights, dtype=np.float32, copy=True)
    assert w.size == n
    lib().tgo_unpack_update(arr, W, L, op, sp, np.float32(eta), _f32(w)[1])
    return w


def average_float(grads_list):
    """plain fp32 average of W float32 arrays [n] (layers that are not ternarized)"""
    keep = [np.ascontiguousarray(g, dtype=np.float32) for g in grads_list]
    n = keep[0].size
    assert all(g.size == n for g in keep)
    fp = ctypes.POINTER(ctypes.c_float)
    arr = (fp * len(keep))(*[g.ctypes.data_as(fp) for g in keep])
    avg = np.empty(n, np.float32)
    lib().tgo_average_float(arr, len(keep), n, _f32(avg)[1])
    return avg


def sum_bits(n_workers: int) -> int:
    """ceil(log2(2N+1)): the narrowest field that holds k in -N .. N"""
    return int(lib().tgo_sum_bits(int(n_workers)))


def sum_pack(codes_list, n: int, bits: int):
    """-> uint8 [ceil(n*bits/8)]: k = sum of the workers' ternary values in `bits`-wide fields"""
    assert 2 <= bits <= 8
    keep = [np.ascontiguousarray(c, dtype=np.uint8) for c in codes_list]
    for c in keep:
        assert c.size >= (n + 3) // 4
    u8p = ctypes.POINTER(ctypes.c_uint8)
    arr = (u8p * len(keep))(*[c.ctypes.data_as(u8p) for c in keep])
    out = np.zeros((n * bits + 7) // 8, np.uint8)
    lib().tgo_sum_pack(arr, len(keep), int(n), int(bits), out.ctypes.data_as(u8p))
    return out


def decode_sum(ksum, bits: int, n_workers: int, off, s_shared):
    off = _check_offsets(off)
    _, op = _i64(off)
    L = off.size - 1
    n = int(off[-1])
    ksum = np.ascontiguousarray(ksum, dtype=np.uint8)
    assert 2 <= bits <= 8 and ksum.size >= (n * bits + 7) // 8
    s_shared, sp = _f32(s_shared)
    avg = np.empty(n, np.float32)
    lib().tgo_decode_sum(ksum.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), int(bits), int(n_workers), L, op, sp,
                         _f32(avg)[1])
    return avg


def unpack_update_momentum(codes_list, off, s_shared, eta, mu, velocity, weights):
    """-> (new velocity, new weights): v = mu*v + avg ; w = w - eta*v  (inputs not modified)"""
    off = _check_offsets(off)
    _, op = _i64(off)
    L = off.size - 1
    n = int(off[-1])
    keep = [np.ascontiguousarray(c, dtype=np.uint8) for c in codes_list]
    for c in keep:
        assert c.size >= (n + 3) // 4
    u8p = ctypes.POINTER(ctypes.c_uint8)
    arr = (u8p * len(keep))(*[c.ctypes.data_as(u8p) for c in keep])
    s_shared, sp = _f32(s_shared)
    v = np.array(velocity, dtype=np.float32, copy=True)
    w = np.array(weights, dtype=np.float32, copy=True)
    assert v.size == n and w.size == n and s_shared.size == L
    lib().tgo_unpack_update_momentum(arr, len(keep), L, op, sp, np.float32(eta), np.float32(mu), _f32(v)[1], _f32(w)[1])
    return v, w


def ternarize_pack_base3(g, off, tau, s_shared, seed, step, worker):
    """-> uint8 [ceil(n/5)]: five ternary values per byte"""
    g, gp = _f32(g)
    off = _check_offsets(off, g.size)
    _, op = _i64(off)
    L = off.size - 1
    tau, tp = _f32(tau)
    s_shared, sp = _f32(s_shared)
    assert tau.size == L and s_shared.size == L
    codes = np.zeros((g.size + 4) // 5, np.uint8)
    lib().tgo_ternarize_pack_base3(gp, L, op, tp, sp, int(seed), int(step), int(worker),
                                   codes.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)))
    return codes


def trit_at(codes3, e: int) -> int:
    codes3 = np.ascontiguousarray(codes3, dtype=np.uint8)
    return int(lib().tgo_trit_at(codes3.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), int(e)))


def unpack_average_base3(codes_list, off, s_shared):
    off = _check_offsets(off)
    _, op = _i64(off)
    L = off.size - 1
    n = int(off[-1])
    keep = [np.ascontiguousarray(c, dtype=np.uint8) for c in codes_list]
    for c in keep:
        assert c.size >= (n + 4) // 5
    u8p = ctypes.POINTER(ctypes.c_uint8)
    arr = (u8p * len(keep))(*[c.ctypes.data_as(u8p) for c in keep])
    s_shared, sp = _f32(s_shared)
    avg = np.empty(n, np.float32)
    lib().tgo_unpack_average_base3(arr, len(keep), L, op, sp, _f32(avg)[1])
    return avg
