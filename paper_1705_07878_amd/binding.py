"""ctypes binding of libterngrad.so: same names as the C ABI (include/terngrad.h).

Argument marshalling only.  Device buffers are torch tensors (or raw integer
device addresses); torch is used for memory and streams, every step of the path
runs in the library's HIP kernels.  There is no fallback: if the library has not
been built, importing fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes
import os
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libterngrad.so")

TG_OK = 0
TG_ERR_INVALID_ARG = -1
TG_ERR_ALIGNMENT = -2
TG_ERR_TOO_MANY_WORKERS = -3
TG_ERR_HIP = -4
TG_ERR_ALLOC = -5
TG_ERR_TOO_LARGE = -6
TG_STATIC_SCRATCH_BYTES = 16 * 1024 * 1024
TG_MAX_WORKERS = 64

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libterngrad.so is not built (expected %s): run `python -m paper_1705_07878_amd.build` "
        "or `python -c 'import __graft_entry__ as g; g.build()'`" % LIB_PATH)

lib = ctypes.CDLL(LIB_PATH)

_vp = ctypes.c_void_p
_i64 = ctypes.c_int64
_pp = ctypes.POINTER(ctypes.c_void_p)

lib.tg_plan_create.argtypes = [_i64, ctypes.POINTER(_i64), ctypes.c_int, ctypes.POINTER(_vp)]
lib.tg_plan_create.restype = ctypes.c_int
lib.tg_plan_destroy.argtypes = [_vp]
lib.tg_plan_destroy.restype = ctypes.c_int
for _f in (lib.tg_num_elements, lib.tg_num_layers, lib.tg_packed_bytes):
    _f.argtypes = [_vp]
    _f.restype = _i64
lib.tg_strerror.argtypes = [ctypes.c_int]
lib.tg_strerror.restype = ctypes.c_char_p
lib.tg_last_hip_error.argtypes = []
lib.tg_last_hip_error.restype = ctypes.c_int
lib.tg_describe_tables.argtypes = [_i64, ctypes.POINTER(_i64), ctypes.c_int,
                                   ctypes.POINTER(_i64), ctypes.POINTER(_i64), ctypes.POINTER(ctypes.c_int32),
                                   ctypes.POINTER(ctypes.c_uint8), _i64,
                                   ctypes.POINTER(_i64), ctypes.POINTER(_i64), ctypes.POINTER(_i64), _i64]
lib.tg_describe_tables.restype = ctypes.c_int
lib.tg_clip_stats.argtypes = [_vp, ctypes.c_int, _pp, ctypes.c_float, _vp, _vp, _vp]
lib.tg_clip_stats.restype = ctypes.c_int
lib.tg_plan_set_update_kernel.argtypes = [_vp, ctypes.c_int]
lib.tg_plan_set_update_kernel.restype = ctypes.c_int
lib.tg_clip_stats_static.argtypes = [_vp, ctypes.c_int, _pp, ctypes.c_float, _vp, _vp, _vp]
lib.tg_clip_stats_static.restype = ctypes.c_int
lib.tg_static_scratch_needed.argtypes = [_vp, ctypes.c_int]
lib.tg_static_scratch_needed.restype = _i64
lib.tg_share_scalers.argtypes = [_vp, ctypes.c_int, _vp, _vp, _vp]
lib.tg_share_scalers.restype = ctypes.c_int
lib.tg_ternarize_pack.argtypes = [_vp, ctypes.c_int, ctypes.c_uint32, _pp, _vp, _vp,
                                  ctypes.c_uint64, ctypes.c_uint32, _pp, _vp]
lib.tg_ternarize_pack.restype = ctypes.c_int
lib.tg_ternarize_pack_devstep.argtypes = [_vp, ctypes.c_int, ctypes.c_uint32, _pp, _vp, _vp,
                                          ctypes.c_uint64, _vp, _pp, _vp]
lib.tg_ternarize_pack_devstep.restype = ctypes.c_int
lib.tg_step_advance.argtypes = [_vp, ctypes.c_uint32, _vp]
lib.tg_step_advance.restype = ctypes.c_int
lib.tg_unpack_average.argtypes = [_vp, ctypes.c_int, _pp, _vp, _vp, _vp]
lib.tg_unpack_average.restype = ctypes.c_int
lib.tg_unpack_average_scalers.argtypes = [_vp, ctypes.c_int, _pp, _vp, _vp, _vp]
lib.tg_unpack_average_scalers.restype = ctypes.c_int
lib.tg_plan_set_layer_modes.argtypes = [_vp, _vp]
lib.tg_plan_set_layer_modes.restype = ctypes.c_int
lib.tg_unpack_average_mixed.argtypes = [_vp, ctypes.c_int, _pp, _pp, _vp, _vp, _vp]
lib.tg_unpack_average_mixed.restype = ctypes.c_int
lib.tg_unpack_update.argtypes = [_vp, ctypes.c_int, _pp, _vp, ctypes.c_float, _vp, _vp]
lib.tg_unpack_update.restype = ctypes.c_int
lib.tg_unpack_update_momentum.argtypes = [_vp, ctypes.c_int, _pp, _vp, ctypes.c_float, ctypes.c_float, _vp, _vp, _vp]
lib.tg_unpack_update_momentum.restype = ctypes.c_int
lib.tg_sum_bits.argtypes = [ctypes.c_int]
lib.tg_sum_bits.restype = ctypes.c_int
lib.tg_sum_bytes.argtypes = [_vp, ctypes.c_int]
lib.tg_sum_bytes.restype = _i64
lib.tg_unpack_sum_pack.argtypes = [_vp, ctypes.c_int, _pp, ctypes.c_int, _vp, _vp]
lib.tg_unpack_sum_pack.restype = ctypes.c_int
lib.tg_decode_sum.argtypes = [_vp, ctypes.c_int, _vp, ctypes.c_int, _vp, _vp, _vp]
lib.tg_decode_sum.restype = ctypes.c_int
lib.tg_packed_bytes_base3.argtypes = [_vp]
lib.tg_packed_bytes_base3.restype = _i64
lib.tg_ternarize_pack_base3.argtypes = lib.tg_ternarize_pack.argtypes
lib.tg_ternarize_pack_base3.restype = ctypes.c_int
lib.tg_unpack_average_base3.argtypes = lib.tg_unpack_average.argtypes
lib.tg_unpack_average_base3.restype = ctypes.c_int
lib.tg_average_float.argtypes = [ctypes.c_int, _i64, _pp, _vp, _vp]
lib.tg_average_float.restype = ctypes.c_int


class TgError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        msg = lib.tg_strerror(int(status)).decode()
        if status == TG_ERR_HIP:
            msg += " [hipError_t %d]" % lib.tg_last_hip_error()
        super().__init__("%s: %s (%d)" % (where, msg, status))


def _check(status: int, where: str):
    if status != TG_OK:
        raise TgError(status, where)


def _ptr(x) -> int:
    """device address of a torch tensor, or an int passed through"""
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _ptr_array(xs: Sequence):
    arr = (ctypes.c_void_p * len(xs))(*[_ptr(x) for x in xs])
    return ctypes.cast(arr, _pp), arr


def _stream(stream) -> int:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)


def tg_sum_bits(n_workers: int) -> int:
    return int(lib.tg_sum_bits(int(n_workers)))


def tg_strerror(status: int) -> str:
    return lib.tg_strerror(int(status)).decode()


def tg_last_hip_error() -> int:
    return int(lib.tg_last_hip_error())


def tg_describe_tables(offsets, max_workers: int = 1):
    """-> dict(tile_elems, tile_layer[n_tiles], tile_whole[n_tiles], chunk_elems, segments[n_segs, 3])  (host only)"""
    off = np.ascontiguousarray(offsets, dtype=np.int64)
    L = off.size - 1
    offp = off.ctypes.data_as(ctypes.POINTER(_i64))
    te, nt, ce, ns = _i64(), _i64(), _i64(), _i64()
    _check(lib.tg_describe_tables(L, offp, int(max_workers), ctypes.byref(te), ctypes.byref(nt), None, None, 0,
                                  ctypes.byref(ce), ctypes.byref(ns), None, 0), "tg_describe_tables")
    tl = np.empty(nt.value, np.int32)
    tw = np.empty(nt.value, np.uint8)
    seg = np.empty((ns.value, 3), np.int64)
    _check(lib.tg_describe_tables(L, offp, int(max_workers), ctypes.byref(te), ctypes.byref(nt),
                                  tl.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                  tw.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), tl.size,
                                  ctypes.byref(ce), ctypes.byref(ns),
                                  seg.ctypes.data_as(ctypes.POINTER(_i64)), seg.shape[0]), "tg_describe_tables")
    return {"tile_elems": te.value, "tile_layer": tl, "tile_whole": tw, "chunk_elems": ce.value, "segments": seg}


def tg_average_float(grads: Sequence, n: int, avg, stream=None):
    gp, _keep = _ptr_array(grads)
    _check(lib.tg_average_float(len(grads), int(n), gp, _ptr(avg), _stream(stream)), "tg_average_float")


def tg_step_advance(step_dev, by: int = 1, stream=None):
    _check(lib.tg_step_advance(_ptr(step_dev), int(by), _stream(stream)), "tg_step_advance")


class Plan:
    """Owns a tg_plan*.  Methods carry the names of the C calls."""

    def __init__(self, offsets, max_workers: int):
        off = np.ascontiguousarray(offsets, dtype=np.int64)
        if off.ndim != 1 or off.size < 2:
            raise TgError(TG_ERR_INVALID_ARG, "tg_plan_create")
        h = _vp()
        _check(lib.tg_plan_create(off.size - 1, off.ctypes.data_as(ctypes.POINTER(_i64)),
                                  int(max_workers), ctypes.byref(h)), "tg_plan_create")
        self._h = h
        self.offsets = off
        self.max_workers = int(max_workers)

    def close(self):
        if getattr(self, "_h", None):
            lib.tg_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def n(self) -> int:
        return int(lib.tg_num_elements(self._h))

    @property
    def n_layers(self) -> int:
        return int(lib.tg_num_layers(self._h))

    @property
    def packed_bytes(self) -> int:
        return int(lib.tg_packed_bytes(self._h))

    def tg_clip_stats(self, grads: Sequence, c: float, tau, s_local, stream=None):
        gp, _keep = _ptr_array(grads)
        _check(lib.tg_clip_stats(self._h, len(grads), gp, float(c), _ptr(tau), _ptr(s_local),
                                 _stream(stream)), "tg_clip_stats")

    def tg_plan_set_update_kernel(self, mode: int):
        _check(lib.tg_plan_set_update_kernel(self._h, int(mode)), "tg_plan_set_update_kernel")

    def tg_clip_stats_static(self, grads: Sequence, c: float, tau, s_local, stream=None):
        gp, _keep = _ptr_array(grads)
        _check(lib.tg_clip_stats_static(self._h, len(grads), gp, float(c), _ptr(tau), _ptr(s_local),
                                        _stream(stream)), "tg_clip_stats_static")

    def tg_static_scratch_needed(self, n_workers: int) -> int:
        return int(lib.tg_static_scratch_needed(self._h, int(n_workers)))

    def tg_share_scalers(self, n_workers: int, s_local, s_shared, stream=None):
        _check(lib.tg_share_scalers(self._h, int(n_workers), _ptr(s_local), _ptr(s_shared),
                                    _stream(stream)), "tg_share_scalers")

    def tg_ternarize_pack(self, grads: Sequence, tau, s_shared, seed: int, step: int, codes: Sequence,
                          worker_base: int = 0, stream=None):
        gp, _k1 = _ptr_array(grads)
        cp, _k2 = _ptr_array(codes)
        if len(grads) != len(codes):
            raise TgError(TG_ERR_INVALID_ARG, "tg_ternarize_pack")
        _check(lib.tg_ternarize_pack(self._h, len(grads), int(worker_base), gp, _ptr(tau), _ptr(s_shared),
                                     int(seed) & 0xFFFFFFFFFFFFFFFF, int(step) & 0xFFFFFFFF, cp,
                                     _stream(stream)), "tg_ternarize_pack")

    def tg_unpack_average(self, codes: Sequence, s_shared, avg, stream=None):
        cp, _k = _ptr_array(codes)
        _check(lib.tg_unpack_average(self._h, len(codes), cp, _ptr(s_shared), _ptr(avg),
                                     _stream(stream)), "tg_unpack_average")

    def tg_plan_set_layer_modes(self, layer_float):
        """layer_float: L flags (1 = layer kept in floating point), or None for all ternarized"""
        if layer_float is None:
            _check(lib.tg_plan_set_layer_modes(self._h, None), "tg_plan_set_layer_modes")
            return
        flags = np.ascontiguousarray(layer_float, dtype=np.uint8)
        if flags.shape != (self.n_layers,):
            raise ValueError("layer_float must hold one flag per layer")
        _check(lib.tg_plan_set_layer_modes(self._h, flags.ctypes.data_as(ctypes.c_void_p)),
               "tg_plan_set_layer_modes")

    def tg_unpack_average_mixed(self, codes: Sequence, grads, s_shared, avg, stream=None):
        cp, _k = _ptr_array(codes)
        gp, _k2 = _ptr_array(grads) if grads is not None else (None, None)
        _check(lib.tg_unpack_average_mixed(self._h, len(codes), cp, gp, _ptr(s_shared), _ptr(avg),
                                           _stream(stream)), "tg_unpack_average_mixed")

    def tg_unpack_average_scalers(self, codes: Sequence, s_workers, avg, stream=None):
        cp, _k = _ptr_array(codes)
        _check(lib.tg_unpack_average_scalers(self._h, len(codes), cp, _ptr(s_workers), _ptr(avg),
                                             _stream(stream)), "tg_unpack_average_scalers")

    def tg_unpack_update(self, codes: Sequence, s_shared, eta: float, weights, stream=None):
        cp, _k = _ptr_array(codes)
        _check(lib.tg_unpack_update(self._h, len(codes), cp, _ptr(s_shared), float(eta), _ptr(weights),
                                    _stream(stream)), "tg_unpack_update")

    def tg_sum_bytes(self, bits: int) -> int:
        return int(lib.tg_sum_bytes(self._h, int(bits)))

    def tg_unpack_sum_pack(self, codes: Sequence, bits: int, ksum, stream=None):
        cp, _k = _ptr_array(codes)
        _check(lib.tg_unpack_sum_pack(self._h, len(codes), cp, int(bits), _ptr(ksum), _stream(stream)),
               "tg_unpack_sum_pack")

    def tg_decode_sum(self, n_workers: int, ksum, bits: int, s_shared, avg, stream=None):
        _check(lib.tg_decode_sum(self._h, int(n_workers), _ptr(ksum), int(bits), _ptr(s_shared), _ptr(avg),
                                 _stream(stream)), "tg_decode_sum")

    def tg_unpack_update_momentum(self, codes: Sequence, s_shared, eta: float, mu: float, velocity, weights,
                                  stream=None):
        cp, _k = _ptr_array(codes)
        _check(lib.tg_unpack_update_momentum(self._h, len(codes), cp, _ptr(s_shared), float(eta), float(mu),
                                             _ptr(velocity), _ptr(weights), _stream(stream)),
               "tg_unpack_update_momentum")

    def tg_ternarize_pack_devstep(self, grads: Sequence, tau, s_shared, seed: int, step_dev, codes: Sequence,
                                  worker_base: int = 0, stream=None):
        gp, _k1 = _ptr_array(grads)
        cp, _k2 = _ptr_array(codes)
        if len(grads) != len(codes):
            raise TgError(TG_ERR_INVALID_ARG, "tg_ternarize_pack_devstep")
        _check(lib.tg_ternarize_pack_devstep(self._h, len(grads), int(worker_base), gp, _ptr(tau), _ptr(s_shared),
                                             int(seed) & 0xFFFFFFFFFFFFFFFF, _ptr(step_dev), cp,
                                             _stream(stream)), "tg_ternarize_pack_devstep")

    @property
    def packed_bytes_base3(self) -> int:
        return int(lib.tg_packed_bytes_base3(self._h))

    def tg_ternarize_pack_base3(self, grads: Sequence, tau, s_shared, seed: int, step: int, codes3: Sequence,
                                worker_base: int = 0, stream=None):
        gp, _k1 = _ptr_array(grads)
        cp, _k2 = _ptr_array(codes3)
        if len(grads) != len(codes3):
            raise TgError(TG_ERR_INVALID_ARG, "tg_ternarize_pack_base3")
        _check(lib.tg_ternarize_pack_base3(self._h, len(grads), int(worker_base), gp, _ptr(tau), _ptr(s_shared),
                                           int(seed) & 0xFFFFFFFFFFFFFFFF, int(step) & 0xFFFFFFFF, cp,
                                           _stream(stream)), "tg_ternarize_pack_base3")

    def tg_unpack_average_base3(self, codes3: Sequence, s_shared, avg, stream=None):
        cp, _k = _ptr_array(codes3)
        _check(lib.tg_unpack_average_base3(self._h, len(codes3), cp, _ptr(s_shared), _ptr(avg),
                                           _stream(stream)), "tg_unpack_average_base3")
