"""ctypes binding of include/svdcache_probes.h: memory-system probes the benchmark times (no SVD-Cache arithmetic)."""
from __future__ import annotations

import ctypes as C
import os

import torch

PKG_DIR = os.path.dirname(os.path.abspath(__file__))

EXPORTS = {
    "svdc_probe_copy": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "svdc_probe_read": (C.c_int32, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]),
    "svdc_probe_tile_copy": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                         C.c_void_p]),
    "svdc_probe_burst_copy": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]),
}

_lib = None


def lib_path() -> str:
    return os.path.join(PKG_DIR, "libsvdcache_probes.so")


def load_library():
    global _lib
    if _lib is None:
        if not os.path.exists(lib_path()):
            raise RuntimeError(f"{lib_path()} is missing: build it with `python -m paper_2601_07396_amd.build`")
        lib = C.CDLL(lib_path())
        for name, (res, args) in EXPORTS.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _ok(rc, what):
    if rc != 0:
        raise RuntimeError(f"{what}: status {rc}")


def _bytes(t):
    return t.numel() * t.element_size()


def copy(dst, src):
    _ok(load_library().svdc_probe_copy(dst.data_ptr(), src.data_ptr(), _bytes(src), _stream()), "svdc_probe_copy")


def read(src, sink, nbytes=None):
    _ok(load_library().svdc_probe_read(src.data_ptr(), _bytes(src) if nbytes is None else nbytes, sink.data_ptr(),
                                       _stream()), "svdc_probe_read")


def tile_copy(dst, src, rows, tiles_per_group, interleave, groups_per_cu=0):
    assert _bytes(src) >= rows * 6144 and _bytes(dst) >= rows * 6144
    _ok(load_library().svdc_probe_tile_copy(dst.data_ptr(), src.data_ptr(), rows, tiles_per_group, int(interleave),
                                            int(groups_per_cu), _stream()), "svdc_probe_tile_copy")


def burst_copy(dst, src, rows, tile_rows):
    assert _bytes(src) >= rows * 6144 and _bytes(dst) >= rows * 6144
    _ok(load_library().svdc_probe_burst_copy(dst.data_ptr(), src.data_ptr(), rows, tile_rows, _stream()),
        "svdc_probe_burst_copy")
