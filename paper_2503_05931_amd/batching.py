"""ctypes binding of the host-side 2D bucketing batch former (include/aed_batching.h).
Argument marshalling only."""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import binding as _b

STRICT, FLEXIBLE = 0, 1
EXPORTS = ("aed_bucketing_estimate", "aed_bucketing_free", "aed_bucketing_bounds", "aed_bucketing_allocate",
           "aed_tps_keep", "aed_bucketing_batch_sizes", "aed_bucketing_form_batches", "aed_bucket_select")
_i32p = C.POINTER(C.c_int32)
_configured = False


def _lib():
    global _configured
    lib = _b.load()
    if not _configured:
        lib.aed_bucketing_estimate.argtypes = [_i32p, _i32p, C.c_int64, C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]
        lib.aed_bucketing_free.argtypes = [C.c_void_p]
        lib.aed_bucketing_free.restype = None
        lib.aed_bucketing_bounds.argtypes = [C.c_void_p, _i32p, _i32p]
        lib.aed_bucketing_allocate.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32]
        lib.aed_bucketing_allocate.restype = C.c_int32
        lib.aed_tps_keep.argtypes = [C.c_int32, C.c_int32, C.c_double, C.c_double]
        lib.aed_tps_keep.restype = C.c_int32
        lib.aed_bucketing_batch_sizes.argtypes = [C.c_void_p, C.c_int64, C.c_int32, _i32p]
        lib.aed_bucketing_form_batches.argtypes = [C.c_void_p, _i32p, _i32p, C.c_int64, C.c_int32, _i32p, _i32p, _i32p,
                                                   _i32p]
        lib.aed_bucket_select.argtypes = [C.c_uint64, C.c_uint64, _i32p, C.c_int32]
        lib.aed_bucket_select.restype = C.c_int32
        _configured = True
    return lib


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(_i32p)


class Bucketing:
    def __init__(self, in_len, out_len, n_in_bins: int, n_out_bins: int):
        self.lib = _lib()
        a, pa = _i32(in_len)
        b, pb = _i32(out_len)
        self.handle = C.c_void_p(None)
        st = self.lib.aed_bucketing_estimate(pa, pb, len(a), n_in_bins, n_out_bins, C.byref(self.handle))
        if st != 0:
            raise ValueError("aed_bucketing_estimate: bad argument")
        self.n_in, self.n_out = n_in_bins, n_out_bins

    def __del__(self):
        if getattr(self, "handle", None):
            self.lib.aed_bucketing_free(self.handle)
            self.handle = None

    def aed_bucketing_bounds(self):
        iu = np.zeros(self.n_in, np.int32)
        ou = np.zeros(self.n_in * self.n_out, np.int32)
        self.lib.aed_bucketing_bounds(self.handle, iu.ctypes.data_as(_i32p), ou.ctypes.data_as(_i32p))
        return iu, ou.reshape(self.n_in, self.n_out)

    def aed_bucketing_allocate(self, in_len: int, out_len: int, mode: int) -> int:
        return int(self.lib.aed_bucketing_allocate(self.handle, int(in_len), int(out_len), int(mode)))

    def aed_bucketing_batch_sizes(self, budget_frames: int, max_batch: int):
        out = np.zeros(self.n_in * self.n_out, np.int32)
        if self.lib.aed_bucketing_batch_sizes(self.handle, int(budget_frames), int(max_batch),
                                              out.ctypes.data_as(_i32p)) != 0:
            raise ValueError("aed_bucketing_batch_sizes: bad argument")
        return out

    def aed_bucketing_form_batches(self, in_len, out_len, mode: int, batch_sizes):
        a, pa = _i32(in_len)
        b, pb = _i32(out_len)
        s, ps = _i32(batch_sizes)
        batch_of = np.zeros(len(a), np.int32)
        bucket_of_batch = np.zeros(len(a), np.int32)
        nb = C.c_int32(0)
        if self.lib.aed_bucketing_form_batches(self.handle, pa, pb, len(a), int(mode), ps, batch_of.ctypes.data_as(_i32p),
                                               bucket_of_batch.ctypes.data_as(_i32p), C.byref(nb)) != 0:
            raise ValueError("aed_bucketing_form_batches: bad argument")
        return batch_of, bucket_of_batch[:nb.value].copy()


def aed_tps_keep(in_len: int, out_len: int, frames_per_second: float, max_tps: float) -> bool:
    return bool(_lib().aed_tps_keep(int(in_len), int(out_len), float(frames_per_second), float(max_tps)))


def aed_bucket_select(seed: int, step: int, available) -> int:
    a, pa = _i32(available)
    return int(_lib().aed_bucket_select(C.c_uint64(seed), C.c_uint64(step), pa, len(a)))
