"""ctypes binding of libhero_probe.so (include/hero_probe.h): the measuring instruments bench.py uses to
establish what the machine sustains.  Not part of the product: nothing else imports this."""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(os.path.dirname(_HERE), "libhero_probe.so")

vp, i64, i32 = C.c_void_p, C.c_int64, C.c_int
SYMBOLS = {
    "hero_probe_mfma_i8": (i32, [i32, i64, vp, C.POINTER(C.c_double), vp]),
    "hero_probe_coissue": (i32, [i32, i32, i64, vp, C.POINTER(C.c_double), C.POINTER(C.c_double), vp]),
    "hero_probe_copy": (i32, [vp, vp, i64, i32, vp]),
    "hero_probe_read": (i32, [vp, i64, vp, vp]),
    "hero_probe_write": (i32, [vp, i64, vp]),
    "hero_probe_memcpy": (i32, [vp, vp, i64, vp]),
}


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Probe:
    def __init__(self, path: str = LIB_PATH):
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it with `python -m paper_2310_17723_amd.build`")
        self.lib = C.CDLL(path)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(self.lib, name)
            fn.restype, fn.argtypes = res, args

    @staticmethod
    def _check(rc):
        if rc != 0:
            raise RuntimeError(f"libhero_probe: status {rc}")

    def mfma_i8(self, random_bytes, iters, sink) -> float:
        ops = C.c_double(0.0)
        self._check(self.lib.hero_probe_mfma_i8(int(bool(random_bytes)), int(iters), sink.data_ptr(), C.byref(ops), _stream()))
        return ops.value

    def coissue(self, mode, valu_per_mfma, iters, sink):
        mo, vi = C.c_double(0.0), C.c_double(0.0)
        self._check(self.lib.hero_probe_coissue(int(mode), int(valu_per_mfma), int(iters), sink.data_ptr(), C.byref(mo), C.byref(vi), _stream()))
        return mo.value, vi.value

    def copy(self, src, dst, loads_in_flight=1):
        n = src.numel() * src.element_size()
        assert dst.numel() * dst.element_size() == n
        self._check(self.lib.hero_probe_copy(src.data_ptr(), dst.data_ptr(), n, int(loads_in_flight), _stream()))

    def read(self, src, sink):
        self._check(self.lib.hero_probe_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(), _stream()))

    def write(self, dst):
        self._check(self.lib.hero_probe_write(dst.data_ptr(), dst.numel() * dst.element_size(), _stream()))

    def memcpy(self, src, dst):
        n = src.numel() * src.element_size()
        self._check(self.lib.hero_probe_memcpy(src.data_ptr(), dst.data_ptr(), n, _stream()))
