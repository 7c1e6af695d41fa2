"""ctypes binding of libpc_probe.so (include/pc_probe.h): the benchmark's achievable-peak probes.
Not part of the attention library; nothing in binding.py or libpc.so depends on it."""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpc_probe.so")

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2512_23049_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.pc_probe_mfma_bf16.restype = i32
        L.pc_probe_mfma_bf16.argtypes = [vp, i64, i32, i32, i32, vp, C.POINTER(C.c_double), vp]
        L.pc_probe_hbm_read.restype = i32
        L.pc_probe_hbm_read.argtypes = [vp, i64, i32, vp, C.POINTER(C.c_double), vp]
        _lib = L
    return _lib


class ProbeError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what} failed with code {code}")
        self.code = code


def probe_mfma_bf16(operands_ptr: int, operand_bytes: int, sink_ptr: int, iters: int = 4096, waves_per_simd: int = 2,
                    reps: int = 3, stream: int = 0) -> float:
    """Sustained TFLOP/s of bare 32x32x16 bf16 matrix instructions on the operands given (device)."""
    out = C.c_double(0.0)
    rc = lib().pc_probe_mfma_bf16(operands_ptr or None, operand_bytes, iters, waves_per_simd, reps, sink_ptr or None,
                                  C.byref(out), stream or None)
    if rc != 0:
        raise ProbeError(rc, "pc_probe_mfma_bf16")
    return out.value


def probe_hbm_read(src_ptr: int, nbytes: int, sink_ptr: int, reps: int = 5, stream: int = 0) -> float:
    """Sustained GB/s of a streaming read of the device buffer given."""
    out = C.c_double(0.0)
    rc = lib().pc_probe_hbm_read(src_ptr or None, nbytes, reps, sink_ptr or None, C.byref(out), stream or None)
    if rc != 0:
        raise ProbeError(rc, "pc_probe_hbm_read")
    return out.value
