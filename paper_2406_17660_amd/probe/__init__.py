"""Binding of probe/libgrass_probe.so (mfma_rate_probe.h): a measurement aid that bench.py
uses to state what the matrix cores of the machine at hand sustain.  Not part of the GRASS
library: nothing of the method's path imports this module."""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgrass_probe.so")
CONSTANTS, REGISTERS, LDS = 0, 1, 2
OK, ERR_NULL, ERR_SIZE, ERR_SOURCE, ERR_DEVICE = range(5)
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2406_17660_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.mfma_rate_probe.argtypes = [C.c_int, C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t,
                                      C.c_int, C.POINTER(C.c_double), C.c_void_p]
        L.mfma_rate_probe.restype = C.c_int
        _lib = L
    return _lib


def mfma_rate(iters=10000, source=CONSTANTS, operands=None):
    """TFLOP/s of a kernel that only issues the GEMM's bf16 matrix instruction on every compute
    unit.  `operands`: at least 32768 bf16 values on the device for the sources that take the
    caller's values (held in registers, or read from LDS like the GEMM's operand fragments)."""
    out = torch.empty(256 * 256, dtype=torch.float32, device="cuda")
    flops = C.c_double(0.0)
    ptr, nbytes = (None, 0) if operands is None else (C.c_void_p(operands.data_ptr()),
                                                      operands.numel() * operands.element_size())
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)

    def launch():
        code = lib().mfma_rate_probe(source, ptr, nbytes, C.c_void_p(out.data_ptr()), out.numel(),
                                     iters, C.byref(flops), stream)
        if code != OK:
            raise RuntimeError(f"mfma_rate_probe: error {code}")
    for _ in range(3):  # the clock settles over the first launches
        launch()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    launch()
    b.record()
    torch.cuda.synchronize()
    return flops.value / (a.elapsed_time(b) * 1e-3) / 1e12
