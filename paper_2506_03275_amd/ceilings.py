"""ctypes binding of the device-ceiling probes (probe/ceilings.h): argument marshalling only."""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


def load():
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "libchipmunk_ceilings.so")
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: run `python paper_2506_03275_amd/build.py`")
        lib = ctypes.CDLL(path)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        lib.chipmunk_probe_mfma_flops.argtypes, lib.chipmunk_probe_mfma_flops.restype = [i32, i32], ctypes.c_double
        lib.chipmunk_probe_mfma_bf16.argtypes, lib.chipmunk_probe_mfma_bf16.restype = [i32] * 3 + [vp, vp], ctypes.c_int32
        lib.chipmunk_probe_read.argtypes, lib.chipmunk_probe_read.restype = [vp, sz, vp, vp], ctypes.c_int32
        lib.chipmunk_probe_copy.argtypes, lib.chipmunk_probe_copy.restype = [vp, vp, sz, vp], ctypes.c_int32
        _LIB = lib
    return _LIB


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(code, what):
    if code != 0:
        raise RuntimeError(f"{what} failed with status {code}")


def mfma_flops(blocks_per_cu, iters):
    return float(load().chipmunk_probe_mfma_flops(blocks_per_cu, iters))


def mfma_bf16(shape, blocks_per_cu, iters, sink):
    _check(load().chipmunk_probe_mfma_bf16(shape, blocks_per_cu, iters, sink.data_ptr(), _stream()),
           "chipmunk_probe_mfma_bf16")


def read(src, sink):
    _check(load().chipmunk_probe_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(), _stream()),
           "chipmunk_probe_read")


def copy(src, dst):
    _check(load().chipmunk_probe_copy(src.data_ptr(), dst.data_ptr(), src.numel() * src.element_size(), _stream()),
           "chipmunk_probe_copy")
