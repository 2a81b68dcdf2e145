"""ctypes binding of libabq_probe.so (include/abq_probe.h): the benchmark's measurement aids.  Not part of the
matmul path; nothing in the package's product code imports this module."""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libabq_probe.so")

_c = ctypes
_SIGNATURES = {
    "abq_probe_stream_read": (_c.c_int, [_c.c_void_p, _c.c_size_t, _c.c_void_p, _c.c_void_p]),
    "abq_probe_l2_read": (_c.c_int, [_c.c_void_p, _c.c_size_t, _c.c_int, _c.c_int, _c.c_void_p, _c.c_void_p]),
    "abq_probe_l2_read_bytes": (_c.c_double, [_c.c_size_t, _c.c_int, _c.c_int]),
    "abq_probe_mfma_i8": (_c.c_int, [_c.c_int, _c.c_int, _c.c_void_p, _c.c_void_p]),
    "abq_probe_mfma_i8_ops": (_c.c_double, [_c.c_int]),
    "abq_probe_mfma_f4": (_c.c_int, [_c.c_int, _c.c_int, _c.c_void_p, _c.c_void_p]),
    "abq_probe_mfma_f4_ops": (_c.c_double, [_c.c_int]),
}
_lib = None


def load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2408_08554_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _run(status, where):
    if status != 0:
        raise RuntimeError(f"{where}: status {status}")


def abq_probe_stream_read(buf, nbytes, sink):
    _run(load().abq_probe_stream_read(buf.data_ptr(), nbytes, sink.data_ptr(), torch.cuda.current_stream().cuda_stream),
         "abq_probe_stream_read")


def abq_probe_l2_read(buf, region_bytes, passes, wgs_per_cu, sink):
    _run(load().abq_probe_l2_read(buf.data_ptr(), region_bytes, passes, wgs_per_cu, sink.data_ptr(), torch.cuda.current_stream().cuda_stream),
         "abq_probe_l2_read")


def abq_probe_l2_read_bytes(region_bytes, passes, wgs_per_cu):
    return float(load().abq_probe_l2_read_bytes(region_bytes, passes, wgs_per_cu))


def abq_probe_mfma_i8(iters, pattern, sink):
    _run(load().abq_probe_mfma_i8(iters, pattern, sink.data_ptr(), torch.cuda.current_stream().cuda_stream), "abq_probe_mfma_i8")


def abq_probe_mfma_i8_ops(iters):
    return load().abq_probe_mfma_i8_ops(iters)


def abq_probe_mfma_f4(iters, pattern, sink):
    _run(load().abq_probe_mfma_f4(iters, pattern, sink.data_ptr(), torch.cuda.current_stream().cuda_stream), "abq_probe_mfma_f4")


def abq_probe_mfma_f4_ops(iters):
    return load().abq_probe_mfma_f4_ops(iters)
