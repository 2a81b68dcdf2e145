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


def l2_read_table(regions_mib=(0.5, 1, 2, 3, 8, 32), wgs_per_cu=(1, 2, 4, 8)):
    """Times abq_probe_l2_read over region sizes and workgroups per compute unit; rows of (MiB per XCD, passes,
    workgroups per CU, microseconds, TB/s).  `python -m paper_2408_08554_amd.probe` prints them."""
    sink = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    rows = []
    for region_mib in regions_mib:
        region = int(region_mib * (1 << 20))
        passes = max(1, int(8 // region_mib))
        buf = torch.randint(0, 255, (8 * region,), dtype=torch.uint8, device="cuda")
        for wgs in wgs_per_cu:
            for _ in range(2):
                abq_probe_l2_read(buf, region, passes, wgs, sink)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            abq_probe_l2_read(buf, region, passes, wgs, sink)
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) * 1e-3
            rows.append((region_mib, passes, wgs, t * 1e6, abq_probe_l2_read_bytes(region, passes, wgs) / t / 1e12))
    return rows


if __name__ == "__main__":
    print("| MiB per XCD | passes | workgroups per CU | us | TB/s |\n|---|---|---|---|---|")
    for r in l2_read_table():
        print(f"| {r[0]} | {r[1]} | {r[2]} | {r[3]:.0f} | {r[4]:.1f} |")
