"""numpy front end of the CPU oracle (oracle/abq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and bench.py's cpu_baseline
leg.  Holds no arithmetic of its own beyond argument marshalling; every function forwards to
the C file, which cites the passages of the paper it follows.
"""
import ctypes
import os

import numpy as np

from .build import LIB, build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            _build()
        lib = ctypes.CDLL(LIB)
        lib.abq_oracle_threads.restype = ctypes.c_int
        lib.abq_oracle_half_bits.restype = ctypes.c_uint16
        lib.abq_oracle_half_bits.argtypes = [ctypes.c_double]
        _lib = lib
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _u8(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint8, a.dtype
    return a


def _i32(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.int32)


def threads() -> int:
    return int(_load().abq_oracle_threads())


def acc(A, W):
    """int64 [M,N] = sum_k A[m,k]*W[n,k] over raw codes (Sec. 3.4, Appendix B)."""
    A, W = _u8(A), _u8(W)
    M, K = A.shape
    N, K2 = W.shape
    assert K == K2
    out = np.empty((M, N), dtype=np.int64)
    _load().abq_oracle_acc(M, N, K, _p(A), _p(W), _p(out))
    return out


def acc_sampled(A, W, ms, ns):
    A, W = _u8(A), _u8(W)
    M, K = A.shape
    N, _ = W.shape
    ms, ns = _i32(ms), _i32(ns)
    assert ms.shape == ns.shape and ms.ndim == 1
    assert ms.min(initial=0) >= 0 and ms.max(initial=0) < M and ns.min(initial=0) >= 0 and ns.max(initial=0) < N
    out = np.empty(ms.shape[0], dtype=np.int64)
    _load().abq_oracle_acc_sampled(M, N, K, _p(A), _p(W), ctypes.c_int64(ms.shape[0]), _p(ms), _p(ns), _p(out))
    return out


def acc_centered(A, W, az, wz):
    """int64 [M,N] = sum_k (A-az[m])*(W-wz[n]), computed term by term (Eq. 3 semantics)."""
    A, W = _u8(A), _u8(W)
    M, K = A.shape
    N, _ = W.shape
    az, wz = _i32(az), _i32(wz)
    assert az.shape == (M,) and wz.shape == (N,)
    out = np.empty((M, N), dtype=np.int64)
    _load().abq_oracle_acc_centered(M, N, K, _p(A), _p(W), _p(az), _p(wz), _p(out))
    return out


def acc_centered_sampled(A, W, az, wz, ms, ns):
    A, W = _u8(A), _u8(W)
    M, K = A.shape
    N, _ = W.shape
    az, wz, ms, ns = _i32(az), _i32(wz), _i32(ms), _i32(ns)
    assert az.shape == (M,) and wz.shape == (N,)
    assert ms.min(initial=0) >= 0 and ms.max(initial=0) < M and ns.min(initial=0) >= 0 and ns.max(initial=0) < N
    out = np.empty(ms.shape[0], dtype=np.int64)
    _load().abq_oracle_acc_centered_sampled(M, N, K, _p(A), _p(W), _p(az), _p(wz),
                                            ctypes.c_int64(ms.shape[0]), _p(ms), _p(ns), _p(out))
    return out


def dequant(accc, a_scale, w_scale):
    """(double Y, uint16 half bits) from the centered accumulator and the two scale vectors."""
    accc = np.ascontiguousarray(accc, dtype=np.int64)
    M, N = accc.shape
    a_scale = np.ascontiguousarray(a_scale, dtype=np.float32)
    w_scale = np.ascontiguousarray(w_scale, dtype=np.float32)
    assert a_scale.shape == (M,) and w_scale.shape == (N,)
    y = np.empty((M, N), dtype=np.float64)
    y16 = np.empty((M, N), dtype=np.uint16)
    _load().abq_oracle_dequant(M, N, _p(accc), _p(a_scale), _p(w_scale), _p(y), _p(y16))
    return y, y16


def dequant_grouped(A, W, a_zero, a_scale, w_zero, w_scale_half, gs=128, want_mag=False):
    """Per-group weight scales / zero-points [N][ceil(K/gs)] (scales as binary16 bit patterns):
    (double Y, uint16 half bits[, double size of the summed terms])."""
    A = np.ascontiguousarray(A, dtype=np.uint8)
    W = np.ascontiguousarray(W, dtype=np.uint8)
    (M, K), (N, K2) = A.shape, W.shape
    assert K == K2 and gs >= 1
    G = (K + gs - 1) // gs
    a_zero = np.ascontiguousarray(a_zero, dtype=np.int32)
    a_scale = np.ascontiguousarray(a_scale, dtype=np.float32)
    w_zero = np.ascontiguousarray(w_zero, dtype=np.int32)
    w_scale_half = np.ascontiguousarray(w_scale_half, dtype=np.uint16)
    assert a_zero.shape == (M,) and a_scale.shape == (M,) and w_zero.shape == (N, G) and w_scale_half.shape == (N, G)
    y = np.empty((M, N), dtype=np.float64)
    y16 = np.empty((M, N), dtype=np.uint16)
    mag = np.empty((M, N), dtype=np.float64) if want_mag else None
    _load().abq_oracle_dequant_grouped(M, N, K, gs, _p(A), _p(W), _p(a_zero), _p(a_scale), _p(w_zero), _p(w_scale_half),
                                       _p(y), _p(y16), _p(mag) if want_mag else None)
    return (y, y16, mag) if want_mag else (y, y16)


def half_bits(v: float) -> int:
    return int(_load().abq_oracle_half_bits(float(v)))


def plane_words(K: int) -> int:
    """Words per plane row used by the oracle's packers (K rounded up to 32 bits)."""
    return (K + 31) // 32


def pack_planes(codes, bits, Kw=None):
    """uint32 [bits,R,Kw]: plane s = (codes >> s) & 1, bit k%32 of word k/32 (Sec. 3.4 step 1)."""
    codes = _u8(codes)
    R, K = codes.shape
    Kw = plane_words(K) if Kw is None else Kw
    assert Kw * 32 >= K
    out = np.empty((bits, R, Kw), dtype=np.uint32)
    _load().abq_oracle_pack_planes(bits, R, K, Kw, _p(codes), _p(out))
    return out


def unpack_planes(planes, K):
    planes = np.ascontiguousarray(planes, dtype=np.uint32)
    bits, R, Kw = planes.shape
    out = np.empty((R, K), dtype=np.uint8)
    _load().abq_oracle_unpack_planes(bits, R, K, Kw, _p(planes), _p(out))
    return out


def acc_bitplane(a_planes, w_planes):
    """Literal Appendix B: sum_{s,t} 2^(s+t) popcount(A_t AND W_s) on packed planes."""
    a_planes = np.ascontiguousarray(a_planes, dtype=np.uint32)
    w_planes = np.ascontiguousarray(w_planes, dtype=np.uint32)
    q, M, Kw = a_planes.shape
    p, N, Kw2 = w_planes.shape
    assert Kw == Kw2
    out = np.empty((M, N), dtype=np.int64)
    _load().abq_oracle_acc_bitplane(p, q, M, N, Kw, _p(a_planes), _p(w_planes), _p(out))
    return out


def quant_act(x_half, q):
    """Per-token quantizer: (codes uint8 [M,K], a_scale float32 [M], a_zero int32 [M])."""
    x_half = np.ascontiguousarray(x_half)
    assert x_half.dtype == np.float16
    M, K = x_half.shape
    codes = np.empty((M, K), dtype=np.uint8)
    sc = np.empty(M, dtype=np.float32)
    zp = np.empty(M, dtype=np.int32)
    _load().abq_oracle_quant_act(q, M, K, _p(x_half.view(np.uint16)), _p(codes), _p(sc), _p(zp))
    return codes, sc, zp


def requant(y_half, q, scale, zero):
    """Codes of a binary16 matrix under given per-row (Delta, z): uint8 [M,N]."""
    y_half = np.ascontiguousarray(y_half)
    assert y_half.dtype == np.float16
    M, N = y_half.shape
    scale = np.ascontiguousarray(scale, dtype=np.float32)
    zero = np.ascontiguousarray(zero, dtype=np.int32)
    assert scale.shape == (M,) and zero.shape == (M,)
    codes = np.empty((M, N), dtype=np.uint8)
    _load().abq_oracle_requant(q, M, N, _p(y_half.view(np.uint16)), _p(scale), _p(zero), _p(codes))
    return codes


def add_half(a_half, b_half):
    """Element-wise binary16 sum: one binary32 addition, one rounding to binary16 (the residual add in front of RMSNorm)."""
    a_half = np.ascontiguousarray(a_half)
    b_half = np.ascontiguousarray(b_half)
    assert a_half.dtype == np.float16 and b_half.dtype == np.float16 and a_half.shape == b_half.shape
    h = np.empty(a_half.shape, dtype=np.float16)
    fn = _load().abq_oracle_add_half
    fn.argtypes = [ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    fn.restype = None
    fn(a_half.size, _p(a_half.view(np.uint16)), _p(b_half.view(np.uint16)), _p(h.view(np.uint16)))
    return h


def rmsnorm_half(x_half, gamma_half, eps):
    """RMSNorm of binary16 rows to binary16 (exact sum of squares, roundings as stated in the C source)."""
    x_half = np.ascontiguousarray(x_half)
    gamma_half = np.ascontiguousarray(gamma_half)
    assert x_half.dtype == np.float16 and gamma_half.dtype == np.float16
    M, K = x_half.shape
    assert gamma_half.shape == (K,)
    y = np.empty((M, K), dtype=np.float16)
    fn = _load().abq_oracle_rmsnorm_half
    fn.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p]
    fn.restype = None
    fn(M, K, _p(x_half.view(np.uint16)), _p(gamma_half.view(np.uint16)), float(eps), _p(y.view(np.uint16)))
    return y


def silu_mul_half(gate_half, up_half):
    """silu(gate) * up in binary16 (exp as the stated sequence of binary32 operations; see the C source)."""
    gate_half = np.ascontiguousarray(gate_half)
    up_half = np.ascontiguousarray(up_half)
    assert gate_half.dtype == np.float16 and up_half.dtype == np.float16 and gate_half.shape == up_half.shape
    M, K = gate_half.shape
    h = np.empty((M, K), dtype=np.float16)
    fn = _load().abq_oracle_silu_mul_half
    fn.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    fn.restype = None
    fn(M, K, _p(gate_half.view(np.uint16)), _p(up_half.view(np.uint16)), _p(h.view(np.uint16)))
    return h
