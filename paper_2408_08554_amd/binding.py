"""ctypes binding of libabq.so — the same names as include/abq.h, argument marshalling only.

torch is used for device memory (tensors own every buffer) and for the current stream; every
step of the path runs in the library's HIP kernels.  A missing library is an error: there is
no fallback of any kind.
"""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libabq.so")

ABQ_OK = 0
ABQ_ERR_NULL, ABQ_ERR_BITS, ABQ_ERR_SHAPE, ABQ_ERR_ALIGN = -1, -2, -3, -4
ABQ_ERR_SIZE, ABQ_ERR_LAYOUT, ABQ_ERR_HIP = -5, -6, -7
ABQ_LAYOUT_AUTO, ABQ_LAYOUT_PLANES, ABQ_LAYOUT_FIELDS, ABQ_LAYOUT_BOTH = 0, 1, 2, 3
ABQ_LAYOUT_FIELDS_G128 = 4
ABQ_USE_PLANES, ABQ_USE_FIELDS = 0x10, 0x20
ABQ_MAX_K = 131072
ABQ_STATIC_SCRATCH_BYTES = 32 << 20

# every symbol include/abq.h declares: (restype, argtypes)
_c = ctypes
_SIGNATURES = {
    "abq_version": (_c.c_int, []),
    "abq_status_string": (_c.c_char_p, [_c.c_int]),
    "abq_last_hip_error": (_c.c_int, []),
    "abq_last_decode_kernel": (_c.c_int, []),
    "abq_packed_weight_bytes": (_c.c_size_t, [_c.c_int] * 4),
    "abq_pack_weights": (_c.c_int, [_c.c_int] * 3 + [_c.c_void_p] * 3 + [_c.c_int, _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "abq_pack_weights_g128": (_c.c_int, [_c.c_int] * 3 + [_c.c_void_p] * 3 + [_c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "abq_plan_set": (_c.c_int, [_c.c_int] * 5 + [_c.c_void_p]),
    "abq_plan_get": (_c.c_int, [_c.c_int] * 5 + [_c.c_void_p]),
    "abq_plan_clear": (None, []),
    "abq_f4_packed_bytes": (_c.c_size_t, [_c.c_int] * 3),
    "abq_f4_pack_codes": (_c.c_int, [_c.c_int] * 3 + [_c.c_void_p] * 3 + [_c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "abq_f4_gemm": (_c.c_int, [_c.c_int] * 5 + [_c.c_void_p] * 4 + [_c.c_void_p]),
    "abq_unpack_weights": (_c.c_int, [_c.c_int] * 4 + [_c.c_void_p, _c.c_int, _c.c_void_p, _c.c_void_p]),
    "abq_packed_act_bytes": (_c.c_size_t, [_c.c_int] * 4),
    "abq_quant_pack_act": (_c.c_int, [_c.c_int] * 3 + [_c.c_void_p, _c.c_int, _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "abq_pack_act_codes": (_c.c_int, [_c.c_int] * 3 + [_c.c_void_p] * 3 + [_c.c_int, _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "abq_unpack_act": (_c.c_int, [_c.c_int] * 4 + [_c.c_void_p, _c.c_int] + [_c.c_void_p] * 5),
    "abq_gemm_workspace_bytes": (_c.c_size_t, [_c.c_int] * 5),
    "abq_gemm": (_c.c_int, [_c.c_int] * 5 + [_c.c_void_p, _c.c_int, _c.c_void_p, _c.c_int, _c.c_void_p, _c.c_void_p,
                                             _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "abq_gemm_act_codes_workspace_bytes": (_c.c_size_t, [_c.c_int] * 6),
    "abq_gemm_grouped_workspace_bytes": (_c.c_size_t, [_c.c_int] * 4 + [_c.c_void_p, _c.c_int, _c.c_int]),
    "abq_gemm_grouped": (_c.c_int, [_c.c_int] * 4 + [_c.c_void_p, _c.c_int, _c.c_int, _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "abq_rmsnorm_quant_act": (_c.c_int, [_c.c_int] * 3 + [_c.c_void_p, _c.c_void_p, _c.c_float] + [_c.c_void_p] * 5),
    "abq_add_rmsnorm_quant_act": (_c.c_int, [_c.c_int] * 3 + [_c.c_void_p] * 3 + [_c.c_float] + [_c.c_void_p] * 6),
    "abq_silu_mul_quant_act": (_c.c_int, [_c.c_int] * 3 + [_c.c_void_p] * 7),
    "abq_gemm_act_codes": (_c.c_int, [_c.c_int] * 5 + [_c.c_void_p] * 4 + [_c.c_int, _c.c_void_p, _c.c_void_p,
                                                                          _c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "abq_gemm_act_codes_requant": (_c.c_int, [_c.c_int] * 5 + [_c.c_void_p] * 4 + [_c.c_int, _c.c_int] + [_c.c_void_p] * 5 + [_c.c_size_t, _c.c_void_p]),
    "abq_check_packed": (_c.c_int, [_c.c_int] * 5 + [_c.c_void_p, _c.c_size_t, _c.c_void_p]),
    "abq_gemm_act_codes_static": (_c.c_int, [_c.c_int] * 5 + [_c.c_void_p] * 4 + [_c.c_int, _c.c_void_p, _c.c_void_p, _c.c_void_p]),
}

_lib = None


class AbqError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = _lib.abq_status_string(status).decode() if _lib is not None else "?"
        extra = f" (hipError {_lib.abq_last_hip_error()})" if status == ABQ_ERR_HIP and _lib is not None else ""
        super().__init__(f"{where}: {msg} [{status}]{extra}")


def load():
    """Load libabq.so (built by paper_2408_08554_amd.build); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2408_08554_amd.build` "
                               "(there is no fallback path)")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def raw():
    """The ctypes library object, for tests that exercise the error paths directly."""
    return load()


def _check(status, where):
    if status != ABQ_OK:
        raise AbqError(status, where)


def _ptr(t):
    return 0 if t is None else t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _dev(t, dtype, shape=None):
    assert t.is_cuda and t.is_contiguous() and t.dtype == dtype, (t.device, t.dtype, t.is_contiguous())
    if shape is not None:
        assert tuple(t.shape) == tuple(shape), (tuple(t.shape), shape)
    return t


def abq_version():
    return load().abq_version()


def abq_packed_weight_bytes(p, N, K, layout=ABQ_LAYOUT_AUTO):
    return load().abq_packed_weight_bytes(p, N, K, layout)


def abq_packed_act_bytes(q, M, K, layout=ABQ_LAYOUT_AUTO):
    return load().abq_packed_act_bytes(q, M, K, layout)


def abq_gemm_workspace_bytes(p, q, M, N, K):
    return load().abq_gemm_workspace_bytes(p, q, M, N, K)


def abq_pack_weights(p, w_codes, w_scale, w_zero, layout=ABQ_LAYOUT_AUTO, out=None):
    """w_codes uint8 [N,K], w_scale float32 [N], w_zero int32 [N] (device) -> packed uint8 blob."""
    lib = load()
    N, K = w_codes.shape
    _dev(w_codes, torch.uint8), _dev(w_scale, torch.float32, (N,)), _dev(w_zero, torch.int32, (N,))
    nbytes = lib.abq_packed_weight_bytes(p, N, K, layout)
    if out is None:
        out = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=w_codes.device)
    _check(lib.abq_pack_weights(p, N, K, _ptr(w_codes), _ptr(w_scale), _ptr(w_zero), layout, _ptr(out), out.numel(),
                                _stream()), "abq_pack_weights")
    return out


def abq_pack_weights_g128(p, w_codes, w_scale_fp16, w_zero, out=None):
    """w_codes uint8 [N,K], w_scale_fp16 float16 [N,G], w_zero int32 [N,G] (device), G = ceil(K/128) -> packed blob
    for w_layout = ABQ_LAYOUT_FIELDS_G128."""
    lib = load()
    N, K = w_codes.shape
    G = (K + 127) // 128
    _dev(w_codes, torch.uint8), _dev(w_scale_fp16, torch.float16, (N, G)), _dev(w_zero, torch.int32, (N, G))
    nbytes = lib.abq_packed_weight_bytes(p, N, K, ABQ_LAYOUT_FIELDS_G128)
    if out is None:
        out = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=w_codes.device)
    _check(lib.abq_pack_weights_g128(p, N, K, _ptr(w_codes), _ptr(w_scale_fp16), _ptr(w_zero), _ptr(out), out.numel(),
                                     _stream()), "abq_pack_weights_g128")
    return out


def abq_check_packed(kind, bits, rows, K, layout, packed):
    """Status of the load-time header check (0 = the blob matches; synchronises)."""
    return load().abq_check_packed(kind, bits, rows, K, layout, _ptr(packed), packed.numel(), _stream())


def abq_unpack_weights(p, N, K, layout, packed, which):
    lib = load()
    out = torch.empty((N, K), dtype=torch.uint8, device=packed.device)
    _check(lib.abq_unpack_weights(p, N, K, layout, _ptr(packed), which, _ptr(out), _stream()), "abq_unpack_weights")
    return out


def abq_quant_pack_act(q, x_fp16, layout=ABQ_LAYOUT_AUTO, out=None):
    """x_fp16 float16 [M,K] (device) -> packed activation blob."""
    lib = load()
    M, K = x_fp16.shape
    _dev(x_fp16, torch.float16)
    nbytes = lib.abq_packed_act_bytes(q, M, K, layout)
    if out is None:
        out = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=x_fp16.device)
    _check(lib.abq_quant_pack_act(q, M, K, _ptr(x_fp16), layout, _ptr(out), out.numel(), _stream()), "abq_quant_pack_act")
    return out


def abq_pack_act_codes(q, a_codes, a_scale, a_zero, layout=ABQ_LAYOUT_AUTO, out=None):
    lib = load()
    M, K = a_codes.shape
    _dev(a_codes, torch.uint8), _dev(a_scale, torch.float32, (M,)), _dev(a_zero, torch.int32, (M,))
    nbytes = lib.abq_packed_act_bytes(q, M, K, layout)
    if out is None:
        out = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=a_codes.device)
    _check(lib.abq_pack_act_codes(q, M, K, _ptr(a_codes), _ptr(a_scale), _ptr(a_zero), layout, _ptr(out), out.numel(),
                                  _stream()), "abq_pack_act_codes")
    return out


def abq_f4_pack_codes(bits, codes, scale, zero, out=None):
    """codes uint8 [rows,K] (weights: rows = N; activations: rows = M) -> blob of the 4-bit floating-point MFMA path."""
    lib = load()
    rows, K = codes.shape
    _dev(codes, torch.uint8), _dev(scale, torch.float32, (rows,)), _dev(zero, torch.int32, (rows,))
    nbytes = lib.abq_f4_packed_bytes(bits, rows, K)
    if out is None:
        out = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=codes.device)
    _check(lib.abq_f4_pack_codes(bits, rows, K, _ptr(codes), _ptr(scale), _ptr(zero), _ptr(out), out.numel(), _stream()),
           "abq_f4_pack_codes")
    return out


def abq_f4_gemm(p, q, M, N, K, packed_act, packed_w, y=None, acc=None, want_acc=False):
    """-> (y float16 [M,N], acc int32 [M,N] or None)."""
    dev = packed_w.device
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=dev)
    if acc is None and want_acc:
        acc = torch.empty((M, N), dtype=torch.int32, device=dev)
    _check(load().abq_f4_gemm(p, q, M, N, K, _ptr(packed_act), _ptr(packed_w), _ptr(y), _ptr(acc), _stream()), "abq_f4_gemm")
    return y, acc


def abq_unpack_act(q, M, K, layout, packed, which):
    """-> (codes uint8 [M,K], scale float32 [M], zero int32 [M], sum int32 [M])."""
    lib = load()
    dev = packed.device
    codes = torch.empty((M, K), dtype=torch.uint8, device=dev)
    scale = torch.empty(M, dtype=torch.float32, device=dev)
    zero = torch.empty(M, dtype=torch.int32, device=dev)
    asum = torch.empty(M, dtype=torch.int32, device=dev)
    _check(lib.abq_unpack_act(q, M, K, layout, _ptr(packed), which, _ptr(codes), _ptr(scale), _ptr(zero), _ptr(asum),
                              _stream()), "abq_unpack_act")
    return codes, scale, zero, asum


def abq_gemm(p, q, M, N, K, packed_act, a_layout, packed_w, w_layout, y=None, acc=None, want_acc=False, workspace=None):
    """-> (y float16 [M,N], acc int32 [M,N] or None).  Buffers are allocated when not given."""
    lib = load()
    dev = packed_w.device
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=dev)
    if acc is None and want_acc:
        acc = torch.empty((M, N), dtype=torch.int32, device=dev)
    need = lib.abq_gemm_workspace_bytes(p, q, M, N, K)
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    _check(lib.abq_gemm(p, q, M, N, K, _ptr(packed_act), a_layout, _ptr(packed_w), w_layout, _ptr(y), _ptr(acc),
                        _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream()), "abq_gemm")
    return y, acc


def abq_gemm_act_codes_workspace_bytes(p, q, M, N, K, w_layout):
    return load().abq_gemm_act_codes_workspace_bytes(p, q, M, N, K, w_layout)


def abq_gemm_act_codes(p, q, M, N, K, a_codes, a_scale, a_zero, packed_w, w_layout, y=None, acc=None, want_acc=False,
                       workspace=None):
    """Activation packing fused into the matmul -> (y float16 [M,N], acc int32 [M,N] or None)."""
    lib = load()
    dev = packed_w.device
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=dev)
    if acc is None and want_acc:
        acc = torch.empty((M, N), dtype=torch.int32, device=dev)
    need = lib.abq_gemm_act_codes_workspace_bytes(p, q, M, N, K, w_layout)
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    _check(lib.abq_gemm_act_codes(p, q, M, N, K, _ptr(a_codes), _ptr(a_scale), _ptr(a_zero), _ptr(packed_w), w_layout,
                                  _ptr(y), _ptr(acc), _ptr(workspace), 0 if workspace is None else workspace.numel(),
                                  _stream()), "abq_gemm_act_codes")
    return y, acc


def abq_gemm_act_codes_requant(p, q, M, N, K, a_codes, a_scale, a_zero, packed_w, w_layout, q_out, out_scale, out_zero,
                               want_y=True, workspace=None):
    """-> (codes uint8 [M,N] of the next layer under (out_scale, out_zero), y float16 [M,N] or None)."""
    lib = load()
    dev = packed_w.device
    _dev(out_scale, torch.float32, (M,)), _dev(out_zero, torch.int32, (M,))
    codes = torch.empty((M, N), dtype=torch.uint8, device=dev)
    y = torch.empty((M, N), dtype=torch.float16, device=dev) if want_y else None
    need = lib.abq_gemm_act_codes_workspace_bytes(p, q, M, N, K, w_layout)
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    _check(lib.abq_gemm_act_codes_requant(p, q, M, N, K, _ptr(a_codes), _ptr(a_scale), _ptr(a_zero), _ptr(packed_w), w_layout, q_out,
                                          _ptr(out_scale), _ptr(out_zero), _ptr(codes), _ptr(y), _ptr(workspace),
                                          0 if workspace is None else workspace.numel(), _stream()), "abq_gemm_act_codes_requant")
    return codes, y


def abq_gemm_act_codes_static(p, q, M, N, K, a_codes, a_scale, a_zero, packed_w, w_layout, y, acc=None):
    """abq_gemm_act_codes without a workspace and without any allocation: the caller passes every buffer."""
    _check(load().abq_gemm_act_codes_static(p, q, M, N, K, _ptr(a_codes), _ptr(a_scale), _ptr(a_zero), _ptr(packed_w), w_layout,
                                            _ptr(y), _ptr(acc), _stream()), "abq_gemm_act_codes_static")
    return y, acc


class AbqProblem(_c.Structure):
    """struct abq_problem of include/abq.h (host descriptor holding device pointers)."""
    _fields_ = [("N", _c.c_int), ("K", _c.c_int), ("packed_w", _c.c_void_p), ("packed_act", _c.c_void_p),
                ("a_codes", _c.c_void_p), ("a_scale", _c.c_void_p), ("a_zero", _c.c_void_p), ("y_fp16", _c.c_void_p),
                ("acc_i32", _c.c_void_p)]


def make_problems(problems):
    """problems: list of dicts with N, K, packed_w, y and either packed_act or a_codes/a_scale/a_zero (torch tensors),
    optionally acc.  Returns the ctypes array (keep the tensors alive while it is in use)."""
    arr = (AbqProblem * len(problems))()
    for d, pr in zip(arr, problems):
        d.N, d.K = pr["N"], pr["K"]
        d.packed_w = _ptr(pr["packed_w"])
        d.packed_act = _ptr(pr.get("packed_act"))
        d.a_codes = _ptr(pr.get("a_codes"))
        d.a_scale = _ptr(pr.get("a_scale"))
        d.a_zero = _ptr(pr.get("a_zero"))
        d.y_fp16 = _ptr(pr["y"])
        d.acc_i32 = _ptr(pr.get("acc"))
    return arr


def abq_gemm_grouped_workspace_bytes(p, q, M, problems, a_layout, w_layout):
    arr = problems if isinstance(problems, _c.Array) else make_problems(problems)
    return load().abq_gemm_grouped_workspace_bytes(p, q, M, len(arr), _c.addressof(arr), a_layout, w_layout)


def abq_gemm_grouped(p, q, M, problems, a_layout, w_layout, workspace=None):
    """One call for a list of independent problems that share p, q, M (see make_problems); outputs are written to
    the y / acc tensors of each problem."""
    lib = load()
    arr = problems if isinstance(problems, _c.Array) else make_problems(problems)
    need = lib.abq_gemm_grouped_workspace_bytes(p, q, M, len(arr), _c.addressof(arr), a_layout, w_layout)
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device="cuda")
    _check(lib.abq_gemm_grouped(p, q, M, len(arr), _c.addressof(arr), a_layout, w_layout, _ptr(workspace),
                                0 if workspace is None else workspace.numel(), _stream()), "abq_gemm_grouped")


class AbqPlan(_c.Structure):
    """struct abq_plan of include/abq.h (0 = keep the library's rule for that knob)."""
    _fields_ = [(n, _c.c_int) for n in ("skinny_waves", "skinny_kgroups", "tiled_mt", "tiled_ntw", "tiled_wd", "tiled_band", "direct_r")]


def abq_plan_set(p, q, M, N, K, plan=None, **knobs):
    """plan: an AbqPlan, or knobs as keywords; neither removes the entry."""
    if plan is None and knobs:
        plan = AbqPlan(**knobs)
    _check(load().abq_plan_set(p, q, M, N, K, None if plan is None else _c.addressof(plan)), "abq_plan_set")


def abq_plan_get(p, q, M, N, K):
    out = AbqPlan()
    _check(load().abq_plan_get(p, q, M, N, K, _c.addressof(out)), "abq_plan_get")
    return {n: getattr(out, n) for n, _ in AbqPlan._fields_}


ABQ_DECODE_DIRECT, ABQ_DECODE_STREAMING, ABQ_DECODE_SHARED_OPERAND = 1, 2, 3


def abq_last_decode_kernel():
    """Test hook: ABQ_DECODE_* of the last M <= 16 matmul call of this thread."""
    return load().abq_last_decode_kernel()


def abq_plan_clear():
    load().abq_plan_clear()


def abq_rmsnorm_quant_act(q, x_fp16, gamma_fp16, eps, want_y=False):
    """-> (codes uint8 [M,K], a_scale float32 [M], a_zero int32 [M], y float16 [M,K] or None)."""
    M, K = x_fp16.shape
    dev = x_fp16.device
    codes = torch.empty((M, K), dtype=torch.uint8, device=dev)
    scale = torch.empty(M, dtype=torch.float32, device=dev)
    zero = torch.empty(M, dtype=torch.int32, device=dev)
    y = torch.empty((M, K), dtype=torch.float16, device=dev) if want_y else None
    _check(load().abq_rmsnorm_quant_act(q, M, K, _ptr(x_fp16), _ptr(gamma_fp16), float(eps), _ptr(codes), _ptr(scale),
                                        _ptr(zero), _ptr(y), _stream()), "abq_rmsnorm_quant_act")
    return codes, scale, zero, y


def abq_add_rmsnorm_quant_act(q, x_fp16, residual_fp16, gamma_fp16, eps, want_y=False, sum_out=None):
    """-> (codes, a_scale, a_zero, h = x + residual as float16 [M,K], y float16 [M,K] or None)."""
    M, K = x_fp16.shape
    dev = x_fp16.device
    codes = torch.empty((M, K), dtype=torch.uint8, device=dev)
    scale = torch.empty(M, dtype=torch.float32, device=dev)
    zero = torch.empty(M, dtype=torch.int32, device=dev)
    h = torch.empty((M, K), dtype=torch.float16, device=dev) if sum_out is None else sum_out
    y = torch.empty((M, K), dtype=torch.float16, device=dev) if want_y else None
    _check(load().abq_add_rmsnorm_quant_act(q, M, K, _ptr(x_fp16), _ptr(residual_fp16), _ptr(gamma_fp16), float(eps), _ptr(codes),
                                            _ptr(scale), _ptr(zero), _ptr(h), _ptr(y), _stream()), "abq_add_rmsnorm_quant_act")
    return codes, scale, zero, h, y


def abq_silu_mul_quant_act(q, gate_fp16, up_fp16, want_h=False):
    """-> (codes uint8 [M,K], a_scale float32 [M], a_zero int32 [M], h float16 [M,K] or None)."""
    M, K = gate_fp16.shape
    dev = gate_fp16.device
    codes = torch.empty((M, K), dtype=torch.uint8, device=dev)
    scale = torch.empty(M, dtype=torch.float32, device=dev)
    zero = torch.empty(M, dtype=torch.int32, device=dev)
    h = torch.empty((M, K), dtype=torch.float16, device=dev) if want_h else None
    _check(load().abq_silu_mul_quant_act(q, M, K, _ptr(gate_fp16), _ptr(up_fp16), _ptr(codes), _ptr(scale), _ptr(zero),
                                         _ptr(h), _stream()), "abq_silu_mul_quant_act")
    return codes, scale, zero, h
