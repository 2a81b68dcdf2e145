"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2408_08554_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    header = open(os.path.join(ROOT, "include", "abq.h")).read()
    declared = set(re.findall(r"\b(abq_[a-z_0-9]+)\s*\(", header))
    assert declared == set(B._SIGNATURES), declared ^ set(B._SIGNATURES)
    for name in declared:
        assert getattr(lib, name) is not None
    # the measurement aids are a library and a header of their own
    from paper_2408_08554_amd import probe
    plib = probe.load()
    pdeclared = set(re.findall(r"\b(abq_[a-z_0-9]+)\s*\(", open(os.path.join(ROOT, "include", "abq_probe.h")).read()))
    assert pdeclared == set(probe._SIGNATURES) and not (pdeclared & declared)
    for name in pdeclared:
        assert getattr(plib, name) is not None
        assert not hasattr(lib, name), "the product library must not export measurement probes"
    assert lib.abq_version() >= 100
    assert lib.abq_status_string(0) == b"ok"
    for st in range(-7, 0):
        assert len(lib.abq_status_string(st)) > 3


def test_size_queries():
    lib = B.load()
    # header + params + fields for W4 4096x4096: the streamed part is exactly p*N*K/8
    nb = lib.abq_packed_weight_bytes(4, 4096, 4096, B.ABQ_LAYOUT_FIELDS)
    assert nb == 256 + 4096 * 16 + 4 * 4096 * 4096 // 8
    both = lib.abq_packed_weight_bytes(4, 4096, 4096, B.ABQ_LAYOUT_BOTH)
    planes = lib.abq_packed_weight_bytes(4, 4096, 4096, B.ABQ_LAYOUT_PLANES)
    assert both == nb + planes - 256 - 4096 * 16
    assert lib.abq_packed_weight_bytes(0, 16, 16, 0) == 0
    assert lib.abq_packed_weight_bytes(9, 16, 16, 0) == 0
    assert lib.abq_packed_weight_bytes(4, 0, 16, 0) == 0
    assert lib.abq_packed_weight_bytes(4, 16, B.ABQ_MAX_K + 1, 0) == 0
    assert lib.abq_packed_weight_bytes(4, 16, 16, 7) == 0
    assert lib.abq_packed_act_bytes(8, 1, 4096, B.ABQ_LAYOUT_FIELDS) == 256 + 256 + 4096
    assert lib.abq_packed_act_bytes(8, 3, 100, B.ABQ_LAYOUT_PLANES) == 256 + 256 + 512   # 8 planes x 3 rows x 4 words x 4 B = 384, sections are 256-B aligned
    assert lib.abq_gemm_workspace_bytes(2, 8, 1, 4096, 4096) == 0
    assert lib.abq_gemm_workspace_bytes(8, 8, 1, 16, 40000) == 0   # overflow bound -> 0


A16 = 0x1000  # any non-null 16-byte aligned value; validation fails before it is dereferenced


@pytest.mark.parametrize("args,want", [
    ((4, 16, 64, 0, A16, A16, 0, A16, 1 << 20, None), B.ABQ_ERR_NULL),
    ((0, 16, 64, A16, A16, A16, 0, A16, 1 << 20, None), B.ABQ_ERR_BITS),
    ((9, 16, 64, A16, A16, A16, 0, A16, 1 << 20, None), B.ABQ_ERR_BITS),
    ((4, 0, 64, A16, A16, A16, 0, A16, 1 << 20, None), B.ABQ_ERR_SHAPE),
    ((4, 16, B.ABQ_MAX_K + 1, A16, A16, A16, 0, A16, 1 << 30, None), B.ABQ_ERR_SHAPE),
    ((4, 16, 64, A16, A16, A16, 9, A16, 1 << 20, None), B.ABQ_ERR_LAYOUT),
    ((4, 16, 64, A16 + 4, A16, A16, 0, A16, 1 << 20, None), B.ABQ_ERR_ALIGN),
    ((4, 16, 64, A16, A16, A16, 0, A16, 100, None), B.ABQ_ERR_SIZE),
])
def test_pack_weights_rejects(args, want):
    assert B.load().abq_pack_weights(*args) == want


@pytest.mark.parametrize("args,want", [
    ((8, 1, 64, None, 0, A16, 1 << 20, None), B.ABQ_ERR_NULL),
    ((0, 1, 64, A16, 0, A16, 1 << 20, None), B.ABQ_ERR_BITS),
    ((8, 1, 0, A16, 0, A16, 1 << 20, None), B.ABQ_ERR_SHAPE),
    ((8, 1, 64, A16 + 2, 0, A16, 1 << 20, None), B.ABQ_ERR_ALIGN),
    ((8, 1, 64, A16, 0, A16, 10, None), B.ABQ_ERR_SIZE),
    ((8, 1, 64, A16, 5, A16, 1 << 20, None), B.ABQ_ERR_LAYOUT),
])
def test_quant_pack_act_rejects(args, want):
    assert B.load().abq_quant_pack_act(*args) == want


def test_g128_pack_rejects_and_size_query():
    lib = B.load()
    G128 = B.ABQ_LAYOUT_FIELDS_G128
    # the field-packed blob plus one 256-byte record block per (16-channel tile, 512-k super-chunk)
    assert lib.abq_packed_weight_bytes(4, 4096, 4096, G128) == lib.abq_packed_weight_bytes(4, 4096, 4096, B.ABQ_LAYOUT_FIELDS) + 256 * 8 * 256
    assert lib.abq_packed_weight_bytes(2, 17, 100, G128) == lib.abq_packed_weight_bytes(2, 17, 100, B.ABQ_LAYOUT_FIELDS) + 2 * 256
    assert lib.abq_packed_act_bytes(8, 1, 4096, G128) == 0          # a weight-side layout only
    f = lib.abq_pack_weights_g128
    assert f(4, 16, 256, A16, A16, None, A16, 1 << 20, None) == B.ABQ_ERR_NULL
    assert f(4, 16, 256, A16, None, A16, A16, 1 << 20, None) == B.ABQ_ERR_NULL
    assert f(9, 16, 256, A16, A16, A16, A16, 1 << 20, None) == B.ABQ_ERR_BITS
    assert f(4, 16, 0, A16, A16, A16, A16, 1 << 20, None) == B.ABQ_ERR_SHAPE
    assert f(4, 16, 256, A16, A16 + 2, A16, A16, 1 << 20, None) == B.ABQ_ERR_ALIGN
    assert f(4, 16, 256, A16, A16, A16, A16, 1000, None) == B.ABQ_ERR_SIZE
    # the per-channel packer does not write this layout; the matmuls cannot return the raw accumulator from it
    assert lib.abq_pack_weights(4, 16, 256, A16, A16, A16, G128, A16, 1 << 20, None) == B.ABQ_ERR_LAYOUT
    assert gemm(lib, al=B.ABQ_LAYOUT_FIELDS, wl=G128, acc=A16) == B.ABQ_ERR_LAYOUT
    assert gemm(lib, al=B.ABQ_LAYOUT_PLANES, wl=G128) == B.ABQ_ERR_LAYOUT
    assert gemm_fused(lib, wl=G128, acc=A16) == B.ABQ_ERR_LAYOUT
    q = lib.abq_gemm_act_codes_workspace_bytes
    assert q(4, 8, 1, 4096, 4096, G128) == 0 and q(4, 8, 16, 4096, 4096, G128) == 0       # one launch up to 16 rows
    assert q(4, 8, 300, 4096, 4096, G128) == lib.abq_packed_act_bytes(8, 300, 4096, B.ABQ_LAYOUT_FIELDS)   # above: pack + tiled per-group kernel
    assert q(4, 8, 2, 64, 1000, G128) == lib.abq_packed_act_bytes(8, 2, 1000, B.ABQ_LAYOUT_FIELDS)   # K not a multiple of 16


def test_plan_table_set_get_clear_and_rejects():
    B.load()
    B.abq_plan_clear()
    zero = dict(skinny_waves=0, skinny_kgroups=0, tiled_mt=0, tiled_ntw=0, tiled_wd=0, tiled_band=0, direct_r=0)
    assert B.abq_plan_get(4, 8, 1, 4096, 4096) == zero
    B.abq_plan_set(4, 8, 1, 4096, 4096, skinny_waves=6)
    B.abq_plan_set(2, 8, 1, 4096, 11008, direct_r=-1)
    assert B.abq_plan_get(2, 8, 1, 4096, 11008) == dict(zero, direct_r=-1)
    B.abq_plan_set(6, 6, 512, 11008, 4096, tiled_mt=4, tiled_ntw=2, tiled_wd=4, tiled_band=8)
    assert B.abq_plan_get(4, 8, 1, 4096, 4096) == dict(zero, skinny_waves=6)
    assert B.abq_plan_get(6, 6, 512, 11008, 4096) == dict(zero, tiled_mt=4, tiled_ntw=2, tiled_wd=4, tiled_band=8)
    assert B.abq_plan_get(4, 8, 2, 4096, 4096) == zero                      # exact problem sizes only
    B.abq_plan_set(4, 8, 1, 4096, 4096)                                     # no plan: removes the entry
    assert B.abq_plan_get(4, 8, 1, 4096, 4096) == zero
    assert B.abq_plan_get(6, 6, 512, 11008, 4096)["tiled_mt"] == 4
    B.abq_plan_clear()
    assert B.abq_plan_get(6, 6, 512, 11008, 4096) == zero
    lib = B.load()
    for bad in (dict(skinny_waves=3), dict(skinny_waves=9), dict(skinny_kgroups=5), dict(tiled_mt=6), dict(tiled_ntw=3),
                dict(tiled_wd=3), dict(tiled_band=-1), dict(direct_r=3), dict(direct_r=-3)):
        plan = B.AbqPlan(**bad)
        assert lib.abq_plan_set(4, 8, 1, 64, 64, ctypes.addressof(plan)) == B.ABQ_ERR_LAYOUT, bad
    plan = B.AbqPlan(skinny_waves=4)
    assert lib.abq_plan_set(9, 8, 1, 64, 64, ctypes.addressof(plan)) == B.ABQ_ERR_BITS
    assert lib.abq_plan_set(4, 8, 0, 64, 64, ctypes.addressof(plan)) == B.ABQ_ERR_SHAPE
    assert lib.abq_plan_get(4, 8, 1, 64, 64, None) == B.ABQ_ERR_NULL
    assert B.abq_plan_get(4, 8, 1, 64, 64) == zero                          # rejected plans left nothing behind


def test_pack_act_codes_rejects():
    lib = B.load()
    assert lib.abq_pack_act_codes(8, 1, 64, A16, None, A16, 0, A16, 1 << 20, None) == B.ABQ_ERR_NULL
    assert lib.abq_pack_act_codes(8, -1, 64, A16, A16, A16, 0, A16, 1 << 20, None) == B.ABQ_ERR_SHAPE
    assert lib.abq_pack_act_codes(12, 1, 64, A16, A16, A16, 0, A16, 1 << 20, None) == B.ABQ_ERR_BITS
    assert lib.abq_pack_act_codes(8, 1, 64, A16, A16, A16, 0, A16, 16, None) == B.ABQ_ERR_SIZE


def gemm(lib, p=4, q=8, M=1, N=16, K=64, pa=A16, al=0, pw=A16, wl=0, y=A16, acc=None, ws=None, wsb=0):
    return lib.abq_gemm(p, q, M, N, K, pa, al, pw, wl, y, acc, ws, wsb, None)


def test_gemm_rejects():
    lib = B.load()
    assert gemm(lib, pa=None) == B.ABQ_ERR_NULL
    assert gemm(lib, y=None) == B.ABQ_ERR_NULL
    assert gemm(lib, p=0) == B.ABQ_ERR_BITS
    assert gemm(lib, q=9) == B.ABQ_ERR_BITS
    assert gemm(lib, M=0) == B.ABQ_ERR_SHAPE
    # 32-bit accumulator bound: K*(2^p-1)*(2^q-1) must fit int32
    assert gemm(lib, p=8, q=8, K=33026) == B.ABQ_ERR_SHAPE
    assert gemm(lib, p=8, q=8, K=33025, y=A16 + 8) == B.ABQ_ERR_ALIGN   # shape accepted, next check trips
    assert gemm(lib, K=B.ABQ_MAX_K + 1) == B.ABQ_ERR_SHAPE
    # the two blobs must share a representation
    assert gemm(lib, al=B.ABQ_LAYOUT_PLANES, wl=B.ABQ_LAYOUT_FIELDS) == B.ABQ_ERR_LAYOUT
    assert gemm(lib, al=B.ABQ_LAYOUT_FIELDS, wl=B.ABQ_LAYOUT_FIELDS | B.ABQ_USE_PLANES) == B.ABQ_ERR_LAYOUT
    assert gemm(lib, al=B.ABQ_LAYOUT_BOTH, wl=B.ABQ_LAYOUT_BOTH | B.ABQ_USE_PLANES | B.ABQ_USE_FIELDS) == B.ABQ_ERR_LAYOUT
    assert gemm(lib, al=4) == B.ABQ_ERR_LAYOUT    # the group layout exists for weights only
    assert gemm(lib, al=5) == B.ABQ_ERR_LAYOUT
    assert gemm(lib, acc=A16 + 4) == B.ABQ_ERR_ALIGN


def gemm_fused(lib, p=4, q=8, M=1, N=16, K=64, a=A16, sc=A16, zp=A16, pw=A16, wl=0, y=A16, acc=None, ws=None, wsb=0):
    return lib.abq_gemm_act_codes(p, q, M, N, K, a, sc, zp, pw, wl, y, acc, ws, wsb, None)


def test_gemm_act_codes_rejects_and_workspace_query():
    lib = B.load()
    assert gemm_fused(lib, a=None) == B.ABQ_ERR_NULL
    assert gemm_fused(lib, zp=None) == B.ABQ_ERR_NULL
    assert gemm_fused(lib, y=None) == B.ABQ_ERR_NULL
    assert gemm_fused(lib, p=9) == B.ABQ_ERR_BITS
    assert gemm_fused(lib, N=0) == B.ABQ_ERR_SHAPE
    assert gemm_fused(lib, p=8, q=8, K=33026) == B.ABQ_ERR_SHAPE
    assert gemm_fused(lib, wl=7) == B.ABQ_ERR_LAYOUT
    assert gemm_fused(lib, wl=B.ABQ_LAYOUT_FIELDS | B.ABQ_USE_PLANES) == B.ABQ_ERR_LAYOUT
    assert gemm_fused(lib, a=A16 + 1) == B.ABQ_ERR_ALIGN
    q = lib.abq_gemm_act_codes_workspace_bytes
    # one kernel: decode shapes on field-packed weights with K a multiple of 16
    assert q(4, 8, 1, 4096, 4096, B.ABQ_LAYOUT_FIELDS) == 0
    assert q(2, 8, 8, 4096, 11008, B.ABQ_LAYOUT_AUTO) == 0
    assert q(6, 6, 16, 64, 48, B.ABQ_LAYOUT_BOTH) == 0
    assert q(1, 1, 1, 13824, 5120, B.ABQ_LAYOUT_BOTH) == 0          # a blob with both representations takes the MFMA path
    # two kernels: the packed activations live in the workspace
    for args in [(4, 8, 1, 4096, 4090, B.ABQ_LAYOUT_FIELDS),      # K not a multiple of 16
                 (6, 6, 128, 11008, 4096, B.ABQ_LAYOUT_FIELDS),   # prefill shape
                 (2, 8, 1, 4096, 4096, B.ABQ_LAYOUT_PLANES),      # bit-serial family
                 (4, 8, 1, 4096, 4096, B.ABQ_LAYOUT_BOTH | B.ABQ_USE_PLANES)]:
        p_, q_, M, N, K, wl = args
        assert q(*args) == lib.abq_packed_act_bytes(q_, M, K, wl & 3) + lib.abq_gemm_workspace_bytes(p_, q_, M, N, K)
        assert q(*args) > 0
    assert q(0, 8, 1, 16, 64, 0) == 0 and q(4, 8, 1, 16, 64, 9) == 0
    # a needed workspace that is missing or too small is an error before any HIP call
    assert gemm_fused(lib, M=128, N=11008, K=4096) == B.ABQ_ERR_NULL
    assert gemm_fused(lib, M=128, N=11008, K=4096, ws=A16, wsb=64) == B.ABQ_ERR_SIZE
    assert gemm_fused(lib, K=40, ws=A16, wsb=64) == B.ABQ_ERR_SIZE


def _problems(*items):
    arr = (B.AbqProblem * len(items))()
    for d, it in zip(arr, items):
        for k, v in it.items():
            setattr(d, k, v)
    return arr


def test_gemm_grouped_rejects_and_workspace_query():
    import ctypes
    lib = B.load()
    packed = dict(N=64, K=4096, packed_w=A16, packed_act=A16, y_fp16=A16)
    codes = dict(N=64, K=4096, packed_w=A16, a_codes=A16, a_scale=A16, a_zero=A16, y_fp16=A16)

    def call(arr, p=4, q=8, M=1, count=None, al=0, wl=0, ws=None, wsb=0):
        return lib.abq_gemm_grouped(p, q, M, len(arr) if count is None else count, ctypes.addressof(arr), al, wl, ws, wsb, None)

    def query(arr, p=4, q=8, M=1, al=0, wl=0):
        return lib.abq_gemm_grouped_workspace_bytes(p, q, M, len(arr), ctypes.addressof(arr), al, wl)

    assert lib.abq_gemm_grouped(4, 8, 1, 1, None, 0, 0, None, 0, None) == B.ABQ_ERR_NULL
    assert call(_problems(packed), count=0) == B.ABQ_ERR_SHAPE
    assert call(_problems(dict(packed, packed_w=None))) == B.ABQ_ERR_NULL
    assert call(_problems(dict(packed, y_fp16=None))) == B.ABQ_ERR_NULL
    assert call(_problems(dict(packed, packed_act=None))) == B.ABQ_ERR_NULL
    assert call(_problems(dict(codes, a_zero=None))) == B.ABQ_ERR_NULL
    assert call(_problems(packed, codes)) == B.ABQ_ERR_LAYOUT                  # mixed activation forms
    assert call(_problems(dict(codes, packed_act=A16))) == B.ABQ_ERR_LAYOUT    # both forms in one descriptor
    assert call(_problems(packed), p=9) == B.ABQ_ERR_BITS
    assert call(_problems(dict(packed, N=0))) == B.ABQ_ERR_SHAPE
    assert call(_problems(packed, dict(packed, K=B.ABQ_MAX_K + 1))) == B.ABQ_ERR_SHAPE
    assert call(_problems(dict(packed, y_fp16=A16 + 2))) == B.ABQ_ERR_ALIGN
    assert call(_problems(packed), wl=B.ABQ_USE_PLANES | B.ABQ_USE_FIELDS) == B.ABQ_ERR_LAYOUT
    assert call(_problems(packed), al=9) == B.ABQ_ERR_LAYOUT
    # workspace: none when one launch serves the group, none for packed activations
    assert query(_problems(codes, dict(codes, N=11008), dict(codes, K=11008))) == 0
    assert query(_problems(packed, dict(packed, K=100))) == 0
    # unpacked codes that cannot be grouped (a short K here) fall back to single calls: the largest of their needs
    short = dict(codes, K=1000)
    need = query(_problems(codes, short))
    assert need == lib.abq_gemm_act_codes_workspace_bytes(4, 8, 1, 64, 1000, 0) and need > 0
    assert call(_problems(codes, short)) == B.ABQ_ERR_NULL
    assert call(_problems(codes, short), ws=A16, wsb=16) == B.ABQ_ERR_SIZE
    assert query(_problems(codes), p=0) == 0


def test_f4_entry_points_reject_bad_arguments():
    lib = B.load()
    assert lib.abq_f4_packed_bytes(2, 16, 128) == 256 + 256 + 1024
    assert lib.abq_f4_packed_bytes(2, 17, 129) == 256 + 512 + 4 * 1024
    assert lib.abq_f4_packed_bytes(3, 16, 128) == 0 and lib.abq_f4_packed_bytes(2, 0, 128) == 0
    assert lib.abq_f4_pack_codes(2, 16, 128, None, A16, A16, A16, 4096, None) == B.ABQ_ERR_NULL
    assert lib.abq_f4_pack_codes(3, 16, 128, A16, A16, A16, A16, 4096, None) == B.ABQ_ERR_BITS
    assert lib.abq_f4_pack_codes(2, 0, 128, A16, A16, A16, A16, 4096, None) == B.ABQ_ERR_SHAPE
    assert lib.abq_f4_pack_codes(2, 16, 128, A16 + 4, A16, A16, A16, 4096, None) == B.ABQ_ERR_ALIGN
    assert lib.abq_f4_pack_codes(2, 16, 128, A16, A16, A16, A16, 1535, None) == B.ABQ_ERR_SIZE
    assert lib.abq_f4_gemm(2, 2, 1, 1, 1, None, A16, A16, None, None) == B.ABQ_ERR_NULL
    assert lib.abq_f4_gemm(3, 2, 1, 1, 1, A16, A16, A16, None, None) == B.ABQ_ERR_BITS
    assert lib.abq_f4_gemm(2, 2, 1, 0, 1, A16, A16, A16, None, None) == B.ABQ_ERR_SHAPE
    assert lib.abq_f4_gemm(2, 2, 1, 1, 1, A16, A16, A16 + 2, None, None) == B.ABQ_ERR_ALIGN


def test_probe_rejects():
    from paper_2408_08554_amd import probe
    lib = probe.load()
    assert lib.abq_probe_stream_read(None, 4096, A16, None) == B.ABQ_ERR_NULL
    assert lib.abq_probe_stream_read(A16, 4096, None, None) == B.ABQ_ERR_NULL
    assert lib.abq_probe_stream_read(A16, 8, A16, None) == B.ABQ_ERR_SHAPE
    assert lib.abq_probe_stream_read(A16, 4100, A16, None) == B.ABQ_ERR_SHAPE
    assert lib.abq_probe_stream_read(A16 + 4, 4096, A16, None) == B.ABQ_ERR_ALIGN
    assert lib.abq_probe_l2_read(None, 1 << 20, 1, 1, A16, None) == B.ABQ_ERR_NULL
    assert lib.abq_probe_l2_read(A16, 1 << 20, 1, 1, None, None) == B.ABQ_ERR_NULL
    assert lib.abq_probe_l2_read(A16, 1000, 1, 1, A16, None) == B.ABQ_ERR_SHAPE          # not a multiple of 32 KiB
    assert lib.abq_probe_l2_read(A16, 1 << 20, 0, 1, A16, None) == B.ABQ_ERR_SHAPE
    assert lib.abq_probe_l2_read(A16, 1 << 20, 1, 9, A16, None) == B.ABQ_ERR_SHAPE
    assert lib.abq_probe_l2_read(A16 + 4, 1 << 20, 1, 1, A16, None) == B.ABQ_ERR_ALIGN
    assert lib.abq_probe_mfma_i8(10, 0, None, None) == B.ABQ_ERR_NULL
    assert lib.abq_probe_mfma_i8(0, 0, A16, None) == B.ABQ_ERR_SHAPE
    assert lib.abq_probe_mfma_i8(10, 2, A16, None) == B.ABQ_ERR_SHAPE
    assert lib.abq_probe_mfma_i8_ops(0) == 0.0
    assert lib.abq_probe_mfma_f4(10, 0, None, None) == B.ABQ_ERR_NULL
    assert lib.abq_probe_mfma_f4(0, 0, A16, None) == B.ABQ_ERR_SHAPE
    assert lib.abq_probe_mfma_f4(10, 2, A16, None) == B.ABQ_ERR_SHAPE
    assert lib.abq_probe_mfma_f4_ops(0) == 0.0


def test_rmsnorm_quant_act_rejects():
    lib = B.load()

    def call(q=8, M=1, K=64, x=A16, g=A16, eps=1e-5, c=A16, s=A16, z=A16, y=None):
        return lib.abq_rmsnorm_quant_act(q, M, K, x, g, eps, c, s, z, y, None)

    assert call(x=None) == B.ABQ_ERR_NULL
    assert call(g=None) == B.ABQ_ERR_NULL
    assert call(z=None) == B.ABQ_ERR_NULL
    assert call(q=0) == B.ABQ_ERR_BITS
    assert call(M=0) == B.ABQ_ERR_SHAPE
    assert call(K=B.ABQ_MAX_K + 1) == B.ABQ_ERR_SHAPE
    assert call(eps=-1.0) == B.ABQ_ERR_SHAPE
    assert call(eps=float("nan")) == B.ABQ_ERR_SHAPE
    assert call(y=A16 + 2) == B.ABQ_ERR_ALIGN
    assert call(c=A16 + 1) == B.ABQ_ERR_ALIGN


def test_add_rmsnorm_quant_act_rejects():
    f = B.load().abq_add_rmsnorm_quant_act
    ok = dict(q=8, M=2, K=64, x=A16, r=A16, g=A16, eps=1e-5, c=A16, s=A16, z=A16, h=A16, y=None)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["q"], a["M"], a["K"], a["x"], a["r"], a["g"], a["eps"], a["c"], a["s"], a["z"], a["h"], a["y"], None)

    assert call(r=None) == B.ABQ_ERR_NULL
    assert call(h=None) == B.ABQ_ERR_NULL          # the sum is the next residual: always written
    assert call(q=0) == B.ABQ_ERR_BITS
    assert call(K=0) == B.ABQ_ERR_SHAPE
    assert call(eps=-1.0) == B.ABQ_ERR_SHAPE
    assert call(r=A16 + 2) == B.ABQ_ERR_ALIGN
    assert call(y=A16 + 8) == B.ABQ_ERR_ALIGN


def test_silu_mul_quant_act_rejects():
    lib = B.load()

    def call(q=8, M=1, K=64, g=A16, u=A16, c=A16, s=A16, z=A16, h=None):
        return lib.abq_silu_mul_quant_act(q, M, K, g, u, c, s, z, h, None)

    assert call(g=None) == B.ABQ_ERR_NULL
    assert call(u=None) == B.ABQ_ERR_NULL
    assert call(s=None) == B.ABQ_ERR_NULL
    assert call(q=9) == B.ABQ_ERR_BITS
    assert call(K=0) == B.ABQ_ERR_SHAPE
    assert call(u=A16 + 2) == B.ABQ_ERR_ALIGN
    assert call(h=A16 + 6) == B.ABQ_ERR_ALIGN


def test_unpack_rejects():
    lib = B.load()
    assert lib.abq_unpack_weights(4, 16, 64, B.ABQ_LAYOUT_FIELDS, A16, B.ABQ_LAYOUT_PLANES, A16, None) == B.ABQ_ERR_LAYOUT
    assert lib.abq_unpack_weights(4, 16, 64, B.ABQ_LAYOUT_FIELDS, None, B.ABQ_LAYOUT_FIELDS, A16, None) == B.ABQ_ERR_NULL
    assert lib.abq_unpack_act(8, 1, 64, B.ABQ_LAYOUT_PLANES, A16, B.ABQ_LAYOUT_FIELDS, A16, None, None, None, None) == B.ABQ_ERR_LAYOUT


def test_tuner_candidate_plans_are_valid_plan_table_entries():
    """Every plan the search would try must be one the table accepts (no GPU needed: the table is host state)."""
    from paper_2408_08554_amd import tune
    B.load()
    B.abq_plan_clear()
    for shape in [(4, 8, 1, 4096, 4096), (8, 8, 16, 5120, 13824), (2, 8, 40, 100, 1536), (6, 6, 128, 11008, 4096),
                  (4, 4, 2048, 13824, 5120), (1, 1, 1, 16, 100)]:
        plans = tune.candidates(*shape)
        assert plans[0] == {} and len({tuple(sorted(pl.items())) for pl in plans}) == len(plans)      # the rule first, no duplicates
        for plan in plans:
            assert set(plan) <= set(tune.KNOBS)
            B.abq_plan_set(*shape, **plan) if plan else B.abq_plan_set(*shape)
            assert {k: v for k, v in B.abq_plan_get(*shape).items() if v} == plan
    B.abq_plan_clear()


def test_shipped_plan_table_is_well_formed():
    import json
    from paper_2408_08554_amd import tune
    table = json.load(open(tune.DEFAULT_PLANS))
    B.load()
    B.abq_plan_clear()
    assert tune.load_plans() == len(table)
    for key, plan in table.items():
        shape = tuple(int(v) for v in key.split(","))
        assert len(shape) == 5 and set(plan) <= set(tune.KNOBS)
        assert {k: v for k, v in B.abq_plan_get(*shape).items() if v} == plan
    B.abq_plan_clear()


def test_check_packed_rejects_before_touching_the_device():
    lib = B.load()
    F = B.ABQ_LAYOUT_FIELDS
    big = 1 << 30
    assert lib.abq_check_packed(0, 4, 64, 512, F, None, big, None) == B.ABQ_ERR_NULL
    assert lib.abq_check_packed(0, 0, 64, 512, F, A16, big, None) == B.ABQ_ERR_BITS
    assert lib.abq_check_packed(0, 4, 0, 512, F, A16, big, None) == B.ABQ_ERR_SHAPE
    assert lib.abq_check_packed(0, 4, 64, 512, 9, A16, big, None) == B.ABQ_ERR_LAYOUT
    assert lib.abq_check_packed(2, 4, 64, 512, F, A16, big, None) == B.ABQ_ERR_LAYOUT          # unknown kind
    assert lib.abq_check_packed(1, 4, 64, 512, B.ABQ_LAYOUT_FIELDS_G128, A16, big, None) == B.ABQ_ERR_LAYOUT   # weights-only layout
    assert lib.abq_check_packed(0, 4, 64, 512, F, A16 + 8, big, None) == B.ABQ_ERR_ALIGN
    assert lib.abq_check_packed(0, 4, 64, 512, F, A16, lib.abq_packed_weight_bytes(4, 64, 512, F) - 1, None) == B.ABQ_ERR_SIZE
    assert lib.abq_check_packed(1, 8, 3, 512, F, A16, lib.abq_packed_act_bytes(8, 3, 512, F) - 1, None) == B.ABQ_ERR_SIZE


def test_static_entry_point_rejects_before_touching_the_device():
    lib = B.load()
    F = B.ABQ_LAYOUT_FIELDS

    def call(p=4, q=8, M=300, N=64, K=512, a=A16, s=A16, z=A16, w=A16, wl=F, y=A16, acc=None):
        return lib.abq_gemm_act_codes_static(p, q, M, N, K, a, s, z, w, wl, y, acc, None)

    assert call(a=None) == B.ABQ_ERR_NULL
    assert call(y=None) == B.ABQ_ERR_NULL
    assert call(p=9) == B.ABQ_ERR_BITS
    assert call(K=0) == B.ABQ_ERR_SHAPE
    assert call(wl=9) == B.ABQ_ERR_LAYOUT
    # 4096 rows of K = 13824 need 54 MiB of packed activations: beyond the static buffer
    assert lib.abq_gemm_act_codes_workspace_bytes(8, 8, 4096, 5120, 13824, F) > B.ABQ_STATIC_SCRATCH_BYTES
    assert call(p=8, q=8, M=4096, N=5120, K=13824) == B.ABQ_ERR_SIZE


def test_requant_entry_point_rejects_before_touching_the_device():
    lib = B.load()
    F = B.ABQ_LAYOUT_FIELDS

    def call(p=4, q=8, M=1, N=64, K=512, a=A16, s=A16, z=A16, w=A16, wl=F, qo=8, osc=A16, ozp=A16, codes=A16, y=None, ws=None, wsb=0):
        return lib.abq_gemm_act_codes_requant(p, q, M, N, K, a, s, z, w, wl, qo, osc, ozp, codes, y, ws, wsb, None)

    assert call(codes=None) == B.ABQ_ERR_NULL
    assert call(osc=None) == B.ABQ_ERR_NULL
    assert call(a=None) == B.ABQ_ERR_NULL
    assert call(qo=0) == B.ABQ_ERR_BITS and call(qo=9) == B.ABQ_ERR_BITS and call(q=0) == B.ABQ_ERR_BITS
    assert call(codes=A16 + 1) == B.ABQ_ERR_ALIGN
    assert call(K=0) == B.ABQ_ERR_SHAPE
    assert call(wl=B.ABQ_LAYOUT_FIELDS_G128) == B.ABQ_ERR_LAYOUT            # per-group blobs: not built
    assert call(M=300) == B.ABQ_ERR_NULL                                      # the two-kernel path needs its workspace
    assert call(M=300, ws=A16, wsb=16) == B.ABQ_ERR_SIZE
    assert lib.abq_gemm_act_codes(4, 8, 1, 64, 512, A16, A16, A16, A16, F, None, None, None, 0, None) == B.ABQ_ERR_NULL   # y stays required there


def test_build_refuses_scratch_memory_in_kernels_with_hand_written_loads(tmp_path, monkeypatch):
    """The F4 matmul kernel fills registers with load instructions the compiler does not track; a spill of such a
    register would save it before the data lands.  The build reads the compiler's resource-usage remarks and must fail
    on any scratch memory in that kernel, and when the remarks are missing."""
    from paper_2408_08554_amd import build as bld

    def remarks(scratch):
        return ("abq_f4.hip:1:0: remark: Function Name: _ZN3abq14f4_gemm_kernelILi4EEEvNS_8F4ParamsE [-Rpass-analysis=kernel-resource-usage]\n"
                "abq_f4.hip:1:0: remark:     VGPRs: 228 [-Rpass-analysis=kernel-resource-usage]\n"
                f"abq_f4.hip:1:0: remark:     ScratchSize [bytes/lane]: {scratch} [-Rpass-analysis=kernel-resource-usage]\n"
                "abq_f4.hip:2:0: remark: Function Name: _ZN3abq14f4_pack_kernelEPKh [-Rpass-analysis=kernel-resource-usage]\n"
                "abq_f4.hip:2:0: remark:     ScratchSize [bytes/lane]: 16 [-Rpass-analysis=kernel-resource-usage]\n")

    monkeypatch.setattr(bld, "OBJ", str(tmp_path))
    src = os.path.join(bld.CSRC, "abq_f4.hip")
    obj = tmp_path / "abq_f4.hip.o"
    bld._check_no_scratch(src, remarks(0), "f4_gemm_kernel")      # other kernels may use scratch; this one does not: passes
    obj.write_bytes(b"x")
    with pytest.raises(RuntimeError, match="scratch"):
        bld._check_no_scratch(src, remarks(48), "f4_gemm_kernel")
    assert not obj.exists()                                       # the object of a refused build is removed
    with pytest.raises(RuntimeError, match="did not run"):
        bld._check_no_scratch(src, "", "f4_gemm_kernel")
    assert "abq_f4.hip" in bld.NO_SCRATCH
