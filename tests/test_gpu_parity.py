"""GPU parity: every step of the hot path through the C ABI against the CPU oracle.
int32 accumulator bit-exact, codes/planes bit-exact, fp16 output within the stated tolerance."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2408_08554_amd import synth
from helpers import check_against_oracle, check_g128, check_sampled, gpu_gemm, gpu_gemm_fused, to_dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

PLANES, FIELDS, BOTH = 1, 2, 3


def say(*a):
    print(*a, flush=True)


# ---- packers ------------------------------------------------------------------------------

@pytest.mark.parametrize("p,N,K", [(1, 16, 512), (2, 33, 100), (3, 17, 1000), (4, 64, 4096), (5, 7, 96),
                                   (6, 100, 640), (7, 31, 513), (8, 48, 32), (8, 5, 2049)])
def test_weight_pack_roundtrip(abq, p, N, K):
    say("weights roundtrip", p, N, K)
    c = synth.make_case(p, 8, 1, N, K, seed=1000 + p)
    pw = abq.abq_pack_weights(p, to_dev(torch, c.W), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero), BOTH)
    for which in (PLANES, FIELDS):
        back = abq.abq_unpack_weights(p, N, K, BOTH, pw, which).cpu().numpy()
        assert np.array_equal(back, c.W), which
    # the plane section is the paper's [p][N][K] BitPacking: compare with the oracle's packer word for word
    lib_bytes = pw.cpu().numpy()
    Kw = (K + 127) // 128 * 4
    off = 256 + (N * 16 + 255) // 256 * 256
    planes = lib_bytes[off:off + p * N * Kw * 4].view(np.uint32).reshape(p, N, Kw)
    assert np.array_equal(planes, oracle.pack_planes(c.W, p, Kw=Kw))


@pytest.mark.parametrize("q,M,K", [(1, 1, 512), (2, 3, 100), (4, 16, 4096), (6, 5, 1000), (8, 2, 96), (8, 9, 11008), (7, 1, 31)])
def test_act_pack_roundtrip(abq, q, M, K):
    say("acts roundtrip", q, M, K)
    c = synth.make_case(2, q, M, 16, K, seed=2000 + q)
    pa = abq.abq_pack_act_codes(q, to_dev(torch, c.A), to_dev(torch, c.a_scale), to_dev(torch, c.a_zero), BOTH)
    for which in (PLANES, FIELDS):
        codes, sc, zp, sm = abq.abq_unpack_act(q, M, K, BOTH, pa, which)
        assert np.array_equal(codes.cpu().numpy(), c.A)
        assert np.array_equal(sc.cpu().numpy(), c.a_scale) and np.array_equal(zp.cpu().numpy(), c.a_zero)
        assert np.array_equal(sm.cpu().numpy().astype(np.int64), c.A.astype(np.int64).sum(axis=1))


@pytest.mark.parametrize("q", [1, 2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("M,K", [(1, 4096), (5, 1000), (3, 96)])
def test_quant_pack_act_matches_oracle(abq, q, M, K):
    say("quantizer", q, M, K)
    x = synth.act_fp16(3000 + 10 * q + M, M, K)
    if M >= 3:
        x[1] = 0
        x[2] = np.abs(x[2])
    ref_codes, ref_scale, ref_zero = oracle.quant_act(x, q)
    pa = abq.abq_quant_pack_act(q, to_dev(torch, x), BOTH)
    for which in (PLANES, FIELDS):
        codes, sc, zp, sm = abq.abq_unpack_act(q, M, K, BOTH, pa, which)
        assert np.array_equal(sc.cpu().numpy(), ref_scale)
        assert np.array_equal(zp.cpu().numpy(), ref_zero)
        assert np.array_equal(codes.cpu().numpy(), ref_codes)
        assert np.array_equal(sm.cpu().numpy().astype(np.int64), ref_codes.astype(np.int64).sum(axis=1))


# ---- matmul: every (p,q), both kernel families -------------------------------------------------

@pytest.mark.parametrize("layout", [FIELDS, PLANES], ids=["mfma", "bitserial"])
@pytest.mark.parametrize("p,q", list(itertools.product(range(1, 9), range(1, 9))))
def test_all_pq_small(abq, layout, p, q):
    say("all pq", layout, p, q)
    c = synth.make_case(p, q, 3, 40, 1100, seed=synth.case_seed(9, p, q), name=f"W{p}A{q} 3x40x1100")
    y, acc = gpu_gemm(torch, abq, c, layout, layout)
    check_against_oracle(c, y, acc)


SHAPES = [(1, 256, 512), (1, 17, 100), (2, 16, 32), (8, 100, 96), (16, 64, 2048), (5, 33, 1), (7, 1, 513),
          (1, 48, 5120), (4, 31, 13824), (17, 20, 700), (33, 50, 1536), (64, 16, 640), (16, 70, 13824), (15, 33, 9000)]


@pytest.mark.parametrize("layout", [FIELDS, PLANES], ids=["mfma", "bitserial"])
@pytest.mark.parametrize("M,N,K", SHAPES)
@pytest.mark.parametrize("p,q", [(2, 8), (4, 8), (6, 6), (8, 8), (3, 5), (7, 7), (1, 1), (5, 2)])
def test_shapes(abq, layout, M, N, K, p, q):
    say("shape", layout, M, N, K, p, q)
    c = synth.make_case(p, q, M, N, K, seed=synth.case_seed(8, p, q) + M + N + K, name=f"W{p}A{q} {M}x{N}x{K}")
    y, acc = gpu_gemm(torch, abq, c, layout, layout)
    check_against_oracle(c, y, acc)


TILED_SHAPES = [(65, 40, 700), (128, 128, 512), (200, 150, 1100), (129, 257, 64), (300, 16, 2048), (257, 130, 1536),
                (128, 4096, 4096), (96, 300, 5632), (512, 11008, 1024), (70, 129, 3584)]


@pytest.mark.parametrize("M,N,K", TILED_SHAPES)
@pytest.mark.parametrize("p,q", [(1, 1), (2, 8), (3, 3), (4, 8), (5, 5), (6, 6), (7, 7), (8, 8), (8, 2)])
def test_prefill_shapes(abq, M, N, K, p, q):
    say("prefill shape", M, N, K, p, q)
    c = synth.make_case(p, q, M, N, K, seed=synth.case_seed(7, p, q) + M + N + K, name=f"W{p}A{q} {M}x{N}x{K}")
    y, acc = gpu_gemm(torch, abq, c, FIELDS, FIELDS)
    if M * N * K <= 1 << 28:
        check_against_oracle(c, y, acc)
    else:
        check_sampled(c, y, acc)


@pytest.mark.parametrize("p,q,M,N,K", [(4, 4, 2050, 6000, 200),     # 64x256 workgroup tiles by the rule, ragged on every side
                                       (2, 8, 1030, 5500, 300),     # 64x128 tiles by the rule
                                       (3, 8, 1024, 13824, 128),    # K of half a super-chunk
                                       (8, 8, 520, 5100, 8200)])    # p = 8, long K: deep rings past one workgroup per CU
def test_prefill_large_ragged_rule_paths(abq, p, q, M, N, K):
    say("prefill rule path", p, q, M, N, K)
    c = synth.make_case(p, q, M, N, K, seed=synth.case_seed(7, p, q) + M + N + K, name=f"W{p}A{q} {M}x{N}x{K}")
    y, acc = gpu_gemm(torch, abq, c, FIELDS, FIELDS)
    check_sampled(c, y, acc, count=8192)
    # the last row and column blocks in full (partial tiles at both edges)
    ms = np.arange(M - 70, M)
    ns = np.arange(N - 300, N)
    sub = synth.Case(p, q, len(ms), len(ns), K, c.W[ns], c.A[ms], c.w_scale[ns], c.w_zero[ns], c.a_scale[ms], c.a_zero[ms], c.seed, c.name)
    check_against_oracle(sub, y[np.ix_(ms, ns)], acc[np.ix_(ms, ns)])


def test_prefill_bitserial(abq):
    c = synth.make_case(3, 5, 70, 50, 600, seed=123)
    y, acc = gpu_gemm(torch, abq, c, PLANES, PLANES)
    check_against_oracle(c, y, acc)


def test_both_layout_and_forced_family(abq):
    c = synth.make_case(4, 8, 2, 48, 1024, seed=77)
    for flag in (0, 0x10, 0x20):
        y, acc = gpu_gemm(torch, abq, c, BOTH, BOTH, gemm_w_layout=BOTH | flag)
        check_against_oracle(c, y, acc)


def test_auto_dispatch_on_both_blobs_narrow_single_token(abq):
    # M = 1, p <= 2, q <= 4, many output tiles: the dispatcher takes the bit-serial kernel when both
    # representations are present; the result must not depend on that choice
    c = synth.make_case(2, 4, 1, 8200, 640, seed=31)
    y0, acc0 = gpu_gemm(torch, abq, c, BOTH, BOTH)
    check_against_oracle(c, y0, acc0)
    y1, acc1 = gpu_gemm(torch, abq, c, BOTH, BOTH, gemm_w_layout=BOTH | 0x20)
    assert np.array_equal(acc0, acc1) and np.array_equal(y0.view(np.uint16), y1.view(np.uint16))


@pytest.mark.parametrize("layout", [FIELDS, PLANES], ids=["mfma", "bitserial"])
def test_degenerate_shapes(abq, layout):
    for p, q, M, N, K in [(1, 1, 1, 1, 1), (8, 8, 1, 1, 1), (3, 7, 2, 1, 5), (5, 2, 1, 3, 17), (4, 4, 17, 1, 64)]:
        c = synth.make_case(p, q, M, N, K, seed=900 + p + q + M + N + K)
        y, acc = gpu_gemm(torch, abq, c, layout, layout)
        check_against_oracle(c, y, acc)


def test_longest_k(abq):
    # K at the ABI limit (131072); W1A1 keeps the accumulator far inside int32
    K = 131072
    c = synth.make_case(1, 1, 2, 20, K, seed=4)
    for layout in (FIELDS, PLANES):
        y, acc = gpu_gemm(torch, abq, c, layout, layout)
        check_against_oracle(c, y, acc)
    c = synth.make_case(2, 6, 1, 16, K, seed=5)       # 131072*3*63 < 2^31
    y, acc = gpu_gemm(torch, abq, c, FIELDS, FIELDS)
    check_against_oracle(c, y, acc)


def test_prefill_long_k_sums_of_codes_beyond_24_bits(abq):
    """M > 16 with K * (2^q - 1) or K * (2^p - 1) at or above 2^23: the prefill kernel's epilogue must leave its 24-bit
    multiply-adds for 32-bit multiplies (the host decides), with and without the accumulator output."""
    for p, q, M, N, K in [(2, 8, 40, 70, 40000), (8, 2, 33, 130, 36000), (1, 8, 70, 24, 131072)]:
        assert K * ((1 << max(p, q)) - 1) >= 1 << 23
        c = synth.make_case(p, q, M, N, K, seed=31 + p + q)
        say(c.name)
        y, acc = gpu_gemm(torch, abq, c, FIELDS, FIELDS)
        check_against_oracle(c, y, acc)
        pw = abq.abq_pack_weights(p, to_dev(torch, c.W), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero), FIELDS)
        pa = abq.abq_pack_act_codes(q, to_dev(torch, c.A), to_dev(torch, c.a_scale), to_dev(torch, c.a_zero), FIELDS)
        y_only, _ = abq.abq_gemm(p, q, M, N, K, pa, FIELDS, pw, FIELDS)
        torch.cuda.synchronize()
        assert np.array_equal(y_only.cpu().numpy().view(np.uint16), np.asarray(y).view(np.uint16))


# Long K with up to 16 rows of A: the streaming kernel stages A one K group at a time and keeps per-tile
# partial sums between the groups (several tiles per workgroup at the larger N).
KGROUP_SHAPES = [(16, 70, 13824), (16, 4096, 11008), (12, 40, 20000), (9, 48, 16384), (16, 8200, 11008),
                 (16, 5120, 13824), (8, 64, 28672), (16, 32, 28672), (13, 100, 33024), (16, 24, 131072)]


@pytest.mark.parametrize("fused", [False, True], ids=["packed", "fused"])
@pytest.mark.parametrize("M,N,K", KGROUP_SHAPES)
def test_long_k_groups(abq, M, N, K, fused):
    for p, q in [(4, 8), (8, 8), (1, 3), (7, 2), (3, 8)]:
        if K * ((1 << p) - 1) * ((1 << q) - 1) > 2 ** 31 - 1:
            p, q = min(p, 2), min(q, 4)
        say("long K", M, N, K, p, q, "fused" if fused else "packed")
        c = synth.make_case(p, q, M, N, K, seed=synth.case_seed(4, p, q) + M + N + K, name=f"longK W{p}A{q} {M}x{N}x{K}")
        y, acc = gpu_gemm_fused(torch, abq, c, FIELDS) if fused else gpu_gemm(torch, abq, c, FIELDS, FIELDS)
        if M * N * K <= 1 << 27:
            check_against_oracle(c, y, acc)
        else:
            check_sampled(c, y, acc)


def test_zero_and_constant_operands(abq):
    c = synth.make_case(4, 8, 3, 40, 1000, seed=6)
    c.A[:] = 0
    y, acc = gpu_gemm(torch, abq, c, FIELDS, FIELDS)
    assert (acc == 0).all()
    check_against_oracle(c, y, acc)
    c = synth.make_case(4, 8, 3, 40, 1000, seed=7)
    c.A[1] = 255
    c.W[:] = 15
    y, acc = gpu_gemm(torch, abq, c, FIELDS, FIELDS)
    assert (acc[1] == 1000 * 255 * 15).all()
    check_against_oracle(c, y, acc)


def test_extreme_codes_and_no_acc_output(abq):
    # all-max codes hit the largest accumulator value the ABI admits for this K; acc pointer NULL
    for p, q, K in [(8, 8, 33025), (1, 8, 4096), (8, 1, 700), (4, 4, 8192)]:
        M, N = 2, 20
        c = synth.make_case(p, q, M, N, K, seed=5)
        c.A[:] = (1 << q) - 1
        c.W[:] = (1 << p) - 1
        c.a_zero[:] = 0
        c.w_zero[:] = 0
        c.a_scale[:] = np.float32(2.0 ** -20)
        c.w_scale[:] = np.float32(2.0 ** -8)
        for layout in (FIELDS, PLANES):
            y, acc = gpu_gemm(torch, abq, c, layout, layout)
            assert (acc == K * ((1 << p) - 1) * ((1 << q) - 1)).all()
            check_against_oracle(c, y, acc)
            y2, none = gpu_gemm(torch, abq, c, layout, layout, want_acc=False)
            assert none is None and np.array_equal(y2.view(np.uint16), y.view(np.uint16))


def test_output_overwrites_poison_and_is_deterministic(abq):
    c = synth.make_case(2, 8, 3, 70, 1500, seed=11)
    pw = abq.abq_pack_weights(c.p, to_dev(torch, c.W), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero), FIELDS)
    pa = abq.abq_pack_act_codes(c.q, to_dev(torch, c.A), to_dev(torch, c.a_scale), to_dev(torch, c.a_zero), FIELDS)
    outs = []
    for fill in (0xFF, 0x00):
        y = torch.full((c.M, c.N), 0, dtype=torch.float16, device="cuda").view(torch.uint8).fill_(fill).view(torch.float16)
        acc = torch.full((c.M, c.N), -1 if fill else 0, dtype=torch.int32, device="cuda")
        abq.abq_gemm(c.p, c.q, c.M, c.N, c.K, pa, FIELDS, pw, FIELDS, y=y, acc=acc)
        torch.cuda.synchronize()
        outs.append((y.cpu().numpy().view(np.uint16), acc.cpu().numpy()))
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])
    check_against_oracle(c, outs[0][0].view(np.float16), outs[0][1])


# ---- the benchmark configurations at full size -------------------------------------------------

# ---- activation packing fused into the matmul ------------------------------------------------------

@pytest.mark.parametrize("p,q", list(itertools.product(range(1, 9), range(1, 9))))
def test_fused_act_all_pq(abq, p, q):
    say("fused pq", p, q)
    c = synth.make_case(p, q, 3, 40, 1104, seed=synth.case_seed(7, p, q), name=f"fused W{p}A{q} 3x40x1104")
    assert abq.abq_gemm_act_codes_workspace_bytes(p, q, c.M, c.N, c.K, FIELDS) == 0
    y, acc = gpu_gemm_fused(torch, abq, c, FIELDS)
    check_against_oracle(c, y, acc)


FUSED_SHAPES = [(1, 256, 512), (1, 17, 112), (2, 16, 32), (8, 100, 96), (16, 64, 2048), (5, 33, 16), (7, 1, 528),
                (1, 48, 5120), (4, 31, 13824), (13, 4096, 4096), (16, 300, 8192), (16, 70, 13824), (33, 50, 1536),
                (64, 16, 640), (1, 13824, 5120)]


@pytest.mark.parametrize("M,N,K", FUSED_SHAPES)
@pytest.mark.parametrize("p,q", [(2, 8), (4, 8), (6, 6), (8, 8), (3, 5), (7, 7), (1, 1), (5, 2)])
def test_fused_act_shapes(abq, M, N, K, p, q):
    say("fused shape", M, N, K, p, q)
    c = synth.make_case(p, q, M, N, K, seed=synth.case_seed(6, p, q) + M + N + K, name=f"fused W{p}A{q} {M}x{N}x{K}")
    assert abq.abq_gemm_act_codes_workspace_bytes(p, q, M, N, K, FIELDS) == 0
    y, acc = gpu_gemm_fused(torch, abq, c, FIELDS)
    if M * N * K <= 1 << 28:
        check_against_oracle(c, y, acc)
    else:
        check_sampled(c, y, acc)


@pytest.mark.parametrize("M,N,K,layout,flag", [(1, 64, 1000, FIELDS, 0),        # K not a multiple of 16
                                               (128, 130, 512, FIELDS, 0),      # prefill shape: tiled kernel
                                               (3, 40, 640, PLANES, 0),         # bit-serial family
                                               (2, 48, 512, BOTH, 0x10),        # planes forced on a blob with both
                                               (2, 48, 512, BOTH, 0x20),        # fields forced: one kernel again
                                               (1, 8192, 512, BOTH, 0)])        # both representations, nothing forced: the MFMA path, one kernel (p=2, q=4)
def test_fused_act_two_step_paths(abq, M, N, K, layout, flag):
    say("fused fallback", M, N, K, layout, flag)
    p, q = (2, 4) if N == 8192 else (4, 8)
    c = synth.make_case(p, q, M, N, K, seed=synth.case_seed(5, p, q) + M + N + K, name=f"fused2 W{p}A{q} {M}x{N}x{K}")
    need = abq.abq_gemm_act_codes_workspace_bytes(p, q, M, N, K, layout | flag)
    assert (need == 0) == (flag == 0x20 or (layout == BOTH and flag == 0 and M <= 16))
    y, acc = gpu_gemm_fused(torch, abq, c, layout, gemm_w_layout=layout | flag)
    check_against_oracle(c, y, acc)


def test_fused_act_equals_two_calls_bitwise(abq):
    """The fused call and pack + gemm give the same bits (config-3 activations: rounded Gaussian codes)."""
    for M in (1, 8):
        c = synth.config3(M)
        say("fused vs two calls", c.name)
        y1, acc1 = gpu_gemm(torch, abq, c, FIELDS, FIELDS)
        y2, acc2 = gpu_gemm_fused(torch, abq, c, FIELDS)
        assert np.array_equal(acc1, acc2)
        assert np.array_equal(y1.view(np.uint16), y2.view(np.uint16))
        check_against_oracle(c, y2, acc2)


def test_fused_act_extreme_codes(abq):
    """All-maximum codes: the largest row sums and the q = 8 offset at its limit."""
    for p, q, K in [(8, 8, 33024), (4, 8, 4096), (8, 4, 2048)]:
        c = synth.make_case(p, q, 5, 48, K, seed=3, name=f"fused max W{p}A{q} K={K}")
        c.A[:] = (1 << q) - 1
        c.W[:] = (1 << p) - 1
        c.A[1] = 0
        say(c.name)
        y, acc = gpu_gemm_fused(torch, abq, c, FIELDS)
        check_against_oracle(c, y, acc)


# ---- grouped decode launch -------------------------------------------------------------------------

def run_group(abq, p, q, M, shapes, fused, seed0, w_layout=FIELDS, a_layout=FIELDS, gemm_w_layout=None):
    """shapes: list of (N, K).  Returns [(case, y, acc)] after one abq_gemm_grouped call."""
    cases, problems, keep = [], [], []
    for i, (N, K) in enumerate(shapes):
        c = synth.make_case(p, q, M, N, K, seed=seed0 + 17 * i, name=f"group[{i}] W{p}A{q} {M}x{N}x{K}")
        pw = abq.abq_pack_weights(p, to_dev(torch, c.W), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero), w_layout)
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        acc = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
        pr = dict(N=N, K=K, packed_w=pw, y=y, acc=acc)
        if fused:
            pr.update(a_codes=to_dev(torch, c.A), a_scale=to_dev(torch, c.a_scale), a_zero=to_dev(torch, c.a_zero))
        else:
            pr.update(packed_act=abq.abq_pack_act_codes(q, to_dev(torch, c.A), to_dev(torch, c.a_scale), to_dev(torch, c.a_zero), a_layout))
        cases.append(c)
        problems.append(pr)
    abq.abq_gemm_grouped(p, q, M, problems, a_layout, w_layout if gemm_w_layout is None else gemm_w_layout)
    torch.cuda.synchronize()
    return [(c, pr["y"].cpu().numpy(), pr["acc"].cpu().numpy()) for c, pr in zip(cases, problems)]


GROUP_SHAPES = [(4096, 4096), (33, 2048), (1000, 11008), (16, 2560), (4097, 4096), (250, 5120), (64, 13824), (7, 2064),
                (300, 4096), (48, 8192), (129, 2048)]


@pytest.mark.parametrize("fused", [False, True], ids=["packed", "fused"])
@pytest.mark.parametrize("p,q,M", [(4, 8, 1), (2, 8, 5), (8, 8, 2), (1, 1, 16), (7, 3, 3), (3, 4, 8), (6, 6, 1), (5, 8, 12)])
def test_grouped_launch(abq, p, q, M, fused):
    say("grouped", p, q, M, fused)
    shapes = GROUP_SHAPES[: 11 if M <= 5 else 6]        # 11 problems: two launches (8 + 3)
    for c, y, acc in run_group(abq, p, q, M, shapes, fused, synth.case_seed(3, p, q) + M):
        if M * c.N * c.K <= 1 << 27:
            check_against_oracle(c, y, acc)
        else:
            check_sampled(c, y, acc)


def test_grouped_launch_equals_single_calls_bitwise(abq):
    p, q, M = 4, 8, 3
    shapes = [(4096, 4096), (200, 11008), (31, 2048)]
    for fused in (False, True):
        for c, y, acc in run_group(abq, p, q, M, shapes, fused, 77):
            y1, acc1 = gpu_gemm_fused(torch, abq, c, FIELDS) if fused else gpu_gemm(torch, abq, c, FIELDS, FIELDS)
            assert np.array_equal(acc, acc1)
            assert np.array_equal(y.view(np.uint16), y1.view(np.uint16))


@pytest.mark.parametrize("fused", [False, True], ids=["packed", "fused"])
@pytest.mark.parametrize("kind", ["short_k", "many_rows", "planes", "ragged_k", "long_k16"])
def test_grouped_falls_back_to_single_calls(abq, kind, fused):
    """Groups that one launch cannot serve run problem by problem with the same results."""
    say("grouped fallback", kind, fused)
    p, q, M, shapes, wl, al = 4, 8, 2, [(64, 4096), (40, 512)], FIELDS, FIELDS
    if kind == "many_rows":
        M, shapes = 40, [(64, 2048), (130, 2560)]
    elif kind == "planes":
        wl = al = PLANES
    elif kind == "ragged_k":
        shapes = [(64, 4096), (40, 4100)]
    elif kind == "long_k16":
        M, shapes = 16, [(64, 4096), (48, 13824)]
    for c, y, acc in run_group(abq, p, q, M, shapes, fused, 91, w_layout=wl, a_layout=al):
        check_against_oracle(c, y, acc)


# ---- RMSNorm with the quantizer fused in -----------------------------------------------------------

def _norm_inputs(M, K, seed, kind="normal"):
    rng = np.random.Generator(np.random.PCG64(seed))
    x = (rng.standard_normal((M, K)) * rng.uniform(0.05, 8.0, (M, 1))).astype(np.float16)
    x[:, rng.integers(0, K, 4)] *= np.float16(20.0)
    if kind == "extremes":      # huge and tiny magnitudes, subnormals, zeros, an all-zero row, a constant row
        x[0, : K // 2] = np.float16(6e-5)
        x[0, 0] = np.float16(60000.0)
        x[0, 1] = np.float16(5.96e-8)
        if M > 1:
            x[1] = 0
        if M > 2:
            x[2] = np.float16(-3.0)
    g = (1.0 + 0.2 * rng.standard_normal(K)).astype(np.float16)
    return x, g


@pytest.mark.parametrize("q", [1, 4, 6, 8])
@pytest.mark.parametrize("M,K,eps,kind", [(1, 4096, 1e-5, "normal"), (5, 1000, 1e-6, "normal"), (3, 37, 0.0, "normal"),
                                          (2, 11008, 1e-5, "normal"), (16, 5120, 1e-5, "normal"), (4, 4096, 1e-5, "extremes"),
                                          (3, 1, 1e-5, "normal"), (2, 131072, 1e-6, "normal")])
def test_rmsnorm_quant_act_matches_oracle(abq, q, M, K, eps, kind):
    say("rmsnorm quant", q, M, K, eps, kind)
    x, g = _norm_inputs(M, K, 4000 + 13 * q + K + M, kind)
    y_ref = oracle.rmsnorm_half(x, g, eps)
    codes_ref, scale_ref, zero_ref = oracle.quant_act(y_ref, q)
    codes, scale, zero, y = abq.abq_rmsnorm_quant_act(q, to_dev(torch, x), to_dev(torch, g), eps, want_y=True)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy().view(np.uint16), y_ref.view(np.uint16))
    assert np.array_equal(scale.cpu().numpy(), scale_ref)
    assert np.array_equal(zero.cpu().numpy(), zero_ref)
    assert np.array_equal(codes.cpu().numpy(), codes_ref)
    # without the optional output the codes are the same
    codes2, _, _, none = abq.abq_rmsnorm_quant_act(q, to_dev(torch, x), to_dev(torch, g), eps)
    assert none is None and np.array_equal(codes2.cpu().numpy(), codes_ref)


@pytest.mark.parametrize("q", [4, 8])
@pytest.mark.parametrize("M,K", [(1, 4096), (5, 1000), (3, 37), (16, 11008), (2, 16392), (4, 8)])
def test_add_rmsnorm_quant_act_matches_oracle(abq, q, M, K):
    say(f"add+rmsnorm q={q} M={M} K={K}")
    x, gamma = _norm_inputs(M, K, 3100 + K)
    res, _ = _norm_inputs(M, K, 3200 + K)
    res[0, : min(K, 8)] = -x[0, : min(K, 8)]                    # exact cancellation inside a row
    h_ref = oracle.add_half(x, res)
    y_ref = oracle.rmsnorm_half(h_ref, gamma, 1e-5)
    c_ref, s_ref, z_ref = oracle.quant_act(y_ref, q)
    codes, sc, zp, h, y = abq.abq_add_rmsnorm_quant_act(q, to_dev(torch, x), to_dev(torch, res), to_dev(torch, gamma), 1e-5, want_y=True)
    torch.cuda.synchronize()
    assert np.array_equal(h.cpu().numpy().view(np.uint16), h_ref.view(np.uint16))
    assert np.array_equal(y.cpu().numpy().view(np.uint16), y_ref.view(np.uint16))
    assert np.array_equal(codes.cpu().numpy(), c_ref) and np.array_equal(zp.cpu().numpy(), z_ref)
    assert np.array_equal(sc.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    # the sum written over the residual buffer itself
    r_dev = to_dev(torch, res)
    codes2, _, _, h2, _ = abq.abq_add_rmsnorm_quant_act(q, to_dev(torch, x), r_dev, to_dev(torch, gamma), 1e-5, sum_out=r_dev)
    torch.cuda.synchronize()
    assert h2.data_ptr() == r_dev.data_ptr() and np.array_equal(r_dev.cpu().numpy().view(np.uint16), h_ref.view(np.uint16))
    assert np.array_equal(codes2.cpu().numpy(), c_ref)


def test_rmsnorm_quant_then_fused_gemm_end_to_end(abq):
    """fp16 hidden state -> RMSNorm + quantizer (one kernel) -> fused decode matmul (one kernel), against the
    oracle chain rmsnorm -> quantizer -> centered product sum -> dequant."""
    p, q, M, N, K = 4, 8, 3, 200, 4096
    x, g = _norm_inputs(M, K, 99)
    c = synth.make_case(p, q, M, N, K, seed=98)
    codes_ref, scale_ref, zero_ref = oracle.quant_act(oracle.rmsnorm_half(x, g, 1e-5), q)
    pw = abq.abq_pack_weights(p, to_dev(torch, c.W), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero), FIELDS)
    codes, scale, zero, _ = abq.abq_rmsnorm_quant_act(q, to_dev(torch, x), to_dev(torch, g), 1e-5)
    y, acc = abq.abq_gemm_act_codes(p, q, M, N, K, codes, scale, zero, pw, FIELDS, want_acc=True)
    torch.cuda.synchronize()
    c.A, c.a_scale, c.a_zero = codes_ref, scale_ref, zero_ref
    check_against_oracle(c, y.cpu().numpy(), acc.cpu().numpy())


@pytest.mark.parametrize("q", [2, 4, 8])
@pytest.mark.parametrize("M,K", [(1, 11008), (5, 1000), (3, 37), (16, 4096), (2, 13824), (4, 16392), (2, 131072), (3, 8)])
def test_silu_mul_quant_act_matches_oracle(abq, q, M, K):
    say("silu quant", q, M, K)
    rng = np.random.Generator(np.random.PCG64(7000 + 11 * q + K + M))
    g = (rng.standard_normal((M, K)) * rng.uniform(0.1, 12.0, (M, 1))).astype(np.float16)
    u = (rng.standard_normal((M, K)) * 3.0).astype(np.float16)
    g[0, :8] = np.array([0.0, -0.0, 100.0, -100.0, 60000.0, -60000.0, 1e-4, -1e-4], dtype=np.float16)[: min(8, K)]
    u[0, :8] = np.float16(1.0)                         # (keeps the products of the extreme gates finite)
    if M > 1:
        u[1] = 0                                      # a row of zeros: Delta = 1, z = 0
    h_ref = oracle.silu_mul_half(g, u)
    codes_ref, scale_ref, zero_ref = oracle.quant_act(h_ref, q)
    codes, scale, zero, h = abq.abq_silu_mul_quant_act(q, to_dev(torch, g), to_dev(torch, u), want_h=True)
    torch.cuda.synchronize()
    assert np.array_equal(h.cpu().numpy().view(np.uint16), h_ref.view(np.uint16))
    assert np.array_equal(scale.cpu().numpy(), scale_ref)
    assert np.array_equal(zero.cpu().numpy(), zero_ref)
    assert np.array_equal(codes.cpu().numpy(), codes_ref)
    codes2, _, _, none = abq.abq_silu_mul_quant_act(q, to_dev(torch, g), to_dev(torch, u))
    assert none is None and np.array_equal(codes2.cpu().numpy(), codes_ref)


def test_silu_mul_quant_then_down_proj_end_to_end(abq):
    """gate, up fp16 -> SiLU * up + quantizer (one kernel) -> fused decode matmul on a down_proj shape."""
    p, q, M, N, K = 2, 8, 2, 300, 11008
    rng = np.random.Generator(np.random.PCG64(55))
    g = (rng.standard_normal((M, K)) * 2.0).astype(np.float16)
    u = (rng.standard_normal((M, K)) * 1.5).astype(np.float16)
    c = synth.make_case(p, q, M, N, K, seed=56)
    c.A, c.a_scale, c.a_zero = oracle.quant_act(oracle.silu_mul_half(g, u), q)
    pw = abq.abq_pack_weights(p, to_dev(torch, c.W), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero), FIELDS)
    codes, scale, zero, _ = abq.abq_silu_mul_quant_act(q, to_dev(torch, g), to_dev(torch, u))
    y, acc = abq.abq_gemm_act_codes(p, q, M, N, K, codes, scale, zero, pw, FIELDS, want_acc=True)
    torch.cuda.synchronize()
    check_against_oracle(c, y.cpu().numpy(), acc.cpu().numpy())


def test_graph_replays_match_eager(abq):
    """The decode entry points captured in one HIP graph (no allocation, no memset inside) and replayed several
    times with new inputs, eager work and synchronizations in between: every replay equals the eager result."""
    p, q, M, K = 4, 8, 2, 4096
    shapes = [(4096, 4096), (300, 4096)]
    rng = np.random.Generator(np.random.PCG64(321))
    cases = [synth.make_case(p, q, M, N, K2, seed=500 + i) for i, (N, K2) in enumerate(shapes)]
    pws = [abq.abq_pack_weights(p, to_dev(torch, c.W), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero), FIELDS) for c in cases]
    g = to_dev(torch, (1.0 + 0.1 * rng.standard_normal(K)).astype(np.float16))
    x = torch.zeros((M, K), dtype=torch.float16, device="cuda")
    codes = torch.empty((M, K), dtype=torch.uint8, device="cuda")
    scale = torch.empty(M, dtype=torch.float32, device="cuda")
    zero = torch.empty(M, dtype=torch.int32, device="cuda")
    y1 = torch.empty((M, shapes[0][0]), dtype=torch.float16, device="cuda")
    ys = [torch.empty((M, N), dtype=torch.float16, device="cuda") for N, _ in shapes]
    lib = abq.load()
    problems = abq.make_problems([dict(N=c.N, K=c.K, packed_w=pw, a_codes=codes, a_scale=scale, a_zero=zero, y=y)
                                  for c, pw, y in zip(cases, pws, ys)])

    def run():
        st = torch.cuda.current_stream().cuda_stream
        assert lib.abq_rmsnorm_quant_act(q, M, K, x.data_ptr(), g.data_ptr(), 1e-5, codes.data_ptr(), scale.data_ptr(),
                                         zero.data_ptr(), None, st) == 0
        abq.abq_gemm_act_codes(p, q, M, shapes[0][0], K, codes, scale, zero, pws[0], FIELDS, y=y1)
        abq.abq_gemm_grouped(p, q, M, problems, FIELDS, FIELDS)

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        run()
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            run()
        for rep in range(4):
            xin = (rng.standard_normal((M, K)) * (rep + 1)).astype(np.float16)
            x.copy_(torch.from_numpy(xin).cuda())
            for t in (y1, *ys):
                t.fill_(float("nan"))
            graph.replay()
            stream.synchronize()
            got = [y1.clone()] + [t.clone() for t in ys]
            for t in (y1, *ys):
                t.fill_(float("nan"))
            run()                               # eager, same inputs
            stream.synchronize()
            for a, b in zip(got, [y1, *ys]):
                assert torch.equal(a.view(torch.int16), b.view(torch.int16)), f"replay {rep} differs from the eager run"
            # and the eager run is right: first problem against the oracle chain
            cr, sr, zr = oracle.quant_act(oracle.rmsnorm_half(xin, g.cpu().numpy(), 1e-5), q)
            c0 = cases[0]
            c0.A, c0.a_scale, c0.a_zero = cr, sr, zr
            check_against_oracle(c0, y1.cpu().numpy(), None)


def test_graph_replays_match_eager_on_the_shared_operand_kernel(abq):
    """Sixteen rows over more tiles than compute units (the shared-operand decode kernel, by rule), captured and replayed
    with new activations: every replay equals the eager result and the oracle."""
    p, q, M, N, K = 2, 8, 16, 4400, 2048
    c = synth.make_case(p, q, M, N, K, seed=611)
    pw = abq.abq_pack_weights(p, to_dev(torch, c.W), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero), FIELDS)
    codes = torch.zeros((M, K), dtype=torch.uint8, device="cuda")
    scale, zero = to_dev(torch, c.a_scale), to_dev(torch, c.a_zero)
    y = torch.empty((M, N), dtype=torch.float16, device="cuda")
    rng = np.random.Generator(np.random.PCG64(612))

    def run():
        abq.abq_gemm_act_codes(p, q, M, N, K, codes, scale, zero, pw, FIELDS, y=y)

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        run()
        stream.synchronize()
        assert abq.abq_last_decode_kernel() == abq.ABQ_DECODE_SHARED_OPERAND
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            run()
        for rep in range(3):
            a = rng.integers(0, 1 << q, size=(M, K), dtype=np.uint8)
            codes.copy_(torch.from_numpy(a).cuda())
            y.fill_(float("nan"))
            graph.replay()
            stream.synchronize()
            got = y.clone()
            y.fill_(float("nan"))
            run()
            stream.synchronize()
            assert torch.equal(got.view(torch.int16), y.view(torch.int16)), f"replay {rep} differs from the eager run"
            c.A = a
            check_against_oracle(c, y.cpu().numpy(), None)


def test_check_packed_reads_the_blob_header(abq):
    """abq_check_packed accepts a blob with the geometry it was packed with and names every mismatch."""
    F, P, G128 = FIELDS, PLANES, abq.ABQ_LAYOUT_FIELDS_G128
    c = synth.make_case(3, 5, 4, 40, 700, seed=77)
    pw = abq.abq_pack_weights(3, to_dev(torch, c.W), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero), F)
    pa = abq.abq_pack_act_codes(5, to_dev(torch, c.A), to_dev(torch, c.a_scale), to_dev(torch, c.a_zero), P)
    assert abq.abq_check_packed(0, 3, 40, 700, F, pw) == abq.ABQ_OK
    assert abq.abq_check_packed(1, 5, 4, 700, P, pa) == abq.ABQ_OK
    big = torch.zeros(1 << 22, dtype=torch.uint8, device="cuda")
    big[:pw.numel()] = pw
    for args in [(0, 4, 40, 700, F), (0, 3, 41, 700, F), (0, 3, 40, 701, F), (0, 3, 40, 700, abq.ABQ_LAYOUT_BOTH), (1, 3, 40, 700, F)]:
        assert abq.abq_check_packed(*args, big) == abq.ABQ_ERR_LAYOUT, args
    sh, zg = synth.group_quant_params(c)
    pg = abq.abq_pack_weights_g128(3, to_dev(torch, c.W), to_dev(torch, sh.view(np.float16)), to_dev(torch, zg))
    assert abq.abq_check_packed(0, 3, 40, 700, G128, pg) == abq.ABQ_OK
    assert abq.abq_check_packed(0, 3, 40, 700, F, pg) == abq.ABQ_ERR_LAYOUT


def test_fused_act_ignores_bits_above_q(abq):
    """Unpacked codes with bits set above q: the one-kernel call masks them while staging, as the packers do."""
    c = synth.make_case(4, 5, 3, 100, 2048, seed=78)
    dirty = (c.A | (np.random.Generator(np.random.PCG64(3)).integers(0, 8, size=c.A.shape, dtype=np.uint8) << 5)).astype(np.uint8)
    pw = abq.abq_pack_weights(4, to_dev(torch, c.W), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero), FIELDS)
    assert abq.abq_gemm_act_codes_workspace_bytes(4, 5, 3, 100, 2048, FIELDS) == 0
    y, acc = abq.abq_gemm_act_codes(4, 5, 3, 100, 2048, to_dev(torch, dirty), to_dev(torch, c.a_scale), to_dev(torch, c.a_zero), pw,
                                    FIELDS, want_acc=True)
    torch.cuda.synchronize()
    check_against_oracle(c, y.cpu().numpy(), acc.cpu().numpy())


def test_measurement_probes_run(abq):
    """The probe kernels (a library of their own, used by the benchmark and the design measurements) launch, finish and leave their sink alone."""
    from paper_2408_08554_amd import probe as abq   # noqa: F811
    buf = torch.ones(8 << 20, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    abq.abq_probe_stream_read(buf, buf.numel(), sink)
    abq.abq_probe_stream_read(buf[256:], 4096 + 16, sink)       # a ragged size: the last workgroup clamps its reads
    abq.abq_probe_mfma_i8(100, 0, sink)
    abq.abq_probe_mfma_i8(100, 1, sink)
    abq.abq_probe_mfma_f4(100, 0, sink)
    abq.abq_probe_mfma_f4(100, 1, sink)
    abq.abq_probe_l2_read(buf, 1 << 20, 2, 2, sink)             # eight regions of 1 MiB: the whole of buf
    abq.abq_probe_l2_read(buf, 32768, 1, 1, sink)               # the smallest region: one round per pass
    assert abq.abq_probe_l2_read_bytes(1 << 20, 2, 2) == float((1 << 20) * 2 * 2 * torch.cuda.get_device_properties(0).multi_processor_count)
    torch.cuda.synchronize()
    assert int(sink.sum()) == 0
    assert abq.abq_probe_mfma_i8_ops(1) == 2.0 * 16 * 16 * 64 * 8 * 4 * 8 * torch.cuda.get_device_properties(0).multi_processor_count


def test_config1_tiny(abq):
    c = synth.config1()
    for layout in (FIELDS, PLANES):
        y, acc = gpu_gemm(torch, abq, c, layout, layout)
        check_against_oracle(c, y, acc)


def test_config2_w4a8_gemv_full(abq):
    c = synth.config2()
    y, acc = gpu_gemm(torch, abq, c, FIELDS, FIELDS)
    check_against_oracle(c, y, acc)
    y, acc = gpu_gemm(torch, abq, c, PLANES, PLANES)
    check_against_oracle(c, y, acc)


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 6, 7, 8])
def test_config3_w2a8_gemv_full(abq, M):
    c = synth.config3(M)
    y, acc = gpu_gemm(torch, abq, c, FIELDS, FIELDS)
    check_against_oracle(c, y, acc)


def test_config3_bitserial(abq):
    c = synth.config3(2)
    y, acc = gpu_gemm(torch, abq, c, PLANES, PLANES)
    check_against_oracle(c, y, acc)


@pytest.mark.parametrize("M,N,K,fused", [(1, 4096, 11008, True), (1, 4096, 11008, False), (8, 4096, 11008, True),
                                          (5, 70, 1000, True), (16, 33, 9000, False), (128, 1000, 2048, False)])
def test_bit_balance_five_level_weights(abq, M, N, K, fused):
    # W2* (Sec. 3.3): levels {-2..2} as p = 3 codes with zero-point 2, on the decode and the tiled path
    c = synth.bit_balance_case(8, M, N, K, seed=777 + M)
    y, acc = (gpu_gemm_fused(torch, abq, c, FIELDS) if fused else gpu_gemm(torch, abq, c, FIELDS, FIELDS))
    yref = check_against_oracle(c, y, acc)
    levels = c.W.astype(np.float64) - 2.0
    real = ((c.A.astype(np.float64) - c.a_zero[:, None]) * c.a_scale[:, None]) @ (levels * c.w_scale[:, None].astype(np.float64)).T
    assert np.allclose(yref, real, rtol=1e-12, atol=0)


# ---- launch-plan table: every candidate plan of the tuner returns the oracle's result -------------------------

@pytest.mark.parametrize("p,q,M,N,K", [(4, 8, 1, 256, 4096), (2, 8, 5, 70, 1000), (8, 8, 16, 70, 13824), (6, 6, 128, 300, 2048),
                                       (3, 5, 40, 100, 1536), (4, 4, 300, 520, 1024)])
def test_every_candidate_plan_gives_the_same_result(abq, p, q, M, N, K):
    from paper_2408_08554_amd import tune
    c = synth.make_case(p, q, M, N, K, seed=9600 + M)
    plans = tune.candidates(p, q, M, N, K)
    assert len(plans) >= 3 and plans[0] == {}
    try:
        for plan in plans:
            say(f"plan {plan} on {p, q, M, N, K}")
            abq.abq_plan_set(p, q, M, N, K, **plan)
            assert {k: v for k, v in abq.abq_plan_get(p, q, M, N, K).items() if v} == plan
            y, acc = gpu_gemm(torch, abq, c, FIELDS, FIELDS)
            check_against_oracle(c, y, acc)
            if K % 16 == 0:
                y, acc = gpu_gemm_fused(torch, abq, c, FIELDS)
                check_against_oracle(c, y, acc)
    finally:
        abq.abq_plan_clear()


def test_shipped_plan_table_loads_and_keeps_results(abq):
    from paper_2408_08554_amd import tune
    import json
    table = json.load(open(tune.DEFAULT_PLANS))
    try:
        assert tune.load_plans() == len(table) > 0
        checked = 0
        for key in sorted(table):
            p, q, M, N, K = (int(v) for v in key.split(","))
            assert {k: v for k, v in abq.abq_plan_get(p, q, M, N, K).items() if v} == table[key]
            c = synth.make_case(p, q, M, N, K, seed=9650 + checked)
            if M * N * K > 16 * 11008 * 4096:       # the oracle takes the small ones in full, the others at sampled outputs
                y, acc = gpu_gemm(torch, abq, c, FIELDS, FIELDS)
                check_sampled(c, y, acc, count=512)
            else:
                y, acc = gpu_gemm_fused(torch, abq, c, FIELDS)
                check_against_oracle(c, y, acc)
            checked += 1
        assert checked == len(table)
    finally:
        abq.abq_plan_clear()


def test_tuner_search_reports_the_rule_and_restores_the_table(abq):
    from paper_2408_08554_amd import tune
    abq.abq_plan_set(4, 8, 1, 512, 2048, skinny_waves=2)
    rows = tune.search(4, 8, 1, 512, 2048, launches=20, rotate_bytes=1 << 24)
    assert any(not plan for _, plan in rows) and all(t > 0 for t, _ in rows)
    assert rows == sorted(rows, key=lambda r: r[0])
    assert abq.abq_plan_get(4, 8, 1, 512, 2048)["skinny_waves"] == 2
    abq.abq_plan_clear()


# ---- per-group weight scales and zero-points, groups of 128 along K (Appendix C) -------------------------

G128 = 4   # ABQ_LAYOUT_FIELDS_G128


def run_g128(abq, c, sh, zg, fused):
    pw = abq.abq_pack_weights_g128(c.p, to_dev(torch, c.W), to_dev(torch, sh.view(np.float16)), to_dev(torch, zg))
    if fused:
        y, _ = abq.abq_gemm_act_codes(c.p, c.q, c.M, c.N, c.K, to_dev(torch, c.A), to_dev(torch, c.a_scale),
                                      to_dev(torch, c.a_zero), pw, G128, want_acc=False)
    else:
        pa = abq.abq_pack_act_codes(c.q, to_dev(torch, c.A), to_dev(torch, c.a_scale), to_dev(torch, c.a_zero), FIELDS)
        y, _ = abq.abq_gemm(c.p, c.q, c.M, c.N, c.K, pa, FIELDS, pw, G128, want_acc=False)
    torch.cuda.synchronize()
    return y.cpu().numpy()


@pytest.mark.parametrize("fused", [False, True], ids=["packed", "fused"])
@pytest.mark.parametrize("p,q", list(itertools.product(range(1, 9), [1, 4, 8])))
def test_g128_all_widths(abq, p, q, fused):
    say(f"g128 p={p} q={q} fused={fused}")
    c = synth.make_case(p, q, 3, 40, 1536, seed=9000 + 10 * p + q)
    sh, zg = synth.group_quant_params(c)
    check_g128(c, sh, zg, run_g128(abq, c, sh, zg, fused))


G128_SHAPES = [(1, 4096, 4096), (1, 4096, 11008), (8, 4096, 11008), (16, 70, 13824), (5, 33, 1000), (2, 17, 128),
               (3, 16, 80), (16, 256, 4096), (40, 100, 2048), (1, 13824, 5120)]


@pytest.mark.parametrize("fused", [False, True], ids=["packed", "fused"])
@pytest.mark.parametrize("M,N,K", G128_SHAPES)
@pytest.mark.parametrize("p,q", [(2, 8), (4, 8), (3, 8), (8, 8), (4, 4)])
def test_g128_shapes(abq, M, N, K, p, q, fused):
    say(f"g128 shape M={M} N={N} K={K} p={p} q={q} fused={fused}")
    c = synth.make_case(p, q, M, N, K, seed=9100 + M + N + K + p)
    sh, zg = synth.group_quant_params(c)
    check_g128(c, sh, zg, run_g128(abq, c, sh, zg, fused))


@pytest.mark.parametrize("fused", [False, True], ids=["packed", "fused"])
@pytest.mark.parametrize("N,K", [(48, 8704), (33, 9000), (20, 16384), (16, 16000), (100, 8320)])
@pytest.mark.parametrize("p,q", [(1, 8), (2, 8), (4, 8), (4, 4), (2, 3)])
def test_g128_one_row_long_k(abq, N, K, p, q, fused):
    # one row of A over more than sixteen super-chunks of K: the decode kernel's waves take two each (an odd count
    # leaves the last wave with one, K = 16384 is the most the variant covers, 9000 and 16000 end inside a group)
    say(f"g128 long K N={N} K={K} p={p} q={q} fused={fused}")
    c = synth.make_case(p, q, 1, N, K, seed=9300 + N + K + p + q)
    sh, zg = synth.group_quant_params(c)
    check_g128(c, sh, zg, run_g128(abq, c, sh, zg, fused))


@pytest.mark.parametrize("p", [1, 2, 4, 7, 8])
@pytest.mark.parametrize("kind", ["zero_points_at_both_ends", "all_codes_maximal", "all_codes_zero", "zero_scales"])
def test_g128_extremes(abq, p, kind):
    # the zero-point rides an MFMA operand byte as -z (p <= 7: down to -127) or is subtracted in integers (p = 8:
    # z - 128 spans -128..127); the ends of those ranges, saturated operands and dead groups
    q, M, N, K = 8, 5, 40, 1300                      # 11 groups, the last of 20 values
    c = synth.make_case(p, q, M, N, K, seed=9700 + p)
    sh, zg = synth.group_quant_params(c)
    top = (1 << p) - 1
    if kind == "zero_points_at_both_ends":
        zg[:, 0::2] = 0
        zg[:, 1::2] = top
        c.a_zero[:] = [0, 255, 128, 1, 254]
    elif kind == "all_codes_maximal":
        c.W[:] = top
        c.A[:] = 255
        zg[:] = 0
        c.a_zero[:] = 0
        c.a_scale[:] = np.float32(1e-4)
    elif kind == "all_codes_zero":
        c.W[:] = 0
        c.A[:] = 0
        zg[:] = top
        c.a_zero[:] = 255
        c.a_scale[:] = np.float32(1e-4)
    else:
        sh[:, 3:7] = 0                               # binary16 +0: groups that contribute nothing
        sh[:, 8] = 0x8000                            # and -0
    for fused in (False, True):
        if fused and K % 16:
            continue
        check_g128(c, sh, zg, run_g128(abq, c, sh, zg, fused))
    c2 = synth.make_case(p, q, 3, 17, 1296, seed=9750 + p)      # K a multiple of 16: the fused entry point as well
    sh2, zg2 = synth.group_quant_params(c2)
    if kind == "zero_points_at_both_ends":
        zg2[:, 0::2] = top
        zg2[:, 1::2] = 0
    check_g128(c2, sh2, zg2, run_g128(abq, c2, sh2, zg2, True))


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (1, 16, 127), (2, 3, 129), (64, 48, 1024), (100, 20, 640), (16, 1, 8192)])
def test_g128_degenerate_and_many_rows(abq, M, N, K):
    c = synth.make_case(4, 8, M, N, K, seed=9800 + M + K)
    sh, zg = synth.group_quant_params(c)
    check_g128(c, sh, zg, run_g128(abq, c, sh, zg, False))
    if K % 16 == 0:
        check_g128(c, sh, zg, run_g128(abq, c, sh, zg, True))


def test_g128_exact_when_the_float_sum_is_exact(abq):
    # power-of-two scales and small codes: every product and partial sum is an integer multiple of 2^-10 below
    # 2^24 ulps, so binary32 accumulates without rounding and the output must equal the oracle's bit for bit
    c = synth.make_case(3, 4, 4, 48, 2048, seed=9200)
    sh, zg = synth.group_quant_params(c)
    rng = np.random.Generator(np.random.PCG64(9201))
    sh = np.float16(2.0) ** rng.integers(-6, -2, size=sh.shape).astype(np.float16)
    sh = sh.astype(np.float16).view(np.uint16)
    c.a_scale = (np.float32(2.0) ** rng.integers(-8, -5, size=c.M)).astype(np.float32)
    for fused in (False, True):
        y = run_g128(abq, c, sh, zg, fused)
        _, y16 = oracle.dequant_grouped(c.A, c.W, c.a_zero, c.a_scale, zg, sh, gs=128)
        assert np.array_equal(y.view(np.uint16), y16)


def test_g128_one_parameter_set_per_channel_matches_the_per_channel_kernel(abq):
    # equal parameters in every group: the same problem as the per-channel path
    c = synth.make_case(4, 8, 2, 64, 4096, seed=9300)
    G = c.K // 128
    sh = np.repeat(c.w_scale.astype(np.float16).view(np.uint16)[:, None], G, axis=1).copy()
    zg = np.repeat(c.w_zero[:, None], G, axis=1).astype(np.int32).copy()
    y = run_g128(abq, c, sh, zg, True)
    y_pc, _ = gpu_gemm_fused(torch, abq, c, FIELDS)
    yref = check_against_oracle(c, y_pc, None)
    check_g128(c, sh, zg, y)
    assert np.all(np.abs(y.astype(np.float64) - y_pc.astype(np.float64)) <= 2 * (2.0 ** (np.floor(np.log2(np.maximum(np.abs(yref), 2.0 ** -14))) - 10)))


@pytest.mark.parametrize("fused", [False, True], ids=["packed", "fused"])
@pytest.mark.parametrize("p,q,M", [(4, 8, 1), (2, 8, 5), (8, 8, 2), (3, 4, 16), (7, 8, 3)])
def test_g128_grouped_launch(abq, p, q, M, fused):
    say(f"g128 grouped p={p} q={q} M={M} fused={fused}")
    shapes = [(100, 2048), (33, 4096), (256, 2560), (16, 6656)]
    cases = [synth.make_case(p, q, M, N, K, seed=9500 + i) for i, (N, K) in enumerate(shapes)]
    gpar = [synth.group_quant_params(c) for c in cases]
    keep, probs = [], []
    for c, (sh, zg) in zip(cases, gpar):
        pw = abq.abq_pack_weights_g128(p, to_dev(torch, c.W), to_dev(torch, sh.view(np.float16)), to_dev(torch, zg))
        y = torch.full((M, c.N), float("nan"), dtype=torch.float16, device="cuda")
        d = dict(N=c.N, K=c.K, packed_w=pw, y=y)
        if fused:
            d.update(a_codes=to_dev(torch, c.A), a_scale=to_dev(torch, c.a_scale), a_zero=to_dev(torch, c.a_zero))
        else:
            d.update(packed_act=abq.abq_pack_act_codes(q, to_dev(torch, c.A), to_dev(torch, c.a_scale), to_dev(torch, c.a_zero), FIELDS))
        probs.append(d)
        keep.append(y)
    assert abq.abq_gemm_grouped_workspace_bytes(p, q, M, probs, FIELDS, G128) == 0     # one launch
    abq.abq_gemm_grouped(p, q, M, probs, FIELDS, G128)
    torch.cuda.synchronize()
    for c, (sh, zg), y in zip(cases, gpar, keep):
        got = y.cpu().numpy()
        check_g128(c, sh, zg, got)
        # the single call may split K over a different number of waves: another order of the binary32 sum, so the
        # two agree to the bound (both were checked against it), not to the bit


def test_g128_rejects_what_it_cannot_do(abq):
    c = synth.make_case(4, 8, 1, 32, 1024, seed=9400)
    sh, zg = synth.group_quant_params(c)
    pw = abq.abq_pack_weights_g128(4, to_dev(torch, c.W), to_dev(torch, sh.view(np.float16)), to_dev(torch, zg))
    with pytest.raises(abq.AbqError):   # no raw integer accumulator on this path
        abq.abq_gemm_act_codes(4, 8, 1, 32, 1024, to_dev(torch, c.A), to_dev(torch, c.a_scale), to_dev(torch, c.a_zero), pw, G128,
                               want_acc=True)
    codes = abq.abq_unpack_weights(4, 32, 1024, G128, pw, FIELDS)
    assert np.array_equal(codes.cpu().numpy(), c.W)


def test_quantize_then_gemm_end_to_end(abq):
    # fp16 activations -> online quantizer -> matmul; the oracle follows the same two steps
    p, q, M, N, K = 4, 8, 4, 64, 2048
    c = synth.make_case(p, q, M, N, K, seed=4242)
    x = synth.act_fp16(4243, M, K)
    codes, sc, zp = oracle.quant_act(x, q)
    c.A, c.a_scale, c.a_zero = codes, sc, zp
    pw = abq.abq_pack_weights(p, to_dev(torch, c.W), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero), FIELDS)
    pa = abq.abq_quant_pack_act(q, to_dev(torch, x), FIELDS)
    y, acc = abq.abq_gemm(p, q, M, N, K, pa, FIELDS, pw, FIELDS, want_acc=True)
    torch.cuda.synchronize()
    check_against_oracle(c, y.cpu().numpy(), acc.cpu().numpy())


@pytest.mark.parametrize("M", [128, 512])
def test_config4_w6a6_gemm_sampled(abq, M):
    c = synth.config4(M)
    y, acc = gpu_gemm(torch, abq, c, FIELDS, FIELDS)
    check_sampled(c, y, acc)


@pytest.mark.parametrize("p,q,shape_idx,m_idx", [(4, 8, 0, 1), (2, 4, 1, 2), (8, 8, 0, 2), (3, 8, 1, 0), (1, 1, 0, 2),
                                                 (4, 4, 0, 3), (7, 8, 1, 3)])
def test_config5_sweep_samples(abq, p, q, shape_idx, m_idx):
    c = synth.config5(p, q, shape_idx, m_idx)
    y, acc = gpu_gemm(torch, abq, c, FIELDS, FIELDS)
    check_sampled(c, y, acc)


# ---- per-group weight parameters in the prefill shape (the tiled per-group kernel, M > 16) --------------------------
@pytest.mark.parametrize("fused", [False, True], ids=["packed", "fused"])
@pytest.mark.parametrize("M,N,K", [(128, 300, 2048), (512, 1000, 4096), (2048, 256, 1024), (70, 130, 1000), (17, 64, 127),
                                   (200, 4100, 640)])
@pytest.mark.parametrize("p,q", [(1, 8), (2, 8), (3, 5), (4, 4), (4, 8), (6, 6), (7, 3), (8, 8)])
def test_g128_prefill_shapes(abq, p, q, M, N, K, fused):
    if (M, N, K) in ((512, 1000, 4096), (2048, 256, 1024), (200, 4100, 640)) and (p, q) not in ((2, 8), (4, 8), (8, 8), (3, 5)):
        pytest.skip("the large shapes run for four width pairs")
    c = synth.make_case(p, q, M, N, K, seed=synth.case_seed(10, p, q, M % 97, N % 89), name=f"g128 prefill W{p}A{q} {M}x{N}x{K}")
    say(c.name)
    sh, zg = synth.group_quant_params(c)
    check_g128(c, sh, zg, run_g128(abq, c, sh, zg, fused))


def test_g128_prefill_exact_when_the_float_sum_is_exact(abq):
    """Power-of-two scales and small codes: every product and partial sum is exact in binary32, so the tiled per-group
    kernel must return the oracle's binary16 values bit for bit."""
    M, N, K = 96, 80, 1024
    c = synth.make_case(2, 4, M, N, K, seed=4242, name="g128 prefill exact")
    rng = np.random.Generator(np.random.PCG64(5))
    G = (K + 127) // 128
    sh = (2.0 ** rng.integers(-6, -2, size=(N, G))).astype(np.float16).view(np.uint16)
    zg = rng.integers(0, 4, size=(N, G)).astype(np.int32)
    c.a_scale = (2.0 ** rng.integers(-8, -4, size=M)).astype(np.float32)
    y = run_g128(abq, c, sh, zg, False)
    _, y16ref = oracle.dequant_grouped(c.A, c.W, c.a_zero, c.a_scale, zg, sh, gs=128)
    assert np.array_equal(y.view(np.uint16), y16ref)


# ---- ReQuant fused into the matmul epilogue (the consumer side of Fig. 3b) --------------------------------------
@pytest.mark.parametrize("p,q,q_out,M,N,K,layout", [(4, 8, 8, 1, 300, 4096, FIELDS),      # direct decode kernel
                                                    (2, 8, 4, 7, 70, 1552, FIELDS),       # direct, ragged
                                                    (8, 8, 8, 16, 2000, 13824, FIELDS),   # streaming decode kernel (long stream, 16 rows)
                                                    (2, 8, 8, 16, 4400, 2048, FIELDS),    # shared-operand decode kernel (more tiles than units)
                                                    (1, 8, 4, 12, 4200, 7168, FIELDS),    # shared-operand, K in two phases
                                                    (6, 6, 6, 130, 200, 2048, FIELDS),    # tiled prefill kernel
                                                    (4, 4, 2, 300, 520, 1000, FIELDS),    # tiled, K ragged
                                                    (3, 5, 3, 5, 33, 200, PLANES),        # bit-serial kernel (two-step path)
                                                    (1, 1, 1, 2, 16, 512, FIELDS)])
def test_gemm_requant_emits_the_next_layers_codes(abq, p, q, q_out, M, N, K, layout):
    """abq_gemm_act_codes_requant: the codes equal the oracle's ReQuant of the kernel's own binary16 output bit for bit, the
    binary16 output is the one abq_gemm_act_codes gives, and leaving it out changes no code."""
    c = synth.make_case(p, q, M, N, K, seed=synth.case_seed(9, p, q, M, q_out), name=f"requant W{p}A{q}->A{q_out} {M}x{N}x{K}")
    say(c.name)
    pw = abq.abq_pack_weights(p, to_dev(torch, c.W), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero), layout)
    a, s, z = to_dev(torch, c.A), to_dev(torch, c.a_scale), to_dev(torch, c.a_zero)
    y_plain, _ = abq.abq_gemm_act_codes(p, q, M, N, K, a, s, z, pw, layout)
    # per-token output parameters as a calibration pass would fix them: the quantizer's own on the reference output
    yref = check_against_oracle(c, y_plain.cpu().numpy(), None)
    _, osc, ozp = oracle.quant_act(yref.astype(np.float16), q_out)
    codes, y = abq.abq_gemm_act_codes_requant(p, q, M, N, K, a, s, z, pw, layout, q_out, to_dev(torch, osc), to_dev(torch, ozp))
    codes_only, none = abq.abq_gemm_act_codes_requant(p, q, M, N, K, a, s, z, pw, layout, q_out, to_dev(torch, osc), to_dev(torch, ozp),
                                                      want_y=False)
    torch.cuda.synchronize()
    assert none is None and torch.equal(codes, codes_only)
    assert torch.equal(y.view(torch.int16), y_plain.view(torch.int16))
    want = oracle.requant(y.cpu().numpy(), q_out, osc, ozp)
    assert np.array_equal(codes.cpu().numpy(), want)
    # against the oracle end to end: the codes can differ only where the binary16 outputs differ (both within tolerance)
    y16ref = yref.astype(np.float16)
    end_to_end = oracle.requant(y16ref, q_out, osc, ozp)
    same_y = y.cpu().numpy().view(np.uint16) == y16ref.view(np.uint16)
    assert np.array_equal(codes.cpu().numpy()[same_y], end_to_end[same_y])
    assert np.abs(codes.cpu().numpy().astype(np.int32) - end_to_end.astype(np.int32)).max() <= 1


def test_gemm_requant_chains_two_layers_without_a_quantizer_kernel(abq):
    """Layer 1's epilogue writes layer 2's activation codes; layer 2 consumes them directly: two launches in all."""
    M, K1, N1, N2 = 3, 2048, 1024, 64
    c1 = synth.make_case(4, 8, M, N1, K1, seed=7701)
    c2 = synth.make_case(4, 8, M, N2, N1, seed=7702)
    pw1 = abq.abq_pack_weights(4, to_dev(torch, c1.W), to_dev(torch, c1.w_scale), to_dev(torch, c1.w_zero), FIELDS)
    pw2 = abq.abq_pack_weights(4, to_dev(torch, c2.W), to_dev(torch, c2.w_scale), to_dev(torch, c2.w_zero), FIELDS)
    acc1 = oracle.acc_centered(c1.A, c1.W, c1.a_zero, c1.w_zero)
    y1ref, _ = oracle.dequant(acc1, c1.a_scale, c1.w_scale)
    _, osc, ozp = oracle.quant_act(y1ref.astype(np.float16), 8)
    codes, _ = abq.abq_gemm_act_codes_requant(4, 8, M, N1, K1, to_dev(torch, c1.A), to_dev(torch, c1.a_scale), to_dev(torch, c1.a_zero), pw1,
                                              FIELDS, 8, to_dev(torch, osc), to_dev(torch, ozp), want_y=False)
    y2, acc2 = abq.abq_gemm_act_codes(4, 8, M, N2, N1, codes, to_dev(torch, osc), to_dev(torch, ozp), pw2, FIELDS, want_acc=True)
    torch.cuda.synchronize()
    c2.A, c2.a_scale, c2.a_zero = codes.cpu().numpy(), osc, ozp     # layer 2 against the oracle on the codes it was given
    check_against_oracle(c2, y2.cpu().numpy(), acc2.cpu().numpy())


# ---- the direct decode kernel: every variant (operand rows 1..16, 1/2/4 super-chunks per wave, both activation forms) ------
@pytest.mark.parametrize("fused", [False, True], ids=["packed", "fused"])
@pytest.mark.parametrize("r", [1, 2, 4])
@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8, 9, 16])
@pytest.mark.parametrize("p,q", [(1, 8), (2, 8), (3, 4), (4, 8), (5, 3), (6, 6), (7, 1), (8, 8)])
def test_direct_decode_kernel_variants(abq, p, q, M, r, fused):
    """The plan table forces the direct kernel with r super-chunks per wave (a value the problem does not fit leaves the
    rule's choice, which the other tests cover); shapes ragged in N and K, K spanning whole and partial super-chunks."""
    for N, K in ((40, 1552), (17, 4096)) if r < 4 else ((40, 2608),):
        c = synth.make_case(p, q, M, N, K, seed=synth.case_seed(8, p, q, M, r), name=f"direct W{p}A{q} M={M} N={N} K={K} r={r}")
        abq.abq_plan_set(p, q, M, N, K, direct_r=r)
        try:
            y, acc = (gpu_gemm_fused if fused else gpu_gemm)(torch, abq, c, FIELDS) if fused else gpu_gemm(torch, abq, c, FIELDS, FIELDS)
        finally:
            abq.abq_plan_set(p, q, M, N, K)
        check_against_oracle(c, y, acc)


def test_direct_and_streaming_decode_kernels_agree_bitwise(abq):
    """Both decode kernels on the same problems: equal accumulators and equal fp16 bits."""
    for p, q, M, N, K in [(4, 8, 1, 256, 4096), (2, 8, 8, 70, 2048), (8, 8, 4, 33, 5120), (3, 5, 16, 64, 1024)]:
        c = synth.make_case(p, q, M, N, K, seed=synth.case_seed(8, p, q, M, 9))
        out = []
        for r in (-1, 1):
            abq.abq_plan_set(p, q, M, N, K, direct_r=r)
            try:
                out.append(gpu_gemm_fused(torch, abq, c, FIELDS))
            finally:
                abq.abq_plan_set(p, q, M, N, K)
        assert np.array_equal(out[0][1], out[1][1]) and np.array_equal(out[0][0].view(np.uint16), out[1][0].view(np.uint16))
        check_against_oracle(c, *out[1])


# ---- the shared-operand decode kernel (one copy of A in LDS per workgroup of several tiles) ------------------------------
@pytest.mark.parametrize("fused", [False, True], ids=["packed", "fused"])
@pytest.mark.parametrize("M", [1, 7, 9, 13, 16])
@pytest.mark.parametrize("p,q", [(1, 8), (2, 8), (3, 4), (4, 8), (5, 3), (6, 6), (7, 1), (8, 8)])
def test_shared_operand_decode_kernel_forced(abq, p, q, M, fused):
    """The plan table forces the kernel on small problems (two tiles per workgroup, the second one partly or wholly past
    the end of N; K spanning whole and partial super-chunks, one to three per wave)."""
    for N, K in ((40, 1552), (17, 4096), (90, 2608), (33, 5120)):
        c = synth.make_case(p, q, M, N, K, seed=synth.case_seed(8, p, q, M, 11), name=f"shared-A W{p}A{q} M={M} N={N} K={K}")
        say(c.name)
        abq.abq_plan_set(p, q, M, N, K, direct_r=-2)
        try:
            y, acc = gpu_gemm_fused(torch, abq, c, FIELDS) if fused else gpu_gemm(torch, abq, c, FIELDS, FIELDS)
        finally:
            abq.abq_plan_set(p, q, M, N, K)
        assert abq.abq_last_decode_kernel() == abq.ABQ_DECODE_SHARED_OPERAND
        check_against_oracle(c, y, acc)


@pytest.mark.parametrize("fused", [False, True], ids=["packed", "fused"])
@pytest.mark.parametrize("p,q,M,N,K", [(1, 8, 16, 4100, 1024), (4, 8, 9, 8200, 3000), (2, 4, 16, 12304, 5120), (6, 6, 12, 12290, 4608),
                                       (8, 8, 16, 8208, 4096), (3, 8, 10, 28000, 2048), (2, 8, 16, 28690, 6144), (4, 4, 16, 13824, 5120)])
def test_shared_operand_decode_kernel_many_tiles(abq, p, q, M, N, K, fused):
    """More tiles than compute units: the kernel's own plans (two to eight tiles per workgroup, up to six super-chunks per
    wave), whichever decode kernel the rule takes being forced aside."""
    c = synth.make_case(p, q, M, N, K, seed=synth.case_seed(8, p, q, M, 12), name=f"shared-A W{p}A{q} M={M} N={N} K={K}")
    say(c.name)
    abq.abq_plan_set(p, q, M, N, K, direct_r=-2)
    try:
        y, acc = gpu_gemm_fused(torch, abq, c, FIELDS) if fused else gpu_gemm(torch, abq, c, FIELDS, FIELDS)
    finally:
        abq.abq_plan_set(p, q, M, N, K)
    assert abq.abq_last_decode_kernel() == abq.ABQ_DECODE_SHARED_OPERAND
    check_against_oracle(c, y, acc)


@pytest.mark.parametrize("fused", [False, True], ids=["packed", "fused"])
@pytest.mark.parametrize("p,q,M,N,K", [(1, 8, 16, 5120, 13824), (2, 8, 9, 5120, 13824), (2, 8, 16, 5120, 13824), (1, 4, 13, 4200, 11008),
                                       (2, 3, 16, 100, 8000), (1, 1, 11, 40, 7000), (2, 8, 16, 33, 12288), (2, 8, 16, 8200, 6656),
                                       (1, 8, 10, 48, 14336)])
def test_shared_operand_decode_kernel_two_phases_of_k(abq, p, q, M, N, K, fused):
    """A larger than LDS: K is cut in two phases whose halves of A take turns in LDS (an odd number of super-chunks, a
    second phase that ends inside a super-chunk, few and many tiles)."""
    c = synth.make_case(p, q, M, N, K, seed=synth.case_seed(8, p, q, M, 14), name=f"shared-A two phases W{p}A{q} M={M} N={N} K={K}")
    say(c.name)
    abq.abq_plan_set(p, q, M, N, K, direct_r=-2)
    try:
        y, acc = gpu_gemm_fused(torch, abq, c, FIELDS) if fused else gpu_gemm(torch, abq, c, FIELDS, FIELDS)
    finally:
        abq.abq_plan_set(p, q, M, N, K)
    assert abq.abq_last_decode_kernel() == abq.ABQ_DECODE_SHARED_OPERAND
    check_against_oracle(c, y, acc)


def test_shared_operand_and_streaming_decode_kernels_agree_bitwise(abq):
    """Same problems on both kernels, with the accumulator output and the ReQuant epilogue: equal bits."""
    for p, q, M, N, K in [(4, 8, 16, 4200, 2048), (2, 8, 11, 70, 2048), (8, 8, 9, 33, 5120)]:
        c = synth.make_case(p, q, M, N, K, seed=synth.case_seed(8, p, q, M, 13))
        out = []
        for r in (-1, -2):
            abq.abq_plan_set(p, q, M, N, K, direct_r=r)
            try:
                out.append(gpu_gemm_fused(torch, abq, c, FIELDS))
            finally:
                abq.abq_plan_set(p, q, M, N, K)
            assert abq.abq_last_decode_kernel() == (abq.ABQ_DECODE_STREAMING if r == -1 else abq.ABQ_DECODE_SHARED_OPERAND)
        assert np.array_equal(out[0][1], out[1][1]) and np.array_equal(out[0][0].view(np.uint16), out[1][0].view(np.uint16))
        check_against_oracle(c, *out[1])


# ---- config 5 in full: every (p, q) on both LLaMA-13B shapes ---------------------------------------------------
@pytest.mark.parametrize("m_idx", [0, 1], ids=["M1", "M16"])
@pytest.mark.parametrize("shape_idx", [0, 1], ids=["5120to13824", "13824to5120"])
@pytest.mark.parametrize("p,q", list(itertools.product(range(1, 9), range(1, 9))))
def test_config5_decode_every_pq(abq, p, q, shape_idx, m_idx):
    """M = 1 and 16 through abq_gemm_act_codes (the one-kernel decode step), every output element against the oracle."""
    c = synth.config5(p, q, shape_idx, m_idx)
    say(c.name)
    assert abq.abq_gemm_act_codes_workspace_bytes(p, q, c.M, c.N, c.K, FIELDS) == 0
    y, acc = gpu_gemm_fused(torch, abq, c, FIELDS)
    check_against_oracle(c, y, acc)


@pytest.mark.parametrize("m_idx", [2, 3], ids=["M256", "M2048"])
@pytest.mark.parametrize("shape_idx", [0, 1], ids=["5120to13824", "13824to5120"])
@pytest.mark.parametrize("p,q", [(p, p) for p in range(1, 9)] + [(p, 8) for p in range(1, 8)])
def test_config5_prefill_every_p(abq, p, q, shape_idx, m_idx):
    """M = 256 and 2048 through abq_pack_act_codes + abq_gemm for every weight width (q = p and q = 8), sampled outputs."""
    c = synth.config5(p, q, shape_idx, m_idx)
    say(c.name)
    y, acc = gpu_gemm(torch, abq, c, FIELDS, FIELDS)
    check_sampled(c, y, acc)
