"""The very-low-bit path on the 4-bit floating-point MFMA (weights and activations of one or two bits): the HIP kernels
through the C ABI against the oracle, element by element — int32 accumulator bit-exact, binary16 output within the same
tolerance as the int8 path, and equal to the int8 path bit for bit."""
import itertools

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from helpers import check_against_oracle, check_sampled, gpu_gemm, to_dev   # noqa: E402
from paper_2408_08554_amd import synth   # noqa: E402


def say(*a):
    print(*a, flush=True)


def run_f4(abq, c):
    pw = abq.abq_f4_pack_codes(c.p, to_dev(torch, c.W), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero))
    pa = abq.abq_f4_pack_codes(c.q, to_dev(torch, c.A), to_dev(torch, c.a_scale), to_dev(torch, c.a_zero))
    y = torch.full((c.M, c.N), float("nan"), dtype=torch.float16, device="cuda")
    acc = torch.full((c.M, c.N), -7, dtype=torch.int32, device="cuda")
    abq.abq_f4_gemm(c.p, c.q, c.M, c.N, c.K, pa, pw, y=y, acc=acc)
    # without the accumulator output the kernel takes its staged epilogue (vector stores): the same bits
    y_only = torch.full((c.M, c.N), float("nan"), dtype=torch.float16, device="cuda")
    abq.abq_f4_gemm(c.p, c.q, c.M, c.N, c.K, pa, pw, y=y_only)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y_only.view(torch.int16)), f"{c.name}: output differs without the accumulator"
    return y.cpu().numpy(), acc.cpu().numpy()


# one tile and less, ragged in every dimension, several workgroup tiles (256 x 128) with ragged tails, odd and even numbers
# of 128-k steps, K ending inside a step
F4_SHAPES = [(1, 1, 1), (1, 16, 128), (5, 33, 200), (16, 16, 129), (17, 130, 1000), (256, 128, 1024), (300, 520, 1000),
             (513, 257, 384), (64, 1000, 2048), (700, 300, 4096 + 64), (260, 136, 256), (31, 8, 64)]


@pytest.mark.parametrize("M,N,K", F4_SHAPES)
@pytest.mark.parametrize("p,q", list(itertools.product([1, 2], [1, 2])))
def test_f4_matmul_against_oracle(abq, p, q, M, N, K):
    c = synth.make_case(p, q, M, N, K, seed=synth.case_seed(11, p, q, M % 97, N % 89), name=f"f4 W{p}A{q} {M}x{N}x{K}")
    say(c.name)
    y, acc = run_f4(abq, c)
    check_against_oracle(c, y, acc)


def test_f4_extreme_codes(abq):
    """All codes maximal (the largest sums: K * 9), all zero, and zero-points at both ends."""
    for p, q, K in [(2, 2, 8192), (1, 2, 3000), (2, 1, 4096), (2, 2, 131072)]:   # (the last: the longest K the ABI takes)
        c = synth.make_case(p, q, 40, 70, K, seed=5, name=f"f4 max W{p}A{q} K={K}")
        c.A[:] = (1 << q) - 1
        c.W[:] = (1 << p) - 1
        c.A[1] = 0
        c.W[3] = 0
        c.a_zero[:] = np.where(np.arange(40) % 2 == 0, 0, (1 << q) - 1)
        c.w_zero[:] = np.where(np.arange(70) % 2 == 0, (1 << p) - 1, 0)
        say(c.name)
        y, acc = run_f4(abq, c)
        check_against_oracle(c, y, acc)


def test_f4_equals_the_int8_path_bitwise(abq):
    for p, q, M, N, K in [(2, 2, 300, 520, 1000), (1, 2, 64, 257, 2048), (2, 1, 1, 100, 512)]:
        c = synth.make_case(p, q, M, N, K, seed=synth.case_seed(11, p, q, M % 97, 7))
        y, acc = run_f4(abq, c)
        y8, acc8 = gpu_gemm(torch, abq, c, abq.ABQ_LAYOUT_FIELDS, abq.ABQ_LAYOUT_FIELDS)
        assert np.array_equal(acc, acc8) and np.array_equal(y.view(np.uint16), y8.view(np.uint16))


def test_f4_drops_bits_above_the_width(abq):
    """Codes with bits above `bits` set are masked, as the other packers mask them."""
    c = synth.make_case(2, 1, 20, 48, 640, seed=9)
    dirty_w = (c.W | (np.arange(c.W.size, dtype=np.uint8).reshape(c.W.shape) << 2)).astype(np.uint8)
    dirty_a = (c.A | 0xFE).astype(np.uint8)
    pw = abq.abq_f4_pack_codes(2, to_dev(torch, dirty_w), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero))
    pa = abq.abq_f4_pack_codes(1, to_dev(torch, dirty_a), to_dev(torch, c.a_scale), to_dev(torch, c.a_zero))
    y, acc = abq.abq_f4_gemm(2, 1, c.M, c.N, c.K, pa, pw, want_acc=True)
    torch.cuda.synchronize()
    check_against_oracle(c, y.cpu().numpy(), acc.cpu().numpy())


def test_f4_large_tile_sampled(abq):
    """256 workgroups of the 256-row tile (one per compute unit: the smallest grid that takes this tile), ragged K (eight
    steps: two turns of the three-buffer ring and a tail of two): sampled outputs.  A second case with several panels of
    row tiles and a partial last panel."""
    for M, N, K in [(1024, 8192, 1000), (2600, 3300, 640)]:
        c = synth.make_case(2, 2, M, N, K, seed=synth.case_seed(11, 2, 2, 55, 66), name=f"f4 W2A2 {M}x{N}x{K}")
        say(c.name)
        y, acc = run_f4(abq, c)
        check_sampled(c, y, acc)


@pytest.mark.parametrize("p,q", [(2, 2), (1, 1)])
def test_f4_config5_prefill_shape_sampled(abq, p, q):
    """M = 2048 on the LLaMA-13B up-projection, the launch the bench times: sampled outputs against the oracle."""
    c = synth.config5(p, q, 0, 3)
    say(c.name)
    y, acc = run_f4(abq, c)
    check_sampled(c, y, acc)
