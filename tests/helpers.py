"""Shared pieces of the GPU parity tests: run one synthetic case through the C ABI and compare
with the CPU oracle (int32 accumulator bit-exact, fp16 output within the stated tolerance)."""
import numpy as np

import oracle


def ulp16(v):
    """Spacing of binary16 at |v| (2^-24 in the subnormal range)."""
    a = np.abs(np.asarray(v, dtype=np.float64))
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -14)))
    return 2.0 ** (e - 10)


def y_tolerance(yref):
    """|y - Yref| <= max(1e-2*|Yref|, 2 ulp16(Yref), 2^-24): the bound the build is held to."""
    return np.maximum(np.maximum(1e-2 * np.abs(yref), 2 * ulp16(yref)), 2.0 ** -24)


def to_dev(torch, arr):
    return torch.from_numpy(np.ascontiguousarray(arr)).cuda()


def gpu_gemm(torch, abq, c, a_layout, w_layout, gemm_w_layout=None, want_acc=True):
    """pack both operands from codes, run abq_gemm; returns (y float16 ndarray, acc int32 ndarray)."""
    pw = abq.abq_pack_weights(c.p, to_dev(torch, c.W), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero), w_layout)
    pa = abq.abq_pack_act_codes(c.q, to_dev(torch, c.A), to_dev(torch, c.a_scale), to_dev(torch, c.a_zero), a_layout)
    y, acc = abq.abq_gemm(c.p, c.q, c.M, c.N, c.K, pa, a_layout, pw, w_layout if gemm_w_layout is None else gemm_w_layout,
                          want_acc=want_acc)
    torch.cuda.synchronize()
    return y.cpu().numpy(), (acc.cpu().numpy() if acc is not None else None)


def gpu_gemm_fused(torch, abq, c, w_layout, gemm_w_layout=None, want_acc=True):
    """pack the weights, then abq_gemm_act_codes on the unpacked activation codes."""
    pw = abq.abq_pack_weights(c.p, to_dev(torch, c.W), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero), w_layout)
    y, acc = abq.abq_gemm_act_codes(c.p, c.q, c.M, c.N, c.K, to_dev(torch, c.A), to_dev(torch, c.a_scale),
                                    to_dev(torch, c.a_zero), pw, w_layout if gemm_w_layout is None else gemm_w_layout,
                                    want_acc=want_acc)
    torch.cuda.synchronize()
    return y.cpu().numpy(), (acc.cpu().numpy() if acc is not None else None)


def check_against_oracle(c, y, acc, tight=True):
    ref_acc = oracle.acc(c.A, c.W)
    assert ref_acc.max() <= np.iinfo(np.int32).max
    if acc is not None:
        bad = np.argwhere(acc.astype(np.int64) != ref_acc)
        assert bad.size == 0, f"{c.name}: int32 accumulator differs at {bad[:5].tolist()} " \
                              f"got {acc[tuple(bad[0])]} want {ref_acc[tuple(bad[0])]} ({len(bad)} of {acc.size})"
    accc = oracle.acc_centered(c.A, c.W, c.a_zero, c.w_zero)
    yref, y16ref = oracle.dequant(accc, c.a_scale, c.w_scale)
    err = np.abs(y.astype(np.float64) - yref)
    tol = y_tolerance(yref)
    assert np.all(err <= tol), f"{c.name}: fp16 output off by {np.max(err / tol):.3g} x tolerance"
    if tight:
        # with an exact integer correction and one fp32 product chain the result is within 1 ulp16
        assert np.all(err <= 1.0 * ulp16(yref) + 1e-30), f"{c.name}: more than 1 ulp16 from the exact value"
    return yref


def check_sampled(c, y, acc, count=4096, seed=1):
    """Large cases: compare at tile-boundary rows/columns and random positions only."""
    rng = np.random.Generator(np.random.PCG64(seed))
    ms = rng.integers(0, c.M, size=count)
    ns = rng.integers(0, c.N, size=count)
    edge_m = np.array([0, c.M - 1, min(15, c.M - 1), min(16, c.M - 1), c.M // 2])
    edge_n = np.array([0, c.N - 1, min(15, c.N - 1), min(16, c.N - 1), c.N // 2, min(255, c.N - 1), min(256, c.N - 1)])
    em, en = np.meshgrid(edge_m, edge_n, indexing="ij")
    ms = np.concatenate([ms, em.ravel()]).astype(np.int32)
    ns = np.concatenate([ns, en.ravel()]).astype(np.int32)
    ref_acc = oracle.acc_sampled(c.A, c.W, ms, ns)
    if acc is not None:
        got = acc[ms, ns].astype(np.int64)
        assert np.array_equal(got, ref_acc), f"{c.name}: sampled int32 accumulator differs"
    accc = oracle.acc_centered_sampled(c.A, c.W, c.a_zero, c.w_zero, ms, ns)
    yref = accc.astype(np.float64) * c.a_scale[ms].astype(np.float64) * c.w_scale[ns].astype(np.float64)
    err = np.abs(y[ms, ns].astype(np.float64) - yref)
    assert np.all(err <= y_tolerance(yref)), f"{c.name}: sampled fp16 output outside tolerance"
    assert np.all(err <= ulp16(yref) + 1e-30)


def g128_tolerance(yref, mag, K):
    """Bound for the group-scaled path.  Its kernel adds G = ceil(K/128) exact integer group sums (both zero-point
    corrections applied in integers), each times a binary16 scale, in binary32: one rounding per fused multiply-add,
    over at most 8 partial sums of different waves, then the activation scale, before the one rounding to binary16.
    With u = 2^-24 every partial result is bounded by the size `mag` of the summed terms (the oracle's
    sum_g |a_scale * s_g * inner_g|), so the value before the last rounding is within (G + 12) u mag of the exact
    one; the last rounding adds half an ulp16, and a value that close to a rounding boundary may land on the
    neighbour: 1 ulp16 in all."""
    G = (K + 127) // 128
    return (G + 12) * 2.0 ** -24 * mag + 1.0 * ulp16(yref) + 2.0 ** -24


def check_g128(c, sh, zg, y):
    yref, _, mag = oracle.dequant_grouped(c.A, c.W, c.a_zero, c.a_scale, zg, sh, gs=128, want_mag=True)
    err = np.abs(y.astype(np.float64) - yref)
    tol = g128_tolerance(yref, mag, c.K)
    assert np.all(err <= tol), f"{c.name}: g128 output off by {np.max(err / tol):.3g} x bound"
    assert np.all(err <= y_tolerance(yref) + (c.K // 128 + 13) * 2.0 ** -24 * mag), f"{c.name}: outside the stated fp16 tolerance"
    return yref
