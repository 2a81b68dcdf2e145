"""Pins for the CPU oracle: every check here compares the oracle with something that is not
the oracle — brute force on the bits, a library matmul, closed forms, long-double
dequantise-then-multiply, numpy's own float16 conversion — so that a dropped term, a wrong
sign/index or a transposed operand in oracle/abq_oracle.c fails at least one of them.
CPU only."""
import itertools
import os

import numpy as np
import pytest

import oracle
from paper_2408_08554_amd import synth, metrics

RNG = np.random.Generator(np.random.PCG64(20240808))


def codes(shape, bits):
    return RNG.integers(0, 1 << bits, size=shape, dtype=np.uint8)


def brute_bits(A, W, p, q):
    """Literal Appendix B in pure Python ints: sum_{s<p,t<q} 2^(s+t) sum_k w^s_k AND x^t_k."""
    M, K = A.shape
    N = W.shape[0]
    out = np.zeros((M, N), dtype=object)
    for m in range(M):
        for n in range(N):
            y = 0
            for s in range(p):
                for t in range(q):
                    c = 0
                    for k in range(K):
                        c += ((int(W[n, k]) >> s) & 1) & ((int(A[m, k]) >> t) & 1)
                    y += c << (s + t)
            out[m, n] = y
    return out.astype(np.int64)


# ---- P1: brute force on tiny inputs -------------------------------------------------------

@pytest.mark.parametrize("p,q", list(itertools.product(range(1, 9), range(1, 9))))
def test_exhaustive_k1_all_codes(p, q):
    # every (a,w) code pair once: M = 2^q rows, N = 2^p rows, K = 1
    A = np.arange(1 << q, dtype=np.uint8).reshape(-1, 1)
    W = np.arange(1 << p, dtype=np.uint8).reshape(-1, 1)
    s = np.arange(p).reshape(1, 1, p, 1)
    t = np.arange(q).reshape(1, 1, 1, q)
    wb = (W.astype(np.int64).reshape(1, -1, 1, 1) >> s) & 1
    ab = (A.astype(np.int64).reshape(-1, 1, 1, 1) >> t) & 1
    expect = ((wb & ab) << (s + t)).sum(axis=(2, 3))
    assert np.array_equal(oracle.acc(A, W), expect)
    assert np.array_equal(oracle.acc_bitplane(oracle.pack_planes(A, q), oracle.pack_planes(W, p)), expect)


@pytest.mark.parametrize("p,q", [(1, 1), (2, 8), (3, 5), (4, 4), (8, 2), (8, 8), (7, 6), (1, 8)])
@pytest.mark.parametrize("K", [1, 2, 3, 31, 32, 33, 130])
def test_bruteforce_random_small(p, q, K):
    M, N = int(RNG.integers(1, 6)), int(RNG.integers(1, 6))
    A, W = codes((M, K), q), codes((N, K), p)
    expect = brute_bits(A, W, p, q)
    assert np.array_equal(oracle.acc(A, W), expect)
    assert np.array_equal(oracle.acc_bitplane(oracle.pack_planes(A, q), oracle.pack_planes(W, p)), expect)


def test_two_bit_worked_identity():
    # Sec. 3.4: w*x = OP(w,x^1)*2 + OP(w,x^0) for a 2-bit x; with 1-bit w, OP is AND.
    for w in (0, 1):
        for x in range(4):
            x1, x0 = (x >> 1) & 1, x & 1
            got = oracle.acc(np.array([[x]], dtype=np.uint8), np.array([[w]], dtype=np.uint8))[0, 0]
            assert got == (w & x1) * 2 + (w & x0) == w * x


# ---- P2: p = q = 8 is an ordinary integer matmul ------------------------------------------

@pytest.mark.parametrize("M,N,K", [(1, 7, 64), (5, 33, 257), (16, 48, 1000)])
def test_w8a8_equals_library_matmul(M, N, K):
    A, W = codes((M, K), 8), codes((N, K), 8)
    lib = A.astype(np.int64) @ W.astype(np.int64).T
    assert np.array_equal(oracle.acc(A, W), lib)
    assert np.array_equal(oracle.acc_bitplane(oracle.pack_planes(A, 8), oracle.pack_planes(W, 8)), lib)
    ms = RNG.integers(0, M, size=50)
    ns = RNG.integers(0, N, size=50)
    assert np.array_equal(oracle.acc_sampled(A, W, ms, ns), lib[ms, ns])


def test_operand_roles_not_transposed():
    # acc is [M,N] with A indexed by m and W by n: a non-square, asymmetric case.
    A = np.array([[1, 2, 3]], dtype=np.uint8)           # M=1
    W = np.array([[1, 0, 0], [0, 1, 0], [0, 0, 1], [1, 1, 1]], dtype=np.uint8)  # N=4
    assert oracle.acc(A, W).tolist() == [[1, 2, 3, 6]]


# ---- P3: closed forms ---------------------------------------------------------------------

@pytest.mark.parametrize("p,q", [(1, 1), (2, 8), (6, 6), (8, 8), (3, 7)])
def test_closed_forms(p, q):
    M, N, K = 3, 4, 517
    amax, wmax = (1 << q) - 1, (1 << p) - 1
    A = np.full((M, K), amax, dtype=np.uint8)
    W = np.full((N, K), wmax, dtype=np.uint8)
    assert (oracle.acc(A, W) == K * amax * wmax).all()
    assert (oracle.acc_bitplane(oracle.pack_planes(A, q), oracle.pack_planes(W, p)) == K * amax * wmax).all()
    Z = np.zeros_like(A)
    Wr = codes((N, K), p)
    assert (oracle.acc(Z, Wr) == 0).all()
    # one-hot activation row picks out one weight column, scaled
    k0, v = 123, amax
    H = np.zeros((1, K), dtype=np.uint8)
    H[0, k0] = v
    assert np.array_equal(oracle.acc(H, Wr)[0], v * Wr[:, k0].astype(np.int64))


# ---- P4: invariants -----------------------------------------------------------------------

def test_plane_composition_and_padding_and_symmetry():
    p, q, M, N, K = 5, 7, 4, 6, 200
    A, W = codes((M, K), q), codes((N, K), p)
    full = oracle.acc(A, W)
    # (1,1) kernel composes every other: acc(p,q) = sum 2^(s+t) acc(1,1)(A_t, W_s)
    comp = np.zeros_like(full)
    for s in range(p):
        for t in range(q):
            comp += oracle.acc(((A >> t) & 1).astype(np.uint8), ((W >> s) & 1).astype(np.uint8)) << (s + t)
    assert np.array_equal(comp, full)
    # zero-padding K changes nothing
    Ap = np.concatenate([A, np.zeros((M, 56), np.uint8)], axis=1)
    Wp = np.concatenate([W, codes((N, 56), p)], axis=1)
    assert np.array_equal(oracle.acc(Ap, Wp), full)
    # row / column permutation equivariance
    pm, pn, pk = RNG.permutation(M), RNG.permutation(N), RNG.permutation(K)
    assert np.array_equal(oracle.acc(A[pm][:, pk], W[pn][:, pk]), full[pm][:, pn])
    # transposition symmetry with the roles (and p,q) swapped
    assert np.array_equal(oracle.acc(W, A), full.T)
    # masking to the low p' bits == dropping the upper planes
    pl = oracle.pack_planes(W, p)
    assert np.array_equal(oracle.acc_bitplane(oracle.pack_planes(A, q), pl[:3]),
                          oracle.acc(A, (W & 7).astype(np.uint8)))


# ---- P5/P6/P7: zero points and dequant ----------------------------------------------------

@pytest.mark.parametrize("p,q,M,N,K", [(2, 8, 1, 9, 512), (6, 6, 7, 5, 333), (8, 8, 3, 3, 1024), (1, 1, 2, 2, 65)])
def test_centered_equals_four_term_expansion(p, q, M, N, K):
    A, W = codes((M, K), q), codes((N, K), p)
    az = RNG.integers(0, 1 << q, size=M).astype(np.int32)
    wz = RNG.integers(0, 1 << p, size=N).astype(np.int32)
    direct = oracle.acc_centered(A, W, az, wz)
    A64, W64 = A.astype(np.int64), W.astype(np.int64)
    raw = A64 @ W64.T
    asum = A64.sum(axis=1)[:, None]
    wsum = W64.sum(axis=1)[None, :]
    expanded = raw - wz[None, :].astype(np.int64) * asum - az[:, None].astype(np.int64) * wsum \
        + K * az[:, None].astype(np.int64) * wz[None, :].astype(np.int64)
    assert np.array_equal(direct, expanded)
    ms = RNG.integers(0, M, size=20)
    ns = RNG.integers(0, N, size=20)
    assert np.array_equal(oracle.acc_centered_sampled(A, W, az, wz, ms, ns), expanded[ms, ns])


def test_unit_scales_zero_points_give_exact_half():
    A, W = codes((2, 40), 3), codes((5, 40), 3)     # acc <= 40*49 = 1960 < 2048: exact in fp16
    raw = oracle.acc(A, W)
    accc = oracle.acc_centered(A, W, np.zeros(2, np.int32), np.zeros(5, np.int32))
    assert np.array_equal(accc, raw)
    y, y16 = oracle.dequant(accc, np.ones(2, np.float32), np.ones(5, np.float32))
    assert np.array_equal(y, raw.astype(np.float64))
    assert np.array_equal(y16.view(np.float16).astype(np.int64), raw)


def test_dequant_equals_dequantise_then_multiply_longdouble():
    c = synth.make_case(4, 8, 3, 17, 300, seed=77)
    accc = oracle.acc_centered(c.A, c.W, c.a_zero, c.w_zero)
    y, _ = oracle.dequant(accc, c.a_scale, c.w_scale)
    ld = np.longdouble
    Ar = c.a_scale.astype(ld)[:, None] * (c.A.astype(ld) - c.a_zero.astype(ld)[:, None])
    Wr = c.w_scale.astype(ld)[:, None] * (c.W.astype(ld) - c.w_zero.astype(ld)[:, None])
    ref = np.zeros((c.M, c.N), dtype=ld)
    for k in range(c.K):
        ref += Ar[:, k][:, None] * Wr[:, k][None, :]
    scale = np.abs(Ar).astype(ld) @ np.abs(Wr).astype(ld).T
    assert np.all(np.abs(y.astype(ld) - ref) <= 1e-12 * scale + 1e-300)


def test_dequant_scale_roles_not_swapped():
    accc = np.array([[1, 1], [1, 1], [1, 1]], dtype=np.int64)      # M=3, N=2
    y, _ = oracle.dequant(accc, np.array([1, 2, 4], np.float32), np.array([8, 16], np.float32))
    assert y.tolist() == [[8, 16], [16, 32], [32, 64]]


# ---- P8: binary16 rounding against the library conversion ---------------------------------

def test_half_rounding_matches_numpy():
    probes = [0.0, -0.0, 1.0, -1.0, 65504.0, 65519.99, 65520.0, 70000.0, -65520.0, 1e-8, 2.0 ** -24,
              2.0 ** -25, 2.0 ** -25 * 1.0000001, 3 * 2.0 ** -25, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25,
              1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -11 + 1e-9, 2047.5, 2048.5, 2049.5, 0.1, 1 / 3,
              float("inf"), float("-inf")]
    vals = np.concatenate([
        np.array(probes, dtype=np.float64),
        RNG.normal(0, 1, 4000) * np.exp(RNG.uniform(-20, 12, 4000)),
        # exact ties between neighbouring halves
        (np.arange(1024, 1536) + 0.5) * 2.0 ** -10,
    ])
    with np.errstate(over="ignore"):
        lib = vals.astype(np.float16).view(np.uint16)
    mine = np.array([oracle.half_bits(v) for v in vals], dtype=np.uint16)
    assert np.array_equal(mine, lib)
    assert oracle.half_bits(float("nan")) & 0x7C00 == 0x7C00 and oracle.half_bits(float("nan")) & 0x3FF


# ---- P9: packers --------------------------------------------------------------------------

@pytest.mark.parametrize("bits,R,K", [(1, 3, 1), (2, 4, 33), (5, 2, 100), (8, 3, 256), (7, 1, 1000)])
def test_pack_unpack_planes(bits, R, K):
    c = codes((R, K), bits)
    pl = oracle.pack_planes(c, bits)
    assert pl.shape == (bits, R, (K + 31) // 32)
    assert np.array_equal(oracle.unpack_planes(pl, K), c)
    # popcount of plane s over a row = number of codes with bit s set; bit order k%32 LSB-first
    for s in range(bits):
        for r in range(R):
            row_bits = np.unpackbits(pl[s, r].view(np.uint8), bitorder="little")
            assert np.array_equal(row_bits[:K], (c[r] >> s) & 1)
            assert row_bits[K:].sum() == 0
    # wider row stride keeps the same bits
    pl2 = oracle.pack_planes(c, bits, Kw=(K + 31) // 32 + 3)
    assert np.array_equal(pl2[:, :, :pl.shape[2]], pl) and pl2[:, :, pl.shape[2]:].sum() == 0


# ---- activation quantizer: invariants only (parity unpinned by the paper) -----------------

@pytest.mark.parametrize("q", [1, 2, 4, 6, 8])
def test_quant_act_invariants(q):
    x = synth.act_fp16(1234 + q, 6, 300)
    x[4] = 0                      # degenerate row
    x[5] = np.abs(x[5])           # one-sided row: lo = 0
    cd, sc, zp = oracle.quant_act(x, q)
    qmax = (1 << q) - 1
    assert cd.max() <= qmax and zp.min() >= 0 and zp.max() <= qmax
    assert sc[4] == 1.0 and zp[4] == 0 and (cd[4] == 0).all()
    assert zp[5] == 0
    xf = x.astype(np.float64)
    recon = sc.astype(np.float64)[:, None] * (cd.astype(np.float64) - zp[:, None])
    # inside the representable range the error is at most half a step (plus fp32 slack);
    # the zero-point rounding can clip up to half a step more at the two ends
    lo = np.minimum(xf.min(axis=1), 0)
    hi = np.maximum(xf.max(axis=1), 0)
    step = sc.astype(np.float64)[:, None]
    assert np.all(np.abs(recon - xf) <= step * (1.0 + 1e-3))
    inner = (xf > (lo[:, None] + step)) & (xf < (hi[:, None] - step))
    assert np.all(np.abs(recon - xf)[inner] <= step.repeat(x.shape[1], 1)[inner] * (0.5 + 1e-3))
    # a row that already lies on a grid round-trips exactly
    grid = (np.arange(300) % (qmax + 1)).astype(np.float16).reshape(1, -1)
    cg, sg, zg = oracle.quant_act(grid, q)
    assert sg[0] == 1.0 and zg[0] == 0 and np.array_equal(cg[0], grid[0].astype(np.uint8))
    # monotone: larger x never gets a smaller code
    order = np.argsort(xf[0], kind="stable")
    assert np.all(np.diff(cd[0][order].astype(np.int32)) >= 0)


# ---- ReQuant with given per-token parameters (parity unpinned by the paper) ---------------------

@pytest.mark.parametrize("q", [1, 3, 4, 8])
def test_requant_pins(q):
    qmax = (1 << q) - 1
    # (1) with the per-token quantizer's own Delta and z it IS that quantizer (a function pinned on its own)
    x = synth.act_fp16(4321 + q, 5, 257)
    cd, sc, zp = oracle.quant_act(x, q)
    assert np.array_equal(oracle.requant(x, q, sc, zp), cd)
    # (2) values on the grid Delta*(c - z) come back as c (Delta a power of two: the grid is exact in binary16)
    for delta, z in ((0.25, 0), (2.0, qmax // 2), (0.5, qmax)):
        c = np.arange(qmax + 1, dtype=np.int64)
        y = (delta * (c - z)).astype(np.float16).reshape(1, -1)
        got = oracle.requant(y, q, np.array([delta], np.float32), np.array([z], np.int32))
        assert np.array_equal(got[0], c.astype(np.uint8))
    # (3) saturation at both ends, also where the quotient is far outside any integer type's comfort
    y = np.array([[65504.0, -65504.0, 0.0, 1e-4, -1e-4]], dtype=np.float16)
    got = oracle.requant(y, q, np.array([1e-7], np.float32), np.array([qmax // 2], np.int32))
    assert list(got[0]) == [qmax, 0, qmax // 2, qmax, 0]
    # (4) ties go to the even integer: y / Delta = 0.5, 1.5, 2.5, -0.5 -> 0, 2, 2, 0 (before the zero-point)
    if q >= 3:
        y = np.array([[0.5, 1.5, 2.5, -0.5, 3.5]], dtype=np.float16)
        got = oracle.requant(y, q, np.array([1.0], np.float32), np.array([1], np.int32))
        assert list(got[0]) == [1, 3, 3, 1, 5]
    # (5) the zero-point and the step are the row's own; monotone in y
    y = np.sort(synth.act_fp16(99, 1, 400)[0]).reshape(1, -1).repeat(2, axis=0)
    got = oracle.requant(y, q, np.array([0.125, 0.5], np.float32), np.array([0, qmax], np.int32))
    assert np.all(np.diff(got.astype(np.int32), axis=1) >= 0)
    assert got[1].max() == qmax and (q == 1 or not np.array_equal(got[0], got[1]))


# ---- the metric itself, against the values the paper prints -------------------------------

def test_tops_definition_matches_table4():
    path = os.path.join(os.path.dirname(__file__), "golden", "table4_latency_tops.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 5
    for M, N, K, us, tops in rows:
        got = metrics.effective_tops(int(M), int(N), int(K), float(us) * 1e-6)
        assert abs(got - float(tops)) <= 0.015, (us, got, tops)
    assert metrics.packed_weight_stream_bytes(4, 4096, 4096) == 8 * 1024 * 1024
    assert metrics.packed_weight_stream_bytes(2, 4096, 11008) == 11272192


# ---- generator sanity (ranges, determinism) -----------------------------------------------

def test_synth_cases():
    c = synth.config1()
    assert (c.p, c.q, c.M, c.N, c.K) == (2, 8, 1, 256, 512)
    assert c.W.max() <= 3 and c.A.dtype == np.uint8 and c.w_zero.max() <= 3
    assert np.array_equal(c.w_scale, c.w_scale.astype(np.float16).astype(np.float32))
    c2 = synth.config1()
    assert np.array_equal(c.W, c2.W) and np.array_equal(c.a_scale, c2.a_scale)
    g = synth.make_case(2, 8, 2, 8, 2048, seed=5, act="gauss")
    assert (g.a_zero == 128).all() and 100 < g.A.mean() < 156
    y, _ = oracle.dequant(oracle.acc_centered(c.A, c.W, c.a_zero, c.w_zero), c.a_scale, c.w_scale)
    assert np.abs(y).max() < 410


# ---- RMSNorm (the producer the activation quantizer is fused into) ---------------------------
# No printed formula or worked example in the paper: pinned against a float64 evaluation of the standard
# definition, closed forms, and invariances that the exact sum of squares gives bit for bit.

def _ulp16(v):
    return 2.0 ** (np.floor(np.log2(np.maximum(np.abs(v), 2.0 ** -14))) - 10)


@pytest.mark.parametrize("M,K,eps", [(1, 512, 1e-5), (3, 1000, 1e-6), (2, 4096, 1e-5), (5, 37, 0.0), (1, 11008, 1e-5)])
def test_rmsnorm_matches_float64_definition(M, K, eps):
    rng = np.random.Generator(np.random.PCG64(1000 + K))
    x = (rng.standard_normal((M, K)) * rng.uniform(0.05, 8.0, (M, 1))).astype(np.float16)
    x[:, rng.integers(0, K, 3)] *= np.float16(20.0)                      # outlier channels
    g = (1.0 + 0.2 * rng.standard_normal(K)).astype(np.float16)
    y = oracle.rmsnorm_half(x, g, eps)
    xr = x.astype(np.float64)
    ref = xr / np.sqrt((xr ** 2).mean(axis=1, keepdims=True) + np.float64(np.float32(eps))) * g.astype(np.float64)
    # one rounding to binary16 (half an ulp) plus three binary32 roundings before it (2^-13 of an ulp16 each)
    assert np.all(np.abs(y.astype(np.float64) - ref) <= 0.501 * _ulp16(ref))


def test_rmsnorm_closed_forms():
    K = 1024
    # constant row, unit gain, no eps: every output is exactly +-1
    for c in (3.0, -0.37, 1000.0, 6e-5):
        x = np.full((1, K), c, dtype=np.float16)
        y = oracle.rmsnorm_half(x, np.ones(K, dtype=np.float16), 0.0)
        assert np.all(y == np.float16(np.sign(c)))
    # one-hot row: mean = a^2/K, so the hot output is sqrt(K) * gamma * sign(a) and the rest stay zero
    x = np.zeros((1, K), dtype=np.float16)
    x[0, 17] = -2.5
    g = np.full(K, 0.75, dtype=np.float16)
    y = oracle.rmsnorm_half(x, g, 0.0)
    assert y[0, 17] == np.float16(-32.0 * 0.75) and np.count_nonzero(y) == 1
    # all-zero row with eps: zeros (0 * finite)
    y = oracle.rmsnorm_half(np.zeros((2, 64), dtype=np.float16), np.ones(64, dtype=np.float16), 1e-5)
    assert not y.any()
    # eps dominates: x = 2^-10 everywhere, eps = 1 -> y = x / sqrt(2^-20 + 1) rounds to x itself
    x = np.full((1, 256), 2.0 ** -10, dtype=np.float16)
    assert np.all(oracle.rmsnorm_half(x, np.ones(256, dtype=np.float16), 1.0) == np.float16(2.0 ** -10))


def test_rmsnorm_invariances_are_bit_exact():
    rng = np.random.Generator(np.random.PCG64(77))
    K = 777
    x = rng.standard_normal((4, K)).astype(np.float16)
    g = rng.uniform(0.5, 1.5, K).astype(np.float16)
    y = oracle.rmsnorm_half(x, g, 0.0)
    # a power-of-two gain on the input cancels exactly when eps = 0 (every step scales exactly)
    for s in (0.25, 4.0):
        assert np.array_equal(oracle.rmsnorm_half((x * np.float16(s)).astype(np.float16), g, 0.0).view(np.uint16), y.view(np.uint16))
    # permuting the channels (of x and gamma alike) permutes the outputs: the sum of squares is exact, so
    # it cannot depend on the order of the terms
    perm = rng.permutation(K)
    yp = oracle.rmsnorm_half(np.ascontiguousarray(x[:, perm]), np.ascontiguousarray(g[perm]), 1e-5)
    assert np.array_equal(yp.view(np.uint16), oracle.rmsnorm_half(x, g, 1e-5)[:, perm].view(np.uint16))
    # rows are independent, and flipping the sign of a row flips its outputs
    assert np.array_equal(oracle.rmsnorm_half(x[1:2], g, 1e-5), oracle.rmsnorm_half(x, g, 1e-5)[1:2])
    assert np.array_equal(oracle.rmsnorm_half(-x, g, 1e-5), -oracle.rmsnorm_half(x, g, 1e-5))
    # the exact sum copes with terms 2^60 apart (a float or double running sum would drop the small ones):
    # one huge element and 4095 tiny ones whose squares together shift the mean by less than one part in 2^53
    x = np.full((1, 4096), 6e-5, dtype=np.float16)
    x[0, 0] = 60000.0
    y = oracle.rmsnorm_half(x, np.ones(4096, dtype=np.float16), 0.0)
    assert y[0, 0] == np.float16(64.0) and np.all(y[0, 1:] == np.float16(np.float64(x[0, 1]) * 64.0 / 60000.0))


# ---- SiLU(gate) * up (the second producer the quantizer is fused into) ------------------------------

def test_silu_mul_matches_float64_definition():
    rng = np.random.Generator(np.random.PCG64(2024))
    g = (rng.standard_normal((6, 3000)) * rng.uniform(0.1, 12.0, (6, 1))).astype(np.float16)
    u = (rng.standard_normal((6, 3000)) * 3.0).astype(np.float16)
    h = oracle.silu_mul_half(g, u)
    gd = g.astype(np.float64)
    ref = gd / (1.0 + np.exp(-gd)) * u.astype(np.float64)
    # half an ulp of binary16 for the final rounding; the binary32 steps before it (polynomial exp within
    # 2e-7, one add, one division, one product) add less than a thousandth of that
    assert np.all(np.abs(h.astype(np.float64) - ref) <= 0.501 * _ulp16(ref))


def test_silu_mul_closed_forms_and_limits():
    one = np.ones((1, 8), dtype=np.float16)
    g = np.array([[0.0, -0.0, 100.0, -100.0, 60000.0, -60000.0, 1e-4, -1e-4]], dtype=np.float16)
    h = oracle.silu_mul_half(g, one)
    assert h[0, 0] == 0 and h[0, 1] == 0                        # silu(0) = 0
    assert h[0, 2] == np.float16(100.0) and h[0, 4] == np.float16(60000.0)     # exp(-g) vanishes: silu(g) = g
    assert h[0, 3] == 0 and h[0, 5] == 0                        # g * exp(g) underflows binary16
    assert h[0, 6] == np.float16(np.float64(g[0, 6]) / 2) and h[0, 7] == np.float16(np.float64(g[0, 7]) / 2)   # silu(g) ~ g/2 near 0
    # the second operand multiplies: zero, sign, and a power of two pass through exactly
    g = np.linspace(-8, 8, 64, dtype=np.float16).reshape(1, 64)
    base = oracle.silu_mul_half(g, np.ones_like(g))
    assert not oracle.silu_mul_half(g, np.zeros_like(g)).any()
    assert np.array_equal(oracle.silu_mul_half(g, -np.ones_like(g)), -base)
    assert np.array_equal(oracle.silu_mul_half(g, np.full_like(g, 4.0)).astype(np.float64), base.astype(np.float64) * 4.0)
    # silu(g) - silu(-g) = g: holds to rounding
    b64 = base.astype(np.float64)[0]
    assert np.all(np.abs(b64 - b64[::-1] - g.astype(np.float64)[0]) <= 2 * _ulp16(g.astype(np.float64)[0]))
    # silu has its minimum -0.2785 at g = -1.2785 and increases from there on
    gpos = np.linspace(-1.25, 12.0, 500, dtype=np.float16).reshape(1, 500)
    hp = oracle.silu_mul_half(gpos, np.ones_like(gpos)).astype(np.float64)[0]
    assert np.all(np.diff(hp) >= 0) and abs(oracle.silu_mul_half(np.array([[-1.2785]], dtype=np.float16), np.ones((1, 1), dtype=np.float16))[0, 0] + 0.2785) < 3e-4


# ---- bit balance (Sec. 3.3): five weight levels carried as three-bit codes ------------------

def test_bit_balance_levels_equal_three_bit_codes_with_zero_point_two():
    """W2* weights take the levels {-2..2}.  The engine has no level type: the levels ride as p = 3 codes
    level + 2 with zero-point 2.  The centered sum over codes must equal the plain integer product with
    the signed levels, and the dequantised value the real-valued product s_a (A - z_a) . s_w level."""
    c = synth.bit_balance_case(8, 3, 7, 300, seed=99)
    levels = c.W.astype(np.int64) - 2
    assert levels.min() == -2 and levels.max() == 2 and set(np.unique(c.W)) <= {0, 1, 2, 3, 4}
    assert abs(float(levels.mean())) < 0.1                      # symmetric level histogram
    direct = (c.A.astype(np.int64) - c.a_zero[:, None]) @ levels.T
    accc = oracle.acc_centered(c.A, c.W, c.a_zero, c.w_zero)
    assert np.array_equal(accc, direct)
    planes = oracle.acc_bitplane(oracle.pack_planes(c.A, 8), oracle.pack_planes(c.W, 3))
    assert np.array_equal(planes, c.A.astype(np.int64) @ c.W.astype(np.int64).T)
    y, _ = oracle.dequant(accc, c.a_scale, c.w_scale)
    real = ((c.A.astype(np.float64) - c.a_zero[:, None]) * c.a_scale[:, None].astype(np.float64)) @ \
           (levels.astype(np.float64) * c.w_scale[:, None].astype(np.float64)).T
    assert np.allclose(y, real, rtol=1e-12, atol=0)


# ---- per-group weight scales and zero-points (Appendix C) ------------------------------------

def _grouped_case(p, q, M, N, K, seed, gs):
    c = synth.make_case(p, q, M, N, K, seed=seed)
    sh, zg = synth.group_quant_params(c, gs)
    return c, sh, zg


def test_grouped_one_group_is_the_per_channel_result():
    c, sh, zg = _grouped_case(4, 8, 3, 9, 200, 501, gs=256)          # gs >= K: one group per row
    assert sh.shape == (9, 1)
    y, y16 = oracle.dequant_grouped(c.A, c.W, c.a_zero, c.a_scale, zg, sh, gs=256)
    accc = oracle.acc_centered(c.A, c.W, c.a_zero, zg[:, 0])
    yc, yc16 = oracle.dequant(accc, c.a_scale, sh.view(np.float16)[:, 0].astype(np.float32))
    assert np.array_equal(y16, yc16) and np.allclose(y, yc, rtol=1e-15, atol=0)


def test_grouped_equal_parameters_in_every_group_is_the_per_channel_result():
    c, sh, zg = _grouped_case(3, 5, 2, 6, 700, 502, gs=128)
    sh[:] = sh[:, :1]
    zg[:] = zg[:, :1]
    y, _ = oracle.dequant_grouped(c.A, c.W, c.a_zero, c.a_scale, zg, sh, gs=128)
    yc, _ = oracle.dequant(oracle.acc_centered(c.A, c.W, c.a_zero, zg[:, 0]), c.a_scale,
                           sh.view(np.float16)[:, 0].astype(np.float32))
    assert np.allclose(y, yc, rtol=1e-13, atol=0)


@pytest.mark.parametrize("p,q,M,N,K,gs", [(4, 8, 3, 5, 300, 128), (2, 8, 1, 7, 1024, 128), (8, 8, 2, 3, 129, 128),
                                          (6, 6, 4, 4, 1000, 64), (1, 1, 2, 2, 513, 128)])
def test_grouped_equals_dequantise_then_multiply(p, q, M, N, K, gs):
    """The definition taken the other way round: dequantise every weight with the parameters of ITS group
    (group of k is k // gs, the last one short), dequantise the activations, multiply as real matrices."""
    c, sh, zg = _grouped_case(p, q, M, N, K, 503 + K, gs)
    y, y16, mag = oracle.dequant_grouped(c.A, c.W, c.a_zero, c.a_scale, zg, sh, gs=gs, want_mag=True)
    gk = np.arange(K) // gs
    s_real = sh.view(np.float16).astype(np.longdouble)[:, gk]                       # [N][K]
    w_real = s_real * (c.W.astype(np.longdouble) - zg[:, gk].astype(np.longdouble))
    a_real = c.a_scale[:, None].astype(np.longdouble) * (c.A.astype(np.longdouble) - c.a_zero[:, None])
    real = a_real @ w_real.T
    assert np.all(np.abs(y - real.astype(np.float64)) <= 1e-12 * mag + 1e-300)
    assert np.all(mag >= np.abs(y) * (1 - 1e-12))
    assert np.array_equal(y16, np.array([[oracle.half_bits(v) for v in row] for row in y], dtype=np.uint16))


def test_grouped_single_live_group_uses_that_groups_scale_and_zero():
    """Weights equal to their group's zero-point contribute nothing; leave one group live and the result is
    that group's scale times its integer sum, for a middle group and for the short last one."""
    c, sh, zg = _grouped_case(4, 8, 2, 5, 300, 504, gs=128)          # groups: 128, 128, 44
    G = 3
    for live in range(G):
        W = np.repeat(zg, 128, axis=1)[:, :300].astype(np.uint8)
        lo, hi = live * 128, min(live * 128 + 128, 300)
        W[:, lo:hi] = c.W[:, lo:hi]
        y, _ = oracle.dequant_grouped(c.A, W, c.a_zero, c.a_scale, zg, sh, gs=128)
        inner = (c.A[:, lo:hi].astype(np.int64) - c.a_zero[:, None]) @ (W[:, lo:hi].astype(np.int64) - zg[:, live:live + 1]).T
        expect = c.a_scale[:, None].astype(np.float64) * sh.view(np.float16)[:, live].astype(np.float64)[None, :] * inner
        assert np.allclose(y, expect, rtol=1e-15, atol=0)


# ---- residual add in front of the normalization ------------------------------------------------

def test_add_half_matches_numpy_two_step_rounding_and_identities():
    rng = np.random.Generator(np.random.PCG64(77))
    with np.errstate(over="ignore"):          # a few values are meant to overflow to infinity
        a = (rng.standard_normal(20000) * rng.choice([1e-4, 1.0, 300.0, 3e4], 20000)).astype(np.float16)
        b = (rng.standard_normal(20000) * rng.choice([1e-6, 1.0, 300.0, 3e4], 20000)).astype(np.float16)
    got = oracle.add_half(a, b)
    with np.errstate(over="ignore"):
        lib = (a.astype(np.float32) + b.astype(np.float32)).astype(np.float16)        # numpy: IEEE add, RNE conversion
    assert np.array_equal(got.view(np.uint16), lib.view(np.uint16))
    assert np.array_equal(oracle.add_half(b, a).view(np.uint16), got.view(np.uint16))                 # commutative
    assert np.array_equal(oracle.add_half(a, np.zeros_like(a)).view(np.uint16), (a + np.float16(0)).view(np.uint16))
    fin = np.isfinite(a)
    assert np.all(oracle.add_half(a[fin], -a[fin]) == 0)
    ties = oracle.add_half(np.array([2048, 2048, 1, 60000], np.float16), np.array([1, 3, 2.0 ** -24, 60000], np.float16))
    assert ties.tolist()[:3] == [2048.0, 2052.0, 1.0] and np.isinf(ties[3])         # ties to even; overflow to infinity
