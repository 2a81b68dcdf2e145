"""Seeded synthetic inputs with the shapes and value distributions of the paper's kernel
benchmark (LLaMA-7B/13B linear-layer shapes, Sec. 4.4 and the appendix throughput tables).

This module only draws numbers.  It holds none of the method's arithmetic and is the one
piece of code that both the GPU tests/bench and the CPU oracle's callers use, so that both
sides see the same arrays.  Imports numpy only.
"""
from dataclasses import dataclass

import numpy as np

BASE_SEED = 24080854


def case_seed(cfg: int, p: int, q: int, shape_idx: int = 0, m_idx: int = 0) -> int:
    return BASE_SEED + 1_000_000 * cfg + 10_000 * (8 * (p - 1) + (q - 1)) + 100 * shape_idx + m_idx


@dataclass
class Case:
    p: int
    q: int
    M: int
    N: int
    K: int
    W: np.ndarray        # uint8 [N,K], codes < 2^p
    A: np.ndarray        # uint8 [M,K], codes < 2^q
    w_scale: np.ndarray  # float32 [N], fp16-representable
    w_zero: np.ndarray   # int32 [N], in code range
    a_scale: np.ndarray  # float32 [M]
    a_zero: np.ndarray   # int32 [M], in code range
    seed: int
    name: str = ""


def make_case(p, q, M, N, K, seed, act="uniform", name="") -> Case:
    """Draw order is fixed: W codes, A codes, w_scale, w_zero, a_scale, a_zero.

    act="uniform": A ~ U{0..2^q-1}, a_zero ~ U{0..2^q-1}.
    act="gauss":   A = clip(rint(N(mu, 30^2)), 0, 2^q-1) with mu = 2^(q-1), a_zero = mu
                   (a bell-shaped code histogram with rare far values, like real activations).
    a_scale = U[0.5,1] * 4096 / (K * 2^(p+q)) keeps |Y| far below the fp16 maximum.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    W = rng.integers(0, 1 << p, size=(N, K), dtype=np.uint8)
    if act == "uniform":
        A = rng.integers(0, 1 << q, size=(M, K), dtype=np.uint8)
    elif act == "gauss":
        mu = float(1 << (q - 1))
        A = np.clip(np.rint(rng.normal(mu, 30.0, size=(M, K))), 0, (1 << q) - 1).astype(np.uint8)
    else:
        raise ValueError(act)
    w_scale = rng.uniform(0.01, 0.1, size=N).astype(np.float16).astype(np.float32)
    w_zero = rng.integers(0, 1 << p, size=N).astype(np.int32)
    a_scale = (rng.uniform(0.5, 1.0, size=M) * 4096.0 / (K * float(1 << (p + q)))).astype(np.float32)
    if act == "gauss":
        a_zero = np.full(M, 1 << (q - 1), dtype=np.int32)
        rng.integers(0, 1 << q, size=M)  # keep the stream position independent of `act`
    else:
        a_zero = rng.integers(0, 1 << q, size=M).astype(np.int32)
    return Case(p, q, M, N, K, W, A, w_scale, w_zero, a_scale, a_zero, seed, name)


# The five benchmark configurations (LLaMA-7B q_proj / down_proj / up_proj, LLaMA-13B MLP).
SWEEP_SHAPES = [(5120, 13824), (13824, 5120)]   # (K, N)
SWEEP_M = [1, 16, 256, 2048]


def config1() -> Case:
    return make_case(2, 8, 1, 256, 512, case_seed(1, 2, 8), name="C1 tiny W2A8 GEMV")


def config2() -> Case:
    return make_case(4, 8, 1, 4096, 4096, case_seed(2, 4, 8), name="C2 W4A8 GEMV 4096x4096")


def config3(M: int) -> Case:
    assert 1 <= M <= 8
    return make_case(2, 8, M, 4096, 11008, case_seed(3, 2, 8, 0, M - 1), act="gauss",
                     name=f"C3 W2A8 GEMV M={M} 11008->4096")


def config4(M: int) -> Case:
    assert M in (128, 512)
    return make_case(6, 6, M, 11008, 4096, case_seed(4, 6, 6, 0, 0 if M == 128 else 1),
                     name=f"C4 W6A6 GEMM M={M} 4096->11008")


def config5(p: int, q: int, shape_idx: int, m_idx: int) -> Case:
    K, N = SWEEP_SHAPES[shape_idx]
    M = SWEEP_M[m_idx]
    return make_case(p, q, M, N, K, case_seed(5, p, q, shape_idx, m_idx),
                     name=f"C5 W{p}A{q} M={M} K={K} N={N}")


def bit_balance_case(q: int, M: int, N: int, K: int, seed: int, name: str = "") -> Case:
    """W2* (bit balance, Sec. 3.3): weights on the five levels {-2,-1,0,1,2}.  Five levels need three
    bits; they are carried as p = 3 codes level + 2 with zero-point 2 in every channel.  Levels are a
    rounded Gaussian (sigma 0.9) clipped to +-2: symmetric, like the near-normal weights the section
    describes.  Everything else as in make_case (same draw order)."""
    c = make_case(3, q, M, N, K, seed, act="gauss" if q == 8 else "uniform", name=name or f"W2*A{q} M={M} {K}->{N}")
    rng = np.random.Generator(np.random.PCG64(seed + 7))
    levels = np.clip(np.rint(rng.normal(0.0, 0.9, size=(N, K))), -2, 2).astype(np.int8)
    c.W = (levels + 2).astype(np.uint8)
    c.w_zero = np.full(N, 2, dtype=np.int32)
    return c


def config3_bit_balance(M: int) -> Case:
    return bit_balance_case(8, M, 4096, 11008, case_seed(3, 3, 8, 1, M - 1), name=f"W2*A8 GEMV M={M} 11008->4096")


def group_quant_params(c: Case, gs: int = 128):
    """Per-group weight parameters for case c (Appendix C, group size gs along K): binary16 scales
    ~ U[0.01, 0.1] as bit patterns [N][G] and zero-points uniform in the code range [N][G], G = ceil(K/gs)."""
    rng = np.random.Generator(np.random.PCG64(c.seed + 13))
    G = (c.K + gs - 1) // gs
    scale = rng.uniform(0.01, 0.1, size=(c.N, G)).astype(np.float16)
    zero = rng.integers(0, 1 << c.p, size=(c.N, G)).astype(np.int32)
    return scale.view(np.uint16).copy(), zero


def act_fp16(seed: int, M: int, K: int, outliers: bool = True) -> np.ndarray:
    """fp16 activations for the online quantizer: N(0,1) rows with a per-row gain and a few
    large-magnitude channels (the outlier structure LLM activations are known for)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.normal(0.0, 1.0, size=(M, K))
    x *= rng.uniform(0.25, 4.0, size=(M, 1))
    if outliers and K >= 8:
        cols = rng.choice(K, size=max(1, K // 512), replace=False)
        x[:, cols] *= 20.0
    return x.astype(np.float16)
