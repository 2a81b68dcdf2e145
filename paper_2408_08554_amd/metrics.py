"""The paper's throughput metric and this build's byte counts (no kernels here)."""


def effective_tops(M: int, N: int, K: int, seconds: float) -> float:
    """TOPS = 2*M*N*K / time, independent of (p,q) (the definition Table 4 of the paper
    implies: 6.68 us <-> 5.01 TOPS for (1,4096)x(4096,4096))."""
    return 2.0 * M * N * K / seconds / 1e12


def packed_weight_stream_bytes(p: int, N: int, K: int) -> int:
    """Algorithmic weight bytes of one matmul: p bit-planes of N*K bits."""
    return p * N * K // 8


def weight_gbs(p: int, N: int, K: int, seconds: float) -> float:
    return packed_weight_stream_bytes(p, N, K) / seconds / 1e9


def gemm_algorithmic_bytes(p: int, q: int, M: int, N: int, K: int) -> int:
    """Bytes one abq_gemm call must move: packed weights, q-bit activations, the per-channel
    and per-token affine parameters and sums (12 B each), and the fp16 output."""
    return p * N * K // 8 + q * M * K // 8 + 12 * N + 12 * M + 2 * M * N
