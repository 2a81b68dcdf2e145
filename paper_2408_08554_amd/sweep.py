"""Timing sweep of the matmul over (p, q, M, shape): `python -m paper_2408_08554_amd.sweep`.

The timed call is abq_gemm_act_codes where that is one kernel (decode shapes: activation pack fused
in) and abq_gemm on pre-packed activations elsewhere; `--entry gemm` times abq_gemm everywhere.
Prints one markdown table row per case: kernel time from a HIP-graph replay over rotating weight
blobs (>= 1 GiB in total, so the last-level cache cannot serve the weight stream), effective
TOPS = 2*M*N*K/t, packed-weight GB/s, and the fraction of the bound that applies (HBM 8 TB/s on
algorithmic bytes while M <= 39*p, else dense int8 MFMA 5 POP/s).  Codes are drawn on the GPU
(uniform, seeded); parity is the tests' business, not this tool's.
"""
import argparse
import sys

import torch

from . import binding as abq, metrics

SHAPES = {"13b_up": (5120, 13824), "13b_down": (13824, 5120), "7b_q": (4096, 4096), "7b_up": (4096, 11008),
          "7b_down": (11008, 4096)}


def time_case(p, q, M, K, N, family, launches, rotate_bytes, entry="auto"):
    layout = abq.ABQ_LAYOUT_PLANES if family == "bitserial" else abq.ABQ_LAYOUT_FIELDS
    g = torch.Generator(device="cuda").manual_seed(1000 * p + 10 * q + M % 7)
    W = torch.randint(0, 1 << p, (N, K), dtype=torch.uint8, device="cuda", generator=g)
    A = torch.randint(0, 1 << q, (M, K), dtype=torch.uint8, device="cuda", generator=g)
    ws = torch.full((N,), 0.05, device="cuda")
    wz = torch.randint(0, 1 << p, (N,), dtype=torch.int32, device="cuda", generator=g)
    a_s = torch.full((M,), 1e-4, device="cuda")
    az = torch.randint(0, 1 << q, (M,), dtype=torch.int32, device="cuda", generator=g)
    blob0 = abq.abq_pack_weights(p, W, ws, wz, layout)
    del W
    nb = blob0.numel()
    stride = (nb + 255) // 256 * 256
    R = max(2, min(launches, -(-rotate_bytes // nb)))
    pool = torch.empty(R * stride, dtype=torch.uint8, device="cuda")
    blobs = [pool[i * stride:i * stride + nb] for i in range(R)]
    for b in blobs:
        b.copy_(blob0)
    pa = abq.abq_pack_act_codes(q, A, a_s, az, layout)
    y = torch.empty((M, N), dtype=torch.float16, device="cuda")
    fused = entry != "gemm" and family != "bitserial" and abq.abq_gemm_act_codes_workspace_bytes(p, q, M, N, K, layout) == 0

    def call(i):
        if fused:
            abq.abq_gemm_act_codes(p, q, M, N, K, A, a_s, az, blobs[i % R], layout, y=y)
        else:
            abq.abq_gemm(p, q, M, N, K, pa, layout, blobs[i % R], layout, y=y)

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for i in range(3):
            call(i)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for i in range(launches):
                call(i)
        graph.replay()
        stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        graph.replay()
        e1.record(stream)
        torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / launches


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--p", default="1,2,3,4,5,6,7,8")
    ap.add_argument("--q", default="1,2,3,4,5,6,7,8")
    ap.add_argument("--m", default="1,16,256,2048")
    ap.add_argument("--shapes", default="13b_up,13b_down")
    ap.add_argument("--family", default="mfma", choices=["mfma", "bitserial"])
    ap.add_argument("--rotate-gib", type=float, default=1.0)
    ap.add_argument("--entry", default="auto", choices=["auto", "gemm"])
    args = ap.parse_args()
    abq.load()
    torch.cuda.set_device(0)
    print("| shape | K | N | M | p | q | us | TOPS | weight GB/s | bound | frac |")
    print("|---|---|---|---|---|---|---|---|---|---|---|")
    for shape in args.shapes.split(","):
        K, N = SHAPES[shape]
        for M in (int(v) for v in args.m.split(",")):
            for p in (int(v) for v in args.p.split(",")):
                for q in (int(v) for v in args.q.split(",")):
                    launches = 200 if M <= 16 else (40 if M <= 256 else 12)
                    t = time_case(p, q, M, K, N, args.family, launches, int(args.rotate_gib * 2 ** 30), args.entry)
                    tops = metrics.effective_tops(M, N, K, t)
                    if M <= 39 * p:
                        bound, frac = "hbm", metrics.gemm_algorithmic_bytes(p, q, M, N, K) / t / 8e12
                    else:
                        bound, frac = "mfma", tops / 5000.0
                    print(f"| {shape} | {K} | {N} | {M} | {p} | {q} | {t * 1e6:.2f} | {tops:.1f} | "
                          f"{metrics.weight_gbs(p, N, K, t):.0f} | {bound} | {frac:.3f} |", flush=True)
                    torch.cuda.empty_cache()


if __name__ == "__main__":
    sys.exit(main())
