"""Launch-plan search on the device: `python -m paper_2408_08554_amd.tune --shape p,q,M,N,K [--save plans.json]`.

The paper's engine picks its kernel configuration per problem size by timing candidates (Appendix D,
auto kernel search).  The library picks launch plans from closed-form rules; this tool times the
candidate plans of one exact problem size through the plan table of the C ABI (abq_plan_set), checks
that every candidate returns the default plan's result bit for bit (accumulator and fp16 output),
and reports them fastest first.  `--save` merges the winner into a JSON file when it beats the rule
by more than `--min-gain`; `load_plans(path)` installs such a file into the running process.

Timing: a HIP-graph replay over rotating weight blobs (>= 1 GiB in total).  The timed
call is abq_gemm_act_codes where that is one kernel, abq_gemm on packed activations elsewhere.
"""
import argparse
import itertools
import json
import os
import sys

import torch

from . import binding as abq

KNOBS = ("skinny_waves", "skinny_kgroups", "tiled_mt", "tiled_ntw", "tiled_wd", "tiled_band", "direct_r")


def candidates(p, q, M, N, K):
    """Plans worth timing for this problem (the knobs of the kernel family that does not run are left 0)."""
    out = [{}]
    nsuper = -(-K // 512)
    if M <= 16:     # the direct decode kernel with 1, 2 or 4 super-chunks per wave (a value that does not fit leaves the rule)
        for r in (1, 2, 4):
            if -(-nsuper // r) <= 16:
                out.append({"direct_r": r})
    if M <= 64:     # the streaming decode kernel (M <= 16 always; up to 64 when there are few output tiles)
        direct_off = {"direct_r": -1} if M <= 16 else {}
        if direct_off:
            out.append(dict(direct_off))
            out.append({"direct_r": -2})    # the shared-operand kernel (falls back to the streaming kernel where it does not fit)
        for w in (1, 2, 4, 5, 6, 7, 8):
            if w <= nsuper:
                out.append({"skinny_waves": w, **direct_off})
        if M > 8 and K >= 8192:
            for w, g in itertools.product((4, 6, 8), (2, 3, 4)):
                out.append({"skinny_waves": w, "skinny_kgroups": g, **direct_off})
    if M > 16:      # prefill kernel
        bands = sorted({b for b in (2, 4, 8, 16) if b <= max(2, -(-M // 64))})
        for mt, ntw in itertools.product((4, 8), (1, 2, 4)):
            for wd in ((2, 4) if mt == 4 and ntw <= 2 else (2,)):
                for band in bands:
                    out.append({"tiled_mt": mt, "tiled_ntw": ntw, "tiled_wd": wd, "tiled_band": band})
    return out


class Problem:
    """Synthetic operands of one problem size, resident on the device, with rotating copies of the weight blob."""

    def __init__(self, p, q, M, N, K, rotate_bytes=1 << 30, launches=100):
        self.shape = (p, q, M, N, K)
        self.launches = launches
        g = torch.Generator(device="cuda").manual_seed(77 + p + 10 * q)
        W = torch.randint(0, 1 << p, (N, K), dtype=torch.uint8, device="cuda", generator=g)
        self.A = torch.randint(0, 1 << q, (M, K), dtype=torch.uint8, device="cuda", generator=g)
        ws = torch.rand((N,), device="cuda", generator=g) * 0.09 + 0.01
        wz = torch.randint(0, 1 << p, (N,), dtype=torch.int32, device="cuda", generator=g)
        self.a_s = torch.rand((M,), device="cuda", generator=g) * 1e-4 + 1e-4
        self.az = torch.randint(0, 1 << q, (M,), dtype=torch.int32, device="cuda", generator=g)
        self.layout = abq.ABQ_LAYOUT_FIELDS
        blob0 = abq.abq_pack_weights(p, W, ws, wz, self.layout)
        nb = blob0.numel()
        stride = (nb + 255) // 256 * 256
        R = max(2, min(launches, -(-rotate_bytes // nb)))
        self.pool = torch.empty(R * stride, dtype=torch.uint8, device="cuda")
        self.blobs = [self.pool[i * stride:i * stride + nb] for i in range(R)]
        for b in self.blobs:
            b.copy_(blob0)
        self.pa = abq.abq_pack_act_codes(q, self.A, self.a_s, self.az, self.layout)
        self.fused = abq.abq_gemm_act_codes_workspace_bytes(p, q, M, N, K, self.layout) == 0
        self.y = torch.empty((M, N), dtype=torch.float16, device="cuda")
        self.acc = torch.empty((M, N), dtype=torch.int32, device="cuda")

    def call(self, i, acc=None):
        p, q, M, N, K = self.shape
        blob = self.blobs[i % len(self.blobs)]
        if self.fused:
            abq.abq_gemm_act_codes(p, q, M, N, K, self.A, self.a_s, self.az, blob, self.layout, y=self.y, acc=acc)
        else:
            abq.abq_gemm(p, q, M, N, K, self.pa, self.layout, blob, self.layout, y=self.y, acc=acc)

    def result(self):
        """(y bits, acc) of one call under the plan currently set."""
        self.y.fill_(float("nan"))
        self.acc.fill_(-1)
        self.call(0, acc=self.acc)
        torch.cuda.synchronize()
        return self.y.view(torch.int16).clone(), self.acc.clone()

    def time(self):
        """Seconds per launch under the plan currently set."""
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            for i in range(3):
                self.call(i)
            stream.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for i in range(self.launches):
                    self.call(i)
            graph.replay()
            stream.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            graph.replay()
            e1.record(stream)
            torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / self.launches


def search(p, q, M, N, K, launches=None, rotate_bytes=1 << 30, log=None, passes=4):
    """Times every candidate plan; returns [(seconds, plan dict)] fastest first.  The entry with the empty
    plan is the library's own rule.  Leaves the plan table as it found it for this problem."""
    if launches is None:
        launches = 200 if M <= 16 else (40 if M <= 256 else 12)
    before = abq.abq_plan_get(p, q, M, N, K)
    prob = Problem(p, q, M, N, K, rotate_bytes, launches)
    abq.abq_plan_set(p, q, M, N, K)          # the rule
    y0, acc0 = prob.result()
    plans = candidates(p, q, M, N, K)
    best = [float("inf")] * len(plans)

    def install(plan):
        if plan:
            abq.abq_plan_set(p, q, M, N, K, **plan)
        else:
            abq.abq_plan_set(p, q, M, N, K)

    try:
        for plan in plans:
            install(plan)
            y, acc = prob.result()
            if not (torch.equal(y, y0) and torch.equal(acc, acc0)):
                raise AssertionError(f"plan {plan} changes the result of {p, q, M, N, K}")
        # Timings depend on what ran before: the clock needs about half a second of load to settle, and a
        # candidate that follows a slow, low-occupancy one reads a few percent high.  So: an untimed warm-up, then
        # every candidate once per pass over several passes, each pass walking the list from another start and
        # in alternating direction, and each candidate keeps its fastest time.
        install(plans[0])
        for _ in range(8):
            prob.time()
        n = len(plans)
        for k in range(passes):
            order = [(k * n // passes + j) % n for j in range(n)]
            if k % 2:
                order.reverse()
            for i in order:
                install(plans[i])
                best[i] = min(best[i], prob.time())
        rows = list(zip(best, plans))
        if log:
            for t, plan in rows:
                log(f"{t * 1e6:9.2f} us  {plan or 'rule'}")
    finally:
        if any(before.values()):
            abq.abq_plan_set(p, q, M, N, K, **before)
        else:
            abq.abq_plan_set(p, q, M, N, K)
    rows.sort(key=lambda r: r[0])
    return rows


DEFAULT_PLANS = os.path.join(os.path.dirname(os.path.abspath(__file__)), "plans", "llama_mi355x.json")
"""Plans found by this search on an MI355X for LLaMA-7B/13B layer shapes (every entry at least 5 % ahead of the rule)."""


def load_plans(path=DEFAULT_PLANS):
    """Installs the plans of a file written by --save (default: the shipped table); returns how many."""
    with open(path) as f:
        table = json.load(f)
    for key, plan in table.items():
        p, q, M, N, K = (int(v) for v in key.split(","))
        abq.abq_plan_set(p, q, M, N, K, **{k: int(plan.get(k, 0)) for k in KNOBS})
    return len(table)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--shape", action="append", required=True, help="p,q,M,N,K (repeatable)")
    ap.add_argument("--save", help="JSON file to merge winning plans into")
    ap.add_argument("--min-gain", type=float, default=0.03, help="keep a plan only if it beats the rule by this fraction")
    args = ap.parse_args()
    abq.load()
    torch.cuda.set_device(0)
    table = {}
    if args.save:
        try:
            with open(args.save) as f:
                table = json.load(f)
        except FileNotFoundError:
            pass
    for shape in args.shape:
        p, q, M, N, K = (int(v) for v in shape.split(","))
        print(f"# W{p}A{q} M={M} N={N} K={K}", flush=True)
        rows = search(p, q, M, N, K, log=lambda s: print(s, flush=True))
        rule = next(t for t, plan in rows if not plan)
        best_t, best = rows[0]
        gain = rule / best_t - 1.0
        print(f"rule {rule * 1e6:.2f} us, best {best_t * 1e6:.2f} us ({best or 'rule'}), gain {gain * 100:.1f} %", flush=True)
        if best and gain >= args.min_gain:
            table[shape] = best
        else:
            table.pop(shape, None)
    if args.save:
        with open(args.save, "w") as f:
            json.dump(table, f, indent=1, sort_keys=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
