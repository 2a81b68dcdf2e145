"""abq_gemm_act_codes_static (the entry point that allocates nothing) against abq_gemm_act_codes, through the
C ABI: two calls in a row, the second on a smaller problem, both on shapes whose packed activations go through
the scratch buffer; outputs must be equal bit for bit, and both are checked against the oracle."""
import numpy as np
import pytest

from paper_2408_08554_amd import synth
from helpers import check_against_oracle, to_dev

FIELDS = 2


@pytest.mark.gpu
def test_static_scratch_entry_point_matches_workspace_entry_point(abq):
    import torch
    #           p, q,   M,   N,    K      (two-kernel path: M above the decode range, or K not a multiple of 16)
    problems = [(4, 8, 300, 520, 2048), (6, 3, 70, 250, 1000), (2, 8, 5, 64, 1001)]
    for i, (p, q, M, N, K) in enumerate(problems):
        print(f"static scratch case W{p}A{q} M={M} N={N} K={K}", flush=True)
        c = synth.make_case(p, q, M, N, K, seed=synth.case_seed(7, p, q, i, 0), name=f"static W{p}A{q} {M}x{N}x{K}")
        need = abq.abq_gemm_act_codes_workspace_bytes(p, q, M, N, K, FIELDS)
        assert 0 < need <= abq.ABQ_STATIC_SCRATCH_BYTES, "the case must use the scratch buffer"
        pw = abq.abq_pack_weights(p, to_dev(torch, c.W), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero), FIELDS)
        a, s, z = to_dev(torch, c.A), to_dev(torch, c.a_scale), to_dev(torch, c.a_zero)
        y_ref, acc_ref = abq.abq_gemm_act_codes(p, q, M, N, K, a, s, z, pw, FIELDS, want_acc=True)
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        acc = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
        abq.abq_gemm_act_codes_static(p, q, M, N, K, a, s, z, pw, FIELDS, y, acc)
        torch.cuda.synchronize()
        assert torch.equal(acc, acc_ref), "int32 accumulator differs from abq_gemm_act_codes"
        assert torch.equal(y.view(torch.int16), y_ref.view(torch.int16)), "fp16 output differs from abq_gemm_act_codes"
        check_against_oracle(c, y.cpu().numpy(), acc.cpu().numpy())
    # a one-kernel decode shape needs no scratch and runs through the same entry point
    c = synth.make_case(4, 8, 3, 100, 2048, seed=synth.case_seed(7, 4, 8, 9, 0), name="static decode")
    assert abq.abq_gemm_act_codes_workspace_bytes(4, 8, 3, 100, 2048, FIELDS) == 0
    pw = abq.abq_pack_weights(4, to_dev(torch, c.W), to_dev(torch, c.w_scale), to_dev(torch, c.w_zero), FIELDS)
    y = torch.empty((3, 100), dtype=torch.float16, device="cuda")
    acc = torch.empty((3, 100), dtype=torch.int32, device="cuda")
    abq.abq_gemm_act_codes_static(4, 8, 3, 100, 2048, to_dev(torch, c.A), to_dev(torch, c.a_scale), to_dev(torch, c.a_zero), pw, FIELDS, y, acc)
    torch.cuda.synchronize()
    check_against_oracle(c, y.cpu().numpy(), acc.cpu().numpy())


@pytest.mark.gpu
def test_static_scratch_entry_point_rejects_what_does_not_fit(abq):
    import torch
    lib = abq.raw()
    # M = 4096 rows of K = 13824: 54 MiB of packed activations, beyond the 32 MiB buffer
    assert abq.abq_gemm_act_codes_workspace_bytes(8, 8, 4096, 5120, 13824, FIELDS) > abq.ABQ_STATIC_SCRATCH_BYTES
    t = torch.empty(64, dtype=torch.uint8, device="cuda")
    st = lib.abq_gemm_act_codes_static(8, 8, 4096, 5120, 13824, t.data_ptr(), t.data_ptr(), t.data_ptr(), t.data_ptr(), FIELDS,
                                       t.data_ptr(), None, None)
    assert st == abq.ABQ_ERR_SIZE
