"""GPU test of fg_gemm_noalloc, the entry point for callers that cannot allocate device memory:
its output against fg_gemm's (and against the oracle) on two calls in a row, the second smaller."""
import numpy as np
import pytest
import torch

from paper_2009_12263_amd import binding as fg
from paper_2009_12263_amd import workloads as W
from tests.parity import run_gemm_case

pytestmark = pytest.mark.gpu


def say(msg):
    print("[case] " + msg, flush=True)


def scratch_bytes(plan: str, M: int, N: int) -> int:
    """Bytes of partial products a split plan keeps: (tiles x K ranges x tile bytes), from the plan name."""
    import re
    m = re.match(r".*_(\d+)x(\d+)x\d+(?:_\w+)?\+splitk(\d+)$", plan)
    bm, bn, S = int(m.group(1)), int(m.group(2)), int(m.group(3))
    return -(-M // bm) * -(-N // bn) * S * bm * bn * 4


def test_noalloc_matches_fg_gemm_two_calls_in_a_row_second_smaller():
    fg.fg_init()
    torch.cuda.synchronize()
    cases = [(1024, 768, 8192, dict(bias_dim=0, act=fg.FG_ACT_RELU)), (300, 200, 4096, dict(c_act=fg.FG_ACT_RELU))]
    held = []
    for (M, N, K, kw) in cases:
        plan = fg.fg_gemm_plan(M, N, K)
        assert "+splitk" in plan and scratch_bytes(plan, M, N) <= 16 << 20, plan
        lda, ldc = (M + 7) // 8 * 8, (M + 3) // 4 * 4
        A = W.uniform_pm1(lda * K, 31, device="cuda"); B = W.uniform_pm1(K * N, 32, device="cuda")
        Cm = W.uniform_pm1(ldc * N, 33, device="cuda", dtype=torch.float32)
        bias = W.uniform_pm1(M, 34, device="cuda", dtype=torch.float32) if "bias_dim" in kw else None
        D0, D1 = torch.full_like(Cm, float("nan")), torch.full_like(Cm, float("nan"))
        held.append((M, N, K, kw, lda, ldc, A, B, Cm, bias, D0, D1))
    torch.cuda.synchronize()

    def both_calls():
        # the two allocation-free calls back to back on one stream, the larger first
        for (M, N, K, kw, lda, ldc, A, B, Cm, bias, D0, D1) in held:
            say("noalloc %dx%dx%d" % (M, N, K))
            D1.fill_(float("nan"))
            fg.fg_gemm(M, N, K, 0.5, fg.Matrix(A, fg.FG_COL, lda), fg.Matrix(B, fg.FG_COL, K), 2.0, fg.Matrix(Cm, fg.FG_COL, ldc),
                       fg.Matrix(D1, fg.FG_COL, ldc), bias=bias, noalloc=True, **kw)
        torch.cuda.synchronize()
    both_calls()      # the HIP runtime's own first-launch work (its argument and signal pools) happens here
    free_before = torch.cuda.mem_get_info()[0]
    both_calls()
    assert torch.cuda.mem_get_info()[0] == free_before, "device memory was allocated during the allocation-free calls"
    for (M, N, K, kw, lda, ldc, A, B, Cm, bias, D0, D1) in held:
        fg.fg_gemm(M, N, K, 0.5, fg.Matrix(A, fg.FG_COL, lda), fg.Matrix(B, fg.FG_COL, K), 2.0, fg.Matrix(Cm, fg.FG_COL, ldc),
                   fg.Matrix(D0, fg.FG_COL, ldc), bias=bias, **kw)
    torch.cuda.synchronize()
    for (M, N, K, kw, lda, ldc, A, B, Cm, bias, D0, D1) in held:
        v0, v1 = D0.view(N, ldc)[:, :M], D1.view(N, ldc)[:, :M]
        assert torch.isfinite(v1).all()
        assert torch.equal(v0, v1), "fg_gemm_noalloc differs from fg_gemm at %dx%dx%d" % (M, N, K)
        if ldc > M:
            assert torch.isnan(D1.view(N, ldc)[:, M:]).all(), "padding of D was written"
    # the same two shapes against the oracle (floats to the tolerance, integers bit-exact), again in a row
    for ints in (False, True):
        for (M, N, K, kw) in cases:
            say("noalloc vs oracle %dx%dx%d ints=%s" % (M, N, K, ints))
            run_gemm_case(M, N, K, alpha=0.5 if not ints else 1.0, beta=2.0, ints=ints, noalloc=True, **kw)


def test_noalloc_without_a_split_and_beyond_the_static_array():
    fg.fg_init()
    say("noalloc, plan without a split"); run_gemm_case(1024, 1024, 1024, noalloc=True)
    say("noalloc, general kernel"); run_gemm_case(70, 50, 27, ints=True, noalloc=True)
    # a plan whose partial products exceed the 16 MiB array is refused, and nothing is written
    # (the first of a few long-K shapes whose plan needs more; which ones split how is the planner's choice)
    for (M, N, K) in [(1536, 1024, 16384), (2048, 1024, 16384), (1024, 1024, 32768), (1024, 1024, 16384)]:
        plan = fg.fg_gemm_plan(M, N, K)
        if "+splitk" in plan and scratch_bytes(plan, M, N) > 16 << 20:
            break
    else:
        pytest.fail("none of the long-K shapes is split beyond 16 MiB by this build's planner")
    say("noalloc, %dx%dx%d planned as %s" % (M, N, K, plan))
    A = W.small_ints(M * K, 1, device="cuda"); B = W.small_ints(K * N, 2, device="cuda")
    D = torch.full((M * N,), float("nan"), dtype=torch.float32, device="cuda")
    st = fg.fg_gemm(M, N, K, 1.0, fg.Matrix(A, fg.FG_COL, M), fg.Matrix(B, fg.FG_COL, K), 0.0, None, fg.Matrix(D, fg.FG_COL, M),
                    noalloc=True, raise_on_error=False)
    torch.cuda.synchronize()
    assert st == fg.FG_ERR_UNSUPPORTED and "static scratch" in fg.fg_last_error()
    assert torch.isnan(D).all()
