"""GPU parity tests of the layout adapters of fg_gemm: diagonal operands (Section 5.2) and
planar-split complex operands (Section 5.4), against the CPU oracle."""
import itertools

import pytest

from paper_2009_12263_amd import binding as fg
from tests.parity import run_cgemm_case, run_diag_case

pytestmark = pytest.mark.gpu
LAYOUTS = [fg.FG_COL, fg.FG_ROW]


def say(msg):
    print("[case] " + msg, flush=True)


@pytest.mark.parametrize("side", ["A", "B"])
@pytest.mark.parametrize("other,ldl", list(itertools.product(LAYOUTS, LAYOUTS)))
def test_diagonal_operand_small(side, other, ldl):
    for (M, N, K) in [(256, 256, 256), (512, 384, 512), (128, 320, 256), (384, 128, 64)]:
        # rectangular diagonal operands hold min(rows, cols) entries; rows/columns beyond are zero
        say("diag %s M=%d N=%d K=%d other=%d D=%d" % (side, M, N, K, other, ldl))
        run_diag_case(M, N, K, side, other, ldl, ints=True)
    run_diag_case(512, 512, 512, side, other, ldl, alpha=0.5, beta=-1.25)


def test_diagonal_config4_4096():
    """BASELINE config 4 variant: D = diag(d) B + C, N = 4096, B column-major; every entry is
    checked against the closed form the oracle was pinned to (d_i B_ij + C_ij)."""
    say("diag A 4096 ints"); run_diag_case(4096, 4096, 4096, "A", ints=True, samples=20000)
    say("diag A 4096 floats"); run_diag_case(4096, 4096, 4096, "A", samples=20000)


@pytest.mark.parametrize("la,lb", list(itertools.product(LAYOUTS, LAYOUTS)))
def test_complex_small_all_layouts(la, lb):
    for (M, N, K) in [(64, 64, 64), (256, 128, 192), (384, 512, 128)]:
        say("cgemm ints M=%d N=%d K=%d la=%d lb=%d" % (M, N, K, la, lb))
        run_cgemm_case(M, N, K, la, lb, ints=True, pad=8)
    say("cgemm floats 512"); run_cgemm_case(512, 512, 512, la, lb, alpha=0.5, beta=2.0)
    say("cgemm row-major D"); run_cgemm_case(256, 384, 128, la, lb, ld_layout=fg.FG_ROW, ints=True)


def test_complex_config4_4096():
    """BASELINE config 4: planar complex D = A B + C at 4096^3, sampled."""
    say("cgemm 4096 floats"); run_cgemm_case(4096, 4096, 4096, samples=4096)
    say("cgemm 4096 ints"); run_cgemm_case(4096, 4096, 4096, ints=True, samples=4096)


def test_edge_tiles_diagonal_and_complex():
    """Sizes that are not multiples of any tile (K a multiple of 8) for the layout adapters."""
    for side in ("A", "B"):
        for other in LAYOUTS:
            say("diag %s edge other=%d" % (side, other))
            run_diag_case(300, 200, 264, side, other, ints=True)
            run_diag_case(70, 333, 72, side, other, fg.FG_ROW, ints=True)
    for la, lb in itertools.product(LAYOUTS, LAYOUTS):
        say("cgemm edge la=%d lb=%d" % (la, lb))
        run_cgemm_case(100, 75, 40, la, lb, ints=True, pad=8)
        run_cgemm_case(300, 513, 136, la, lb, ld_layout=fg.FG_ROW, alpha=0.5, beta=1.5)


@pytest.mark.parametrize("la,lb", list(itertools.product(LAYOUTS, LAYOUTS)))
def test_dual_numbers_all_layouts(la, lb):
    """Dual-number products (Section 5.4, eps^2 = 0) on the planar layout: exact on integers for
    every tile shape, floats within tolerance, edge tiles and a row-major result."""
    for (M, N, K) in [(64, 64, 64), (256, 128, 192), (384, 512, 128), (100, 75, 40)]:
        say("dual ints M=%d N=%d K=%d la=%d lb=%d" % (M, N, K, la, lb))
        run_cgemm_case(M, N, K, la, lb, ints=True, pad=8, dual=True)
    say("dual floats 512"); run_cgemm_case(512, 512, 512, la, lb, alpha=0.5, beta=2.0, dual=True)
    say("dual row-major D"); run_cgemm_case(300, 513, 136, la, lb, ld_layout=fg.FG_ROW, alpha=0.5, beta=1.5, dual=True)
    say("dual no C"); run_cgemm_case(256, 384, 128, la, lb, with_c=False, ints=True, dual=True)


def test_dual_4096():
    say("dual 4096 floats"); run_cgemm_case(4096, 4096, 4096, samples=4096, dual=True)
    say("dual 4096 ints"); run_cgemm_case(4096, 4096, 4096, ints=True, samples=4096, dual=True)


@pytest.mark.parametrize("la,lb", list(itertools.product(LAYOUTS, LAYOUTS)))
def test_interleaved_complex_all_layouts(la, lb):
    """Complex matrices with real and imaginary parts adjacent in memory (Section 5.4's global
    layout); the oracle is fed the same numbers in planar form, which its own pins tie to the
    interleaved form.  Exact on integers for every tile shape, edge tiles, a K tail, no C, and a
    row-major result."""
    for (M, N, K) in [(64, 64, 64), (256, 128, 192), (384, 512, 128), (100, 75, 40)]:
        say("interleaved ints M=%d N=%d K=%d la=%d lb=%d" % (M, N, K, la, lb))
        run_cgemm_case(M, N, K, la, lb, ints=True, pad=8, interleaved=True)
    say("interleaved floats 512"); run_cgemm_case(512, 512, 512, la, lb, alpha=0.5, beta=2.0, interleaved=True)
    say("interleaved row-major D"); run_cgemm_case(300, 513, 136, la, lb, ld_layout=fg.FG_ROW, alpha=0.5, beta=1.5, interleaved=True)
    say("interleaved no C"); run_cgemm_case(256, 384, 128, la, lb, with_c=False, ints=True, interleaved=True)


def test_interleaved_complex_4096():
    say("interleaved 4096 floats"); run_cgemm_case(4096, 4096, 4096, samples=4096, interleaved=True)
    say("interleaved 2048x4096x256 ints, every entry"); run_cgemm_case(2048, 4096, 256, ints=True, interleaved=True)


def test_interleaved_and_planar_matrices_are_not_mixed():
    import torch
    H = torch.zeros(2 * 64 * 64, dtype=torch.float16, device="cuda")
    F = torch.zeros(2 * 64 * 64, dtype=torch.float32, device="cuda")
    il = lambda t, d: fg.Matrix(t, fg.FG_COL, 64, dtype=d)
    kw = dict(raise_on_error=False)
    assert fg.fg_gemm(64, 64, 64, 1.0, il(H, fg.FG_CF16), il(H, fg.FG_CF16), 0.0, None, fg.Matrix(F, fg.FG_COL, 64, im=F), **kw) == fg.FG_ERR_UNSUPPORTED
    assert fg.fg_gemm(64, 64, 64, 1.0, il(H, fg.FG_CF16), fg.Matrix(H, fg.FG_COL, 64), 0.0, None, il(F, fg.FG_CF32), **kw) == fg.FG_ERR_UNSUPPORTED
    assert fg.fg_gemm(64, 64, 64, 1.0, fg.Matrix(H, fg.FG_COL, 64), fg.Matrix(H, fg.FG_COL, 64), 0.0, None, il(F, fg.FG_CF32), **kw) == fg.FG_ERR_UNSUPPORTED
    assert fg.fg_gemm(64, 64, 64, 1.0, il(H, fg.FG_CF16), il(H, fg.FG_CF16), 0.0, None, il(F, fg.FG_CF32), act=fg.FG_ACT_RELU, **kw) == fg.FG_ERR_UNSUPPORTED
    assert fg.fg_gemm(64, 64, 64, 1.0, fg.Matrix(H, fg.FG_COL, 64, im=H, dtype=fg.FG_CF16), il(H, fg.FG_CF16), 0.0, None, il(F, fg.FG_CF32), **kw) == fg.FG_ERR_LAYOUT
