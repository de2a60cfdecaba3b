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
