"""GPU parity tests of fg_gemm against the CPU oracle (run with -m gpu on an MI355X)."""
import itertools

import pytest
import torch

from paper_2009_12263_amd import binding as fg
from tests.parity import delenv, run_gemm_case, run_unaligned_gemm_case, setenv

pytestmark = pytest.mark.gpu

LAYOUTS = [fg.FG_COL, fg.FG_ROW]


def say(msg):
    print("[case] " + msg, flush=True)


def test_config1_256_cube_colmajor():
    """BASELINE config 1: D = A.B + C, 256^3, A, B column-major, alpha = beta = 1; every entry."""
    say("256^3 NN floats"); run_gemm_case(256, 256, 256, config=1)
    say("256^3 NN ints"); run_gemm_case(256, 256, 256, config=1, ints=True)


@pytest.mark.parametrize("la,lb", list(itertools.product(LAYOUTS, LAYOUTS)))
def test_index_mapping_is_bit_exact_all_layouts(la, lb):
    """Integer-valued inputs: the result is unique, so every entry must match bit for bit.
    Sizes span several block tiles of every tile shape and use padded leading dimensions."""
    for (M, N, K) in [(64, 64, 64), (128, 192, 256), (512, 256, 128), (768, 1280, 320)]:
        say("ints M=%d N=%d K=%d la=%d lb=%d" % (M, N, K, la, lb))
        run_gemm_case(M, N, K, la, lb, ints=True, pad=8, config=2)


@pytest.mark.parametrize("la,lb", list(itertools.product(LAYOUTS, LAYOUTS)))
def test_float_parity_1024_all_layouts(la, lb):
    say("1024^3 la=%d lb=%d" % (la, lb))
    run_gemm_case(1024, 1024, 1024, la, lb, config=2)


@pytest.mark.parametrize("ldl", LAYOUTS)
def test_row_major_output_alpha_beta_inplace(ldl):
    say("D layout %d alpha=-1.5 beta=0.25 in place" % ldl)
    run_gemm_case(384, 256, 192, fg.FG_COL, fg.FG_ROW, ldl, alpha=-1.5, beta=0.25, pad=8, inplace=True, config=2)
    say("D layout %d ints" % ldl)
    run_gemm_case(256, 384, 128, fg.FG_ROW, fg.FG_ROW, ldl, alpha=2.0, beta=-1.0, ints=True, config=2)


@pytest.mark.parametrize("bias_dim", [0, 1])
@pytest.mark.parametrize("ldl", LAYOUTS)
def test_bias_and_relu_epilogue(bias_dim, ldl):
    say("bias_dim=%d D layout=%d relu" % (bias_dim, ldl))
    run_gemm_case(256, 320, 128, ld_layout=ldl, with_c=False, bias_dim=bias_dim, act=fg.FG_ACT_RELU, config=3)
    run_gemm_case(256, 320, 128, ld_layout=ldl, with_c=False, bias_dim=bias_dim, act=fg.FG_ACT_RELU, ints=True, config=3)
    run_gemm_case(128, 128, 64, ld_layout=ldl, with_c=True, beta=0.5, bias_dim=bias_dim, act=fg.FG_ACT_NONE, config=3)


def test_k_zero_and_empty():
    # K = 0: D = beta*C; M = 0: nothing happens
    say("K=0"); run_gemm_case(128, 128, 0, beta=2.0, ints=True, config=1)
    A = torch.zeros(64, dtype=torch.float16, device="cuda"); D = torch.zeros(64, dtype=torch.float32, device="cuda")
    assert fg.fg_gemm(0, 64, 64, 1.0, fg.Matrix(A, fg.FG_COL, 8), fg.Matrix(A, fg.FG_COL, 64), 0.0, None, fg.Matrix(D, fg.FG_COL, 8)) == fg.FG_OK


@pytest.mark.parametrize("la,lb", list(itertools.product(LAYOUTS, LAYOUTS)))
def test_full_size_8192_sampled(la, lb):
    """BASELINE config 2 at its headline size, in the launch configuration bench.py times:
    sampled entries (each an exact K-long FP64 dot product in the oracle) incl. every tile seam."""
    say("8192^3 la=%d lb=%d sampled" % (la, lb))
    run_gemm_case(8192, 8192, 8192, la, lb, config=2, samples=4096)


@pytest.mark.parametrize("la,lb", list(itertools.product(LAYOUTS, LAYOUTS)))
def test_full_size_16384_sampled(la, lb):
    """The largest point of the config-2 sweep (3.2 GB of operands, 4096 block tiles = 16 rounds of
    the persistent grid, the largest ld * n offsets of the sweep): sampled entries and every kind
    of tile seam, floats in all four layout pairs, integer-exact in NN and TT."""
    say("16384^3 la=%d lb=%d floats sampled" % (la, lb))
    run_gemm_case(16384, 16384, 16384, la, lb, config=2, samples=4096)
    if la == lb:
        say("16384^3 la=%d lb=%d ints sampled" % (la, lb))
        run_gemm_case(16384, 16384, 16384, la, lb, config=2, samples=4096, ints=True)


@pytest.mark.parametrize("n", [2048, 4096])
@pytest.mark.parametrize("la,lb", list(itertools.product(LAYOUTS, LAYOUTS)))
def test_full_size_2048_4096_sampled_all_layouts(n, la, lb):
    """The middle points of the config-2 sweep in every layout pair: floats and integers."""
    say("%d^3 la=%d lb=%d floats sampled" % (n, la, lb)); run_gemm_case(n, n, n, la, lb, config=2, samples=4096)
    say("%d^3 la=%d lb=%d ints sampled" % (n, la, lb)); run_gemm_case(n, n, n, la, lb, config=2, samples=4096, ints=True)


def test_full_size_4096_ints_sampled():
    say("4096^3 ints sampled"); run_gemm_case(4096, 4096, 4096, ints=True, config=2, samples=8192)


def test_config3_relu_bias_shapes():
    say("config 3: 4096^3 relu+bias"); run_gemm_case(4096, 4096, 4096, with_c=False, bias_dim=0, act=fg.FG_ACT_RELU, config=3, samples=4096)
    say("config 3: 8192x1024x4096 relu+bias"); run_gemm_case(8192, 1024, 4096, with_c=False, bias_dim=0, act=fg.FG_ACT_RELU, config=3, samples=4096)


@pytest.mark.parametrize("la,lb", list(itertools.product(LAYOUTS, LAYOUTS)))
@pytest.mark.parametrize("ldl", LAYOUTS)
def test_arbitrary_sizes_edge_tiles(la, lb, ldl):
    """M and N need not be multiples of any tile, K only of 8: tiles that hang over the edge are
    predicated.  Integer inputs make every stored entry bit-exact; the NaN-filled padding of D must
    stay untouched (checked inside run_gemm_case)."""
    for (M, N, K) in [(1, 1, 8), (7, 5, 16), (65, 63, 72), (100, 260, 200), (257, 129, 264), (300, 520, 136), (777, 1031, 520)]:
        say("edge ints M=%d N=%d K=%d la=%d lb=%d D=%d" % (M, N, K, la, lb, ldl))
        run_gemm_case(M, N, K, la, lb, ldl, ints=True, pad=8, config=2)
    say("edge floats + bias + relu")
    run_gemm_case(333, 1111, 248, la, lb, ldl, alpha=0.5, beta=-1.0, bias_dim=0, act=fg.FG_ACT_RELU, pad=8, config=3)
    run_gemm_case(333, 1111, 248, la, lb, ldl, with_c=False, bias_dim=1, pad=8, config=3)


@pytest.mark.parametrize("la,lb", list(itertools.product(LAYOUTS, LAYOUTS)))
def test_poisoned_padding_never_reaches_a_result(la, lb):
    """Everything between an extent and its leading dimension in A, B and C holds NaN (that covers
    the rest of the last 16-byte chunk of a column or row, and the rows and columns an edge tile
    reads beyond the matrix).  The kernels read some of it by design; no stored entry may depend on
    it: results stay finite and, on integers, bit-exact; D's own padding stays untouched."""
    for (M, N, K) in [(100, 260, 200), (257, 129, 264), (300, 520, 136), (777, 1031, 520), (250, 250, 72)]:
        for ldl in LAYOUTS:
            say("poison ints M=%d N=%d K=%d la=%d lb=%d D=%d" % (M, N, K, la, lb, ldl))
            run_gemm_case(M, N, K, la, lb, ldl, ints=True, pad=8, config=2, poison=True)
    say("poison floats bias relu"); run_gemm_case(333, 1111, 248, la, lb, alpha=0.5, beta=-1.0, bias_dim=0, act=fg.FG_ACT_RELU, pad=8, config=3, poison=True)
    say("poison in place"); run_gemm_case(259, 131, 200, la, lb, ints=True, pad=8, inplace=True, poison=True)
    say("poison split-K 300x200x4096"); run_gemm_case(300, 200, 4096, la, lb, ints=True, pad=8, bias_dim=0, act=fg.FG_ACT_RELU, c_act=fg.FG_ACT_RELU, poison=True)
    say("poison split-K with K tail 250x120x4104"); run_gemm_case(250, 120, 4104, la, lb, ints=True, pad=8, poison=True)
    say("poison tail split 4100x4100x1032"); run_gemm_case(4100, 4100, 1032, la, lb, ints=True, pad=8, samples=6000, poison=True)
    say("poison addition on A and B"); run_gemm_case(257, 129, 264, la, lb, ints=True, pad=8, ab_add=(1.0, -2.0), poison=True)
    say("poison bf16"); run_gemm_case(257, 129, 264, la, lb, ints=True, pad=8, bf16=True, poison=True)
    say("poison binary16 C and D"); run_gemm_case(257, 129, 264, la, lb, ints=True, pad=8, cd16=True, poison=True)


def test_poisoned_padding_complex_dual_diagonal():
    from tests.parity import run_cgemm_case, run_diag_case
    for la, lb in itertools.product(LAYOUTS, LAYOUTS):
        say("poison complex la=%d lb=%d" % (la, lb)); run_cgemm_case(130, 200, 72, la, lb, ints=True, pad=8, poison=True)
    say("poison dual"); run_cgemm_case(130, 200, 72, ints=True, pad=8, dual=True, poison=True)
    say("poison interleaved complex"); run_cgemm_case(130, 200, 72, fg.FG_ROW, fg.FG_COL, ints=True, pad=8, interleaved=True, poison=True)


def test_non_finite_values_propagate_like_the_definition():
    """NaN and infinities in A, B and C reach D exactly where the definition puts them (the oracle
    evaluates the same IEEE expression in FP64): without activation they pass through, with ReLU
    the comparison y > 0 turns NaN into 0.  With beta == 0, C is never read: a NaN-filled C (the
    in-place call on uninitialised memory) leaves the product untouched."""
    import numpy as np
    from oracle import cpu_oracle as O
    from paper_2009_12263_amd import workloads as W
    from tests.parity import np16
    for (M, N, K, force) in [(300, 260, 136, None), (300, 200, 4096, None), (70, 50, 27, None)]:
        for act in (fg.FG_ACT_NONE, fg.FG_ACT_RELU):
            say("non-finite M=%d N=%d K=%d act=%d" % (M, N, K, act))
            lda, ldb, ldc = (M + 7) // 8 * 8, (K + 7) // 8 * 8, (M + 3) // 4 * 4
            A = W.small_ints(lda * K, 1, device="cuda"); B = W.small_ints(ldb * N, 2, device="cuda")
            Cm = W.small_ints(ldc * N, 3, device="cuda", dtype=torch.float32)
            A.view(K, lda)[5, 17] = float("nan"); A.view(K, lda)[K - 1, 3] = float("inf")
            B.view(N, ldb)[7, 2] = float("-inf")
            Cm.view(N, ldc)[9, 40] = float("nan"); Cm.view(N, ldc)[11, 41] = float("-inf")
            D = torch.full_like(Cm, 7.0)
            fg.fg_gemm(M, N, K, 1.0, fg.Matrix(A, fg.FG_COL, lda), fg.Matrix(B, fg.FG_COL, ldb), 1.0, fg.Matrix(Cm, fg.FG_COL, ldc),
                       fg.Matrix(D, fg.FG_COL, ldc), act=act)
            torch.cuda.synchronize()
            with np.errstate(invalid="ignore"):
                r = O.gemm(M, N, K, 1.0, O.Operand(np16(A), O.COL, lda), O.Operand(np16(B), O.COL, ldb), 1.0, np16(Cm), None, O.COL, ldc, act=act)
            got = np16(D).reshape(N, ldc)[:, :M].T.astype(np.float64)
            assert np.isnan(r["D"]).any() or act == fg.FG_ACT_RELU
            assert np.array_equal(got, r["D"], equal_nan=True), "non-finite entries differ from the definition"
    say("beta == 0 with a NaN-filled C, in place")
    M = N = 256; K = 128
    A = W.small_ints(M * K, 1, device="cuda"); B = W.small_ints(K * N, 2, device="cuda")
    D = torch.full((M * N,), float("nan"), dtype=torch.float32, device="cuda")
    fg.fg_gemm(M, N, K, 1.0, fg.Matrix(A, fg.FG_COL, M), fg.Matrix(B, fg.FG_COL, K), 0.0, fg.Matrix(D, fg.FG_COL, M), fg.Matrix(D, fg.FG_COL, M))
    torch.cuda.synchronize()
    r = O.gemm(M, N, K, 1.0, O.Operand(np16(A), O.COL, M), O.Operand(np16(B), O.COL, K), 0.0, None, None, O.COL, M)
    assert np.array_equal(np16(D).reshape(N, M).T.astype(np.float64), r["D"])


def test_arbitrary_sizes_large():
    say("5000x3000x1000 ints sampled"); run_gemm_case(5000, 3000, 1000, ints=True, config=2, samples=6000)
    say("4100x4100x4104 floats sampled"); run_gemm_case(4100, 4100, 4104, fg.FG_ROW, fg.FG_COL, config=2, samples=6000)


@pytest.mark.parametrize("la,lb", list(itertools.product(LAYOUTS, LAYOUTS)))
def test_bf16_inputs_all_layouts(la, lb):
    """bfloat16 A and B (Section 2.2: the matrix unit's other 16-bit input type): exact on integers
    for every tile shape, floats within tolerance, epilogue, edge tiles and a row-major result."""
    for (M, N, K) in [(64, 64, 64), (128, 192, 256), (768, 1280, 320), (100, 75, 40)]:
        say("bf16 ints M=%d N=%d K=%d la=%d lb=%d" % (M, N, K, la, lb))
        run_gemm_case(M, N, K, la, lb, ints=True, pad=8, bf16=True)
    say("bf16 floats 512"); run_gemm_case(512, 512, 512, la, lb, alpha=0.5, beta=2.0, bf16=True)
    say("bf16 bias relu row-major D")
    run_gemm_case(300, 513, 136, la, lb, ld_layout=fg.FG_ROW, bias_dim=1, act=fg.FG_ACT_RELU, bf16=True)


def test_bf16_large_sampled():
    say("bf16 4096 floats"); run_gemm_case(4096, 4096, 4096, samples=4096, bf16=True)
    say("bf16 8192x1024x4096 ints"); run_gemm_case(8192, 1024, 4096, ints=True, samples=4096, bf16=True)


def test_bf16_is_rejected_where_unsupported():
    A = torch.zeros(64 * 64, dtype=torch.bfloat16, device="cuda")
    H = torch.zeros(64 * 64, dtype=torch.float16, device="cuda")
    D = torch.zeros(64 * 64, dtype=torch.float32, device="cuda")
    m = lambda t, **kw: fg.Matrix(t, fg.FG_COL, 64, **kw)
    assert fg.fg_gemm(64, 64, 64, 1.0, m(A), m(H), 0.0, None, m(D), raise_on_error=False) == fg.FG_ERR_UNSUPPORTED
    assert fg.fg_gemm(64, 64, 64, 1.0, m(A, im=A), m(A, im=A), 0.0, None, m(D, im=D), raise_on_error=False) == fg.FG_ERR_UNSUPPORTED
    assert fg.fg_gemm(64, 64, 64, 1.0, fg.Matrix(A, fg.FG_DIAG, 0), m(A), 0.0, None, m(D), raise_on_error=False) == fg.FG_ERR_UNSUPPORTED


@pytest.mark.parametrize("la,lb", list(itertools.product(LAYOUTS, LAYOUTS)))
def test_transforms_on_loaded_elements_all_layouts(la, lb):
    """Last rows of the fusion table (Section 5.3): ReLU on the loaded C and a constant added to
    the loaded A and B values (in FP16), for every tile shape, with edge tiles and a K that is not
    a multiple of the K tile (the zero fill beyond K must stay zero)."""
    for (M, N, K) in [(64, 64, 64), (128, 192, 256), (768, 1280, 320), (100, 75, 40), (300, 130, 72)]:
        say("ab_add ints M=%d N=%d K=%d la=%d lb=%d" % (M, N, K, la, lb))
        run_gemm_case(M, N, K, la, lb, ints=True, pad=8, ab_add=(2.0, -3.0), c_act=fg.FG_ACT_RELU)
    say("ab_add floats 512"); run_gemm_case(512, 512, 512, la, lb, alpha=0.5, beta=2.0, ab_add=(0.25, 0.0999755859375))
    say("ab_add bias relu row-major D")
    run_gemm_case(300, 513, 136, la, lb, ld_layout=fg.FG_ROW, bias_dim=1, act=fg.FG_ACT_RELU, ab_add=(-0.5, 1.5), c_act=fg.FG_ACT_RELU)
    say("relu on C only"); run_gemm_case(256, 384, 128, la, lb, c_act=fg.FG_ACT_RELU)
    say("a_add only"); run_gemm_case(256, 384, 128, la, lb, ints=True, ab_add=(1.0, 0.0))


def test_transforms_fusion_table_4096():
    """The full last row of the fusion table at the paper's size: bias, ReLU on C and D, addition on
    A and B, N = 4096, sampled."""
    say("fusion table last row, floats")
    run_gemm_case(4096, 4096, 4096, bias_dim=0, act=fg.FG_ACT_RELU, ab_add=(0.5, -0.25), c_act=fg.FG_ACT_RELU, samples=4096, config=3)
    say("fusion table last row, ints")
    run_gemm_case(4096, 4096, 4096, bias_dim=0, act=fg.FG_ACT_RELU, ab_add=(1.0, -2.0), c_act=fg.FG_ACT_RELU, samples=4096, config=3, ints=True)


def test_binding_refuses_tensors_smaller_than_the_matrix():
    """The library sees pointers only; the Python binding checks that every device tensor holds the
    matrix it is said to hold and raises before anything is launched."""
    A = torch.zeros(64 * 64, dtype=torch.float16, device="cuda")
    D = torch.full((64 * 64,), 7.0, dtype=torch.float32, device="cuda")
    m = lambda t, ld=64, lay=fg.FG_COL: fg.Matrix(t, lay, ld)
    short = D[:64 * 64 - 1]
    with pytest.raises(ValueError):
        fg.fg_gemm(64, 64, 64, 1.0, m(A), m(A), 0.0, None, m(short))
    with pytest.raises(ValueError):
        fg.fg_gemm(64, 64, 64, 1.0, m(A, 72), m(A), 0.0, None, m(D))          # 63 * 72 + 64 > 4096
    with pytest.raises(ValueError):
        fg.fg_gemm(64, 64, 64, 1.0, m(A), m(A[:100], 64, fg.FG_ROW), 0.0, None, m(D))
    with pytest.raises(ValueError):
        fg.fg_gemm(64, 64, 64, 1.0, m(A), m(A), 1.0, m(short), m(D))
    with pytest.raises(ValueError):
        fg.fg_contract([0, 1], [1, 64], A, [1, 2], [1, 64], A, [0, 2], [1, 64], None, short, {0: 64, 1: 64, 2: 64})
    torch.cuda.synchronize()
    assert bool((D == 7.0).all())
    assert fg.fg_gemm(64, 64, 64, 1.0, m(A), m(A), 0.0, None, m(D)) == fg.FG_OK     # exactly large enough
    torch.cuda.synchronize()
    assert bool((D == 0.0).all())


def test_transforms_are_rejected_where_unsupported():
    H = torch.zeros(64 * 64, dtype=torch.float16, device="cuda")
    Bf = torch.zeros(64 * 64, dtype=torch.bfloat16, device="cuda")
    D = torch.zeros(64 * 64, dtype=torch.float32, device="cuda")
    m = lambda t, **kw: fg.Matrix(t, fg.FG_COL, 64, **kw)
    kw = dict(raise_on_error=False)
    assert fg.fg_gemm(64, 64, 64, 1.0, m(Bf), m(Bf), 0.0, None, m(D), a_add=1.0, **kw) == fg.FG_ERR_UNSUPPORTED
    assert fg.fg_gemm(64, 64, 64, 1.0, m(H, im=H), m(H, im=H), 0.0, None, m(D, im=D), a_add=1.0, **kw) == fg.FG_ERR_UNSUPPORTED
    assert fg.fg_gemm(64, 64, 64, 1.0, m(H, im=H), m(H, im=H), 0.0, None, m(D, im=D), c_act=fg.FG_ACT_RELU, **kw) == fg.FG_ERR_UNSUPPORTED
    assert fg.fg_gemm(64, 64, 64, 1.0, fg.Matrix(H, fg.FG_DIAG, 0), m(H), 0.0, None, m(D), b_add=1.0, **kw) == fg.FG_ERR_UNSUPPORTED
    assert fg.fg_gemm(64, 64, 64, 1.0, m(H), m(H), 0.0, None, m(D), c_act=7, **kw) == fg.FG_ERR_LAYOUT
    assert fg.fg_gemm(64, 64, 64, 1.0, m(H), m(H), 0.0, None, m(D), a_add=float("nan"), **kw) == fg.FG_ERR_SHAPE


def test_seeded_random_shape_sweep():
    """Forty seeded random problems (sizes up to ~700, K a multiple of 8, every layout triple,
    random epilogue and transform choices), integer-valued so that every entry must be exact."""
    import random
    rng = random.Random(20091226)
    for case in range(40):
        M, N = rng.randint(1, 700), rng.randint(1, 700)
        K = 8 * rng.randint(1, 60)
        la, lb, ld = rng.choice(LAYOUTS), rng.choice(LAYOUTS), rng.choice(LAYOUTS)
        with_c = rng.random() < 0.7
        bias_dim = rng.choice([None, 0, 1])
        act = rng.choice([fg.FG_ACT_NONE, fg.FG_ACT_RELU])
        ab_add = rng.choice([None, None, (1.0, -2.0), (0.0, 3.0)])
        c_act = rng.choice([fg.FG_ACT_NONE, fg.FG_ACT_RELU]) if with_c else fg.FG_ACT_NONE
        bf16 = ab_add is None and rng.random() < 0.25
        alpha, beta = rng.choice([(1.0, 1.0), (0.5, 2.0), (-1.0, 0.25), (2.0, -1.0)])
        say("sweep %d: M=%d N=%d K=%d la=%d lb=%d ld=%d c=%s bias=%s act=%d add=%s c_act=%d bf16=%s" % (
            case, M, N, K, la, lb, ld, with_c, bias_dim, act, ab_add, c_act, bf16))
        run_gemm_case(M, N, K, la, lb, ld, alpha=alpha, beta=beta, with_c=with_c, bias_dim=bias_dim, act=act,
                      ints=True, pad=8 * rng.randint(0, 2), ab_add=ab_add, c_act=c_act, bf16=bf16, seed=1000 + case)


def test_calls_can_be_captured_in_a_hip_graph():
    """After fg_init() a call only enqueues one kernel on the given stream (no allocation, no
    synchronisation), so a sequence of calls can be captured into a HIP graph and replayed.  Every
    replay is checked against the eager result, with eager work and synchronisation between
    replays."""
    from paper_2009_12263_amd import workloads as W
    n = 512
    dev = "cuda"
    A = W.uniform_pm1(n * n, 1, device=dev); B = W.uniform_pm1(n * n, 2, device=dev)
    C = W.uniform_pm1(n * n, 3, device=dev, dtype=torch.float32)
    bias = W.uniform_pm1(n, 4, device=dev, dtype=torch.float32)
    D1, D2 = torch.empty_like(C), torch.empty_like(C)
    m = lambda t, l=fg.FG_COL: fg.Matrix(t, l, n)

    fg.fg_init()

    def chain(out1, out2, stream=None):
        # out1 = A.B + C;  out2 = relu(0.5 A.B^T + out1 + bias): the second call reads the first's result
        fg.fg_gemm(n, n, n, 1.0, m(A), m(B), 1.0, m(C), m(out1), stream=stream)
        fg.fg_gemm(n, n, n, 0.5, m(A), m(B, fg.FG_ROW), 1.0, m(out1), m(out2), bias=bias, bias_dim=0, act=fg.FG_ACT_RELU, stream=stream)

    chain(D1, D2)                                # eager reference
    torch.cuda.synchronize()
    want1, want2 = D1.clone(), D2.clone()
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        D1.zero_(); D2.zero_()
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=s):
            chain(D1, D2, stream=s)
    torch.cuda.synchronize()
    for rep in range(4):
        D1.fill_(float("nan")); D2.fill_(float("nan"))          # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        say("graph replay %d" % rep)
        assert torch.equal(D1, want1) and torch.equal(D2, want2), "replay %d differs from the eager result" % rep


@pytest.mark.parametrize("noalloc", [False, True])
def test_split_k_calls_can_be_captured_in_a_hip_graph(noalloc):
    """A call that splits K enqueues two kernels (partial products, reduction pass) and, outside a
    capture, orders itself against the workspace's previous user with an event; under capture it
    must record nothing but its kernels.  Captured through fg_gemm (library workspace, which exists
    after fg_init) and through the allocation-free entry point; every replay is checked."""
    from paper_2009_12263_amd import workloads as W
    M, N, K = 384, 256, 8192
    assert "+splitk" in fg.fg_gemm_plan(M, N, K)
    A = W.small_ints(M * K, 1, device="cuda"); B = W.small_ints(K * N, 2, device="cuda")
    Cm = W.small_ints(M * N, 3, device="cuda", dtype=torch.float32)
    D = torch.empty_like(Cm)
    fg.fg_init()
    call = lambda stream=None: fg.fg_gemm(M, N, K, 1.0, fg.Matrix(A, fg.FG_COL, M), fg.Matrix(B, fg.FG_COL, K), -1.0, fg.Matrix(Cm, fg.FG_COL, M),
                                          fg.Matrix(D, fg.FG_COL, M), stream=stream, noalloc=noalloc)
    call()
    torch.cuda.synchronize()
    want = D.clone()
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        D.zero_()
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=s):
            call(stream=s)
    torch.cuda.synchronize()
    for rep in range(3):
        D.fill_(float("nan"))
        call_other = torch.empty_like(D)
        fg.fg_gemm(M, N, K, 2.0, fg.Matrix(A, fg.FG_COL, M), fg.Matrix(B, fg.FG_COL, K), 0.0, None, fg.Matrix(call_other, fg.FG_COL, M))   # eager split-K work in between
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        say("split-K graph replay %d noalloc=%s" % (rep, noalloc))
        assert torch.equal(D, want), "replay %d differs from the eager result" % rep


def test_split_k_small_outputs_long_k():
    """Outputs with too few tiles to fill the GPU and a long K are computed as partial products
    over K ranges plus a reduction pass (the cross-workgroup reduction use of the epilogue,
    Section 4.2.5).  Exact on integers; epilogue, transforms, BF16, edge tiles and a row-major
    result go through the reduction pass."""
    assert "+splitk" in fg.fg_gemm_plan(512, 512, 8192)
    assert "+splitk" in fg.fg_gemm_plan(300, 200, 4096)
    say("split 512x512x8192 ints"); run_gemm_case(512, 512, 8192, ints=True)
    say("split 512x512x8192 floats"); run_gemm_case(512, 512, 8192, alpha=0.5, beta=2.0)
    say("split 300x200x4096 ragged, bias, relu, relu on C")
    run_gemm_case(300, 200, 4096, fg.FG_ROW, fg.FG_COL, ints=True, bias_dim=0, act=fg.FG_ACT_RELU, c_act=fg.FG_ACT_RELU, pad=8)
    say("split 300x200x4096 row-major D, bias along N")
    run_gemm_case(300, 200, 4096, fg.FG_COL, fg.FG_ROW, ld_layout=fg.FG_ROW, ints=True, bias_dim=1, alpha=-1.0, beta=0.25)
    say("split 64x64x32768 no C"); run_gemm_case(64, 64, 32768, with_c=False, ints=True)
    say("split 1024x1024x8192 floats sampled"); run_gemm_case(1024, 1024, 8192, fg.FG_ROW, fg.FG_ROW, samples=4096)
    say("split with K tail: 256x128x4104"); run_gemm_case(256, 128, 4104, ints=True)
    say("split bf16"); run_gemm_case(384, 256, 8192, ints=True, bf16=True)
    say("split with addition on A and B"); run_gemm_case(384, 256, 8192, ints=True, ab_add=(1.0, -1.0))
    say("split in place"); run_gemm_case(512, 512, 8192, ints=True, inplace=True)


def test_forced_split_counts(monkeypatch):
    """Every split count the planner can choose, forced on one ragged multi-tile problem, gives the
    same exact result (FG_FORCE_SPLIT is the library's tuning override)."""
    for S in (2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64):
        setenv(monkeypatch, "FG_FORCE_SPLIT", str(S))
        assert ("+splitk%d" % S) in fg.fg_gemm_plan(200, 136, 4160)
        say("forced split %d" % S); run_gemm_case(200, 136, 4160, ints=True, bias_dim=1, act=fg.FG_ACT_RELU)
    setenv(monkeypatch, "FG_FORCE_SPLIT", "1")
    assert "+splitk" not in fg.fg_gemm_plan(512, 512, 8192)
    run_gemm_case(512, 512, 8192, ints=True)


def test_every_entry_of_large_multi_tile_launches():
    """Every output entry (not a sample) of launches in which each persistent workgroup computes
    two tiles, with a short K so that the oracle can afford it: a fault that hits a few lanes of a
    few waves now and then shows up here, while a sample of positions can miss it."""
    say("8192x4096x64 NN ints, every entry"); run_gemm_case(8192, 4096, 64, ints=True)
    say("4096x8192x128 TT ints, bias, relu, every entry")
    run_gemm_case(4096, 8192, 128, fg.FG_ROW, fg.FG_ROW, ints=True, bias_dim=1, act=fg.FG_ACT_RELU)


def test_c_and_d_stored_as_binary16():
    """The type-conversion transform (Section 4.2.3): C and D live in memory as binary16, are
    widened when loaded and rounded to nearest even when stored, the arithmetic stays FP32.
    Integer data: every entry must equal the exact result rounded once to binary16."""
    for la, lb in itertools.product((fg.FG_COL, fg.FG_ROW), repeat=2):
        say("f16 C,D ints, layouts A=%d B=%d, ragged 300x200x256" % (la, lb))
        run_gemm_case(300, 200, 256, la, lb, ints=True, cd16=True)
    say("row-major C and D, odd leading dimension, bias along N, ReLU"); run_gemm_case(260, 190, 128, fg.FG_ROW, fg.FG_COL, ld_layout=fg.FG_ROW, ints=True, cd16=True, pad=8, bias_dim=1, act=fg.FG_ACT_RELU)
    say("no C, bias along M"); run_gemm_case(512, 256, 512, ints=True, cd16=True, with_c=False, bias_dim=0)
    say("in place, ReLU on C, beta = -3"); run_gemm_case(256, 384, 192, ints=True, cd16=True, inplace=True, c_act=fg.FG_ACT_RELU, beta=-3.0)
    say("every entry of a launch with two tiles per workgroup"); run_gemm_case(4096, 8192, 64, ints=True, cd16=True, samples=200000)
    say("floats, 1024x768x2048"); run_gemm_case(1024, 768, 2048, cd16=True, alpha=0.5, beta=-2.0)
    say("floats, 4096^3 sampled (the 256x256 tile)"); run_gemm_case(4096, 4096, 4096, fg.FG_COL, fg.FG_ROW, cd16=True, samples=4000)
    say("small tiles"); run_gemm_case(64, 72, 64, ints=True, cd16=True)


def test_binary16_c_and_d_whole_line_stores(monkeypatch):
    """With binary16 C and D the tiles whose waves hold at least two 32-row accumulators exchange
    half-registers between them so that loads and stores cover whole lines: every epilogue option
    on that path, on each such tile, with interior and edge waves in one launch.  Integer data:
    every entry must equal the exact result rounded once."""
    for tile in (0, 1, 2, 4):
        setenv(monkeypatch, "FG_FORCE_TILE", str(tile))
        say("tile %d: bias along N, ReLU, ReLU on C, beta = -3, in place" % tile)
        run_gemm_case(600, 520, 128, ints=True, cd16=True, bias_dim=1, act=fg.FG_ACT_RELU, c_act=fg.FG_ACT_RELU, beta=-3.0, inplace=True)
        say("tile %d: bias along M, no C, row-major D" % tile)
        run_gemm_case(520, 600, 192, fg.FG_ROW, fg.FG_ROW, ld_layout=fg.FG_ROW, ints=True, cd16=True, bias_dim=0, with_c=False, pad=8)
        say("tile %d: alpha = -2, beta = 1, separate C" % tile)
        run_gemm_case(512, 512, 64, fg.FG_COL, fg.FG_ROW, ints=True, cd16=True, alpha=-2.0)
    delenv(monkeypatch, "FG_FORCE_TILE")


def test_every_tile_shape_in_every_kernel_family(monkeypatch):
    """Each of the block tiles (256x256, 256x128, 128x128, 64x64, the 128x128 tile with a ring of
    four buffers, and the 256x256 tile on 16x16x32 matrix instructions) forced in turn on one
    ragged problem, for the plain, BF16, A/B-addition and binary16-result kernels and all four
    layout pairs: integer data, every entry exact.  The deep-ring tile is also run over a K that
    is shorter than its ring and with K split, the 16x16x32 kernel over short K and with K split."""
    for tile in range(6):
        setenv(monkeypatch, "FG_FORCE_TILE", str(tile))
        for la, lb in itertools.product((fg.FG_COL, fg.FG_ROW), repeat=2):
            say("tile %d layouts A=%d B=%d: plain, bf16, ab_add, f16 C,D" % (tile, la, lb))
            run_gemm_case(300, 264, 448, la, lb, ints=True, bias_dim=0)
            run_gemm_case(300, 264, 448, la, lb, ints=True, bf16=True)
            run_gemm_case(300, 264, 192, la, lb, ints=True, ab_add=(1.0, -2.0), c_act=fg.FG_ACT_RELU)
            run_gemm_case(300, 264, 448, la, lb, ints=True, cd16=True, act=fg.FG_ACT_RELU)
    setenv(monkeypatch, "FG_FORCE_TILE", "4")
    for K in (64, 128, 192, 256, 320):
        say("deep ring, K = %d" % K); run_gemm_case(256, 384, K, ints=True)
    setenv(monkeypatch, "FG_FORCE_SPLIT", "3")
    say("deep ring, K split in 3"); run_gemm_case(384, 256, 1536, fg.FG_ROW, fg.FG_COL, ints=True, bias_dim=1, act=fg.FG_ACT_RELU)
    delenv(monkeypatch, "FG_FORCE_SPLIT")
    setenv(monkeypatch, "FG_FORCE_TILE", "5")
    for K in (8, 64, 72, 128, 192, 520):
        say("16x16x32 kernel, K = %d" % K); run_gemm_case(300, 520, K, fg.FG_COL, fg.FG_ROW, ints=True, pad=8)
    say("16x16x32 kernel, A/B layouts x row-major D, bias along N, ReLU")
    for la, lb in itertools.product((fg.FG_COL, fg.FG_ROW), repeat=2):
        run_gemm_case(520, 300, 200, la, lb, ld_layout=fg.FG_ROW, ints=True, bias_dim=1, act=fg.FG_ACT_RELU, beta=-2.0)
    for la, lb in ((fg.FG_COL, fg.FG_COL), (fg.FG_ROW, fg.FG_ROW)):
        for K in (8, 72, 520, 1000):
            say("16x16x32 kernel with addition on A and B, layouts %d %d, K = %d" % (la, lb, K))
            run_gemm_case(300, 520, K, la, lb, ints=True, pad=8, ab_add=(3.0, -1.0), c_act=fg.FG_ACT_RELU)
    setenv(monkeypatch, "FG_FORCE_SPLIT", "3")
    say("16x16x32 kernel, K split in 3"); run_gemm_case(512, 256, 1536, fg.FG_ROW, fg.FG_COL, ints=True, bias_dim=0)
    say("16x16x32 kernel with addition on A and B, K split in 3"); run_gemm_case(512, 256, 1544, ints=True, ab_add=(1.0, 2.0))
    delenv(monkeypatch, "FG_FORCE_SPLIT")
    delenv(monkeypatch, "FG_FORCE_TILE")
    say("planner's own choice of the deep ring, floats"); assert "deep" in fg.fg_gemm_plan(2048, 2048, 2048)
    run_gemm_case(2048, 2048, 2048, samples=4000)


def test_operands_larger_than_2_gib():
    """A (then B) alone spans more than 2 GiB, once with K along columns and once along rows:
    the panels of the later tiles and the later K steps start beyond the reach of a 32-bit byte
    offset from the matrix base.  Integer data: every sampled entry must be exact."""
    say("A column-major 40000x32768 (2.4 GiB), ragged M"); run_gemm_case(40000, 192, 32768, ints=True, samples=1500)
    torch.cuda.empty_cache()
    say("A row-major 40000x32768"); run_gemm_case(40000, 192, 32768, la=fg.FG_ROW, ints=True, samples=1500, alpha=-1.0, beta=2.0)
    torch.cuda.empty_cache()
    say("B row-major 32768x40000"); run_gemm_case(192, 40000, 32768, lb=fg.FG_ROW, ints=True, samples=1500, with_c=False)
    torch.cuda.empty_cache()
    K = 4194240         # B is stored with K contiguous: its leading dimension must stay below 2^22
    assert "+splitk" in fg.fg_gemm_plan(320, 320, K)
    say("split K, A and B 2.5 GiB each: 320x320x%d" % K); run_gemm_case(320, 320, K, samples=300)
    torch.cuda.empty_cache()


def test_split_k_results_do_not_depend_on_arrival_order(monkeypatch):
    """The K ranges of a tile are computed by workgroups on different XCDs and added up from the
    workspace.  Many launches in a row on fresh data (a stale read would return a previous
    launch's partial products), more work items than resident workgroups, many K ranges per tile
    and ranges that are empty: integer data, every entry exact, every time."""
    cases = [(512, 512, 4096, 3, 8), (640, 1152, 2048, 3, 5), (1100, 900, 1536, 3, 7), (256, 384, 8192, 2, 16),
             (384, 256, 4096, 4, 6), (2100, 2112, 640, 3, 3), (128, 128, 576, 3, 4)]
    for rep in range(4):
        for (m, n, k, tile, S) in cases:
            setenv(monkeypatch, "FG_FORCE_TILE", str(tile))
            setenv(monkeypatch, "FG_FORCE_SPLIT", str(S))
            assert ("+splitk%d" % S) in fg.fg_gemm_plan(m, n, k)
            say("launch %d: %dx%dx%d tile %d split %d" % (rep, m, n, k, tile, S))
            run_gemm_case(m, n, k, fg.FG_COL if rep % 2 else fg.FG_ROW, fg.FG_COL, ints=True, seed=1000 + 17 * rep + S,
                          bias_dim=rep % 2, act=fg.FG_ACT_RELU if rep & 2 else fg.FG_ACT_NONE, beta=1.0 if rep % 3 else -2.0)
    delenv(monkeypatch, "FG_FORCE_TILE")
    delenv(monkeypatch, "FG_FORCE_SPLIT")
    for rep in range(6):
        say("planner's split, launch %d" % rep); run_gemm_case(512, 512, 8192, ints=True, seed=50 + rep)


def test_split_k_calls_on_two_streams_do_not_disturb_each_other():
    """All split-K calls of a GPU share one workspace.  The library orders a call against the
    previous user on another stream with an event, so two streams may issue such calls freely:
    forty launches alternating between two streams, each into its own output, must all equal the
    results of the same calls made one after the other."""
    from paper_2009_12263_amd import workloads as W
    shapes = [(512, 512, 8192), (384, 256, 8192)]
    for (M, N, K) in shapes:
        assert "+splitk" in fg.fg_gemm_plan(M, N, K)
    ops = []
    for i, (M, N, K) in enumerate(shapes):
        A = W.small_ints(M * K, 10 + i, device="cuda"); B = W.small_ints(K * N, 20 + i, device="cuda")
        ref = torch.empty(M * N, dtype=torch.float32, device="cuda")
        fg.fg_gemm(M, N, K, 1.0, fg.Matrix(A, fg.FG_COL, M), fg.Matrix(B, fg.FG_COL, K), 0.0, None, fg.Matrix(ref, fg.FG_COL, M))
        ops.append((M, N, K, A, B, ref))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = []
    for rep in range(20):
        for i, (M, N, K, A, B, ref) in enumerate(ops):
            D = torch.full_like(ref, float("nan"))
            outs.append((i, D))
    torch.cuda.synchronize()
    for n, (i, D) in enumerate(outs):
        M, N, K, A, B, ref = ops[i]
        fg.fg_gemm(M, N, K, 1.0, fg.Matrix(A, fg.FG_COL, M), fg.Matrix(B, fg.FG_COL, K), 0.0, None, fg.Matrix(D, fg.FG_COL, M), stream=streams[i])
    torch.cuda.synchronize()
    for n, (i, D) in enumerate(outs):
        assert torch.equal(D, ops[i][5]), "launch %d on stream %d differs from the serial result" % (n, i)


def test_tail_round_split(monkeypatch):
    """More tiles than the persistent grid holds at once, with a small remainder: the full rounds
    run as one pass and only the leftover tiles are split over K (plus the reduction pass).  Forced
    on small tiles so that the oracle can check every entry, then the planner's own choice."""
    setenv(monkeypatch, "FG_FORCE_TILE", "3")                      # 64x64 tiles: 1024 workgroups resident
    for S in (2, 3, 7):
        setenv(monkeypatch, "FG_FORCE_TAIL", str(S))
        assert ("+tailsplitk%d" % S) in fg.fg_gemm_plan(2100, 2112, 512)
        say("tail split %d on 33x33 tiles of 64x64, ragged edge" % S)
        run_gemm_case(2100, 2112, 512, ints=True, bias_dim=0, act=fg.FG_ACT_RELU)
    say("tail split, row-major operands and result, C with ReLU on C")
    run_gemm_case(2112, 2100, 456, fg.FG_ROW, fg.FG_ROW, ld_layout=fg.FG_ROW, ints=True, c_act=fg.FG_ACT_RELU, alpha=2.0, beta=-1.0)
    delenv(monkeypatch, "FG_FORCE_TILE")
    delenv(monkeypatch, "FG_FORCE_TAIL")
    assert "+tailsplitk" in fg.fg_gemm_plan(4100, 4100, 4096)
    say("planner's choice: 4100x4100x4096 floats sampled"); run_gemm_case(4100, 4100, 4096, samples=6000)
    say("planner's choice: 4100x4100x4096 ints sampled"); run_gemm_case(4100, 4100, 4096, ints=True, samples=6000, bias_dim=1)


@pytest.mark.parametrize("la,lb,ld", list(itertools.product(LAYOUTS, LAYOUTS, LAYOUTS)))
def test_unaligned_operands_use_the_general_kernel(la, lb, ld):
    """Odd leading dimensions, base pointers aligned to an element only and a K that is not a
    multiple of 8: real products fall back to the general kernel with the same semantics."""
    say("odd everything 70x45x13"); run_unaligned_gemm_case(70, 45, 13, la, lb, ld)
    say("several tiles, bias, relu, relu on C"); run_unaligned_gemm_case(150, 131, 77, la, lb, ld, bias_dim=0, act=fg.FG_ACT_RELU, c_act=fg.FG_ACT_RELU, alpha=2.0, beta=-1.0)
    say("floats"); run_unaligned_gemm_case(129, 65, 100, la, lb, ld, ints=False, alpha=0.5, beta=1.5, bias_dim=1)
    say("only K is odd (aligned operands)"); run_unaligned_gemm_case(128, 64, 60, la, lb, ld, pads=(0, 0, 0), offsets=(0, 0, 0))
    say("only a pointer is unaligned"); run_unaligned_gemm_case(128, 64, 64, la, lb, ld, pads=(0, 0, 0), offsets=(4, 0, 0))
    say("bf16"); run_unaligned_gemm_case(70, 45, 21, la, lb, ld, bf16=True)
    say("addition on A and B"); run_unaligned_gemm_case(70, 45, 21, la, lb, ld, ab_add=(1.0, -2.0), with_c=False)


def test_general_kernel_is_only_for_plain_real_products():
    H = torch.zeros(64 * 72 + 8, dtype=torch.float16, device="cuda")
    F = torch.zeros(64 * 72 + 8, dtype=torch.float32, device="cuda")
    kw = dict(raise_on_error=False)
    m = lambda t, **k: fg.Matrix(t, fg.FG_COL, 66, **k)          # ld = 66: not a multiple of 8
    assert fg.fg_gemm(64, 64, 64, 1.0, m(H), m(H), 0.0, None, m(F), **kw) == fg.FG_OK
    assert fg.fg_gemm(64, 64, 64, 1.0, m(H, im=H), m(H, im=H), 0.0, None, fg.Matrix(F, fg.FG_COL, 64, im=F), **kw) == fg.FG_ERR_ALIGN
    assert fg.fg_gemm(64, 64, 64, 1.0, fg.Matrix(H, fg.FG_DIAG, 0), m(H), 0.0, None, m(F), **kw) == fg.FG_ERR_ALIGN
    assert fg.fg_gemm(64, 64, 60, 1.0, fg.Matrix(H, fg.FG_DIAG, 0), fg.Matrix(H, fg.FG_COL, 64), 0.0, None, fg.Matrix(F, fg.FG_COL, 64), **kw) == fg.FG_ERR_UNSUPPORTED
    torch.cuda.synchronize()


def test_mfma_only_probes():
    """The two measurement kernels (32x32x16 and 16x16x32 instruction streams) run on a caller's
    buffer, report the same operation count per iteration, and reject bad arguments."""
    buf = torch.zeros(48 * 1024, dtype=torch.float16, device="cuda")
    for k32 in (False, True):
        assert fg.fg_probe_mfma(buf, 10, k32=k32) == 256 * 8 * 10 * 32 * 32768
    torch.cuda.synchronize()
    with pytest.raises(fg.FlexGemmError):
        fg.fg_probe_mfma(buf, 0, k32=True)
    with pytest.raises(fg.FlexGemmError):
        fg.fg_probe_mfma(buf[1:], 10, k32=True)       # not 16-byte aligned
    with pytest.raises(fg.FlexGemmError):
        fg.fg_probe_mfma(buf[:1024], 10)              # fewer than the 48 KiB the kernels read
    # the K loop's instruction mix: needs 128 KiB, walks a power-of-two window of the buffer (here 256 KiB
    # of a 300 KiB buffer whose tail is never touched), same operation count per iteration
    mix = torch.zeros(150 * 1024, dtype=torch.float16, device="cuda")
    assert fg.fg_probe_mfma(mix, 10, kloop_mix=True) == 256 * 8 * 10 * 32 * 32768
    torch.cuda.synchronize()
    with pytest.raises(fg.FlexGemmError):
        fg.fg_probe_mfma(buf, 10, kloop_mix=True)

