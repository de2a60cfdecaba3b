"""Pins for the CPU oracle: closed forms, identities, brute force and independent library
routines.  None of these tests touches the GPU library.

Each pin is aimed at a different plausible mistake: a transposed operand or leading dimension,
a dropped or mis-signed term, a wrong broadcast direction of the bias, a wrong merged-index
order in a contraction, a bad FP16 decode.
"""
import itertools

import numpy as np
import pytest

from oracle import cpu_oracle as O
from oracle.cpu_oracle import Operand, COL, ROW, DIAG, ACT_NONE, ACT_RELU

RNG = np.random.default_rng(20091226)


def store(mat: np.ndarray, layout: int, pad: int = 0):
    """Store a logical rows x cols float matrix as FP16 in the given layout with ``pad`` extra
    elements per leading dimension; returns (flat float16 buffer, ld, fp16-rounded logical matrix)."""
    rows, cols = mat.shape
    h = mat.astype(np.float16)
    if layout == COL:
        ld = rows + pad
        buf = np.full((cols, ld), np.float16(7.0))     # poison in the padding
        buf[:, :rows] = h.T
    else:
        ld = cols + pad
        buf = np.full((rows, ld), np.float16(7.0))
        buf[:, :cols] = h
    return np.ascontiguousarray(buf).reshape(-1), ld, h.astype(np.float64)


def rand_mat(r, c):
    return RNG.uniform(-1, 1, size=(r, c))


# ---------------------------------------------------------------- FP16 decode
def test_half_decode_matches_numpy_for_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([O.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


# ---------------------------------------------------------------- real GEMM
@pytest.mark.parametrize("la,lb", list(itertools.product([COL, ROW], [COL, ROW])))
@pytest.mark.parametrize("lc", [COL, ROW])
def test_gemm_matches_float64_matmul_all_layouts(la, lb, lc):
    M, N, K = 13, 9, 21
    A, lda, Ah = store(rand_mat(M, K), la, pad=3)
    B, ldb, Bh = store(rand_mat(K, N), lb, pad=5)
    Cm = rand_mat(M, N).astype(np.float32)
    Cbuf = np.ascontiguousarray(Cm.T if lc == COL else Cm).reshape(-1)
    ldc = M if lc == COL else N
    alpha, beta = 0.75, -1.5
    r = O.gemm(M, N, K, alpha, Operand(A, la, lda), Operand(B, lb, ldb), beta, Cbuf, None, lc, ldc, threads=3)
    want = alpha * (Ah @ Bh) + beta * Cm.astype(np.float64)
    assert np.allclose(r["D"], want, rtol=0, atol=1e-12)
    wantG = abs(alpha) * (np.abs(Ah) @ np.abs(Bh)) + abs(beta) * np.abs(Cm.astype(np.float64))
    assert np.allclose(r["G"], wantG, rtol=0, atol=1e-12)


def test_non_square_transposed_operand_is_not_confused_with_its_transpose():
    # A is 2x3 with distinct entries; a swapped (rows, cols) or ld reading gives a different product
    Am = np.array([[1., 2., 3.], [4., 5., 6.]])
    Bm = np.array([[1., 0.], [0., 1.], [2., -1.]])
    want = Am @ Bm
    for la, lb in itertools.product([COL, ROW], repeat=2):
        A, lda, _ = store(Am, la, pad=1)
        B, ldb, _ = store(Bm, lb, pad=2)
        r = O.gemm(2, 2, 3, 1.0, Operand(A, la, lda), Operand(B, lb, ldb))
        assert np.array_equal(r["D"], want), (la, lb)


@pytest.mark.parametrize("la,lb", list(itertools.product([COL, ROW], [COL, ROW])))
def test_identity_and_permutation(la, lb):
    n = 8
    Bm = RNG.integers(-5, 6, size=(n, n)).astype(np.float64)
    Cm = RNG.integers(-5, 6, size=(n, n)).astype(np.float32)
    perm = RNG.permutation(n)
    P = np.zeros((n, n)); P[np.arange(n), perm] = 1.0       # (P B)[i, :] = B[perm[i], :]
    B, ldb, _ = store(Bm, lb)
    for Amat, want_prod in ((np.eye(n), Bm), (P, Bm[perm, :])):
        A, lda, _ = store(Amat, la)
        r = O.gemm(n, n, n, 2.0, Operand(A, la, lda), Operand(B, lb, ldb), 3.0, Cm.T.copy().reshape(-1), None, COL, n)
        assert np.array_equal(r["D"], 2.0 * want_prod + 3.0 * Cm)
    # identity on the B side: A I = A
    A, lda, _ = store(Bm, la)
    I, ldi, _ = store(np.eye(n), lb)
    r = O.gemm(n, n, n, 1.0, Operand(A, la, lda), Operand(I, lb, ldi))
    assert np.array_equal(r["D"], Bm)


def test_rank_one_closed_form_is_exact():
    M, N, K = 6, 5, 37
    u = RNG.integers(-4, 5, size=M).astype(np.float64)
    v = RNG.integers(-4, 5, size=N).astype(np.float64)
    A, lda, _ = store(np.repeat(u[:, None], K, axis=1), COL)
    B, ldb, _ = store(np.repeat(v[None, :], K, axis=0), COL)
    r = O.gemm(M, N, K, 1.0, Operand(A, COL, lda), Operand(B, COL, ldb))
    assert np.array_equal(r["D"], K * np.outer(u, v))
    assert np.array_equal(r["G"], K * np.outer(np.abs(u), np.abs(v)))


def test_alpha_beta_linearity():
    M, N, K = 7, 6, 11
    A, lda, _ = store(rand_mat(M, K), ROW)
    B, ldb, _ = store(rand_mat(K, N), COL)
    Cb = rand_mat(M, N).astype(np.float32).T.copy().reshape(-1)
    a, b = 1.25, -0.5
    f = lambda al, be: O.gemm(M, N, K, al, Operand(A, ROW, lda), Operand(B, COL, ldb), be, Cb, None, COL, M)["D"]
    assert np.allclose(f(a, b), a * f(1, 0) + b * f(0, 1), rtol=0, atol=1e-13)
    assert np.array_equal(f(0, 1), Cb.reshape(N, M).T.astype(np.float64))


def test_transpose_consistency():
    # the same memory read as row-major rows x cols or as column-major cols x rows: A^T
    M, N, K = 5, 4, 6
    Am = rand_mat(M, K)
    A_row, ld_row, Ah = store(Am, ROW, pad=2)              # M x K row-major, ld = K + 2
    B, ldb, Bh = store(rand_mat(K, N), COL)
    r1 = O.gemm(M, N, K, 1.0, Operand(A_row, ROW, ld_row), Operand(B, COL, ldb))["D"]
    # explicit transpose stored column-major is the same buffer
    A_col, ld_col, _ = store(Am.T, COL, pad=2)             # K x M col-major, ld = K + 2
    assert np.array_equal(A_row, A_col) and ld_row == ld_col
    # and A^T used as the left operand of a (K x M)(M x N') product needs M x N' right operand
    Bm2 = rand_mat(M, 3); B2, ldb2, B2h = store(Bm2, COL)
    r2 = O.gemm(K, 3, M, 1.0, Operand(A_col, COL, ld_col), Operand(B2, COL, ldb2))["D"]
    assert np.allclose(r1, Ah @ Bh, atol=1e-13) and np.allclose(r2, Ah.T @ B2h, atol=1e-13)


def test_at_mode_equals_full_mode():
    M, N, K = 10, 12, 9
    A, lda, _ = store(rand_mat(M, K), COL, 1); B, ldb, _ = store(rand_mat(K, N), ROW, 1)
    bias = rand_mat(1, M).astype(np.float32).reshape(-1)
    kw = dict(bias=bias, bias_dim=0, act=ACT_RELU)
    full = O.gemm(M, N, K, 1.0, Operand(A, COL, lda), Operand(B, ROW, ldb), **kw)
    I = RNG.integers(0, M, size=40); J = RNG.integers(0, N, size=40)
    part = O.gemm(M, N, K, 1.0, Operand(A, COL, lda), Operand(B, ROW, ldb), at=(I, J), **kw)
    assert np.array_equal(part["D"], full["D"][I, J]) and np.array_equal(part["G"], full["G"][I, J])


def test_thread_count_does_not_change_results():
    M, N, K = 17, 19, 23
    A, lda, _ = store(rand_mat(M, K), COL); B, ldb, _ = store(rand_mat(K, N), COL)
    r1 = O.gemm(M, N, K, 1.0, Operand(A, COL, lda), Operand(B, COL, ldb), threads=1)["D"]
    r8 = O.gemm(M, N, K, 1.0, Operand(A, COL, lda), Operand(B, COL, ldb), threads=8)["D"]
    assert np.array_equal(r1, r8)


# ---------------------------------------------------------------- epilogues
def test_bias_direction_and_relu_by_brute_force():
    M, N, K = 4, 3, 5
    Am = RNG.integers(-3, 4, size=(M, K)).astype(np.float64)
    Bm = RNG.integers(-3, 4, size=(K, N)).astype(np.float64)
    A, lda, _ = store(Am, COL); B, ldb, _ = store(Bm, COL)
    bias_m = np.array([100., 200., 300., 400.], np.float32)       # per row i
    bias_n = np.array([1000., 2000., 3000.], np.float32)          # per column j
    for dim, bias in ((0, bias_m), (1, bias_n)):
        for act in (ACT_NONE, ACT_RELU):
            r = O.gemm(M, N, K, -1.0, Operand(A, COL, lda), Operand(B, COL, ldb), bias=bias, bias_dim=dim, act=act)["D"]
            for i in range(M):
                for j in range(N):
                    y = -sum(Am[i, k] * Bm[k, j] for k in range(K)) + float(bias[i] if dim == 0 else bias[j])
                    assert r[i, j] == (max(y, 0.0) if act == ACT_RELU else y)


def test_relu_properties_and_order_of_operations():
    M = N = K = 16
    A, lda, _ = store(rand_mat(M, K), COL); B, ldb, _ = store(rand_mat(K, N), COL)
    Cb = (4 * rand_mat(M, N)).astype(np.float32).T.copy().reshape(-1)
    bias = (2 * rand_mat(1, M)).astype(np.float32).reshape(-1)
    kw = dict(beta=0.5, C_re=Cb, ldc=M, bias=bias, bias_dim=0)
    y = O.gemm(M, N, K, 1.0, Operand(A, COL, lda), Operand(B, COL, ldb), **kw)["D"]
    d = O.gemm(M, N, K, 1.0, Operand(A, COL, lda), Operand(B, COL, ldb), act=ACT_RELU, **kw)["D"]
    assert (y < 0).any() and (y > 0).any()
    assert (d >= 0).all() and np.array_equal(d[y > 0], y[y > 0]) and (d[y <= 0] == 0).all()


# ---------------------------------------------------------------- diagonal operands
def test_diagonal_equals_materialised_dense_and_closed_form():
    n = 12
    d = RNG.uniform(-1, 1, n).astype(np.float16)
    Bm = rand_mat(n, n); B, ldb, Bh = store(Bm, COL)
    Cm = rand_mat(n, n).astype(np.float32); Cb = Cm.T.copy().reshape(-1)
    dense, ldd, _ = store(np.diag(d.astype(np.float64)), COL)
    r_diag = O.gemm(n, n, n, 1.0, Operand(d, DIAG, 0), Operand(B, COL, ldb), 1.0, Cb, None, COL, n)
    r_dense = O.gemm(n, n, n, 1.0, Operand(dense, COL, ldd), Operand(B, COL, ldb), 1.0, Cb, None, COL, n)
    assert np.array_equal(r_diag["D"], r_dense["D"]) and np.array_equal(r_diag["G"], r_dense["G"])
    assert np.allclose(r_diag["D"], d.astype(np.float64)[:, None] * Bh + Cm, atol=1e-14)
    # diagonal on the right: column scaling
    A, lda, Ah = store(rand_mat(n, n), ROW)
    r = O.gemm(n, n, n, 1.0, Operand(A, ROW, lda), Operand(d, DIAG, 0))
    assert np.allclose(r["D"], Ah * d.astype(np.float64)[None, :], atol=1e-14)


# ---------------------------------------------------------------- planar complex
def test_complex_matches_complex128_product():
    M, N, K = 7, 5, 9
    Ar, lda, Arh = store(rand_mat(M, K), COL, 1); Ai, _, Aih = store(rand_mat(M, K), COL, 1)
    Br, ldb, Brh = store(rand_mat(K, N), ROW, 2); Bi, _, Bih = store(rand_mat(K, N), ROW, 2)
    Cr = rand_mat(M, N).astype(np.float32); Ci = rand_mat(M, N).astype(np.float32)
    r = O.gemm(M, N, K, 1.0, Operand(Ar, COL, lda, Ai), Operand(Br, ROW, ldb, Bi), 1.0,
               Cr.T.copy().reshape(-1), Ci.T.copy().reshape(-1), COL, M)
    want = (Arh + 1j * Aih) @ (Brh + 1j * Bih) + (Cr + 1j * Ci)
    assert np.allclose(r["D"], want.real, atol=1e-13) and np.allclose(r["D_im"], want.imag, atol=1e-13)
    Gr = np.abs(Arh) @ np.abs(Brh) + np.abs(Aih) @ np.abs(Bih) + np.abs(Cr)
    Gi = np.abs(Arh) @ np.abs(Bih) + np.abs(Aih) @ np.abs(Brh) + np.abs(Ci)
    assert np.allclose(r["G"], Gr, atol=1e-13) and np.allclose(r["G_im"], Gi, atol=1e-13)


def test_complex_closed_form_i_times_identity():
    n = 6
    Z, ldz, _ = store(np.zeros((n, n)), COL); I, _, _ = store(np.eye(n), COL)
    Br, ldb, Brh = store(RNG.integers(-4, 5, (n, n)).astype(float), COL)
    Bi, _, Bih = store(RNG.integers(-4, 5, (n, n)).astype(float), COL)
    r = O.gemm(n, n, n, 1.0, Operand(Z, COL, ldz, I), Operand(Br, COL, ldb, Bi))    # A = i * I
    assert np.array_equal(r["D"], -Bih) and np.array_equal(r["D_im"], Brh)          # i (Br + i Bi) = -Bi + i Br


# ---------------------------------------------------------------- contractions
def brute_contract(ext, mA, sA, A, mB, sB, B, mC, sC, alpha=1.0, beta=0.0, Cin=None):
    """Independent brute force: enumerate every assignment of every mode with itertools.product."""
    labels = sorted(set(mA) | set(mB) | set(mC))
    out = {}
    for assign in itertools.product(*[range(ext[l]) for l in labels]):
        ix = dict(zip(labels, assign))
        oa = sum(ix[m] * s for m, s in zip(mA, sA)); ob = sum(ix[m] * s for m, s in zip(mB, sB))
        oc = sum(ix[m] * s for m, s in zip(mC, sC))
        out[oc] = out.get(oc, 0.0) + float(A[oa]) * float(B[ob])
    res = {}
    for oc, v in out.items():
        res[oc] = alpha * v + (beta * float(Cin[oc]) if Cin is not None else 0.0)
    return res


def dense(ext, modes):
    return O_col_strides([ext[m] for m in modes])


def O_col_strides(e):
    st, s = [], 1
    for x in e:
        st.append(s); s *= x
    return st


CASES = [
    # (extents, modesA, modesB, modesC): labels are small integers
    ({0: 4, 1: 3, 2: 2, 3: 5}, [0, 3, 2], [3, 1], [0, 1, 2]),              # C[a,b,c] = sum_d A[a,d,c] B[d,b]
    ({0: 2, 1: 3, 2: 2, 3: 3, 4: 4, 5: 2}, [0, 4, 1, 5], [3, 5, 2, 4], [0, 1, 2, 3]),  # two contracted modes
    ({0: 3, 1: 2, 2: 4, 3: 3}, [1, 3, 0], [3, 2], [0, 1, 2]),              # D_abc = A_bda B_dc (Section 5.5)
    ({0: 3, 1: 4}, [0, 1], [1], [0]),                                       # matrix-vector
    ({0: 3, 1: 2, 2: 4, 3: 3, 4: 2}, [0, 3, 4], [3, 1, 4], [0, 1, 4]),      # batch mode 4: in A, B and C
    ({0: 3, 1: 2, 3: 3, 4: 2, 5: 3}, [4, 0, 3, 5], [5, 3, 1, 4], [4, 0, 5, 1]),  # two batch modes, interleaved
]


@pytest.mark.parametrize("ext,mA,mB,mC", CASES)
def test_contraction_matches_brute_force_and_einsum(ext, mA, mB, mC):
    sA, sB, sC = dense(ext, mA), dense(ext, mB), dense(ext, mC)
    nA = int(np.prod([ext[m] for m in mA])); nB = int(np.prod([ext[m] for m in mB])); nC = int(np.prod([ext[m] for m in mC]))
    A = RNG.integers(-4, 5, nA).astype(np.float16); B = RNG.integers(-4, 5, nB).astype(np.float16)
    Cin = RNG.integers(-4, 5, nC).astype(np.float32)
    r = O.contract(ext, mA, sA, A, mB, sB, B, mC, sC, Cin, alpha=2.0, beta=-1.0, threads=2)
    want = brute_contract(ext, mA, sA, A, mB, sB, B, mC, sC, 2.0, -1.0, Cin)
    assert len(want) == nC
    for oc, v in want.items():
        assert r["D"][oc] == v
    # numpy.einsum on Fortran-ordered views (first listed mode fastest)
    letters = "abcdefgh"
    sub = lambda ms: "".join(letters[m] for m in ms)
    At = A.astype(np.float64).reshape([ext[m] for m in mA], order="F")
    Bt = B.astype(np.float64).reshape([ext[m] for m in mB], order="F")
    Ct = Cin.astype(np.float64).reshape([ext[m] for m in mC], order="F")
    E = 2.0 * np.einsum(f"{sub(mA)},{sub(mB)}->{sub(mC)}", At, Bt) - Ct
    assert np.array_equal(r["D"].reshape(E.shape, order="F"), E)
    G = 2.0 * np.einsum(f"{sub(mA)},{sub(mB)}->{sub(mC)}", np.abs(At), np.abs(Bt)) + np.abs(Ct)
    assert np.array_equal(r["G"].reshape(E.shape, order="F"), G)


def test_contraction_non_dense_strides_and_at_mode():
    ext = {0: 3, 1: 2, 2: 4}
    mA, mB, mC = [0, 2], [2, 1], [1, 0]            # C[b,a] = sum_c A[a,c] B[c,b], C stored transposed
    sA, sB, sC = [1, 5], [2, 9], [1, 4]            # padded / strided storage
    A = RNG.integers(-4, 5, 1 + 2 * 1 + 3 * 5).astype(np.float16)
    B = RNG.integers(-4, 5, 1 + 3 * 2 + 1 * 9).astype(np.float16)
    r = O.contract(ext, mA, sA, A, mB, sB, B, mC, sC)
    want = brute_contract(ext, mA, sA, A, mB, sB, B, mC, sC)
    for oc, v in want.items():
        assert r["D"][oc] == v
    at = np.array([[1, 2], [0, 0], [1, 1]])          # (b, a) pairs
    ra = O.contract(ext, mA, sA, A, mB, sB, B, mC, sC, at=at)
    for (b, a), v in zip(at, ra["D"]):
        assert v == want[b * 1 + a * 4]


def test_contraction_with_delta_is_a_mode_permutation():
    # C[a,b,c] = sum_d A[a,d,c] delta[d,b]  =>  C[a,b,c] = A[a,b,c]
    n = 4
    ext = {0: n, 1: n, 2: n, 3: n}
    A = RNG.integers(-8, 9, n ** 3).astype(np.float16)
    delta = np.eye(n, dtype=np.float16).reshape(-1)
    st3 = O_col_strides([n, n, n])
    r = O.contract(ext, [0, 3, 2], st3, A, [3, 1], [1, n], delta, [0, 1, 2], st3)
    assert np.array_equal(r["D"], A.astype(np.float64))


def test_merged_index_convention_of_the_gett_layout():
    """Section 5.5 maps A_bda to a matrix A_mk with m = (b a), k = d, and gives the element
    position as b + d*Nb + a*Nb*Nd (zero-based) with a = m div Nb, b = m mod Nb: the first
    written mode of a merged index is the fastest.  The GEMM oracle on matrices built with that
    formula must reproduce the contraction oracle, with D_(ba),c unshuffled to D_abc."""
    Na, Nb, Nc, Nd = 3, 4, 5, 6
    ext = {0: Na, 1: Nb, 2: Nc, 3: Nd}
    A = RNG.integers(-4, 5, Nb * Nd * Na).astype(np.float16)     # A[b,d,a], b fastest
    B = RNG.integers(-4, 5, Nd * Nc).astype(np.float16)          # B[d,c]
    r = O.contract(ext, [1, 3, 0], [1, Nb, Nb * Nd], A, [3, 2], [1, Nd], B, [0, 1, 2], [1, Na, Na * Nb])
    M, K, N = Na * Nb, Nd, Nc
    Amat = np.zeros((M, K), np.float64)
    for m in range(M):
        a, b = m // Nb, m % Nb
        for k in range(K):
            Amat[m, k] = float(A[b + k * Nb + a * Nb * Nd])
    Am, lda, _ = store(Amat, COL)
    g = O.gemm(M, N, K, 1.0, Operand(Am, COL, lda), Operand(B, COL, Nd))["D"]        # rows m = (b a)
    D = r["D"].reshape((Na, Nb, Nc), order="F")
    for a in range(Na):
        for b in range(Nb):
            assert np.array_equal(D[a, b, :], g[b + a * Nb, :])


def test_bad_descriptions_are_rejected():
    A = np.zeros(4, np.float16)
    with pytest.raises(ValueError):
        O.gemm(2, 2, 2, 1.0, Operand(A, COL, 1), Operand(A, COL, 2))          # ld too small
    with pytest.raises(ValueError):
        O.gemm(2, 2, 3, 1.0, Operand(A, COL, 2), Operand(A, COL, 3))          # buffer too short
    with pytest.raises(ValueError):
        O.contract({0: 2, 1: 2}, [0, 1], [1, 2], A, [1], [1], A[:2], [0, 5], [1, 2])  # unknown mode in C
    with pytest.raises(ValueError):
        O.gemm(2, 2, 2, 1.0, Operand(A, COL, 2, A), Operand(A, COL, 2), act=ACT_RELU)  # ReLU of a complex value


# ---------------------------------------------------------------- bfloat16 inputs
def test_bf16_decode_matches_torch_for_every_bit_pattern():
    import torch
    bits = torch.arange(65536, dtype=torch.int32).to(torch.int16)
    want = bits.view(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([O.bf16_to_double(int(b) & 0xFFFF) for b in bits.tolist()])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_bf16_gemm_matches_float64_matmul():
    import torch
    M, N, K = 9, 7, 13
    At = torch.from_numpy(rand_mat(M, K)).to(torch.bfloat16)          # logical M x K
    Bt = torch.from_numpy(rand_mat(K, N)).to(torch.bfloat16)
    bits = lambda t: t.contiguous().view(torch.int16).numpy().view(np.uint16).reshape(-1)
    A = bits(At.t())                                                  # column-major storage, ld = M
    B = bits(Bt)                                                      # row-major storage, ld = N
    r = O.gemm(M, N, K, 1.0, Operand(A, COL, M, dtype=O.BF16), Operand(B, ROW, N, dtype=O.BF16))
    want = At.to(torch.float64).numpy() @ Bt.to(torch.float64).numpy()
    assert np.allclose(r["D"], want, rtol=0, atol=1e-12)
    # the same bits read as binary16 give a different (wrong) product: the dtype flag matters
    r16 = O.gemm(M, N, K, 1.0, Operand(A, COL, M, dtype=O.F16), Operand(B, ROW, N, dtype=O.F16))
    assert not np.allclose(r16["D"], want, rtol=1e-3, atol=1e-3)


# ---------------------------------------------------------------- dual numbers
def test_dual_product_is_value_and_first_derivative():
    # A(t) = Ar + t Ad, B(t) = Br + t Bd:  A(t) B(t) = Ar Br + t (Ar Bd + Ad Br) + t^2 Ad Bd.
    # The dual product keeps the first two coefficients; with integers, the coefficient of t is
    # (P(1) - P(-1)) / 2 exactly, evaluated here with two ordinary matrix products.
    M, N, K = 6, 5, 9
    Ar, Ad = (RNG.integers(-4, 5, size=(M, K)).astype(np.float64) for _ in range(2))
    Br, Bd = (RNG.integers(-4, 5, size=(K, N)).astype(np.float64) for _ in range(2))
    Cr, Cd = (RNG.integers(-4, 5, size=(M, N)).astype(np.float32) for _ in range(2))
    a_re, lda, _ = store(Ar, ROW); a_du, _, _ = store(Ad, ROW)
    b_re, ldb, _ = store(Br, COL); b_du, _, _ = store(Bd, COL)
    r = O.gemm(M, N, K, 2.0, Operand(a_re, ROW, lda, a_du), Operand(b_re, COL, ldb, b_du), 3.0,
               Cr.T.copy().reshape(-1), Cd.T.copy().reshape(-1), COL, M, dual=True)
    P = lambda t: (Ar + t * Ad) @ (Br + t * Bd)
    assert np.array_equal(r["D"], 2.0 * (Ar @ Br) + 3.0 * Cr)
    assert np.array_equal(r["D_im"], 2.0 * (P(1) - P(-1)) / 2 + 3.0 * Cd)
    # and it differs from the complex product exactly by the eps.eps term
    c = O.gemm(M, N, K, 2.0, Operand(a_re, ROW, lda, a_du), Operand(b_re, COL, ldb, b_du), 3.0,
               Cr.T.copy().reshape(-1), Cd.T.copy().reshape(-1), COL, M)
    assert np.array_equal(r["D"] - c["D"], 2.0 * (Ad @ Bd))
    assert np.array_equal(r["D_im"], c["D_im"])
    assert np.array_equal(r["G"], 2.0 * (np.abs(Ar) @ np.abs(Br)) + 3.0 * np.abs(Cr))


# ---------------------------------------------------------------- transforms on loaded elements
def _nearest_half_exact(x):
    """Round a Fraction to binary16 with ties to even by searching the table of all finite values."""
    from fractions import Fraction
    import bisect
    if not hasattr(_nearest_half_exact, "tab"):
        bits = np.arange(0, 0x7C00, dtype=np.uint16)                 # non-negative finite values, ascending
        _nearest_half_exact.tab = [Fraction(float(v)) for v in bits.view(np.float16)]
    tab = _nearest_half_exact.tab
    sign, ax = (-1, -x) if x < 0 else (1, x)
    if ax >= Fraction(65520):
        return sign * float("inf")
    hi = bisect.bisect_left(tab, ax)
    if hi == len(tab):
        return sign * float(tab[-1])
    if tab[hi] == ax or hi == 0:
        return sign * float(tab[hi])
    lo = hi - 1
    dl, dh = ax - tab[lo], tab[hi] - ax
    pick = lo if dl < dh else hi if dh < dl else (lo if lo % 2 == 0 else hi)   # even bit pattern = even mantissa
    return sign * float(tab[pick])


def test_round_to_half_against_exact_rational_rounding():
    from fractions import Fraction
    bits = RNG.integers(0, 65536, size=(6000, 2)).astype(np.uint16)
    vals = bits.view(np.float16).astype(np.float64)
    ok = np.isfinite(vals).all(axis=1)
    # add pairs that straddle binades, subnormals and the overflow threshold
    extra = np.array([[65504.0, 16.0], [65504.0, 15.99], [65504.0, 8.0], [2.0 ** -24, 2.0 ** -24], [2.0 ** -14, -2.0 ** -24],
                      [1.0, 2.0 ** -11], [1.0, 3 * 2.0 ** -12], [1.0 + 2.0 ** -10, 2.0 ** -11], [-2048.0, -1.0], [0.1, -0.1]])
    extra = extra.astype(np.float16).astype(np.float64)
    for a, b in np.concatenate([vals[ok], extra]):
        want = _nearest_half_exact(Fraction(a) + Fraction(b))
        got = O.round_to_half(a + b)          # a + b is exact in double
        assert got == want, (a, b, got, want)


def test_ab_add_and_relu_on_c_by_brute_force():
    M, N, K = 5, 4, 7
    Am, Bm = rand_mat(M, K), rand_mat(K, N)
    A, lda, Ah = store(Am, ROW, pad=1); B, ldb, Bh = store(Bm, ROW, pad=2)
    Cm = rand_mat(M, N).astype(np.float32)
    bias = rand_mat(1, N).astype(np.float32).reshape(-1)
    a_add, b_add = float(np.float16(0.3)), float(np.float16(-1.7))
    r = O.gemm(M, N, K, 1.5, Operand(A, ROW, lda), Operand(B, ROW, ldb), -0.5, Cm.T.copy().reshape(-1), None, COL, M,
               bias=bias, bias_dim=1, act=ACT_RELU, ab_add=(a_add, b_add), c_act=ACT_RELU)
    # numpy float16 addition of moderate values rounds once (float32 holds the exact sum)
    A2 = (Ah.astype(np.float16) + np.float16(a_add)).astype(np.float64)
    B2 = (Bh.astype(np.float16) + np.float16(b_add)).astype(np.float64)
    want = np.zeros((M, N))
    for i in range(M):
        for j in range(N):
            acc = sum(A2[i, k] * B2[k, j] for k in range(K))
            want[i, j] = max(1.5 * acc - 0.5 * max(float(Cm[i, j]), 0.0) + float(bias[j]), 0.0)
    assert np.allclose(r["D"], want, rtol=0, atol=1e-12)
    # the tolerance denominator under the transforms: |alpha| sum_k |A'_ik| |B'_kj| + |beta| |relu(C_ij)|,
    # with the transformed elements (the bias is not part of it)
    want_g = np.zeros((M, N))
    for i in range(M):
        for j in range(N):
            want_g[i, j] = 1.5 * sum(abs(A2[i, k]) * abs(B2[k, j]) for k in range(K)) + 0.5 * max(float(Cm[i, j]), 0.0)
    assert np.allclose(r["G"], want_g, rtol=0, atol=1e-12)
    # ... and it must differ from the denominator of the untransformed product (so that a G that
    # ignored the transforms would fail here): negative C entries exist, and the addends change |A'||B'|
    r_plain = O.gemm(M, N, K, 1.5, Operand(A, ROW, lda), Operand(B, ROW, ldb), -0.5, Cm.T.copy().reshape(-1), None, COL, M,
                     bias=bias, bias_dim=1, act=ACT_RELU)
    assert (Cm < 0).any() and not np.allclose(r_plain["G"], want_g, rtol=1e-3, atol=0)
    # each transform alone
    r_c = O.gemm(M, N, K, 1.5, Operand(A, ROW, lda), Operand(B, ROW, ldb), -0.5, Cm.T.copy().reshape(-1), None, COL, M, c_act=ACT_RELU)
    g_c = 1.5 * np.abs(Ah.astype(np.float64)) @ np.abs(Bh.astype(np.float64)) + 0.5 * np.maximum(Cm.astype(np.float64), 0.0)
    assert np.allclose(r_c["G"], g_c, rtol=0, atol=1e-12)
    r_ab = O.gemm(M, N, K, 1.5, Operand(A, ROW, lda), Operand(B, ROW, ldb), -0.5, Cm.T.copy().reshape(-1), None, COL, M, ab_add=(a_add, b_add))
    g_ab = 1.5 * np.abs(A2) @ np.abs(B2) + 0.5 * np.abs(Cm.astype(np.float64))
    assert np.allclose(r_ab["G"], g_ab, rtol=0, atol=1e-12)
    # a zero addend and no activation on C give back the plain product
    r0 = O.gemm(M, N, K, 1.5, Operand(A, ROW, lda), Operand(B, ROW, ldb), -0.5, Cm.T.copy().reshape(-1), None, COL, M, ab_add=(0.0, 0.0))
    r1 = O.gemm(M, N, K, 1.5, Operand(A, ROW, lda), Operand(B, ROW, ldb), -0.5, Cm.T.copy().reshape(-1), None, COL, M)
    assert np.array_equal(r0["D"], r1["D"])
    with pytest.raises(ValueError):
        O.gemm(M, N, K, 1.0, Operand(A, ROW, lda), Operand(B, ROW, ldb), ab_add=(0.3, 0.0))     # 0.3 is not a binary16 value


# ---------------------------------------------------------------- interleaved complex storage
@pytest.mark.parametrize("la,lb,lc", list(itertools.product([COL, ROW], [COL, ROW], [COL, ROW])))
def test_interleaved_complex_matches_complex128_matmul(la, lb, lc):
    M, N, K = 7, 5, 9

    def store_c(re, im, layout, pad):
        buf_r, ld, hr = store(re, layout, pad)
        buf_i, _, hi = store(im, layout, pad)
        inter = np.empty(buf_r.size * 2, buf_r.dtype)
        inter[0::2], inter[1::2] = buf_r, buf_i
        return inter, ld, hr + 1j * hi

    A, lda, Ac = store_c(rand_mat(M, K), rand_mat(M, K), la, 2)
    B, ldb, Bc = store_c(rand_mat(K, N), rand_mat(K, N), lb, 1)
    Cr, Ci = rand_mat(M, N).astype(np.float32), rand_mat(M, N).astype(np.float32)
    lead = Cr.T if lc == COL else Cr
    Cint = np.empty(2 * M * N, np.float32)
    Cint[0::2] = np.ascontiguousarray(Cr.T if lc == COL else Cr).reshape(-1)
    Cint[1::2] = np.ascontiguousarray(Ci.T if lc == COL else Ci).reshape(-1)
    ldc = M if lc == COL else N
    r = O.gemm(M, N, K, 0.5, Operand(A, la, lda, interleaved=True), Operand(B, lb, ldb, interleaved=True), -2.0,
               Cint, None, lc, ldc, c_interleaved=True)
    want = 0.5 * (Ac @ Bc) - 2.0 * (Cr.astype(np.float64) + 1j * Ci.astype(np.float64))
    assert np.allclose(r["D"] + 1j * r["D_im"], want, rtol=0, atol=1e-12)
    # the same numbers in planar storage give the same result
    Ar, _, _ = store(Ac.real, la, 2); Ai, _, _ = store(Ac.imag, la, 2)
    Br, _, _ = store(Bc.real, lb, 1); Bi, _, _ = store(Bc.imag, lb, 1)
    r2 = O.gemm(M, N, K, 0.5, Operand(Ar, la, lda, Ai), Operand(Br, lb, ldb, Bi), -2.0,
                np.ascontiguousarray(Cr.T if lc == COL else Cr).reshape(-1), np.ascontiguousarray(Ci.T if lc == COL else Ci).reshape(-1), lc, ldc)
    assert np.array_equal(r["D"], r2["D"]) and np.array_equal(r["D_im"], r2["D_im"])


def test_round_array_to_half_matches_an_independent_conversion():
    """The rounding applied to results stored as binary16, against numpy's own double -> half
    conversion (an independent implementation of round-to-nearest-even): random values over the
    whole exponent range, exact ties at every scale, the subnormal range, and values at and
    beyond the largest finite binary16 number."""
    rng = np.random.default_rng(7)
    x = np.concatenate([
        rng.standard_normal(4000) * 10.0 ** rng.integers(-9, 5, 4000),
        (np.arange(1, 4097) + 0.5) * 2.0 ** -3,                     # ties between neighbours, ulp 2^-3 .. 2^-1
        (2048 + np.arange(0, 600)) * 1.0 + 0.0,                      # integers above 2048: every other one is a tie
        np.arange(-40, 40) * 2.0 ** -25,                             # around the smallest subnormal 2^-24
        np.array([65504.0, 65519.99, 65520.0, 65535.0, 1e6, -65520.0, 0.0, -0.0]),
    ])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).astype(np.float64)
    got = O.round_array_to_half(x)
    assert np.array_equal(got, want)
    assert np.array_equal(np.signbit(got), np.signbit(want))


def test_gemm_with_binary16_c_uses_the_stored_values():
    """C stored as binary16 is widened exactly: with A = I the result is alpha B + beta C on the
    binary16 values of C, and the same problem with C widened by hand gives the same numbers."""
    n = 24
    rng = np.random.default_rng(3)
    A = np.eye(n, dtype=np.float16)
    B = rng.uniform(-1, 1, (n, n)).astype(np.float16)
    Ch = rng.uniform(-4, 4, n * n).astype(np.float16)
    r = O.gemm(n, n, n, 2.0, O.Operand(A.T.copy().reshape(-1), O.COL, n), O.Operand(B.T.copy().reshape(-1), O.COL, n),
               -0.5, Ch, None, O.COL, n)
    want = 2.0 * B.astype(np.float64) - 0.5 * Ch.astype(np.float64).reshape(n, n).T
    assert np.array_equal(r["D"], want)
    r32 = O.gemm(n, n, n, 2.0, O.Operand(A.T.copy().reshape(-1), O.COL, n), O.Operand(B.T.copy().reshape(-1), O.COL, n),
                 -0.5, Ch.astype(np.float32), None, O.COL, n)
    assert np.array_equal(r["D"], r32["D"]) and np.array_equal(r["G"], r32["G"])
