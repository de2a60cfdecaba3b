"""CPU-only tests of the C ABI: the library loads, exports every declared symbol, and rejects
bad descriptions with the documented status codes before anything is launched."""
import ctypes as C
import os
import re

import pytest

from paper_2009_12263_amd import binding as fg


def delenv(monkeypatch, name, raising=True):
    monkeypatch.delenv(name, raising=raising)
    fg.fg_reload_tuning()


def setenv(monkeypatch, name, value):
    monkeypatch.setenv(name, value)
    fg.fg_reload_tuning()

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "flexgemm.h")).read()
    declared = set(re.findall(r"\b(fg_[a-z0-9_]+)\s*\(", header))
    assert declared == set(fg.EXPORTS)
    lib = fg.load_library()
    for name in declared:
        assert getattr(lib, name) is not None
    assert fg.fg_version() >= 100


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 (and as C++), and a C program that only
    includes it links against the shared library and can make the calls that need no GPU."""
    import shutil
    import subprocess
    if not shutil.which("gcc"):
        pytest.skip("no host C compiler")
    src = tmp_path / "use.c"
    src.write_text(
        '#include <stdio.h>\n#include "flexgemm.h"\n'
        "int main(void) {\n"
        "    char name[64];\n"
        "    fg_matrix m; m.re = 0; m.im = 0; m.dtype = FG_F16; m.layout = FG_COL; m.ld = 8;\n"
        "    if (fg_version() < 100) return 1;\n"
        "    if (fg_gemm_plan(8192, 8192, 8192, FG_COL, FG_COL, FG_COL, FG_PLAN_REAL, name, (int32_t)sizeof name) != FG_OK) return 2;\n"
        "    if (fg_gemm(8, 8, 8, 1.0f, 0, &m, 0.0f, 0, &m, 0, 0) != FG_ERR_NULL) return 3;\n"
        '    printf("%s|%s\\n", name, fg_last_error());\n'
        "    return 0;\n}\n")
    inc = os.path.join(ROOT, "include")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, "-fsyntax-only", str(src)])
    if shutil.which("g++"):
        subprocess.check_call(["g++", "-std=c++11", "-Wall", "-I", inc, "-fsyntax-only", "-x", "c++", str(src)])
    exe = tmp_path / "use"
    libdir = os.path.dirname(fg.LIB_PATH)
    subprocess.check_call(["gcc", "-std=c99", "-I", inc, str(src), "-o", str(exe), "-L", libdir, "-l:libflexgemm.so", "-Wl,-rpath," + libdir])
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0, out
    plan, err = out.stdout.strip().split("|")
    assert plan == "gemm_nn_256x256x64_k32" and "A is NULL" in err


class FakeTensor:
    """Stands in for a device tensor: the library only looks at the pointer value before launch."""
    def __init__(self, ptr, dtype):
        self._p, self.dtype = ptr, dtype

    def data_ptr(self):
        return self._p


def mats(M=256, N=256, K=256, la=fg.FG_COL, lb=fg.FG_COL, ld=fg.FG_COL, lda=None, ldb=None, ldd=None, pa=0x1000, pb=0x2000, pd=0x3000):
    import torch
    A = fg.Matrix(FakeTensor(pa, torch.float16), la, lda if lda is not None else (M if la == fg.FG_COL else K))
    B = fg.Matrix(FakeTensor(pb, torch.float16), lb, ldb if ldb is not None else (K if lb == fg.FG_COL else N))
    D = fg.Matrix(FakeTensor(pd, torch.float32), ld, ldd if ldd is not None else (M if ld == fg.FG_COL else N))
    return A, B, D


def status(*args, **kw):
    return fg.fg_gemm(*args, raise_on_error=False, **kw)


def test_gemm_argument_errors():
    A, B, D = mats()
    assert status(256, 256, 256, 1.0, None, B, 0.0, None, D) == fg.FG_ERR_NULL
    assert status(256, 256, 256, 1.0, A, B, 0.0, None, None) == fg.FG_ERR_NULL
    assert status(-1, 256, 256, 1.0, A, B, 0.0, None, D) == fg.FG_ERR_SHAPE
    A2, B2, D2 = mats(lda=128)
    assert status(256, 256, 256, 1.0, A2, B2, 0.0, None, D2) == fg.FG_ERR_SHAPE
    # a pointer that is not aligned to an element is rejected for every kind of product
    A4, B4, D4 = mats(pa=0x1001)
    assert status(256, 256, 256, 1.0, A4, B4, 0.0, None, D4) == fg.FG_ERR_ALIGN
    # what the general kernel absorbs for real products (K % 8, ld % 8, 16-byte alignment) stays an
    # error for complex ones, which have no general kernel
    import torch
    im = lambda m: fg.Matrix(m.re, m.layout, m.ld, im=m.re)
    Ac, Bc, Dc = mats()
    assert status(256, 256, 250, 1.0, im(Ac), im(Bc), 0.0, None, im(Dc)) == fg.FG_ERR_UNSUPPORTED
    assert "multiple of 8" in fg.fg_last_error()
    A3, B3, D3 = mats(lda=260)
    assert status(256, 256, 256, 1.0, im(A3), im(B3), 0.0, None, im(D3)) == fg.FG_ERR_ALIGN
    A8, B8, D8 = mats(pa=0x1008)
    assert status(256, 256, 256, 1.0, im(A8), im(B8), 0.0, None, im(D8)) == fg.FG_ERR_ALIGN
    A5, B5, D5 = mats()
    A5.layout = 7
    assert status(256, 256, 256, 1.0, A5, B5, 0.0, None, D5) == fg.FG_ERR_LAYOUT
    A6, B6, D6 = mats()
    A6.dtype = fg.FG_F32
    assert status(256, 256, 256, 1.0, A6, B6, 0.0, None, D6) == fg.FG_ERR_LAYOUT
    A7, B7, D7 = mats()
    C7 = fg.Matrix(D7.re, fg.FG_ROW, 256)
    assert status(256, 256, 256, 1.0, A7, B7, 1.0, C7, D7) == fg.FG_ERR_LAYOUT      # C and D layouts differ
    import torch
    assert status(256, 256, 256, 1.0, A, B, 0.0, None, D, bias=FakeTensor(0x5000, torch.float32), bias_dim=3) == fg.FG_ERR_LAYOUT
    assert status(256, 256, 256, 1.0, A, B, 0.0, None, D, act=9) == fg.FG_ERR_LAYOUT


def test_binary16_c_and_d_rules():
    """C and D stored as binary16: accepted for real FG_F16 products with any leading dimension of
    C and D; C and D must agree in type; no K split (the reduction pass writes FP32), no general
    kernel, no BF16 inputs, no planar complex."""
    import torch
    A, B, D = mats()
    Dh = fg.Matrix(FakeTensor(0x3002, torch.float16), fg.FG_COL, 259)      # odd ld, 2-byte aligned pointer
    Ch = fg.Matrix(FakeTensor(0x7002, torch.float16), fg.FG_COL, 301)
    assert status(256, 256, 256, 1.0, A, B, 1.0, fg.Matrix(D.re, fg.FG_COL, 256), Dh) == fg.FG_ERR_UNSUPPORTED   # FP32 C, binary16 D
    assert "same element type" in fg.fg_last_error()
    assert status(256, 256, 256, 1.0, A, B, 1.0, Ch, D) == fg.FG_ERR_UNSUPPORTED
    assert status(256, 256, 250, 1.0, A, B, 1.0, Ch, Dh) == fg.FG_ERR_UNSUPPORTED          # K % 8: no general kernel
    assert "general kernel" in fg.fg_last_error()
    assert status(256, 256, 256, 1.0, A, B, 1.0, Ch, fg.Matrix(FakeTensor(0x3001, torch.float16), fg.FG_COL, 256)) == fg.FG_ERR_ALIGN
    Ab, Bb, _ = mats()
    Ab.dtype = Bb.dtype = fg.FG_BF16
    assert status(256, 256, 256, 1.0, Ab, Bb, 0.0, None, Dh) == fg.FG_ERR_UNSUPPORTED
    im = lambda m: fg.Matrix(m.re, m.layout, m.ld, im=m.re)
    assert status(256, 256, 256, 1.0, im(A), im(B), 0.0, None, im(Dh)) == fg.FG_ERR_UNSUPPORTED
    assert status(256, 256, 256, 1.0, A, B, 0.0, None, Dh, a_add=0.5) == fg.FG_ERR_UNSUPPORTED
    assert fg.fg_gemm_plan(8192, 8192, 8192, variant=fg.FG_PLAN_REAL_F16_CD) == "gemm_h16_nn_256x256x64_k32"
    assert fg.fg_gemm_plan(4096, 4096, 4096, fg.FG_ROW, fg.FG_ROW, fg.FG_ROW, variant=fg.FG_PLAN_REAL_F16_CD) == "gemm_h16_nn_256x256x64_k32"
    assert "+" not in fg.fg_gemm_plan(512, 512, 8192, variant=fg.FG_PLAN_REAL_F16_CD)
    assert "+" not in fg.fg_gemm_plan(4100, 4100, 4096, variant=fg.FG_PLAN_REAL_F16_CD)
    with pytest.raises(fg.FlexGemmError):
        fg.fg_gemm_plan(128, 64, 60, variant=fg.FG_PLAN_REAL_F16_CD)


def test_empty_problem_is_ok_without_a_gpu():
    A, B, D = mats(M=0)
    assert status(0, 256, 256, 1.0, A, B, 0.0, None, D) == fg.FG_OK


def test_plan_names_follow_sizes_and_layouts():
    # outputs with a 256x256 tile for at least three quarters of the compute units: the kernel built on
    # 16x16x32 matrix instructions (k32), which holds a higher rate once the chip is at its power limit
    assert fg.fg_gemm_plan(8192, 8192, 8192) == "gemm_nn_256x256x64_k32"
    assert fg.fg_gemm_plan(8192, 8192, 8192, fg.FG_ROW, fg.FG_ROW) == "gemm_tt_256x256x64_k32"
    assert fg.fg_gemm_plan(8192, 8192, 8192, fg.FG_COL, fg.FG_ROW) == "gemm_nt_256x256x64"     # neither operand K-contiguous: measured no faster
    assert fg.fg_gemm_plan(8192, 1024, 4096) == "gemm_nn_256x128x64"
    # 2048^2 outputs: 256 medium tiles, one per compute unit, with the ring of four buffers that a
    # workgroup alone on its unit needs to cover the memory latency
    assert fg.fg_gemm_plan(2048, 2048, 2048, fg.FG_ROW, fg.FG_COL) == "gemm_tn_128x128x64_deep"
    assert fg.fg_gemm_plan(1024, 1024, 1024) == "gemm_nn_64x64x64"
    assert fg.fg_gemm_plan(4096, 2048, 2048) == "gemm_nn_256x128x64"        # 512 medium tiles would share units: two buffers
    # 4100^2: 289 big tiles are one full round of 256 plus 33 leftover tiles, which are split over K
    assert fg.fg_gemm_plan(4100, 4100, 4096) == "gemm_nn_256x256x64_k32+tailsplitk4"
    assert fg.fg_gemm_plan(256, 256, 256, fg.FG_COL, fg.FG_ROW) == "gemm_nt_64x64x64"
    # a row-major D is computed as the transposed problem: the operands swap roles
    assert fg.fg_gemm_plan(4096, 4096, 4096, fg.FG_ROW, fg.FG_ROW, fg.FG_ROW) == "gemm_nn_256x256x64_k32"
    # sizes need not be multiples of the tile: edge tiles are predicated
    assert fg.fg_gemm_plan(100, 72, 64) == "gemm_nn_64x64x64"
    assert fg.fg_gemm_plan(5000, 3000, 1000) == "gemm_nn_256x256x64_k32"  # 240 tiles: one round
    assert fg.fg_gemm_plan(3072, 3072, 3072) == "gemm_nn_256x256x64"      # 144 tiles, under three quarters of the units: the 32x32x16 kernel
    assert fg.fg_gemm_plan(128, 64, 60) == "gemm_general_64x64x32"       # K % 8 != 0: the general kernel
    with pytest.raises(fg.FlexGemmError):
        fg.fg_gemm_plan(128, 64, 60, variant=fg.FG_PLAN_COMPLEX)


def test_planner_splits_k_only_for_small_outputs_with_long_k(monkeypatch):
    delenv(monkeypatch, "FG_FORCE_SPLIT", raising=False)
    delenv(monkeypatch, "FG_FORCE_TILE", raising=False)
    delenv(monkeypatch, "FG_FORCE_TAIL", raising=False)
    for shape in [(8192, 8192, 8192), (4096, 4096, 4096), (2048, 2048, 2048), (1024, 1024, 1024), (65536, 256, 256), (256, 256, 256)]:
        assert "+splitk" not in fg.fg_gemm_plan(*shape), shape
    for shape in [(512, 512, 8192), (256, 256, 65536), (64, 64, 32768), (1024, 1024, 8192), (128, 4096, 16384)]:
        assert "+splitk" in fg.fg_gemm_plan(*shape), shape
    # every share of K keeps at least four K tiles, and the partial products fit the workspace
    name = fg.fg_gemm_plan(64, 64, 1024)
    assert "+splitk" not in name or int(name.split("+splitk")[1]) <= 4
    assert "+splitk" not in fg.fg_gemm_plan(4096, 4096, 65536)          # output alone fills the GPU
    # complex, dual and diagonal products are never split
    assert "+splitk" not in fg.fg_gemm_plan(256, 256, 65536, variant=fg.FG_PLAN_COMPLEX)
    assert "+splitk" not in fg.fg_gemm_plan(256, 256, 65536, fg.FG_DIAG, fg.FG_COL)
    assert fg.fg_gemm_plan(4096, 4096, 4096, variant=fg.FG_PLAN_COMPLEX_INTERLEAVED) == "cgemm_il_nn_256x128x32"
    assert fg.fg_gemm_plan(4096, 4096, 4096, variant=fg.FG_PLAN_DUAL) == "dgemm_nn_256x128x32"
    # complex tiles by estimated time: one partly filled round of the large tile beats two of a smaller one
    assert fg.fg_gemm_plan(2560, 2560, 2560, variant=fg.FG_PLAN_COMPLEX) == "cgemm_nn_256x128x32"
    assert fg.fg_gemm_plan(2048, 2048, 2048, variant=fg.FG_PLAN_COMPLEX) == "cgemm_nn_128x128x32"
    assert fg.fg_gemm_plan(1024, 1024, 1024, variant=fg.FG_PLAN_DUAL) == "dgemm_nn_64x64x32"
    assert fg.fg_gemm_plan(8192, 8192, 8192, variant=fg.FG_PLAN_REAL_BF16) == "gemm_bf16_nn_256x256x64_k32"
    # a short K (a pass over C and D): the 256x128 tile instead of the 256x256 one
    assert fg.fg_gemm_plan(8192, 8192, 256) == "gemm_nn_256x128x64"
    assert fg.fg_gemm_plan(8192, 8192, 320) == "gemm_nn_256x256x64_k32"
    # a diagonal operand: the smallest tile while the product's traffic fits the memory-side cache
    assert fg.fg_gemm_plan(4096, 4096, 4096, fg.FG_DIAG, fg.FG_COL) == "gemm_diagA_n_64x64x64"
    assert fg.fg_gemm_plan(8192, 8192, 8192, fg.FG_DIAG, fg.FG_COL) == "gemm_diagA_n_256x256x64"
    assert fg.fg_gemm_plan(8192, 1024, 1024, fg.FG_ROW, fg.FG_DIAG) == "gemm_t_diagB_64x64x64"
    # addition on A and B: the 16x16x32 kernel for the two layout pairs that have one
    assert fg.fg_gemm_plan(4096, 4096, 4096, variant=fg.FG_PLAN_REAL_AB_ADD) == "gemm_abadd_nn_256x256x64_k32"
    assert fg.fg_gemm_plan(4096, 4096, 4096, fg.FG_ROW, fg.FG_ROW, variant=fg.FG_PLAN_REAL_AB_ADD) == "gemm_abadd_tt_256x256x64_k32"
    assert fg.fg_gemm_plan(4096, 4096, 4096, fg.FG_COL, fg.FG_ROW, variant=fg.FG_PLAN_REAL_AB_ADD) == "gemm_abadd_nt_256x256x64"
    assert fg.fg_gemm_plan(4096, 4096, 4096, fg.FG_ROW, fg.FG_COL, variant=fg.FG_PLAN_REAL_AB_ADD) == "gemm_abadd_tn_256x256x64"
    assert fg.fg_gemm_plan(2048, 2048, 2048, variant=fg.FG_PLAN_REAL_AB_ADD) == "gemm_abadd_nn_128x128x64_deep"


def contract_status(mA, sA, mB, sB, mC, sC, ext, pa=0x1000, pb=0x2000, pc=0x3000):
    import torch
    return fg.fg_contract(mA, sA, FakeTensor(pa, torch.float16), mB, sB, FakeTensor(pb, torch.float16), mC, sC, None,
                          FakeTensor(pc, torch.float32), ext, raise_on_error=False)


def contract_plan(mA, sA, mB, sB, mC, sC, ext, pa=0x1000, pb=0x2000, pc=0x3000):
    import torch
    return fg.fg_contract_plan(mA, sA, FakeTensor(pa, torch.float16), mB, sB, FakeTensor(pb, torch.float16), mC, sC, None,
                               FakeTensor(pc, torch.float32), ext)


def test_contraction_descriptions_the_tiled_kernels_cannot_take_go_to_the_general_kernel():
    a, b, c, d, e = 0, 1, 2, 3, 4
    ext = {a: 64, b: 64, c: 64, d: 64}
    dense3 = [1, 64, 4096]
    assert contract_plan([a, d, c], dense3, [d, b], [1, 64], [a, b, c], dense3, ext).startswith("gett_")
    assert "general" not in contract_plan([a, d, c], dense3, [d, b], [1, 64], [a, b, c], dense3, ext)
    general = lambda *args, **kw: contract_plan(*args, **kw).startswith("gett_general_64x64x32 (")
    # no unit-stride mode in A
    assert general([a, d, c], [2, 128, 8192], [d, b], [1, 64], [a, b, c], dense3, ext)
    # B is contiguous along the summed mode, whose extent is not a multiple of 8
    ext2 = {a: 64, b: 64, c: 64, d: 36}
    assert general([a, d, c], [1, 64, 2304], [d, b], [1, 36], [a, b, c], dense3, ext2)
    # base pointer aligned to an element only
    assert general([a, d, c], dense3, [d, b], [1, 64], [a, b, c], dense3, ext, pa=0x1002)
    assert general([a, d, c], dense3, [d, b], [1, 64], [a, b, c], dense3, ext, pc=0x3004)
    # a stride of A that would put 16-byte pieces at 2-byte alignment (padded tensor)
    assert general([a, d, c], [1, 65, 65 * 64], [d, b], [1, 64], [a, b, c], dense3, ext)
    assert not general([a, d, c], [1, 72, 72 * 64], [d, b], [1, 64], [a, b, c], dense3, ext)
    # A and B contiguous along different summed modes
    ext5 = {a: 64, b: 64, d: 64, e: 64}
    assert general([d, e, a], dense3, [e, d, b], dense3, [a, b], [1, 64], ext5)
    # an outer product
    assert general([a], [1], [b], [1], [a, b], [1, 64], {a: 64, b: 64})
    # a tensor of 2 GiB
    big = {a: 1 << 15, b: 64, d: 1 << 15}
    assert general([a, d], [1, 1 << 15], [d, b], [1, 1 << 15], [a, b], [1, 1 << 15], big)


def test_contract_argument_errors():
    a, b, c, d = 0, 1, 2, 3
    ext = {a: 64, b: 64, c: 64, d: 64}
    dense3 = [1, 64, 4096]
    # a mode in one tensor only (no reduction or broadcast modes)
    assert contract_status([a, d, c], dense3, [d, b], [1, 64], [a, b], [1, 64], ext) == fg.FG_ERR_MODES
    # mode without extent
    assert contract_status([a, d, 9], dense3, [d, b], [1, 64], [a, b, 9], dense3, ext) == fg.FG_ERR_MODES
    # repeated mode inside one tensor
    assert contract_status([a, a, d], dense3, [d, b], [1, 64], [a, b], [1, 64], ext) == fg.FG_ERR_MODES
    # a base pointer that is not aligned to an element
    assert contract_status([a, d, c], dense3, [d, b], [1, 64], [a, b, c], dense3, ext, pa=0x1001) == fg.FG_ERR_ALIGN
    assert contract_status([a, d, c], dense3, [d, b], [1, 64], [a, b, c], dense3, ext, pc=0x3002) == fg.FG_ERR_ALIGN
    # negative stride; more than four modes in a group
    assert contract_status([a, d, c], [1, -64, 4096], [d, b], [1, 64], [a, b, c], dense3, ext) == fg.FG_ERR_UNSUPPORTED
    many = {i: 2 for i in range(7)}
    assert contract_status([0, 1, 2, 3, 4, 5], [1, 2, 4, 8, 16, 32], [5, 6], [1, 2], [0, 1, 2, 3, 4, 6], [1, 2, 4, 8, 16, 32], many) == fg.FG_ERR_UNSUPPORTED
    # an empty mode: nothing to do, OK without a GPU
    ext3 = {a: 64, b: 0, c: 64, d: 64}
    assert contract_status([a, d, c], dense3, [d, b], [1, 64], [a, b, c], [1, 64, 0], ext3) == fg.FG_OK


def test_planner_over_random_shapes_never_fails_and_its_splits_fit_the_workspace():
    """Seeded random M, N, K over six orders of magnitude, every layout pair and variant: the plan
    query succeeds, names a kernel, and a split plan's partial products (tiles x K ranges x tile
    bytes) fit the 64 MiB workspace."""
    import random
    rng = random.Random(7)
    for _ in range(400):
        M = rng.choice([1, 7, 64, 100, 256, 300, 1000, 1024, 2048, 4100, 8192, 20000])
        N = rng.choice([1, 5, 64, 128, 200, 512, 1111, 4096, 8192, 16384])
        K = 8 * rng.choice([1, 2, 8, 33, 64, 128, 513, 1024, 4096, 8192, 65536])
        la, lb, ld = rng.choice([0, 1]), rng.choice([0, 1]), rng.choice([0, 1])
        variant = rng.choice([fg.FG_PLAN_REAL, fg.FG_PLAN_REAL, fg.FG_PLAN_REAL_BF16, fg.FG_PLAN_COMPLEX, fg.FG_PLAN_DUAL,
                              fg.FG_PLAN_COMPLEX_INTERLEAVED, fg.FG_PLAN_REAL_F16_CD, fg.FG_PLAN_REAL_AB_ADD])
        plan = fg.fg_gemm_plan(M, N, K, la, lb, ld, variant)
        m = re.match(r"^[a-z0-9_]+_(\d+)x(\d+)x(\d+)(?:_[a-z0-9]+)?(?:\+(tail)?splitk(\d+))?$", plan)
        assert m, plan
        bm, bn = int(m.group(1)), int(m.group(2))
        if m.group(5) and not m.group(4):
            S = int(m.group(5))
            Mn, Nn = (M, N) if ld == 0 else (N, M)
            tiles = -(-Mn // bm) * -(-Nn // bn)
            assert 2 <= S <= 64 and tiles * S * bm * bn * 4 <= 64 << 20, (plan, M, N, K)
            assert variant in (fg.FG_PLAN_REAL, fg.FG_PLAN_REAL_BF16, fg.FG_PLAN_REAL_AB_ADD), plan     # the reduction pass writes FP32 real results
