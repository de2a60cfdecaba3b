"""Thin ctypes binding of libflexgemm.so: argument marshalling only.

The functions have the names and arguments of the C ABI (include/flexgemm.h).  Torch is used
for device memory and streams; every step of the computation runs in the library's kernels.
There is no fallback: if the shared library is missing, importing the entry points raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libflexgemm.so")

FG_OK = 0
FG_ERR_NULL, FG_ERR_SHAPE, FG_ERR_LAYOUT, FG_ERR_ALIGN, FG_ERR_UNSUPPORTED, FG_ERR_MODES, FG_ERR_LAUNCH = range(1, 8)
FG_F16, FG_BF16, FG_F32, FG_CF16, FG_CF32 = 0, 1, 2, 3, 4
FG_COL, FG_ROW, FG_DIAG, FG_ZERO = 0, 1, 2, 3
FG_ACT_NONE, FG_ACT_RELU = 0, 1

EXPORTS = ("fg_init", "fg_gemm", "fg_gemm_ex", "fg_gemm_noalloc", "fg_gemm_dual", "fg_contract", "fg_contract_plan", "fg_last_error", "fg_version",
           "fg_reload_tuning", "fg_gemm_plan", "fg_probe_mfma", "fg_probe_mfma_k32", "fg_probe_kloop_mix")
FG_PLAN_REAL, FG_PLAN_COMPLEX, FG_PLAN_DUAL, FG_PLAN_REAL_BF16, FG_PLAN_COMPLEX_INTERLEAVED, FG_PLAN_REAL_F16_CD = 0, 1, 2, 3, 4, 5
FG_PLAN_REAL_AB_ADD = 6


class fg_matrix(C.Structure):
    _fields_ = [("re", C.c_void_p), ("im", C.c_void_p), ("dtype", C.c_int32), ("layout", C.c_int32), ("ld", C.c_int64)]


class fg_epilogue(C.Structure):
    _fields_ = [("bias", C.c_void_p), ("bias_dim", C.c_int32), ("act", C.c_int32)]


class fg_load_transforms(C.Structure):
    _fields_ = [("a_add", C.c_float), ("b_add", C.c_float), ("c_act", C.c_int32)]


class FlexGemmError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("flexgemm status %d: %s" % (status, message))
        self.status = status


_lib = None


def load_library() -> C.CDLL:
    """Load libflexgemm.so (built in-tree by ``paper_2009_12263_amd.build``).  Fails loudly."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libflexgemm.so is not built: run `python -m paper_2009_12263_amd.build` "
                              "(there is no CPU or PyTorch fallback)")
        lib = C.CDLL(LIB_PATH)
        i32, i64, f32, vp = C.c_int32, C.c_int64, C.c_float, C.c_void_p
        lib.fg_gemm.restype = C.c_int
        lib.fg_gemm.argtypes = [i64, i64, i64, f32, C.POINTER(fg_matrix), C.POINTER(fg_matrix), f32,
                                C.POINTER(fg_matrix), C.POINTER(fg_matrix), C.POINTER(fg_epilogue), vp]
        lib.fg_gemm_ex.restype = C.c_int
        lib.fg_gemm_ex.argtypes = [i64, i64, i64, f32, C.POINTER(fg_matrix), C.POINTER(fg_matrix), f32,
                                   C.POINTER(fg_matrix), C.POINTER(fg_matrix), C.POINTER(fg_epilogue),
                                   C.POINTER(fg_load_transforms), vp]
        lib.fg_gemm_noalloc.restype = C.c_int
        lib.fg_gemm_noalloc.argtypes = lib.fg_gemm_ex.argtypes
        lib.fg_reload_tuning.restype = None
        lib.fg_reload_tuning.argtypes = []
        lib.fg_gemm_dual.restype = C.c_int
        lib.fg_gemm_dual.argtypes = [i64, i64, i64, f32, C.POINTER(fg_matrix), C.POINTER(fg_matrix), f32,
                                     C.POINTER(fg_matrix), C.POINTER(fg_matrix), vp]
        lib.fg_contract.restype = C.c_int
        lib.fg_contract.argtypes = [i32, vp, vp, vp, i32, vp, vp, vp, i32, vp, vp, vp, vp, i32, vp, vp, f32, f32, vp]
        lib.fg_contract_plan.restype = C.c_int
        lib.fg_contract_plan.argtypes = [i32, vp, vp, vp, i32, vp, vp, vp, i32, vp, vp, vp, vp, i32, vp, vp, C.c_char_p, i32]
        lib.fg_last_error.restype = C.c_char_p
        lib.fg_last_error.argtypes = []
        lib.fg_version.restype = i32
        lib.fg_version.argtypes = []
        lib.fg_init.restype = C.c_int
        lib.fg_init.argtypes = []
        lib.fg_gemm_plan.restype = C.c_int
        lib.fg_gemm_plan.argtypes = [i64, i64, i64, i32, i32, i32, i32, C.c_char_p, i32]
        lib.fg_probe_mfma.restype = C.c_int
        lib.fg_probe_mfma.argtypes = [vp, i64, i32, C.POINTER(C.c_int64), vp]
        lib.fg_probe_mfma_k32.restype = C.c_int
        lib.fg_probe_mfma_k32.argtypes = [vp, i64, i32, C.POINTER(C.c_int64), vp]
        lib.fg_probe_kloop_mix.restype = C.c_int
        lib.fg_probe_kloop_mix.argtypes = [vp, i64, i32, C.POINTER(C.c_int64), vp]
        _lib = lib
    return _lib


@dataclass
class Matrix:
    """Host-side description of a device matrix: the tensors only provide the pointers."""
    re: Optional[torch.Tensor]
    layout: int = FG_COL
    ld: int = 0
    im: Optional[torch.Tensor] = None
    dtype: Optional[int] = None

    def _struct(self) -> fg_matrix:
        m = fg_matrix()
        m.re = self.re.data_ptr() if self.re is not None else None
        m.im = self.im.data_ptr() if self.im is not None else None
        if self.dtype is not None:
            m.dtype = self.dtype
        else:
            t = self.re if self.re is not None else self.im
            m.dtype = {torch.float16: FG_F16, torch.bfloat16: FG_BF16, torch.float32: FG_F32,
                       torch.complex32: FG_CF16, torch.complex64: FG_CF32}.get(
                t.dtype if t is not None else torch.float32, -1)
        m.layout, m.ld = self.layout, self.ld
        return m


def _check_extent(m: Optional["Matrix"], rows: int, cols: int, name: str) -> None:
    """The library sees pointers only and cannot know how much memory is behind them: before a call
    that will launch kernels, check here that every device tensor holds the matrix it is said to
    hold (a matrix larger than its tensor would be read or written out of bounds on the GPU).
    Descriptions the library rejects by itself (a leading dimension that is too small, ...) are
    left to it."""
    if m is None or rows <= 0 or cols <= 0:
        return
    for t in (m.re, m.im):
        if t is None or not getattr(t, "is_cuda", False):     # only real device tensors are checked
            continue
        per_entry = 2 if (m.dtype in (FG_CF16, FG_CF32) and not t.is_complex()) else 1
        if m.layout == FG_DIAG:
            need = min(rows, cols)
        elif m.layout == FG_COL:
            need = (cols - 1) * m.ld + rows if m.ld >= rows else 0
        elif m.layout == FG_ROW:
            need = (rows - 1) * m.ld + cols if m.ld >= cols else 0
        else:
            need = 0
        if need * per_entry > t.numel():
            raise ValueError("%s: a %d x %d matrix with leading dimension %d needs %d elements, the tensor has %d"
                             % (name, rows, cols, m.ld, need * per_entry, t.numel()))


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def fg_last_error() -> str:
    return load_library().fg_last_error().decode()


def fg_version() -> int:
    return int(load_library().fg_version())


def fg_init(raise_on_error: bool = True) -> int:
    """Prepare every kernel variant on the current device; see fg_init in include/flexgemm.h."""
    return _check(load_library().fg_init(), raise_on_error)


def fg_reload_tuning() -> None:
    """Re-read the FG_FORCE_* tuning overrides from the environment (read once at load otherwise)."""
    load_library().fg_reload_tuning()


def _check(status: int, raise_on_error: bool) -> int:
    if status != FG_OK and raise_on_error:
        raise FlexGemmError(status, fg_last_error())
    return status


def fg_gemm(M: int, N: int, K: int, alpha: float, A: Optional[Matrix], B: Optional[Matrix], beta: float,
            C_: Optional[Matrix], D: Optional[Matrix], bias: Optional[torch.Tensor] = None, bias_dim: int = 0,
            act: int = FG_ACT_NONE, stream=None, raise_on_error: bool = True,
            a_add: float = 0.0, b_add: float = 0.0, c_act: int = FG_ACT_NONE, noalloc: bool = False) -> int:
    """D = act(alpha * op(A) * op(B) + beta * C + bias); see fg_gemm in include/flexgemm.h.
    With ``a_add``, ``b_add`` or ``c_act`` the call goes to fg_gemm_ex (transforms on loaded elements);
    with ``noalloc`` to fg_gemm_noalloc (same arguments as fg_gemm_ex)."""
    lib = load_library()
    if M > 0 and N > 0:          # an empty result launches nothing
        _check_extent(A, M, K, "A"); _check_extent(B, K, N, "B"); _check_extent(C_, M, N, "C"); _check_extent(D, M, N, "D")
    sa = A._struct() if A is not None else None
    sb = B._struct() if B is not None else None
    sc = C_._struct() if C_ is not None else None
    sd = D._struct() if D is not None else None
    ep = None
    if bias is not None or act != FG_ACT_NONE:
        ep = fg_epilogue()
        ep.bias = bias.data_ptr() if bias is not None else None
        ep.bias_dim, ep.act = bias_dim, act
    ref = lambda s: C.byref(s) if s is not None else None
    if noalloc:
        lt = fg_load_transforms(a_add, b_add, c_act)
        st = lib.fg_gemm_noalloc(M, N, K, alpha, ref(sa), ref(sb), beta, ref(sc), ref(sd), ref(ep), C.byref(lt), _stream_handle(stream))
    elif a_add != 0.0 or b_add != 0.0 or c_act != FG_ACT_NONE:
        lt = fg_load_transforms(a_add, b_add, c_act)
        st = lib.fg_gemm_ex(M, N, K, alpha, ref(sa), ref(sb), beta, ref(sc), ref(sd), ref(ep), C.byref(lt), _stream_handle(stream))
    else:
        st = lib.fg_gemm(M, N, K, alpha, ref(sa), ref(sb), beta, ref(sc), ref(sd), ref(ep), _stream_handle(stream))
    return _check(st, raise_on_error)


def fg_gemm_dual(M: int, N: int, K: int, alpha: float, A: Optional[Matrix], B: Optional[Matrix], beta: float,
                 C_: Optional[Matrix], D: Optional[Matrix], stream=None, raise_on_error: bool = True) -> int:
    """Dual-number product on planar (value, dual part) matrices; see fg_gemm_dual in include/flexgemm.h."""
    lib = load_library()
    if M > 0 and N > 0:          # an empty result launches nothing
        _check_extent(A, M, K, "A"); _check_extent(B, K, N, "B"); _check_extent(C_, M, N, "C"); _check_extent(D, M, N, "D")
    sa = A._struct() if A is not None else None
    sb = B._struct() if B is not None else None
    sc = C_._struct() if C_ is not None else None
    sd = D._struct() if D is not None else None
    ref = lambda s: C.byref(s) if s is not None else None
    st = lib.fg_gemm_dual(M, N, K, alpha, ref(sa), ref(sb), beta, ref(sc), ref(sd), _stream_handle(stream))
    return _check(st, raise_on_error)


def fg_gemm_plan(M: int, N: int, K: int, layoutA: int = FG_COL, layoutB: int = FG_COL, layoutD: int = FG_COL,
                 variant: int = FG_PLAN_REAL) -> str:
    buf = C.create_string_buffer(128)
    st = load_library().fg_gemm_plan(M, N, K, layoutA, layoutB, layoutD, int(variant), buf, 128)
    _check(st, True)
    return buf.value.decode()


def fg_contract(modesA: Sequence[int], stridesA: Sequence[int], A: torch.Tensor,
                modesB: Sequence[int], stridesB: Sequence[int], B: torch.Tensor,
                modesC: Sequence[int], stridesC: Sequence[int], Cin: Optional[torch.Tensor], Cout: torch.Tensor,
                extents: dict, alpha: float = 1.0, beta: float = 0.0, stream=None, raise_on_error: bool = True) -> int:
    """Cout = alpha * contraction(A, B) + beta * Cin; see fg_contract in include/flexgemm.h.
    ``extents`` maps each integer mode label to its extent."""
    lib = load_library()
    for name, t, modes, strides in (("A", A, modesA, stridesA), ("B", B, modesB, stridesB), ("Cin", Cin, modesC, stridesC),
                                    ("Cout", Cout, modesC, stridesC)):
        # the same protection as _check_extent: the last element the description reaches must exist
        if t is not None and getattr(t, "is_cuda", False) and all(int(v) > 0 for v in extents.values()) and len(modes) == len(strides) and all(m in extents and extents[m] > 0 for m in modes) \
                and all(int(x) >= 0 for x in strides):
            need = 1 + sum((int(extents[m]) - 1) * int(x) for m, x in zip(modes, strides))
            if need > t.numel():
                raise ValueError("%s: the modes and strides reach element %d, the tensor has %d" % (name, need - 1, t.numel()))
    i32 = lambda xs: (C.c_int32 * len(xs))(*[int(x) for x in xs])
    i64 = lambda xs: (C.c_int64 * len(xs))(*[int(x) for x in xs])
    mA, sA, mB, sB, mC, sC = i32(modesA), i64(stridesA), i32(modesB), i64(stridesB), i32(modesC), i64(stridesC)
    labels, exts = i32(list(extents.keys())), i64([extents[k] for k in extents])
    ptr = lambda t: t.data_ptr() if t is not None else None
    st = lib.fg_contract(len(mA), mA, sA, ptr(A), len(mB), mB, sB, ptr(B), len(mC), mC, sC, ptr(Cin), ptr(Cout),
                         len(labels), labels, exts, alpha, beta, _stream_handle(stream))
    return _check(st, raise_on_error)


def fg_contract_plan(modesA: Sequence[int], stridesA: Sequence[int], A, modesB: Sequence[int], stridesB: Sequence[int], B,
                     modesC: Sequence[int], stridesC: Sequence[int], Cin, Cout, extents: dict) -> str:
    """Name of the kernel fg_contract would use; see fg_contract_plan in include/flexgemm.h."""
    lib = load_library()
    i32 = lambda xs: (C.c_int32 * len(xs))(*[int(x) for x in xs])
    i64 = lambda xs: (C.c_int64 * len(xs))(*[int(x) for x in xs])
    mA, sA, mB, sB, mC, sC = i32(modesA), i64(stridesA), i32(modesB), i64(stridesB), i32(modesC), i64(stridesC)
    labels, exts = i32(list(extents.keys())), i64([extents[k] for k in extents])
    ptr = lambda t: t.data_ptr() if t is not None else None
    buf = C.create_string_buffer(256)
    st = lib.fg_contract_plan(len(mA), mA, sA, ptr(A), len(mB), mB, sB, ptr(B), len(mC), mC, sC, ptr(Cin), ptr(Cout),
                              len(labels), labels, exts, buf, 256)
    _check(st, True)
    return buf.value.decode()


def fg_probe_mfma(fp16_operands: torch.Tensor, iters: int, stream=None, k32: bool = False, kloop_mix: bool = False) -> int:
    """Launch the MFMA-only measurement kernel on operands from ``fp16_operands``; returns the
    number of floating-point operations of the launch (see fg_probe_mfma, fg_probe_mfma_k32 and
    fg_probe_kloop_mix in include/flexgemm.h; ``k32`` selects the 16x16x32 instruction,
    ``kloop_mix`` that instruction together with the K loop's LDS reads and direct loads)."""
    flops = C.c_int64(0)
    lib = load_library()
    fn = lib.fg_probe_kloop_mix if kloop_mix else lib.fg_probe_mfma_k32 if k32 else lib.fg_probe_mfma
    st = fn(fp16_operands.data_ptr(), fp16_operands.numel() * fp16_operands.element_size(), iters, C.byref(flops), _stream_handle(stream))
    _check(st, True)
    return int(flops.value)
