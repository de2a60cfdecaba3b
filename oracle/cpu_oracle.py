"""ctypes front end of the CPU oracle (``flexgemm_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
CPU-baseline leg of the benchmark.  The product package never imports this
module, and this module never imports the product package.

Every function takes numpy arrays (float16 for A and B, float32 for C and the
bias), hands their buffers to the C code unchanged and returns float64 arrays.
No arithmetic of the method happens in this file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "flexgemm_oracle.c")
_LIB = os.path.join(_HERE, "libflexgemm_oracle.so")

COL, ROW, DIAG = 0, 1, 2
ACT_NONE, ACT_RELU = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no fast-math) and return the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm", "-lpthread"])
        os.replace(tmp, _LIB)
    return _LIB


class _GemmProblem(C.Structure):
    _fields_ = [
        ("M", C.c_int64), ("N", C.c_int64), ("K", C.c_int64),
        ("alpha", C.c_double), ("beta", C.c_double),
        ("A_re", C.c_void_p), ("A_im", C.c_void_p), ("layoutA", C.c_int32), ("lda", C.c_int64),
        ("B_re", C.c_void_p), ("B_im", C.c_void_p), ("layoutB", C.c_int32), ("ldb", C.c_int64),
        ("C_re", C.c_void_p), ("C_im", C.c_void_p), ("layoutC", C.c_int32), ("ldc", C.c_int64),
        ("bias", C.c_void_p), ("bias_dim", C.c_int32), ("act", C.c_int32), ("ab_dtype", C.c_int32), ("dual", C.c_int32),
        ("ab_add", C.c_int32), ("a_add", C.c_double), ("b_add", C.c_double), ("c_act", C.c_int32),
        ("interleaved_ab", C.c_int32), ("interleaved_c", C.c_int32),
    ]


class _ContractProblem(C.Structure):
    _fields_ = [
        ("n_modes", C.c_int32), ("labels", C.c_void_p), ("extents", C.c_void_p),
        ("nA", C.c_int32), ("modesA", C.c_void_p), ("stridesA", C.c_void_p), ("A", C.c_void_p),
        ("nB", C.c_int32), ("modesB", C.c_void_p), ("stridesB", C.c_void_p), ("B", C.c_void_p),
        ("nC", C.c_int32), ("modesC", C.c_void_p), ("stridesC", C.c_void_p), ("Cin", C.c_void_p),
        ("alpha", C.c_double), ("beta", C.c_double),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        l = C.CDLL(build())
        l.oracle_half_to_double.restype = C.c_double
        l.oracle_half_to_double.argtypes = [C.c_uint16]
        l.oracle_round_to_half.restype = C.c_double
        l.oracle_round_to_half.argtypes = [C.c_double]
        l.oracle_bf16_to_double.restype = C.c_double
        l.oracle_bf16_to_double.argtypes = [C.c_uint16]
        pd = C.c_void_p
        l.oracle_gemm_full.restype = C.c_int
        l.oracle_gemm_full.argtypes = [C.POINTER(_GemmProblem), pd, pd, pd, pd, C.c_int]
        l.oracle_gemm_at.restype = C.c_int
        l.oracle_gemm_at.argtypes = [C.POINTER(_GemmProblem), C.c_int64, pd, pd, pd, pd, pd, pd, C.c_int]
        l.oracle_contract_full.restype = C.c_int
        l.oracle_contract_full.argtypes = [C.POINTER(_ContractProblem), pd, pd, C.c_int]
        l.oracle_contract_at.restype = C.c_int
        l.oracle_contract_at.argtypes = [C.POINTER(_ContractProblem), C.c_int64, pd, pd, pd, C.c_int]
        _lib = l
    return _lib


def default_threads() -> int:
    try:
        return max(1, len(os.sched_getaffinity(0)))
    except AttributeError:  # pragma: no cover
        return max(1, os.cpu_count() or 1)


def half_to_double(bits: int) -> float:
    return float(lib().oracle_half_to_double(int(bits) & 0xFFFF))


def bf16_to_double(bits: int) -> float:
    return float(lib().oracle_bf16_to_double(int(bits) & 0xFFFF))


def round_to_half(x: float) -> float:
    return float(lib().oracle_round_to_half(float(x)))


def round_array_to_half(x: np.ndarray) -> np.ndarray:
    """Every element rounded to the nearest binary16 value (ties to even), as float64: what a
    result stored in binary16 holds when the value before the store is ``x`` (the type
    conversion before a store, Section 4.2.3).  Element by element through round_to_half."""
    f = lib().oracle_round_to_half
    flat = np.asarray(x, np.float64).reshape(-1)
    return np.array([f(float(v)) for v in flat], np.float64).reshape(np.shape(x))


F16, BF16 = 0, 1


@dataclass
class Operand:
    """A stored 16-bit operand: ``re`` (and ``im`` for planar complex) are flat or 2-D arrays whose
    memory is read as-is; ``layout`` and ``ld`` say how element (r, c) is found.  float16 arrays
    hold binary16 values; uint16 arrays hold the bit patterns of ``dtype`` (F16 or BF16)."""
    re: np.ndarray
    layout: int = COL
    ld: int = 0
    im: Optional[np.ndarray] = None
    dtype: int = F16
    interleaved: bool = False   # complex with (real, imaginary) adjacent in ``re``; ``im`` unused, ld in complex elements


def _ptr(a: Optional[np.ndarray], dtype) -> Optional[int]:
    if a is None:
        return None
    if dtype == np.float16 and a.dtype == np.uint16:
        dtype = np.uint16                       # raw 16-bit patterns
    if a.dtype != dtype or not a.flags["C_CONTIGUOUS"] and not a.flags["F_CONTIGUOUS"]:
        raise ValueError("oracle buffers must be contiguous %s arrays" % np.dtype(dtype).name)
    return a.ctypes.data


def _check_span(a: Optional[np.ndarray], need: int, what: str):
    if a is not None and a.size < need:
        raise ValueError("%s holds %d elements, the described operand needs %d" % (what, a.size, need))


def _gemm_problem(M, N, K, alpha, A: Operand, B: Operand, beta, Cre, Cim, layoutC, ldc, bias, bias_dim, act,
                  c_interleaved=False):
    q = _GemmProblem()
    q.M, q.N, q.K, q.alpha, q.beta = M, N, K, float(alpha), float(beta)

    def span(layout, ld, rows, cols):
        if rows == 0 or cols == 0:
            return 0
        if layout == COL:
            return (cols - 1) * ld + rows
        if layout == ROW:
            return (rows - 1) * ld + cols
        return min(rows, cols)

    if A.interleaved != B.interleaved:
        raise ValueError("A and B must both be interleaved or both planar")
    for name, op, rows, cols in (("A", A, M, K), ("B", B, K, N)):
        if op.layout == COL and op.ld < rows or op.layout == ROW and op.ld < cols:
            raise ValueError("leading dimension of %s too small" % name)
        need = span(op.layout, op.ld, rows, cols) * (2 if op.interleaved else 1)
        _check_span(op.re, need, name + ".re")
        if not op.interleaved:
            _check_span(op.im, need, name + ".im")
    im_of = lambda op: (_ptr(op.re, np.float16) + 2) if op.interleaved else _ptr(op.im, np.float16)
    q.A_re, q.A_im, q.layoutA, q.lda = _ptr(A.re, np.float16), im_of(A), A.layout, A.ld
    q.B_re, q.B_im, q.layoutB, q.ldb = _ptr(B.re, np.float16), im_of(B), B.layout, B.ld
    q.interleaved_ab = 1 if A.interleaved else 0
    if Cre is not None:
        need = span(layoutC, ldc, M, N) * (2 if c_interleaved else 1)
        _check_span(Cre, need, "C.re")
        if not c_interleaved:
            _check_span(Cim, need, "C.im")
    q.C_re, q.C_im, q.layoutC, q.ldc = _ptr(Cre, np.float32), _ptr(Cim, np.float32), layoutC, ldc
    if c_interleaved and Cre is not None:
        q.C_im, q.interleaved_c = _ptr(Cre, np.float32) + 4, 1
    if bias is not None:
        _check_span(bias, M if bias_dim == 0 else N, "bias")
    q.bias, q.bias_dim, q.act = _ptr(bias, np.float32), bias_dim, act
    if A.dtype != B.dtype:
        raise ValueError("A and B must have the same element type")
    q.ab_dtype = A.dtype
    return q


def gemm(M: int, N: int, K: int, alpha: float, A: Operand, B: Operand, beta: float = 0.0,
         C_re: Optional[np.ndarray] = None, C_im: Optional[np.ndarray] = None, layoutC: int = COL, ldc: int = 0,
         bias: Optional[np.ndarray] = None, bias_dim: int = 0, act: int = ACT_NONE,
         at: Optional[Sequence[np.ndarray]] = None, threads: Optional[int] = None, dual: bool = False,
         ab_add: Optional[Sequence[float]] = None, c_act: int = ACT_NONE, c_interleaved: bool = False):
    """Evaluate the GEMM definition.  ``dual``: the ``im`` planes hold dual parts (eps^2 = 0).
    Interleaved complex operands: ``Operand(..., interleaved=True)`` for A and B, and
    ``c_interleaved`` for C (then ``C_re`` is the interleaved array and ``C_im`` is unused).
    ``ab_add=(a, b)``: every loaded element of A (B) becomes half(element + a) (half(element + b)),
    a and b binary16 values; ``c_act``: activation applied to C before it is scaled by beta.

    Returns a dict with ``D`` and ``G`` (float64; complex problems also ``D_im`` and ``G_im``).
    Without ``at`` the arrays are (M, N); with ``at=(I, J)`` they are 1-D, one value per listed
    position.
    """
    threads = threads or default_threads()
    if C_re is not None and C_re.dtype == np.float16:
        # C stored as binary16: every element is widened exactly when it is loaded (the type
        # conversion after a load, Section 4.2.3)
        C_re = C_re.astype(np.float32)
    q = _gemm_problem(M, N, K, alpha, A, B, beta, C_re, C_im, layoutC, ldc, bias, bias_dim, act, c_interleaved)
    q.dual = 1 if dual else 0
    if ab_add is not None:
        q.ab_add, q.a_add, q.b_add = 1, float(ab_add[0]), float(ab_add[1])
    q.c_act = c_act
    is_complex = A.im is not None or B.im is not None or A.interleaved
    if at is None:
        shape, order = (M, N), "F"
    else:
        I = np.ascontiguousarray(at[0], dtype=np.int64)
        J = np.ascontiguousarray(at[1], dtype=np.int64)
        if I.shape != J.shape or I.ndim != 1:
            raise ValueError("at=(I, J) must be two 1-D arrays of equal length")
        shape, order = (I.size,), "C"
    out = {"D": np.zeros(shape, np.float64, order=order), "G": np.zeros(shape, np.float64, order=order)}
    if is_complex:
        out["D_im"] = np.zeros(shape, np.float64, order=order)
        out["G_im"] = np.zeros(shape, np.float64, order=order)
    p = lambda k: out[k].ctypes.data if k in out else None
    if at is None:
        rc = lib().oracle_gemm_full(C.byref(q), p("D"), p("D_im"), p("G"), p("G_im"), threads)
    else:
        rc = lib().oracle_gemm_at(C.byref(q), I.size, I.ctypes.data, J.ctypes.data,
                                  p("D"), p("D_im"), p("G"), p("G_im"), threads)
    if rc != 0:
        raise ValueError("oracle rejected the GEMM description (code %d)" % rc)
    return out


def contract(extents: dict, modesA: Sequence[int], stridesA: Sequence[int], A: np.ndarray,
             modesB: Sequence[int], stridesB: Sequence[int], B: np.ndarray,
             modesC: Sequence[int], stridesC: Sequence[int], Cin: Optional[np.ndarray] = None,
             alpha: float = 1.0, beta: float = 0.0, at: Optional[np.ndarray] = None,
             threads: Optional[int] = None):
    """Evaluate the contraction definition.

    ``extents`` maps an integer mode label to its extent.  Without ``at`` returns ``D`` and ``G``
    as flat float64 arrays indexed by C's own element offsets (length = span of C); with ``at``
    (count x len(modesC) indices) returns one value per listed position.
    """
    threads = threads or default_threads()
    labels = np.array(list(extents.keys()), dtype=np.int32)
    exts = np.array([extents[k] for k in extents], dtype=np.int64)
    keep = []

    def arr(x, dt):
        a = np.ascontiguousarray(np.array(list(x), dtype=dt))
        keep.append(a)
        return a

    mA, sA = arr(modesA, np.int32), arr(stridesA, np.int64)
    mB, sB = arr(modesB, np.int32), arr(stridesB, np.int64)
    mC, sC = arr(modesC, np.int32), arr(stridesC, np.int64)
    if len(mA) != len(sA) or len(mB) != len(sB) or len(mC) != len(sC):
        raise ValueError("one stride per mode is required")

    def span(modes, strides):
        s = 1
        for m, st in zip(modes, strides):
            if int(m) not in extents:
                raise ValueError("mode label %d has no extent" % int(m))
            e = extents[int(m)]
            if e == 0:
                return 0
            s += (e - 1) * int(st)
        return s

    _check_span(A, span(mA, sA), "A")
    _check_span(B, span(mB, sB), "B")
    spanC = span(mC, sC)
    _check_span(Cin, spanC, "Cin")
    q = _ContractProblem()
    q.n_modes, q.labels, q.extents = len(labels), labels.ctypes.data, exts.ctypes.data
    q.nA, q.modesA, q.stridesA, q.A = len(mA), mA.ctypes.data, sA.ctypes.data, _ptr(A, np.float16)
    q.nB, q.modesB, q.stridesB, q.B = len(mB), mB.ctypes.data, sB.ctypes.data, _ptr(B, np.float16)
    q.nC, q.modesC, q.stridesC, q.Cin = len(mC), mC.ctypes.data, sC.ctypes.data, _ptr(Cin, np.float32)
    q.alpha, q.beta = float(alpha), float(beta)
    if at is None:
        D = np.zeros(spanC, np.float64)
        G = np.zeros(spanC, np.float64)
        rc = lib().oracle_contract_full(C.byref(q), D.ctypes.data, G.ctypes.data, threads)
    else:
        idx = np.ascontiguousarray(at, dtype=np.int64)
        if idx.ndim != 2 or idx.shape[1] != len(mC):
            raise ValueError("at must be count x len(modesC)")
        D = np.zeros(idx.shape[0], np.float64)
        G = np.zeros(idx.shape[0], np.float64)
        rc = lib().oracle_contract_at(C.byref(q), idx.shape[0], idx.ctypes.data, D.ctypes.data, G.ctypes.data, threads)
    if rc != 0:
        raise ValueError("oracle rejected the contraction description (code %d)" % rc)
    return {"D": D, "G": G}
