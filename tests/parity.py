"""Helpers shared by the GPU parity tests: build seeded inputs, call the library through its
C ABI binding, evaluate the oracle (all entries, or a sample) and compare.

Tolerances (written here once, used by every test):
  * official bar (the tolerance stated for this implementation):
        |D - D_ref| <= 2e-3 * (|alpha| (|A||B|)_ij + |beta| |C_ij|)            elementwise;
  * tight bar, derived from the arithmetic: FP16 x FP16 products are exact in FP32, so the only
    error is FP32 accumulation, at worst K * 2^-24 * G and in practice ~sqrt(K) * 2^-24 * G;
    results must also satisfy  |D - D_ref| <= 4 * sqrt(K) * 2^-24 * G + 2^-22 * |D_ref|
    (the second term covers the final alpha/beta/bias roundings).  A dropped or duplicated
    16-wide k slice changes an entry by ~16/K of |A||B|, far above this bar;
  * integer-valued inputs (|a|, |b| <= 8): every partial sum is an integer below 2^24, the
    result is unique, and the comparison is bit-exact.
"""
from __future__ import annotations

import math
from typing import Optional

import numpy as np
import torch

from oracle import cpu_oracle as O
from paper_2009_12263_amd import binding as fg
from paper_2009_12263_amd import workloads as W

OFFICIAL_RTOL = 2e-3


def setenv(monkeypatch, name: str, value: str):
    """Set one of the library's FG_FORCE_* tuning variables and make the library read it (it reads
    its environment once, at load); tests/conftest.py re-reads after the test has restored it."""
    monkeypatch.setenv(name, value)
    fg.fg_reload_tuning()


def delenv(monkeypatch, name: str, raising: bool = True):
    monkeypatch.delenv(name, raising=raising)
    fg.fg_reload_tuning()


def poison_padding(t: torch.Tensor, lead: int, ld: int, other: int):
    """NaN into every element between the extent and the leading dimension: memory the library may
    read (inside 16-byte chunks and edge tiles) but must never let influence a result."""
    if ld > lead and other > 0:
        t[:ld * other].view(other, ld)[:, lead:] = float("nan")


def make_operand(rows: int, cols: int, layout: int, stream: int, device, ints: bool, pad: int = 0, seed=W.DEFAULT_SEED,
                 dtype=torch.float16, poison: bool = False):
    """A stored rows x cols FP16 (or BF16) operand in FG_COL / FG_ROW layout with ld = extent + pad.
    Returns (device tensor, ld)."""
    lead = rows if layout == fg.FG_COL else cols
    other = cols if layout == fg.FG_COL else rows
    ld = (lead + 7) // 8 * 8 + pad          # leading dimensions of FP16 operands are multiples of 8
    gen = W.small_ints if ints else W.uniform_pm1
    t = gen(ld * other, stream, seed=seed, device=device, dtype=dtype)
    if poison:
        poison_padding(t, lead, ld, other)
    return t, ld


def make_f32(numel: int, stream: int, device, ints: bool, seed=W.DEFAULT_SEED):
    gen = W.small_ints if ints else W.uniform_pm1
    return gen(numel, stream, seed=seed, device=device, dtype=torch.float32)


def np16(t: Optional[torch.Tensor]):
    """Host copy as a numpy array; bfloat16 tensors come back as their uint16 bit patterns."""
    if t is None:
        return None
    if t.dtype == torch.bfloat16:
        return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.detach().cpu().numpy()


def sample_positions(M: int, N: int, count: int, seed: int, tile: int = 256):
    """Random positions plus the corners, the last row/column and both sides of block-tile seams."""
    rng = np.random.default_rng(seed)
    I = list(rng.integers(0, M, count)); J = list(rng.integers(0, N, count))
    edges_m = sorted({0, M - 1} | {x for b in range(tile, M, tile) for x in (b - 1, b)} )
    edges_n = sorted({0, N - 1} | {x for b in range(tile, N, tile) for x in (b - 1, b)} )
    pick_m = edges_m if len(edges_m) <= 24 else list(rng.choice(edges_m, 24, replace=False)) + [0, M - 1]
    pick_n = edges_n if len(edges_n) <= 24 else list(rng.choice(edges_n, 24, replace=False)) + [0, N - 1]
    for i in pick_m:
        for j in pick_n:
            I.append(i); J.append(j)
    return np.array(I, np.int64), np.array(J, np.int64)


def compare(got: np.ndarray, ref: np.ndarray, G: np.ndarray, K: int, exact: bool, what: str, half_out: bool = False):
    """half_out: the result is stored as binary16.  Exact cases: it must equal the exact result
    rounded once to binary16.  Otherwise both bars grow by one binary16 rounding of the result,
    2^-11 |D_ref|, doubled for the few cases in which rounding the FP32 value instead of the
    exact one lands on the other neighbour."""
    got = got.astype(np.float64)
    assert np.isfinite(got).all(), what + ": non-finite output"
    if half_out:
        assert np.abs(ref).max(initial=0.0) < 65504.0, what + ": the test's results do not fit binary16"
        if exact:
            ref = O.round_array_to_half(ref)
    err = np.abs(got - ref)
    if exact:
        bad = np.flatnonzero(err.reshape(-1) != 0)
        assert bad.size == 0, "%s: %d entries differ from the exact result (first at flat index %d: got %r want %r)" % (
            what, bad.size, bad[0], got.reshape(-1)[bad[0]], ref.reshape(-1)[bad[0]])
        return 0.0
    official = OFFICIAL_RTOL * G + (2.0 ** -10 * np.abs(ref) if half_out else 0.0)
    tiny = np.finfo(np.float32).tiny
    worst = float(np.max(err / np.maximum(G, tiny))) if err.size else 0.0
    assert (err <= official + tiny).all(), "%s: official tolerance exceeded, max err/G = %g" % (what, worst)
    tight = 4.0 * math.sqrt(max(K, 1)) * 2.0 ** -24 * G + 2.0 ** -22 * np.abs(ref) + tiny + (2.0 ** -10 * np.abs(ref) if half_out else 0.0)
    assert (err <= tight).all(), "%s: tight tolerance exceeded, max err/G = %g" % (what, worst)
    return worst


def run_gemm_case(M, N, K, la=fg.FG_COL, lb=fg.FG_COL, ld_layout=fg.FG_COL, alpha=1.0, beta=1.0, with_c=True,
                  bias_dim=None, act=fg.FG_ACT_NONE, ints=False, pad=0, config=1, samples: Optional[int] = None,
                  inplace=False, device="cuda", seed=W.DEFAULT_SEED, bf16=False, ab_add=None, c_act=fg.FG_ACT_NONE,
                  cd16=False, poison=False, noalloc=False):
    """Run fg_gemm on seeded inputs and compare with the oracle.  ``samples`` None: every entry.
    ``cd16``: C and D are stored as binary16 (any leading dimension).  ``poison``: the padding of
    A, B and C (everything between an extent and its leading dimension) holds NaN."""
    dt = torch.bfloat16 if bf16 else torch.float16
    odt = O.BF16 if bf16 else O.F16
    A, lda = make_operand(M, K, la, W.stream_id(config, "A"), device, ints, pad, seed, dt, poison)
    B, ldb = make_operand(K, N, lb, W.stream_id(config, "B"), device, ints, pad, seed, dt, poison)
    lead, other = (M, N) if ld_layout == fg.FG_COL else (N, M)
    ldc = (lead + 3) // 4 * 4 + (4 if pad else 0)   # leading dimensions of FP32 operands are multiples of 4
    cd_dtype = torch.float32
    if cd16:
        ldc = lead + (3 if pad else 0)
        cd_dtype = torch.float16
    gen_cd = W.small_ints if ints else W.uniform_pm1
    Cbuf = gen_cd(ldc * other, W.stream_id(config, "C"), seed=seed, device=device, dtype=cd_dtype) if with_c else None
    if poison and with_c:
        poison_padding(Cbuf, lead, ldc, other)
    bias = None
    if bias_dim is not None:
        bias = make_f32(M if bias_dim == 0 else N, W.stream_id(config, "bias"), device, ints, seed)
    Dbuf = Cbuf if (inplace and with_c) else torch.full((ldc * other,), float("nan"), dtype=cd_dtype, device=device)
    C_host = np16(Cbuf).copy() if with_c else None
    fg.fg_gemm(M, N, K, alpha, fg.Matrix(A, la, lda), fg.Matrix(B, lb, ldb), beta,
               fg.Matrix(Cbuf, ld_layout, ldc) if with_c else None, fg.Matrix(Dbuf, ld_layout, ldc),
               bias=bias, bias_dim=bias_dim or 0, act=act,
               a_add=ab_add[0] if ab_add else 0.0, b_add=ab_add[1] if ab_add else 0.0, c_act=c_act, noalloc=noalloc)
    torch.cuda.synchronize()
    D_host = np16(Dbuf)
    # padding of D must be untouched
    Dm = D_host.reshape(other, ldc)
    if ldc > lead and (not inplace or poison):
        assert np.isnan(Dm[:, lead:]).all(), "padding of D was written"
    Dlog = Dm[:, :lead].T if ld_layout == fg.FG_COL else Dm[:, :lead]       # logical M x N view
    at = None
    if samples is not None:
        at = sample_positions(M, N, samples, seed=M * 31 + N * 17 + K)
    r = O.gemm(M, N, K, alpha, O.Operand(np16(A), la, lda, dtype=odt), O.Operand(np16(B), lb, ldb, dtype=odt), beta,
               C_host, None, ld_layout, ldc, bias=np16(bias), bias_dim=bias_dim or 0, act=act, at=at,
               ab_add=ab_add, c_act=c_act)
    got = Dlog if at is None else Dlog[at[0], at[1]]
    what = ("bf16 " if bf16 else "") + ("ab_add=%r c_act=%d " % (ab_add, c_act) if (ab_add or c_act) else "") + "gemm M=%d N=%d K=%d A=%d B=%d D=%d alpha=%g beta=%g ints=%s" % (M, N, K, la, lb, ld_layout, alpha, beta, ints)
    return compare(got, r["D"], r["G"], K, ints, ("f16 C,D " if cd16 else "") + what, half_out=cd16)


def run_unaligned_gemm_case(M, N, K, la=fg.FG_COL, lb=fg.FG_COL, ld_layout=fg.FG_COL, alpha=1.0, beta=1.0, with_c=True,
                            bias_dim=None, act=fg.FG_ACT_NONE, ints=True, pads=(1, 3, 1), offsets=(1, 3, 1), config=2,
                            device="cuda", seed=W.DEFAULT_SEED, bf16=False, ab_add=None, c_act=fg.FG_ACT_NONE):
    """fg_gemm on operands that miss the alignment of the tiled kernels: leading dimensions
    extent + pads[i] (any value), base pointers `offsets[i]` elements into their allocations
    (A, B, C/D), any K.  Every entry is compared with the oracle."""
    dt = torch.bfloat16 if bf16 else torch.float16
    odt = O.BF16 if bf16 else O.F16
    gen = W.small_ints if ints else W.uniform_pm1
    lda = (M if la == fg.FG_COL else K) + pads[0]
    ldb = (K if lb == fg.FG_COL else N) + pads[1]
    lead, other = (M, N) if ld_layout == fg.FG_COL else (N, M)
    ldc = lead + pads[2]
    A = gen(lda * (K if la == fg.FG_COL else M) + offsets[0], W.stream_id(config, "A"), seed=seed, device=device, dtype=dt)[offsets[0]:]
    B = gen(ldb * (N if lb == fg.FG_COL else K) + offsets[1], W.stream_id(config, "B"), seed=seed, device=device, dtype=dt)[offsets[1]:]
    Cbuf = gen(ldc * other + offsets[2], W.stream_id(config, "C"), seed=seed, device=device, dtype=torch.float32)[offsets[2]:] if with_c else None
    bias = None
    if bias_dim is not None:
        bias = gen((M if bias_dim == 0 else N) + 1, W.stream_id(config, "bias"), seed=seed, device=device, dtype=torch.float32)[1:]
    Dbuf = torch.full((ldc * other + offsets[2],), float("nan"), dtype=torch.float32, device=device)[offsets[2]:]
    fg.fg_gemm(M, N, K, alpha, fg.Matrix(A, la, lda), fg.Matrix(B, lb, ldb), beta,
               fg.Matrix(Cbuf, ld_layout, ldc) if with_c else None, fg.Matrix(Dbuf, ld_layout, ldc),
               bias=bias, bias_dim=bias_dim or 0, act=act,
               a_add=ab_add[0] if ab_add else 0.0, b_add=ab_add[1] if ab_add else 0.0, c_act=c_act)
    torch.cuda.synchronize()
    Dm = np16(Dbuf).reshape(other, ldc)
    if ldc > lead:
        assert np.isnan(Dm[:, lead:]).all(), "padding of D was written"
    Dlog = Dm[:, :lead].T if ld_layout == fg.FG_COL else Dm[:, :lead]
    r = O.gemm(M, N, K, alpha, O.Operand(np.ascontiguousarray(np16(A)), la, lda, dtype=odt),
               O.Operand(np.ascontiguousarray(np16(B)), lb, ldb, dtype=odt), beta,
               np.ascontiguousarray(np16(Cbuf)) if with_c else None, None, ld_layout, ldc,
               bias=np.ascontiguousarray(np16(bias)) if bias is not None else None, bias_dim=bias_dim or 0, act=act,
               ab_add=ab_add, c_act=c_act)
    what = "unaligned gemm M=%d N=%d K=%d A=%d B=%d D=%d pads=%s offsets=%s" % (M, N, K, la, lb, ld_layout, pads, offsets)
    return compare(Dlog, r["D"], r["G"], K, ints, what)


def run_contract_case(extents, modesA, modesB, modesC, alpha=1.0, beta=0.0, ints=False, samples: Optional[int] = None,
                      stridesA=None, stridesB=None, stridesC=None, inplace=False, config=5, device="cuda",
                      seed=W.DEFAULT_SEED, B_override=None, poison=False):
    """Run fg_contract on seeded dense (or explicitly strided) tensors and compare with the oracle.
    ``poison``: every position of A, B and Cin that the strided tensors do not reach holds NaN."""
    ext = lambda ms: [extents[m] for m in ms]
    sA = list(stridesA) if stridesA else list(W.col_major_strides(tuple(ext(modesA))))
    sB = list(stridesB) if stridesB else list(W.col_major_strides(tuple(ext(modesB))))
    sC = list(stridesC) if stridesC else list(W.col_major_strides(tuple(ext(modesC))))
    span = lambda ms, st: 1 + sum((extents[m] - 1) * s for m, s in zip(ms, st))
    gen = W.small_ints if ints else W.uniform_pm1
    A = gen(span(modesA, sA), W.stream_id(config, "A"), seed=seed, device=device, dtype=torch.float16)
    B = gen(span(modesB, sB), W.stream_id(config, "B"), seed=seed, device=device, dtype=torch.float16)
    if B_override is not None:
        B = B_override.to(device)
    nC = span(modesC, sC)
    Cin = gen(nC, W.stream_id(config, "C"), seed=seed, device=device, dtype=torch.float32) if beta != 0.0 else None
    if poison:
        def reached_mask(modes, strides, n):
            idx = torch.zeros(1, dtype=torch.int64)
            for m, st in zip(modes, strides):
                idx = (idx[:, None] + torch.arange(extents[m], dtype=torch.int64)[None, :] * st).reshape(-1)
            mask = torch.zeros(n, dtype=torch.bool)
            mask[idx] = True
            return mask.to(device)
        A[~reached_mask(modesA, sA, A.numel())] = float("nan")
        B[~reached_mask(modesB, sB, B.numel())] = float("nan")
        if Cin is not None:
            Cin[~reached_mask(modesC, sC, nC)] = float("nan")
    Cout = Cin if (inplace and Cin is not None) else torch.full((nC,), float("nan"), dtype=torch.float32, device=device)
    Cin_host = np16(Cin).copy() if Cin is not None else None
    fg.fg_contract(modesA, sA, A, modesB, sB, B, modesC, sC, Cin, Cout, extents, alpha=alpha, beta=beta)
    torch.cuda.synchronize()
    got_all = np16(Cout)
    K = 1
    for m in modesA:
        if m in modesB:
            K *= extents[m]
    what = "contract A%s B%s -> C%s extents=%s ints=%s" % (modesA, modesB, modesC, extents, ints)
    if samples is None:
        r = O.contract(extents, modesA, sA, np16(A), modesB, sB, np16(B), modesC, sC, Cin_host, alpha=alpha, beta=beta)
        # compare only the positions the tensor reaches (others must stay untouched)
        idx = np.zeros(1, np.int64)
        for m, s in zip(modesC, sC):
            idx = (idx[:, None] + np.arange(extents[m], dtype=np.int64)[None, :] * s).reshape(-1)
        reached = np.zeros(nC, bool); reached[idx] = True
        if not inplace:
            assert np.isnan(got_all[~reached]).all(), what + ": wrote outside the tensor"
        return compare(got_all[idx], r["D"][idx], r["G"][idx], K, ints, what)
    rng = np.random.default_rng(12345)
    at = np.stack([rng.integers(0, extents[m], samples) for m in modesC], axis=1)
    corners = np.array([[0] * len(modesC), [extents[m] - 1 for m in modesC]])
    at = np.concatenate([at, corners], axis=0)
    r = O.contract(extents, modesA, sA, np16(A), modesB, sB, np16(B), modesC, sC, Cin_host, alpha=alpha, beta=beta, at=at)
    off = (at * np.array(sC, np.int64)[None, :]).sum(axis=1)
    return compare(got_all[off], r["D"], r["G"], K, ints, what)


def run_diag_case(M, N, K, side="A", other_layout=fg.FG_COL, ld_layout=fg.FG_COL, alpha=1.0, beta=1.0, with_c=True,
                  ints=False, config=4, samples: Optional[int] = None, device="cuda", seed=W.DEFAULT_SEED):
    """D = diag(d) . B + C (side 'A') or A . diag(d) + C (side 'B'); d holds min(rows, cols) entries."""
    gen = W.small_ints if ints else W.uniform_pm1
    if side == "A":
        dvec = gen(min(M, K), W.stream_id(config, "d"), seed=seed, device=device, dtype=torch.float16)
        X, ldx = make_operand(K, N, other_layout, W.stream_id(config, "B"), device, ints, 0, seed)
        mA, mB = fg.Matrix(dvec, fg.FG_DIAG, 0), fg.Matrix(X, other_layout, ldx)
        oA, oB = O.Operand(np16(dvec), O.DIAG, 0), O.Operand(np16(X), other_layout, ldx)
    else:
        dvec = gen(min(K, N), W.stream_id(config, "d"), seed=seed, device=device, dtype=torch.float16)
        X, ldx = make_operand(M, K, other_layout, W.stream_id(config, "A"), device, ints, 0, seed)
        mA, mB = fg.Matrix(X, other_layout, ldx), fg.Matrix(dvec, fg.FG_DIAG, 0)
        oA, oB = O.Operand(np16(X), other_layout, ldx), O.Operand(np16(dvec), O.DIAG, 0)
    lead, other = (M, N) if ld_layout == fg.FG_COL else (N, M)
    ldc = (lead + 3) // 4 * 4
    Cbuf = make_f32(ldc * other, W.stream_id(config, "C"), device, ints, seed) if with_c else None
    Dbuf = torch.full((ldc * other,), float("nan"), dtype=torch.float32, device=device)
    fg.fg_gemm(M, N, K, alpha, mA, mB, beta, fg.Matrix(Cbuf, ld_layout, ldc) if with_c else None, fg.Matrix(Dbuf, ld_layout, ldc))
    torch.cuda.synchronize()
    Dm = np16(Dbuf).reshape(other, ldc)
    assert ldc == lead or np.isnan(Dm[:, lead:]).all(), "padding of D was written"
    Dm = Dm[:, :lead]
    Dlog = Dm.T if ld_layout == fg.FG_COL else Dm
    at = sample_positions(M, N, samples, seed=M + N + K) if samples is not None else None
    r = O.gemm(M, N, K, alpha, oA, oB, beta, np16(Cbuf), None, ld_layout, ldc, at=at)
    got = Dlog if at is None else Dlog[at[0], at[1]]
    return compare(got, r["D"], r["G"], 1, ints, "diag-%s gemm M=%d N=%d K=%d other=%d D=%d ints=%s" % (side, M, N, K, other_layout, ld_layout, ints))


def run_cgemm_case(M, N, K, la=fg.FG_COL, lb=fg.FG_COL, ld_layout=fg.FG_COL, alpha=1.0, beta=1.0, with_c=True,
                   ints=False, pad=0, config=4, samples: Optional[int] = None, device="cuda", seed=W.DEFAULT_SEED,
                   dual=False, interleaved=False, poison=False):
    """Planar-split complex (or, with ``dual``, dual-number) D = alpha A B + beta C; the two planes
    are separate arrays.  ``interleaved``: the same numbers stored with real and imaginary parts
    adjacent (FG_CF16 inputs, FG_CF32 C and D).  ``poison``: NaN in the padding of A, B and C."""
    Ar, lda = make_operand(M, K, la, W.stream_id(config, "A"), device, ints, pad, seed, poison=poison)
    Ai, _ = make_operand(M, K, la, W.stream_id(config, "A_im"), device, ints, pad, seed, poison=poison)
    Br, ldb = make_operand(K, N, lb, W.stream_id(config, "B"), device, ints, pad, seed, poison=poison)
    Bi, _ = make_operand(K, N, lb, W.stream_id(config, "B_im"), device, ints, pad, seed, poison=poison)
    lead, other = (M, N) if ld_layout == fg.FG_COL else (N, M)
    ldc = (lead + 3) // 4 * 4 + (4 if pad else 0)
    Cr = make_f32(ldc * other, W.stream_id(config, "C"), device, ints, seed) if with_c else None
    Ci = make_f32(ldc * other, W.stream_id(config, "C_im"), device, ints, seed) if with_c else None
    if poison and with_c:
        poison_padding(Cr, lead, ldc, other)
        poison_padding(Ci, lead, ldc, other)
    Dr = torch.full((ldc * other,), float("nan"), dtype=torch.float32, device=device)
    Di = torch.full((ldc * other,), float("nan"), dtype=torch.float32, device=device)
    if interleaved:
        weave = lambda x, y: torch.stack((x, y), dim=-1).reshape(-1).contiguous()
        Aw, Bw = weave(Ar, Ai), weave(Br, Bi)
        Cw = weave(Cr, Ci) if with_c else None
        Dw = torch.full((2 * ldc * other,), float("nan"), dtype=torch.float32, device=device)
        fg.fg_gemm(M, N, K, alpha, fg.Matrix(Aw, la, lda, dtype=fg.FG_CF16), fg.Matrix(Bw, lb, ldb, dtype=fg.FG_CF16), beta,
                   fg.Matrix(Cw, ld_layout, ldc, dtype=fg.FG_CF32) if with_c else None, fg.Matrix(Dw, ld_layout, ldc, dtype=fg.FG_CF32))
        torch.cuda.synchronize()
        Dr, Di = Dw[0::2].contiguous(), Dw[1::2].contiguous()
        if ldc > lead:
            assert torch.isnan(Dr.reshape(other, ldc)[:, lead:]).all() and torch.isnan(Di.reshape(other, ldc)[:, lead:]).all(), "padding of D was written"
    else:
        call = fg.fg_gemm_dual if dual else fg.fg_gemm
        call(M, N, K, alpha, fg.Matrix(Ar, la, lda, im=Ai), fg.Matrix(Br, lb, ldb, im=Bi), beta,
             fg.Matrix(Cr, ld_layout, ldc, im=Ci) if with_c else None, fg.Matrix(Dr, ld_layout, ldc, im=Di))
    torch.cuda.synchronize()
    view = lambda t: (np16(t).reshape(other, ldc)[:, :lead].T if ld_layout == fg.FG_COL else np16(t).reshape(other, ldc)[:, :lead])
    at = sample_positions(M, N, samples, seed=M * 3 + N * 5 + K) if samples is not None else None
    r = O.gemm(M, N, K, alpha, O.Operand(np16(Ar), la, lda, np16(Ai)), O.Operand(np16(Br), lb, ldb, np16(Bi)), beta,
               np16(Cr), np16(Ci), ld_layout, ldc, at=at, dual=dual)
    gr, gi = view(Dr), view(Di)
    if at is not None:
        gr, gi = gr[at[0], at[1]], gi[at[0], at[1]]
    what = ("dual" if dual else "interleaved complex" if interleaved else "complex") + " gemm M=%d N=%d K=%d A=%d B=%d D=%d ints=%s" % (M, N, K, la, lb, ld_layout, ints)
    w1 = compare(gr, r["D"], r["G"], K if dual else 2 * K, ints, what + " (first plane)")
    w2 = compare(gi, r["D_im"], r["G_im"], 2 * K, ints, what + " (second plane)")
    return max(w1, w2)
