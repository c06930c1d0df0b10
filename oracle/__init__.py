"""CPU oracle -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``tad_oracle.c`` (plain fp64 C).  Only tests, the
smoke check and the benchmark's ``cpu_baseline`` leg may import this package;
the GPU library never does, and this package never imports the GPU library.

Expressions are passed as duck-typed objects with the attributes ``body``,
``f_shape``, ``sums`` (inclusive ``(lo, hi)`` pairs) and ``args`` (each with
``shape`` and the integer index matrix ``A``), i.e. the problem statement of
Sec. 5.1 / 5.2 of the paper.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tad_oracle.c")
_LIB = os.path.join(_HERE, "libtad_oracle.so")

MAX_EXT, MAX_RANK, MAX_ARGS = 8, 4, 6


class _Arg(ctypes.Structure):
    _fields_ = [("rank", ctypes.c_int),
                ("shape", ctypes.c_int64 * MAX_RANK),
                ("A", (ctypes.c_int64 * MAX_EXT) * MAX_RANK)]


MAX_PROGRAM = 64
MAX_COND = 8
# postfix operation names of a program body -> the oracle's own codes (enum O_* in tad_oracle.c)
_OPS = {"const": 0, "arg": 1, "sum": 2, "add": 3, "sub": 4, "mul": 5, "div": 6, "neg": 7, "exp": 8, "log": 9,
        "sin": 10, "cos": 11, "tanh": 12, "sqrt": 13, "powi": 14, "store": 15, "load": 16}


class _Op(ctypes.Structure):
    _fields_ = [("op", ctypes.c_int), ("iarg", ctypes.c_int), ("value", ctypes.c_double)]


class _Expr(ctypes.Structure):
    _fields_ = [("body", ctypes.c_char * 16),
                ("n_f", ctypes.c_int),
                ("f_shape", ctypes.c_int64 * MAX_EXT),
                ("n_sum", ctypes.c_int),
                ("sum_lo", ctypes.c_int64 * MAX_EXT),
                ("sum_hi", ctypes.c_int64 * MAX_EXT),
                ("n_args", ctypes.c_int),
                ("args", _Arg * MAX_ARGS),
                ("n_inner", ctypes.c_int), ("n_outer", ctypes.c_int),
                ("inner", _Op * MAX_PROGRAM), ("outer", _Op * MAX_PROGRAM),
                ("n_cond", ctypes.c_int), ("cond", (ctypes.c_int64 * (MAX_EXT + 1)) * MAX_COND)]


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        assert lib.orc_sizeof_expr() == ctypes.sizeof(_Expr), "struct layout mismatch"
        pp = ctypes.POINTER(ctypes.c_void_p)
        lib.orc_forward.argtypes = [ctypes.POINTER(_Expr), pp, ctypes.c_void_p]
        lib.orc_backward.argtypes = [ctypes.POINTER(_Expr), pp, ctypes.c_void_p, pp, ctypes.c_int]
        lib.orc_gamma.argtypes = [ctypes.POINTER(_Expr), ctypes.c_int, ctypes.c_void_p,
                                  ctypes.c_void_p, ctypes.c_int64, ctypes.POINTER(ctypes.c_int64)]
        lib.orc_gamma_counts.argtypes = [ctypes.POINTER(_Expr), ctypes.c_int, ctypes.c_void_p]
        _lib = lib
    return _lib


def _pack(expr) -> _Expr:
    e = _Expr()
    e.body = expr.body.encode()
    e.n_f = len(expr.f_shape)
    for d, n in enumerate(expr.f_shape):
        e.f_shape[d] = int(n)
    e.n_sum = len(expr.sums)
    for s, (lo, hi) in enumerate(expr.sums):
        e.sum_lo[s], e.sum_hi[s] = int(lo), int(hi)
    e.n_args = len(expr.args)
    n_ext = e.n_f + e.n_sum
    assert n_ext <= MAX_EXT and e.n_args <= MAX_ARGS
    for p, a in enumerate(expr.args):
        e.args[p].rank = len(a.shape)
        assert len(a.A) == len(a.shape)
        for r, n in enumerate(a.shape):
            e.args[p].shape[r] = int(n)
            assert len(a.A[r]) == n_ext
            for d in range(n_ext):
                e.args[p].A[r][d] = int(a.A[r][d])
    cond = list(getattr(expr, "constraints", []) or [])
    assert len(cond) <= MAX_COND
    e.n_cond = len(cond)
    for j, (coef, const) in enumerate(cond):
        assert len(coef) == n_ext
        for d in range(n_ext):
            e.cond[j][d] = int(coef[d])
        e.cond[j][n_ext] = int(const)
    if expr.body == "program":
        for name, dst in (("inner", e.inner), ("outer", e.outer)):
            prog = list(getattr(expr, name))
            assert 1 <= len(prog) <= MAX_PROGRAM
            for i, t in enumerate(prog):
                dst[i].op = _OPS[t[0]]
                dst[i].iarg = int(t[1]) if t[0] in ("arg", "powi", "store", "load") else 0
                dst[i].value = float(t[1]) if t[0] == "const" else 0.0
        e.n_inner, e.n_outer = len(expr.inner), len(expr.outer)
    return e


def _ptrs(arrs: Sequence[Optional[np.ndarray]]):
    arr_t = ctypes.c_void_p * len(arrs)
    return arr_t(*[None if a is None else a.ctypes.data for a in arrs])


def _as_f64(expr, args):
    out = []
    for a, spec in zip(args, expr.args):
        x = np.ascontiguousarray(np.asarray(a, dtype=np.float64))
        assert tuple(x.shape) == tuple(spec.shape), (x.shape, spec.shape)
        out.append(x)
    return out


def max_threads() -> int:
    return int(_load().orc_max_threads())


def forward(expr, args) -> np.ndarray:
    """f for every function index, fp64."""
    lib = _load()
    xs = _as_f64(expr, args)
    f = np.empty(tuple(expr.f_shape), dtype=np.float64)
    e = _pack(expr)
    rc = lib.orc_forward(ctypes.byref(e), _ptrs(xs), f.ctypes.data)
    if rc:
        raise RuntimeError(f"orc_forward failed: {rc}")
    return f


def backward(expr, args, df, wanted: Optional[Sequence[bool]] = None,
             nthreads: int = 1) -> List[Optional[np.ndarray]]:
    """Gradients of every argument by brute-force scatter, fp64."""
    lib = _load()
    xs = _as_f64(expr, args)
    dfa = np.ascontiguousarray(np.asarray(df, dtype=np.float64))
    assert tuple(dfa.shape) == tuple(expr.f_shape)
    wanted = [True] * len(xs) if wanted is None else list(wanted)
    dx = [np.empty_like(x) if w else None for x, w in zip(xs, wanted)]
    e = _pack(expr)
    rc = lib.orc_backward(ctypes.byref(e), _ptrs(xs), dfa.ctypes.data, _ptrs(dx), int(nthreads))
    if rc:
        raise RuntimeError(f"orc_backward failed: {rc}")
    return dx


def backward_by_tensor(expr, args, df, nthreads: int = 1) -> List[Optional[np.ndarray]]:
    """Gradients per tensor when a tensor occurs as several operands (an operand whose ``same_as`` names an
    earlier operand is a further occurrence of that tensor and must be given the same array).  The
    derivative with respect to the tensor is the sum of the per-operand derivatives (Sec. 5.3: the
    gradient is accumulated over all occurrences).  Entries of alias operands are None."""
    per_operand = backward(expr, args, df, nthreads=nthreads)
    out: List[Optional[np.ndarray]] = list(per_operand)
    for p, a in enumerate(expr.args):
        q = getattr(a, "same_as", None)
        if q is not None:
            assert args[p] is args[q] or np.array_equal(args[p], args[q]), "alias operands share their tensor"
            out[q] = out[q] + per_operand[p]
            out[p] = None
    return out


def gamma(expr, arg: int, beta: Sequence[int]) -> np.ndarray:
    """All extended indices in the box mapped onto ``beta`` (lexicographic), shape (n, n_ext)."""
    lib = _load()
    e = _pack(expr)
    n_ext = e.n_f + e.n_sum
    b = np.asarray(beta, dtype=np.int64)
    n = ctypes.c_int64(0)
    rc = lib.orc_gamma(ctypes.byref(e), arg, b.ctypes.data, None, 0, ctypes.byref(n))
    if rc:
        raise RuntimeError(f"orc_gamma failed: {rc}")
    out = np.empty((n.value, n_ext), dtype=np.int64)
    if n.value:
        rc = lib.orc_gamma(ctypes.byref(e), arg, b.ctypes.data, out.ctypes.data, n.value,
                           ctypes.byref(n))
        if rc:
            raise RuntimeError(f"orc_gamma failed: {rc}")
    return out


def gamma_counts(expr, arg: int) -> np.ndarray:
    """|Gamma-hat(beta)| for every beta of argument ``arg``."""
    lib = _load()
    e = _pack(expr)
    counts = np.empty(tuple(expr.args[arg].shape), dtype=np.int64)
    rc = lib.orc_gamma_counts(ctypes.byref(e), arg, counts.ctypes.data)
    if rc:
        raise RuntimeError(f"orc_gamma_counts failed: {rc}")
    return counts
