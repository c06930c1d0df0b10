"""ctypes binding of the C ABI in include/tad.h (argument marshalling only).

Every step of the path runs inside libtad.so; PyTorch supplies device memory
and the stream.  There is no CPU fallback: if the library is missing the
import of this module fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np

MAX_EXT, MAX_RANK, MAX_ARGS, MAX_KERNEL, MAX_CONSTRAINTS = 6, 4, 6, 4, 8

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libtad.so")

F32, F64 = 0, 1
BODY = {"sq": 0, "cube": 1, "sin": 2, "exp": 3, "mul": 4, "worked": 5, "tanh_dot": 6, "program": 7}
MAX_PROGRAM = 64
OPCODE = {"const": 0, "arg": 1, "sum": 2, "add": 3, "sub": 4, "mul": 5, "div": 6, "neg": 7, "exp": 8, "log": 9,
          "sin": 10, "cos": 11, "tanh": 12, "sqrt": 13, "powi": 14, "store": 15, "load": 16}
FAMILY = {0: "generic", 1: "row_reduce", 2: "diagonal", 3: "antidiagonal", 4: "worked",
          5: "worked_mfma", 6: "strided", 7: "contraction", 8: "program"}
PLAN_GENERIC_ONLY = 1
PLAN_DIRECT_FORM = 2
PLAN_KEEP_PROGRAM = 4
PLAN_NO_TERM_LISTS = 8
ROWS_LOWER, ROWS_UPPER, ROWS_FEASIBILITY = 0, 1, 2

EXPORTS = ["tad_plan_derive", "tad_plan_free", "tad_plan_workspace_bytes", "tad_plan_query",
           "tad_plan_bound_row", "tad_plan_enumerate", "tad_plan_count_all", "tad_eval_forward",
           "tad_eval_backward", "tad_plan_forward_family", "tad_strerror", "tad_plan_program_eval", "tad_plan_program_registers",
           "tad_plan_derived_expr", "tad_plan_seed_expr", "tad_eval_backward_static", "tad_derived_create",
           "tad_derived_free", "tad_derived_workspace_bytes", "tad_derived_count", "tad_eval_derived"]
STATIC_SCRATCH_BYTES = 16 << 20


class TadOp(ctypes.Structure):
    _fields_ = [("op", ctypes.c_int32), ("iarg", ctypes.c_int32), ("value", ctypes.c_double)]


class TadExpr(ctypes.Structure):
    _fields_ = [("body", ctypes.c_int32), ("n_f", ctypes.c_int32),
                ("f_shape", ctypes.c_int64 * MAX_EXT), ("n_sum", ctypes.c_int32),
                ("sum_lo", ctypes.c_int64 * MAX_EXT), ("sum_hi", ctypes.c_int64 * MAX_EXT),
                ("n_constraints", ctypes.c_int32), ("constraint", (ctypes.c_int64 * (MAX_EXT + 1)) * MAX_CONSTRAINTS),
                ("n_operands", ctypes.c_int32), ("n_inner", ctypes.c_int32), ("n_outer", ctypes.c_int32),
                ("inner", TadOp * MAX_PROGRAM), ("outer", TadOp * MAX_PROGRAM)]


class TadArg(ctypes.Structure):
    _fields_ = [("rank", ctypes.c_int32), ("shape", ctypes.c_int64 * MAX_RANK),
                ("alias", ctypes.c_int32), ("index", (ctypes.c_int64 * MAX_EXT) * MAX_RANK),
                ("needs_grad", ctypes.c_int32)]


class TadPlanInfo(ctypes.Structure):
    _fields_ = [("rank", ctypes.c_int32), ("kernel_dim", ctypes.c_int32), ("n_cokernel", ctypes.c_int32),
                ("smith", ctypes.c_int64 * MAX_RANK),
                ("U", (ctypes.c_int64 * MAX_RANK) * MAX_RANK),
                ("V", (ctypes.c_int64 * MAX_EXT) * MAX_EXT),
                ("K", (ctypes.c_int64 * MAX_KERNEL) * MAX_EXT),
                ("C", (ctypes.c_int64 * MAX_RANK) * MAX_RANK),
                ("n_lower", ctypes.c_int32 * MAX_KERNEL), ("n_upper", ctypes.c_int32 * MAX_KERNEL),
                ("n_feasibility", ctypes.c_int32), ("family", ctypes.c_int32), ("in_outer", ctypes.c_int32),
                ("gather_layout", ctypes.c_int32), ("gather_splits", ctypes.c_int32),
                ("gather_elements", ctypes.c_int64), ("listed", ctypes.c_int32)]


class TadError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


def _load():
    # PyTorch carries its own copy of the HIP runtime.  It must be loaded first so that libtad.so binds to
    # the same runtime instance as the streams and allocations it is handed; two runtimes in one process
    # make every launch fail.
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64)
    lib.tad_plan_derive.argtypes = [ctypes.POINTER(TadExpr), ctypes.POINTER(TadArg), ctypes.c_int,
                                    ctypes.c_int, ctypes.c_uint32, ctypes.POINTER(vp)]
    lib.tad_plan_free.argtypes = [vp]
    lib.tad_plan_free.restype = None
    lib.tad_plan_workspace_bytes.argtypes = [vp]
    lib.tad_plan_workspace_bytes.restype = ctypes.c_size_t
    lib.tad_plan_query.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(TadPlanInfo)]
    lib.tad_plan_bound_row.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                       i64p, i64p, i64p, i64p]
    lib.tad_plan_enumerate.argtypes = [vp, ctypes.c_int, ctypes.c_int, vp, vp, ctypes.c_size_t,
                                       ctypes.POINTER(ctypes.c_size_t)]
    lib.tad_plan_count_all.argtypes = [vp, ctypes.c_int, vp]
    lib.tad_eval_forward.argtypes = [vp, ctypes.POINTER(vp), vp, vp, ctypes.c_size_t, vp]
    lib.tad_eval_backward.argtypes = [vp, ctypes.POINTER(vp), vp, vp, ctypes.POINTER(vp), vp,
                                      ctypes.c_size_t, vp]
    lib.tad_eval_backward_static.argtypes = [vp, ctypes.POINTER(vp), vp, vp, ctypes.POINTER(vp), vp]
    lib.tad_plan_forward_family.argtypes = [vp]
    lib.tad_plan_program_eval.argtypes = [vp, ctypes.c_int, vp, ctypes.c_double, ctypes.POINTER(ctypes.c_double)]
    lib.tad_plan_program_registers.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
    lib.tad_plan_derived_expr.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.POINTER(TadExpr),
                                          ctypes.POINTER(TadArg), ctypes.POINTER(ctypes.c_int),
                                          ctypes.POINTER(ctypes.c_int)]
    lib.tad_plan_seed_expr.argtypes = [vp, ctypes.c_int, ctypes.POINTER(TadExpr), ctypes.POINTER(TadArg),
                                       ctypes.POINTER(ctypes.c_int)]
    lib.tad_derived_create.argtypes = [vp, ctypes.c_int, ctypes.POINTER(vp)]
    lib.tad_derived_free.argtypes = [vp]
    lib.tad_derived_free.restype = None
    lib.tad_derived_workspace_bytes.argtypes = [vp]
    lib.tad_derived_workspace_bytes.restype = ctypes.c_size_t
    lib.tad_derived_count.argtypes = [vp, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
    lib.tad_eval_derived.argtypes = [vp, ctypes.POINTER(vp), vp, vp, vp, ctypes.c_size_t, vp]
    lib.tad_strerror.argtypes = [ctypes.c_int]
    lib.tad_strerror.restype = ctypes.c_char_p
    return lib


lib = _load()


def strerror(status: int) -> str:
    return lib.tad_strerror(int(status)).decode()


def _check(rc: int, where: str):
    if rc != 0:
        raise TadError(rc, where)


def pack_expr(expr) -> TadExpr:
    e = TadExpr()
    e.body = BODY[expr.body]
    e.n_f = len(expr.f_shape)
    for d, n in enumerate(expr.f_shape):
        e.f_shape[d] = int(n)
    e.n_sum = len(expr.sums)
    for s, (lo, hi) in enumerate(expr.sums):
        e.sum_lo[s], e.sum_hi[s] = int(lo), int(hi)
    cons = list(getattr(expr, "constraints", []) or [])
    if len(cons) > MAX_CONSTRAINTS:
        raise TadError(-1, "tad_plan_derive")
    e.n_constraints = len(cons)
    n_ext = e.n_f + e.n_sum
    for j, (coef, const) in enumerate(cons):     # sum_d coef[d] * [alpha k]_d + const >= 0
        for d in range(n_ext):
            e.constraint[j][d] = int(coef[d])
        e.constraint[j][n_ext] = int(const)
    if expr.body == "program":
        # postfix programs as lists of tuples: ("arg", p), ("const", c), ("sum",), ("powi", n), ("add",), ...
        e.n_operands = len(expr.args)
        for name, dst in (("inner", e.inner), ("outer", e.outer)):
            prog = list(getattr(expr, name))
            if len(prog) > MAX_PROGRAM:
                raise TadError(-1, "tad_plan_derive")
            for i, t in enumerate(prog):
                dst[i].op = OPCODE[t[0]]
                if t[0] in ("arg", "powi", "store", "load"):
                    dst[i].iarg = int(t[1])
                elif t[0] == "const":
                    dst[i].value = float(t[1])
        e.n_inner, e.n_outer = len(expr.inner), len(expr.outer)
    return e


def pack_args(expr, needs_grad: Optional[Sequence[bool]] = None):
    n = len(expr.args)
    arr = (TadArg * n)()
    n_ext = len(expr.f_shape) + len(expr.sums)
    for p, a in enumerate(expr.args):
        arr[p].rank = len(a.shape)
        arr[p].alias = 0 if getattr(a, "same_as", None) is None else int(a.same_as) + 1
        arr[p].needs_grad = 1 if needs_grad is None else int(bool(needs_grad[p]))
        for r, s in enumerate(a.shape):
            arr[p].shape[r] = int(s)
            for d in range(n_ext):
                arr[p].index[r][d] = int(a.A[r][d])
    return arr


class Plan:
    """Owner of one ``tad_plan``."""

    def __init__(self, expr, needs_grad: Optional[Sequence[bool]] = None, generic_only: bool = False,
                 direct_form: bool = False, keep_program: bool = False, term_lists: bool = True):
        self.expr = expr
        self.n_ext = len(expr.f_shape) + len(expr.sums)
        if self.n_ext > MAX_EXT or len(expr.args) > MAX_ARGS:
            raise TadError(-1, "tad_plan_derive")
        if any(len(a.shape) > MAX_RANK for a in expr.args):
            raise TadError(-1, "tad_plan_derive")
        self.dtype = {"f32": F32, "f64": F64}[expr.dtype]
        self._h = ctypes.c_void_p(None)
        e, a = pack_expr(expr), pack_args(expr, needs_grad)
        flags = (PLAN_GENERIC_ONLY if generic_only else 0) | (PLAN_DIRECT_FORM if direct_form else 0) | \
            (PLAN_KEEP_PROGRAM if keep_program else 0) | (0 if term_lists else PLAN_NO_TERM_LISTS)
        _check(lib.tad_plan_derive(ctypes.byref(e), a, len(expr.args), self.dtype, flags,
                                   ctypes.byref(self._h)), "tad_plan_derive")

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and lib is not None:   # lib is None while the interpreter shuts down
            lib.tad_plan_free(h)

    # ---- host introspection -------------------------------------------------------------------
    @property
    def workspace_bytes(self) -> int:
        return int(lib.tad_plan_workspace_bytes(self._h))

    @property
    def forward_family(self) -> str:
        return FAMILY[lib.tad_plan_forward_family(self._h)]

    def query(self, arg: int, occ: int = 0) -> dict:
        info = TadPlanInfo()
        _check(lib.tad_plan_query(self._h, arg, occ, ctypes.byref(info)), "tad_plan_query")
        N, D, R, kap = len(self.expr.args[arg].shape), self.n_ext, info.rank, info.kernel_dim
        mat = lambda m, r, c: np.array([[m[i][j] for j in range(c)] for i in range(r)], dtype=np.int64).reshape(r, c)
        return dict(rank=R, kernel_dim=kap, smith=[info.smith[i] for i in range(R)],
                    U=mat(info.U, N, N), V=mat(info.V, D, D), K=mat(info.K, D, kap),
                    C=mat(info.C, info.n_cokernel, N),
                    n_lower=[info.n_lower[k] for k in range(kap)],
                    n_upper=[info.n_upper[k] for k in range(kap)],
                    n_feasibility=info.n_feasibility, family=FAMILY[info.family], in_outer=bool(info.in_outer),
                    gather_layout=("threads", "blocks", "lanes")[info.gather_layout], gather_splits=info.gather_splits,
                    gather_elements=info.gather_elements, listed=bool(info.listed))

    def bound_rows(self, arg: int, kind: int, level: int = 0) -> List[dict]:
        q = self.query(arg)
        n = q["n_feasibility"] if kind == ROWS_FEASIBILITY else (q["n_lower"] if kind == ROWS_LOWER else q["n_upper"])[level]
        out = []
        for r in range(n):
            scale = ctypes.c_int64(0)
            cb = (ctypes.c_int64 * (2 * MAX_EXT))()
            cz = (ctypes.c_int64 * MAX_KERNEL)()
            cc = (ctypes.c_int64 * MAX_CONSTRAINTS)()
            _check(lib.tad_plan_bound_row(self._h, arg, kind, level, r, ctypes.byref(scale), cb, cz, cc),
                   "tad_plan_bound_row")
            D = self.n_ext
            out.append(dict(scale=scale.value,
                            coef_b=np.array([cb[d] for d in range(D)] + [cb[MAX_EXT + d] for d in range(D)],
                                            dtype=np.int64),
                            coef_z=np.array([cz[m] for m in range(q["kernel_dim"])], dtype=np.int64),
                            coef_c=np.array([cc[j] for j in range(len(getattr(self.expr, "constraints", []) or []))],
                                            dtype=np.int64)))
        return out

    def enumerate(self, arg: int, beta: Sequence[int], occ: int = 0) -> np.ndarray:
        b = np.asarray(beta, dtype=np.int64)
        n = ctypes.c_size_t(0)
        _check(lib.tad_plan_enumerate(self._h, arg, occ, b.ctypes.data, None, 0, ctypes.byref(n)),
               "tad_plan_enumerate")
        out = np.empty((n.value, self.n_ext), dtype=np.int64)
        if n.value:
            _check(lib.tad_plan_enumerate(self._h, arg, occ, b.ctypes.data, out.ctypes.data, n.value,
                                          ctypes.byref(n)), "tad_plan_enumerate")
        return out

    def program_eval(self, which: int, values=None, total: float = 0.0) -> float:
        """Host evaluation of the derived scalar programs: which = -1 inner, p >= 0 d inner / d operand p,
        -2 outer(total), -3 d outer / d total."""
        out = ctypes.c_double(0.0)
        v = None if values is None else np.ascontiguousarray(values, dtype=np.float64)
        _check(lib.tad_plan_program_eval(self._h, which, None if v is None else v.ctypes.data, float(total),
                                         ctypes.byref(out)), "tad_plan_program_eval")
        return out.value

    def program_registers(self, which: int) -> int:
        """Registers of the register form of a derived scalar program (`which` as in program_eval); -1: the
        kernels interpret the form with one temporary per operation; 0: a single operand, a constant or zero."""
        n = ctypes.c_int(0)
        _check(lib.tad_plan_program_registers(self._h, which, ctypes.byref(n)), "tad_plan_program_registers")
        return n.value

    def _unpack_expr(self, e, a, n, names):
        from .workloads import ArgSpec, ExprSpec
        n_ext = e.n_f + e.n_sum
        opname = {v: k for k, v in OPCODE.items()}

        def program(ops, count):
            out = []
            for i in range(count):
                name = opname[ops[i].op]
                out.append((name, ops[i].iarg) if name in ("arg", "powi", "store", "load") else
                           (name, ops[i].value) if name == "const" else (name,))
            return out

        args = [ArgSpec(names[q], tuple(a[q].shape[r] for r in range(a[q].rank)),
                        [[a[q].index[r][d] for d in range(n_ext)] for r in range(a[q].rank)],
                        None if a[q].alias == 0 else a[q].alias - 1) for q in range(n)]
        return ExprSpec("program", tuple(e.f_shape[d] for d in range(e.n_f)),
                        [(e.sum_lo[s], e.sum_hi[s]) for s in range(e.n_sum)], args, self.expr.dtype,
                        inner=program(e.inner, e.n_inner), outer=program(e.outer, e.n_outer),
                        constraints=[([e.constraint[j][d] for d in range(n_ext)], e.constraint[j][n_ext])
                                     for j in range(e.n_constraints)])

    def derived_expr(self, arg: int, occ: int = 0, part: int = 0):
        """The gradient of occurrence `occ` of operand `arg` as an expression of its own: (expression, operands)
        with operands[q] = index of the original operand that new operand q is; operands[0] is -1 for df, -2 for
        the seed g = df * d outer / d sum (``seed_expr(-1)``), -3 - p for the seed of operand p (``seed_expr(p)``).
        part 0: the terms through the sum; part 1: the term of an operand the outer function reads.
        The expression can be planned and evaluated like any other."""
        e, a = TadExpr(), (TadArg * MAX_ARGS)()
        src, n = (ctypes.c_int * MAX_ARGS)(), ctypes.c_int(0)
        _check(lib.tad_plan_derived_expr(self._h, arg, occ, part, ctypes.byref(e), a, src, ctypes.byref(n)),
               "tad_plan_derived_expr")
        operands = [src[q] for q in range(n.value)]
        names = [{-1: "df", -2: "g"}.get(operands[0], "h")]
        names += [self.expr.args[operands[q]].name + ("" if a[q].alias == 0 else f"_{q}") for q in range(1, n.value)]
        return self._unpack_expr(e, a, n.value, names), operands

    def seed_expr(self, which: int = -1):
        """g = df * d outer / d sum (which = -1) or h = df * d outer / d operand `which`, as an expression over the
        function indices of this one; its operands are df followed by the operands of this expression."""
        e, a, n = TadExpr(), (TadArg * MAX_ARGS)(), ctypes.c_int(0)
        _check(lib.tad_plan_seed_expr(self._h, which, ctypes.byref(e), a, ctypes.byref(n)), "tad_plan_seed_expr")
        return self._unpack_expr(e, a, n.value, ["df"] + [x.name for x in self.expr.args])

    def count_all(self, arg: int) -> np.ndarray:
        counts = np.empty(tuple(self.expr.args[arg].shape), dtype=np.int64)
        _check(lib.tad_plan_count_all(self._h, arg, counts.ctypes.data), "tad_plan_count_all")
        return counts

    # ---- device evaluation (torch tensors supply memory and stream) -----------------------------
    def _torch_dtype(self):
        import torch
        return torch.float64 if self.dtype == F64 else torch.float32

    def _check_tensor(self, t, shape, what):
        if t.device.type != "cuda" or not t.is_contiguous() or t.dtype != self._torch_dtype() \
                or tuple(t.shape) != tuple(shape):
            raise ValueError(f"{what}: need a contiguous {self._torch_dtype()} cuda tensor of shape {tuple(shape)}, "
                             f"got {t.dtype} {tuple(t.shape)} on {t.device}")

    def _is_alias(self, p: int) -> bool:
        return getattr(self.expr.args[p], "same_as", None) is not None

    def _arg_ptrs(self, args):
        """One entry per operand; the entry of an alias operand is not used (it may be None)."""
        ptrs = []
        for p, (t, a) in enumerate(zip(args, self.expr.args)):
            if self._is_alias(p):
                ptrs.append(None)
                continue
            self._check_tensor(t, a.shape, a.name)
            ptrs.append(t.data_ptr())
        return (ctypes.c_void_p * len(args))(*ptrs)

    def workspace(self, device="cuda"):
        import torch
        n = self.workspace_bytes
        return torch.empty(max(n, 1), dtype=torch.uint8, device=device)

    def forward(self, args, out=None, ws=None):
        import torch
        ptrs = self._arg_ptrs(args)
        if out is None:
            out = torch.empty(tuple(self.expr.f_shape), dtype=self._torch_dtype(), device=args[0].device)
        self._check_tensor(out, self.expr.f_shape, "f")
        ws = self.workspace(args[0].device) if ws is None else ws
        stream = torch.cuda.current_stream().cuda_stream
        _check(lib.tad_eval_forward(self._h, ptrs, out.data_ptr(), ws.data_ptr(), ws.numel(),
                                    ctypes.c_void_p(stream)), "tad_eval_forward")
        return out

    def backward(self, args, f, df, wanted: Optional[Sequence[bool]] = None, out=None, ws=None, static=False):
        """static=True: tad_eval_backward_static (the library's own fixed scratch array instead of a workspace)."""
        import torch
        ptrs = self._arg_ptrs(args)
        self._check_tensor(f, self.expr.f_shape, "f")
        self._check_tensor(df, self.expr.f_shape, "df")
        wanted = [True] * len(args) if wanted is None else list(wanted)
        wanted = [w and not self._is_alias(p) for p, w in enumerate(wanted)]   # an alias has no gradient of its own
        if out is None:
            out = [torch.empty_like(t) if w else None for t, w in zip(args, wanted)]
        for t, a in zip(out, self.expr.args):
            if t is not None:
                self._check_tensor(t, a.shape, "d" + a.name)
        dptr = (ctypes.c_void_p * len(args))(*[None if t is None else t.data_ptr() for t in out])
        stream = torch.cuda.current_stream().cuda_stream
        if static:
            _check(lib.tad_eval_backward_static(self._h, ptrs, f.data_ptr(), df.data_ptr(), dptr,
                                                ctypes.c_void_p(stream)), "tad_eval_backward_static")
            return out
        ws = self.workspace(args[0].device) if ws is None else ws
        _check(lib.tad_eval_backward(self._h, ptrs, f.data_ptr(), df.data_ptr(), dptr, ws.data_ptr(),
                                     ws.numel(), ctypes.c_void_p(stream)), "tad_eval_backward")
        return out


class DerivedGradient:
    """Owner of one ``tad_derived``: the gradient of tensor `arg` of a plan's expression, evaluated through its
    derived expressions (seed expressions, one part per occurrence, a second part for operands of the outer
    function); ``counts`` = (seed expressions, parts)."""

    def __init__(self, plan: Plan, arg: int):
        self.plan, self.arg = plan, arg
        self._h = ctypes.c_void_p(None)
        _check(lib.tad_derived_create(plan._h, arg, ctypes.byref(self._h)), "tad_derived_create")
        a, b = ctypes.c_int(0), ctypes.c_int(0)
        _check(lib.tad_derived_count(self._h, ctypes.byref(a), ctypes.byref(b)), "tad_derived_count")
        self.counts = (a.value, b.value)

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and lib is not None:
            lib.tad_derived_free(h)

    @property
    def workspace_bytes(self) -> int:
        return int(lib.tad_derived_workspace_bytes(self._h))

    def evaluate(self, args, df, out=None, ws=None):
        import torch
        plan = self.plan
        ptrs = plan._arg_ptrs(args)
        plan._check_tensor(df, plan.expr.f_shape, "df")
        if out is None:
            out = torch.empty_like(args[self.arg])
        plan._check_tensor(out, plan.expr.args[self.arg].shape, "d" + plan.expr.args[self.arg].name)
        if ws is None:
            ws = torch.empty(max(self.workspace_bytes, 1), dtype=torch.uint8, device=df.device)
        stream = torch.cuda.current_stream().cuda_stream
        _check(lib.tad_eval_derived(self._h, ptrs, df.data_ptr(), out.data_ptr(), ws.data_ptr(), ws.numel(),
                                    ctypes.c_void_p(stream)), "tad_eval_derived")
        return out


def plan_derive(expr, needs_grad=None, generic_only=False) -> Plan:
    return Plan(expr, needs_grad, generic_only)


def eval_forward(plan: Plan, args, out=None, ws=None):
    return plan.forward(args, out, ws)


def eval_backward(plan: Plan, args, f, df, wanted=None, out=None, ws=None):
    return plan.backward(args, f, df, wanted, out, ws)


# ---- host utilities of the integer machinery (Sec. 4) -----------------------------------------------
lib.tad_extended_gcd.argtypes = [ctypes.c_int64, ctypes.c_int64] + [ctypes.POINTER(ctypes.c_int64)] * 3
lib.tad_smith_normal_form.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(ctypes.c_int)]
lib.tad_lattice_enumerate.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                      ctypes.POINTER(ctypes.c_size_t)]
EXPORTS += ["tad_extended_gcd", "tad_smith_normal_form", "tad_lattice_enumerate"]


def extended_gcd(a: int, b: int):
    g, x, y = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    _check(lib.tad_extended_gcd(a, b, ctypes.byref(g), ctypes.byref(x), ctypes.byref(y)), "tad_extended_gcd")
    return g.value, x.value, y.value


def smith_normal_form(A):
    A = np.ascontiguousarray(np.asarray(A, dtype=np.int64))
    n, m = A.shape
    S, U, V = np.zeros((n, m), np.int64), np.zeros((n, n), np.int64), np.zeros((m, m), np.int64)
    R = ctypes.c_int(0)
    _check(lib.tad_smith_normal_form(A.ctypes.data, n, m, S.ctypes.data, U.ctypes.data, V.ctypes.data,
                                     ctypes.byref(R)), "tad_smith_normal_form")
    return S, U, V, R.value


def lattice_enumerate(A, lo, hi, beta) -> np.ndarray:
    A = np.ascontiguousarray(np.asarray(A, dtype=np.int64))
    n, m = A.shape
    lo, hi = np.asarray(lo, dtype=np.int64), np.asarray(hi, dtype=np.int64)
    beta = np.asarray(beta, dtype=np.int64)
    assert lo.shape == (m,) and hi.shape == (m,) and beta.shape == (n,)
    cnt = ctypes.c_size_t(0)
    _check(lib.tad_lattice_enumerate(A.ctypes.data, n, m, lo.ctypes.data, hi.ctypes.data, beta.ctypes.data,
                                     None, 0, ctypes.byref(cnt)), "tad_lattice_enumerate")
    out = np.empty((cnt.value, m), dtype=np.int64)
    if cnt.value:
        _check(lib.tad_lattice_enumerate(A.ctypes.data, n, m, lo.ctypes.data, hi.ctypes.data,
                                         beta.ctypes.data, out.ctypes.data, cnt.value, ctypes.byref(cnt)),
               "tad_lattice_enumerate")
    return out


lib.tad_profile_begin.argtypes = [ctypes.c_char_p, ctypes.c_int]
lib.tad_profile_end.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int)]
EXPORTS += ["tad_profile_begin", "tad_profile_end"]
