"""Seeded synthetic workloads: expression descriptions and input tensors.

This module only *describes* element-wise defined tensors (shapes, summation
limits, integer index matrices, the name of the scalar body) and draws random
input values.  It contains none of the method's arithmetic and imports neither
the HIP binding nor the CPU oracle; both are driven from the data built here.

An expression follows the problem statement of Sec. 5.1 / 5.2 of the paper:
    f_alpha = fbar( sum_{k in Psi} s( y^p_{Ahat^p [alpha k]} ... ) )
with every argument index an integer linear map of the function indices alpha
followed by the summation indices k (the "sum-extended" multi-index).
Indices are zero-based (Sec. 6) and tensors are dense, row-major.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

import numpy as np

SEED_BASE = 171101348


@dataclass
class ArgSpec:
    name: str
    shape: Tuple[int, ...]
    # index matrix, one row per argument axis, one column per function index
    # followed by one column per summation index
    A: List[List[int]]
    # a further occurrence of the tensor given as operand `same_as` (an earlier operand), else None
    same_as: int | None = None


@dataclass
class ExprSpec:
    body: str                       # name of the scalar body
    f_shape: Tuple[int, ...]
    sums: List[Tuple[int, int]]     # inclusive (lo, hi) per summation index
    args: List[ArgSpec]
    dtype: str = "f64"              # "f64" or "f32"
    # body "program": the scalar functions as postfix programs, f = outer(sum_k inner(operand values)).
    # Entries: ("arg", p), ("const", c), ("sum",), ("add",), ("sub",), ("mul",), ("div",), ("neg",), ("exp",),
    # ("log",), ("sin",), ("cos",), ("tanh",), ("sqrt",), ("powi", n), ("store", t) (keep a copy of the top of the
    # stack in temporary t), ("load", t) (push temporary t).  ("sum",) belongs to the outer program;
    # ("arg", p) to the inner one and, for operands whose index ignores the summation indices, to the outer one.
    inner: List[tuple] = field(default_factory=list)
    outer: List[tuple] = field(default_factory=list)
    # extra linear conditions on the extended index (summation ranges that depend on other indices, Sec. 5.2):
    # a list of (coef, const); the term at [alpha k] is part of the sum iff sum_d coef[d] [alpha k]_d + const >= 0
    constraints: List[tuple] = field(default_factory=list)

    @property
    def n_ext(self) -> int:
        return len(self.f_shape) + len(self.sums)


@dataclass
class Workload:
    name: str
    expr: ExprSpec
    inputs: Dict[str, np.ndarray]   # argument tensors, in expr.args order
    df: np.ndarray
    notes: str = ""
    arg_order: List[str] = field(default_factory=list)

    def arg_list(self) -> List[np.ndarray]:
        """One array per operand; an alias operand gets the array of the operand it names."""
        args = self.expr.args
        return [self.inputs[(a if a.same_as is None else args[a.same_as]).name] for a in args]


def _np_dtype(dtype: str):
    return {"f64": np.float64, "f32": np.float32}[dtype]


def _round(x: np.ndarray, dtype: str) -> np.ndarray:
    """Values are drawn in fp64 and rounded once to the working precision."""
    return np.ascontiguousarray(x.astype(_np_dtype(dtype)))


def _uniform(rng, lo, hi, shape):
    return rng.uniform(lo, hi, size=shape)


# --------------------------------------------------------------------------
# expression builders
# --------------------------------------------------------------------------

def worked_expr(I: int, J: int, K: int, dtype: str, d_len: int | None = None,
                c_shape: Tuple[int, int] | None = None) -> ExprSpec:
    """f_ij = exp(-sum_k((a_ik + b_jk)^2 c_ii + d_{i+k}^3)), extended index (i, j, k)."""
    d_len = I + K - 1 if d_len is None else d_len
    c_shape = (I, I) if c_shape is None else c_shape
    return ExprSpec(
        body="worked", f_shape=(I, J), sums=[(0, K - 1)], dtype=dtype,
        args=[
            ArgSpec("a", (I, K), [[1, 0, 0], [0, 0, 1]]),
            ArgSpec("b", (J, K), [[0, 1, 0], [0, 0, 1]]),
            ArgSpec("c", c_shape, [[1, 0, 0], [1, 0, 0]]),
            ArgSpec("d", (d_len,), [[1, 0, 1]]),
        ])


def broadcast_sq_expr(I: int, J: int, dtype: str) -> ExprSpec:
    """f_ij = x_i^2."""
    return ExprSpec("sq", (I, J), [], [ArgSpec("x", (I,), [[1, 0]])], dtype)


def diagonal_sq_expr(I: int, dtype: str) -> ExprSpec:
    """f_i = x_ii^2."""
    return ExprSpec("sq", (I,), [], [ArgSpec("x", (I, I), [[1], [1]])], dtype)


def index_sum_exp_expr(I: int, J: int, dtype: str) -> ExprSpec:
    """f_ij = exp(x_{i+j})."""
    return ExprSpec("exp", (I, J), [], [ArgSpec("x", (I + J - 1,), [[1, 1]])], dtype)


def strided_tanh_expr(N: int, I: int, J: int, U: int, V: int, stride: int,
                      dtype: str) -> ExprSpec:
    """f_nij = tanh(sum_{u<U, v<V} x_{n, stride*i+u, stride*j+v} w_uv); extended index (n,i,j,u,v)."""
    P = stride * (I - 1) + U
    Q = stride * (J - 1) + V
    return ExprSpec(
        "tanh_dot", (N, I, J), [(0, U - 1), (0, V - 1)],
        [ArgSpec("x", (N, P, Q), [[1, 0, 0, 0, 0],
                                  [0, stride, 0, 1, 0],
                                  [0, 0, stride, 0, 1]]),
         ArgSpec("w", (U, V), [[0, 0, 0, 1, 0],
                               [0, 0, 0, 0, 1]])],
        dtype)


# --------------------------------------------------------------------------
# the five benchmark configurations
# --------------------------------------------------------------------------

def matmul_expr(I: int, J: int, K: int, dtype: str, x_transposed: bool = False,
                y_transposed: bool = False, swap: bool = False) -> ExprSpec:
    """f_ij = sum_k x_ik y_kj (Sec. 5, f^4), extended index (i, j, k).  x is stored I x K (K x I if
    x_transposed), y is stored K x J (J x K if y_transposed); swap lists y before x."""
    ri, rj, rk = [1, 0, 0], [0, 1, 0], [0, 0, 1]
    x = ArgSpec("x", (K, I), [rk, ri]) if x_transposed else ArgSpec("x", (I, K), [ri, rk])
    y = ArgSpec("y", (J, K), [rj, rk]) if y_transposed else ArgSpec("y", (K, J), [rk, rj])
    return ExprSpec("mul", (I, J), [(0, K - 1)], [y, x] if swap else [x, y], dtype)


def matmul_workload(n: int = 4096) -> Workload:
    """Square fp32 matrix product and its two derived products, uniform[-1,1] inputs."""
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + 6))
    expr = matmul_expr(n, n, n, "f32")
    x = _uniform(rng, -1, 1, (n, n))
    y = _uniform(rng, -1, 1, (n, n))
    df = _uniform(rng, -1, 1, (n, n))
    return Workload(f"matmul_{n}x{n}x{n}_f32", expr, {"x": _round(x, "f32"), "y": _round(y, "f32")},
                    _round(df, "f32"))


# The built-in bodies written as programs (same index maps, scalar part given in postfix form)
PROGRAM_OF_BODY = {
    "sq": ([("arg", 0)], [("sum",), ("powi", 2)]),
    "cube": ([("arg", 0)], [("sum",), ("powi", 3)]),
    "sin": ([("arg", 0)], [("sum",), ("sin",)]),
    "exp": ([("arg", 0)], [("sum",), ("exp",)]),
    "mul": ([("arg", 0), ("arg", 1), ("mul",)], [("sum",)]),
    "tanh_dot": ([("arg", 0), ("arg", 1), ("mul",)], [("sum",), ("tanh",)]),
    # (a + b)^2 c + d^3, exp(-s)
    "worked": ([("arg", 0), ("arg", 1), ("add",), ("powi", 2), ("arg", 2), ("mul",), ("arg", 3), ("powi", 3), ("add",)],
               [("sum",), ("neg",), ("exp",)]),
}


def as_program(expr: ExprSpec) -> ExprSpec:
    """The same expression with its built-in body replaced by the equivalent postfix programs."""
    inner, outer = PROGRAM_OF_BODY[expr.body]
    return ExprSpec("program", expr.f_shape, list(expr.sums), list(expr.args), expr.dtype, list(inner), list(outer),
                    list(expr.constraints))


def softplus_ratio_expr(I: int, J: int, K: int, dtype: str) -> ExprSpec:
    """f_ij = log(1 + sum_k exp(x_ik) * sqrt(y_kj^2 + 1) / (2 + cos(z_{i+k})))  -- a body with no built-in twin."""
    inner = [("arg", 0), ("exp",), ("arg", 1), ("powi", 2), ("const", 1.0), ("add",), ("sqrt",), ("mul",),
             ("const", 2.0), ("arg", 2), ("cos",), ("add",), ("div",)]
    outer = [("const", 1.0), ("sum",), ("add",), ("log",)]
    return ExprSpec("program", (I, J), [(0, K - 1)],
                    [ArgSpec("x", (I, K), [[1, 0, 0], [0, 0, 1]]), ArgSpec("y", (K, J), [[0, 0, 1], [0, 1, 0]]),
                     ArgSpec("z", (I + K - 1,), [[1, 0, 1]])], dtype, inner, outer)


def many_live_values_expr(I: int, K: int, dtype: str) -> ExprSpec:
    """f_i = sum_k (sum of 18 different functions of x_ik and y_k), written so that all 18 values are computed
    before the first addition: more values alive at once than the kernels' register form of a program holds."""
    fns = [("exp",), ("sin",), ("cos",), ("tanh",), ("neg",), ("powi", 2), ("powi", 3), ("powi", 4), ("powi", 5)]
    inner = []
    for a in (0, 1):
        for fn in fns:
            inner += [("arg", a), fn]
    inner += [("add",)] * 17
    return ExprSpec("program", (I,), [(0, K - 1)],
                    [ArgSpec("x", (I, K), [[1, 0], [0, 1]]), ArgSpec("y", (K,), [[0, 1]])], dtype, inner, [("sum",)])


# Operands of the outer function (Sec. 5.2: fbar takes the sum and tensors indexed by the function index alone)

def biased_tanh_expr(I: int, K: int, dtype: str) -> ExprSpec:
    """f_i = tanh(b_i + sum_k x_ik w_k): the bias is read by the outer function, once per i."""
    return ExprSpec("program", (I,), [(0, K - 1)],
                    [ArgSpec("x", (I, K), [[1, 0], [0, 1]]), ArgSpec("w", (K,), [[0, 1]]), ArgSpec("b", (I,), [[1, 0]])],
                    dtype, [("arg", 0), ("arg", 1), ("mul",)], [("arg", 2), ("sum",), ("add",), ("tanh",)])


def dense_layer_expr(I: int, J: int, K: int, dtype: str) -> ExprSpec:
    """f_ij = tanh(b_j + sum_k x_ik w_kj): a dense layer; the gradient of the bias sums over the batch index i."""
    return ExprSpec("program", (I, J), [(0, K - 1)],
                    [ArgSpec("x", (I, K), [[1, 0, 0], [0, 0, 1]]), ArgSpec("w", (K, J), [[0, 0, 1], [0, 1, 0]]),
                     ArgSpec("b", (J,), [[0, 1, 0]])], dtype,
                    [("arg", 0), ("arg", 1), ("mul",)], [("arg", 2), ("sum",), ("add",), ("tanh",)])


def biased_causal_conv_expr(N: int, K: int, dtype: str) -> ExprSpec:
    """f_i = b_i * exp(-(sum_{k <= min(i, K-1)} x_{i-k} w_k)^2): a range that depends on i and an outer operand."""
    return ExprSpec("program", (N,), [(0, K - 1)],
                    [ArgSpec("x", (N,), [[1, -1]]), ArgSpec("w", (K,), [[0, 1]]), ArgSpec("b", (N + 2,), [[1, 0]])], dtype,
                    [("arg", 0), ("arg", 1), ("mul",)], [("arg", 2), ("sum",), ("powi", 2), ("neg",), ("exp",), ("mul",)],
                    constraints=[([1, -1], 0)])


def gated_gauss_expr(I: int, J: int, K: int, dtype: str) -> ExprSpec:
    """f_ij = x_i / (1 + y_j0^2) * exp(-sum_k (x_i + y_jk)^2): x is read inside the sum and by the outer function,
    and so is y through a second occurrence that ignores k."""
    return ExprSpec("program", (I, J), [(0, K - 1)],
                    [ArgSpec("x", (I,), [[1, 0, 0]]), ArgSpec("y", (J, K), [[0, 1, 0], [0, 0, 1]]),
                     ArgSpec("y_first", (J, K), [[0, 1, 0], [0, 0, 0]], same_as=1)], dtype,
                    [("arg", 0), ("arg", 1), ("add",), ("powi", 2)],
                    [("arg", 0), ("const", 1.0), ("arg", 2), ("powi", 2), ("add",), ("div",),
                     ("sum",), ("neg",), ("exp",), ("mul",)])


# Summation ranges that depend on other indices (Sec. 5.2; the form derived expressions have, Sec. 5.3)

def cumulative_sum_expr(N: int, dtype: str, body: str = "exp") -> ExprSpec:
    """f_i = phi(sum_{k <= i} x_k), extended index (i, k) with the condition i - k >= 0."""
    return ExprSpec(body, (N,), [(0, N - 1)], [ArgSpec("x", (N,), [[0, 1]])], dtype,
                    constraints=[([1, -1], 0)])


def causal_convolution_expr(N: int, K: int, dtype: str) -> ExprSpec:
    """f_i = sum_{k <= min(i, K-1)} x_{i-k} w_k, extended index (i, k) with the condition i - k >= 0."""
    return ExprSpec("mul", (N,), [(0, K - 1)],
                    [ArgSpec("x", (N,), [[1, -1]]), ArgSpec("w", (K,), [[0, 1]])], dtype,
                    constraints=[([1, -1], 0)])


def triangular_matmul_expr(I: int, N: int, dtype: str) -> ExprSpec:
    """f_ij = sum_{k <= j} x_ik y_kj (product with an upper triangular matrix), extended index (i, j, k)."""
    return ExprSpec("mul", (I, N), [(0, N - 1)],
                    [ArgSpec("x", (I, N), [[1, 0, 0], [0, 0, 1]]), ArgSpec("y", (N, N), [[0, 0, 1], [0, 1, 0]])], dtype,
                    constraints=[([0, 1, -1], 0)])


def band_expr(N: int, W: int, dtype: str) -> ExprSpec:
    """f_i = tanh(sum_{i <= k <= i + W} x_k w_{k - i}): two conditions, a window that moves with i."""
    return ExprSpec("tanh_dot", (N,), [(0, N - 1)],
                    [ArgSpec("x", (N,), [[0, 1]]), ArgSpec("w", (W + 1,), [[-1, 1]])], dtype,
                    constraints=[([-1, 1], 0), ([1, -1], W)])


def random_expr(seed: int, dtype: str = "f64", long_index: bool = False) -> ExprSpec:
    """A seeded random expression: 1..3 function indices, 0..2 summation indices (at most 4 together), one or two
    operands of rank 1..3 with small non-negative index coefficients, sometimes a negative one made safe by a
    condition, operand shapes with some slack beyond the referenced range.  Every index has 2..5 values; with
    long_index one of them, chosen at random, has 1100..2600 (gradients or function elements with long sums)."""
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + (9000 if long_index else 5000) + seed))
    n_f = int(rng.integers(1, 4))
    n_sum = int(rng.integers(0, min(2, 4 - n_f) + 1))
    D = n_f + n_sum
    ext = [int(rng.integers(2, 6)) for _ in range(D)]
    long_at = -1
    if long_index:
        long_at = int(rng.integers(0, D))
        ext[long_at] = int(rng.integers(1100, 2601))
    sums = []
    for q in range(n_sum):
        lo = int(rng.integers(0, 2))
        sums.append((lo, lo + ext[n_f + q] - 1))
    hi = [ext[d] - 1 for d in range(n_f)] + [h for _, h in sums]
    lo = [0] * n_f + [l for l, _ in sums]
    n_args = 1 if n_sum == 0 and rng.random() < 0.5 else int(rng.integers(1, 3))
    constraints = []
    args = []
    for p in range(n_args):
        rank = int(rng.integers(1, 4))
        A = [[int(rng.choice([0, 0, 0, 1, 1, 2, 3])) for _ in range(D)] for _ in range(rank)]
        if not any(any(row) for row in A):
            A[0][int(rng.integers(0, D))] = 1
        if D >= 2 and not constraints and rng.random() < 0.3:
            # x_{.. + i - k ..}: a negative coefficient, kept inside the tensor by the condition i - k >= 0
            i, k = (int(v) for v in rng.choice(D, 2, replace=False))
            r = int(rng.integers(0, rank))
            A[r] = [0] * D
            A[r][i], A[r][k] = 1, -1
            cond = [0] * D
            cond[i], cond[k] = 1, -1
            constraints.append((cond, 0))
        if long_at >= 0:
            # the long index in one row of an operand only, so that no tensor grows with its square
            rows_with = [r for r in range(rank) if A[r][long_at] != 0]
            for r in rows_with[1:]:
                A[r][long_at] = 0          # a row of zeros is a valid index map (that axis is read at 0)
        shape = tuple(max(1, sum(c * (hi[d] if c > 0 else lo[d]) for d, c in enumerate(row)) + 1) + int(rng.integers(0, 3))
                      for row in A)
        args.append(ArgSpec("xy"[p], shape, A))
    if n_args == 2:
        body = "mul" if rng.random() < 0.5 else "tanh_dot"
    else:
        body = str(rng.choice(["exp"] if n_sum else ["exp", "sq", "cube", "sin"]))
    return ExprSpec(body, tuple(ext[:n_f]), sums, args, dtype, constraints=constraints)


# A tensor that occurs more than once in an expression (Sec. 5.3: its gradient is the sum over the
# occurrences): the later occurrences are alias operands.

def matrix_square_expr(N: int, dtype: str) -> ExprSpec:
    """f_ij = sum_k x_ik x_kj, extended index (i, j, k)."""
    return ExprSpec("mul", (N, N), [(0, N - 1)],
                    [ArgSpec("x", (N, N), [[1, 0, 0], [0, 0, 1]]),
                     ArgSpec("x_again", (N, N), [[0, 0, 1], [0, 1, 0]], same_as=0)], dtype)


def symmetric_product_expr(N: int, M: int, dtype: str) -> ExprSpec:
    """f_ij = x_ij x_ji for i, j < N with x of shape M x M (M >= N), no summation."""
    return ExprSpec("mul", (N, N), [],
                    [ArgSpec("x", (M, M), [[1, 0], [0, 1]]),
                     ArgSpec("x_again", (M, M), [[0, 1], [1, 0]], same_as=0)], dtype)


def autocorrelation_expr(N: int, K: int, dtype: str) -> ExprSpec:
    """f_i = sum_{k<K} x_k x_{i+k}, i < N, x of length N + K - 1."""
    L = N + K - 1
    return ExprSpec("mul", (N,), [(0, K - 1)],
                    [ArgSpec("x", (L,), [[0, 1]]), ArgSpec("x_again", (L,), [[1, 1]], same_as=0)], dtype)


def worked_shared_expr(I: int, K: int, dtype: str) -> ExprSpec:
    """The worked expression with b = a:  f_ij = exp(-sum_k((a_ik + a_jk)^2 c_ii + d_{i+k}^3))."""
    e = worked_expr(I, I, K, dtype)
    e.args[1] = ArgSpec("a_again", e.args[1].shape, e.args[1].A, same_as=0)
    return e


def _worked_workload(name, seed, I, J, K, dtype, c_hi, d_half, d_len=None) -> Workload:
    rng = np.random.Generator(np.random.PCG64(seed))
    expr = worked_expr(I, J, K, dtype, d_len=d_len)
    a = _uniform(rng, -1, 1, (I, K))
    b = _uniform(rng, -1, 1, (J, K))
    c = _uniform(rng, 0, c_hi, (I, I))
    d = _uniform(rng, -d_half, d_half, expr.args[3].shape)
    df = _uniform(rng, -1, 1, (I, J))
    inputs = {"a": _round(a, dtype), "b": _round(b, dtype),
              "c": _round(c, dtype), "d": _round(d, dtype)}
    return Workload(name, expr, inputs, _round(df, dtype))


def config1() -> Workload:
    """Worked expression of the paper (Sec. 1 / Sec. 6) at I=8, J=6, K=5, fp64."""
    return _worked_workload("cfg1_worked_8x6x5_f64", SEED_BASE + 1, 8, 6, 5, "f64", 1.0, 0.5)


def config2(which: int, scale: str = "full") -> Workload:
    """The three index patterns of the introduction, fp32."""
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + 2 * 10 + which))
    dtype = "f32"
    if which == 1:
        I, J = (4096, 4096) if scale == "full" else (203, 516)
        expr = broadcast_sq_expr(I, J, dtype)
        x = _uniform(rng, -1, 1, (I,))
        df = _uniform(rng, -1, 1, (I, J))
        name = f"cfg2_1_broadcast_sq_{I}x{J}"
    elif which == 2:
        I = 8192 if scale == "full" else 388
        expr = diagonal_sq_expr(I, dtype)
        x = _uniform(rng, -1, 1, (I, I))
        df = _uniform(rng, -1, 1, (I,))
        name = f"cfg2_2_diagonal_sq_{I}"
    elif which == 3:
        I, J = (4096, 4096) if scale == "full" else (301, 468)
        expr = index_sum_exp_expr(I, J, dtype)
        x = _uniform(rng, -1, 1, (I + J - 1,))
        df = _uniform(rng, -1, 1, (I, J))
        name = f"cfg2_3_index_sum_exp_{I}x{J}"
    else:
        raise ValueError(which)
    return Workload(name, expr, {"x": _round(x, dtype)}, _round(df, dtype))


def config3(scale: str = "full") -> Workload:
    """Worked expression at scale, fp32, K=5 (memory bound)."""
    I, J = (8192, 8192) if scale == "full" else (333, 1300)
    return _worked_workload(f"cfg3_worked_{I}x{J}x5_f32", SEED_BASE + 3, I, J, 5, "f32", 0.2, 0.5)


def config4(scale: str = "full") -> Workload:
    """Worked expression with a long summed index, fp32, K=256 (compute heavy)."""
    I, J, K = (4096, 4096, 256) if scale == "full" else (200, 328, 256)
    return _worked_workload(f"cfg4_worked_{I}x{J}x{K}_f32", SEED_BASE + 4, I, J, K, "f32",
                            1.0 / 256, 0.2)


def config5(scale: str = "full") -> Workload:
    """Strided (stride 2) 3x3 map, fp32."""
    N, I, J = (32, 128, 128) if scale == "full" else (3, 21, 37)
    dtype = "f32"
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + 5))
    expr = strided_tanh_expr(N, I, J, 3, 3, 2, dtype)
    x = _uniform(rng, -1, 1, expr.args[0].shape)
    w = _uniform(rng, -0.5, 0.5, (3, 3))
    df = _uniform(rng, -1, 1, (N, I, J))
    return Workload(f"cfg5_strided_tanh_{N}x{I}x{J}", expr,
                    {"x": _round(x, dtype), "w": _round(w, dtype)}, _round(df, dtype))


def all_configs(scale: str = "small") -> List[Workload]:
    out = [config1()]
    out += [config2(w, scale) for w in (1, 2, 3)]
    out += [config3(scale), config4(scale), config5(scale)]
    return out


# --------------------------------------------------------------------------
# generic random inputs for an arbitrary expression (used by property tests)
# --------------------------------------------------------------------------

def random_inputs(expr: ExprSpec, seed: int, lo: float = -1.0, hi: float = 1.0) -> Workload:
    rng = np.random.Generator(np.random.PCG64(seed))
    inputs = {a.name: _round(_uniform(rng, lo, hi, a.shape), expr.dtype) for a in expr.args
              if a.same_as is None}
    df = _round(_uniform(rng, -1, 1, expr.f_shape), expr.dtype)
    return Workload(f"random_{expr.body}_{seed}", expr, inputs, df)
