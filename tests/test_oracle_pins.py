"""Pins for the CPU oracle: closed forms, printed expressions, finite differences.

Every check compares the oracle's brute-force scatter with something fixed by
the paper or by mathematics, never with the oracle's own formula.
"""
import os
import re

import numpy as np
import pytest

import oracle
from paper_1711_01348_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RNG = np.random.default_rng(12345)


def _expr(body, f_shape, sums, args, dtype="f64"):
    return wl.ExprSpec(body, tuple(f_shape), list(sums),
                       [wl.ArgSpec(n, tuple(s), A) for n, s, A in args], dtype)


# ---------------------------------------------------------------- Sec. 1 closed forms

def test_intro_broadcast_square():
    # f_ij = x_i^2  ->  dx_i = sum_j df_ij 2 x_i          (Sec. 1)
    I, J = 7, 11
    e = wl.broadcast_sq_expr(I, J, "f64")
    x, df = RNG.uniform(-1, 1, I), RNG.uniform(-1, 1, (I, J))
    assert np.allclose(oracle.forward(e, [x]), np.repeat((x * x)[:, None], J, 1), rtol=0, atol=1e-15)
    (dx,) = oracle.backward(e, [x], df)
    assert np.allclose(dx, 2 * x * df.sum(1), rtol=1e-14, atol=1e-15)


def test_intro_diagonal_square():
    # f_i = x_ii^2  ->  dx_ij = delta_ij df_i 2 x_ii       (Sec. 1)
    I = 9
    e = wl.diagonal_sq_expr(I, "f64")
    x, df = RNG.uniform(-1, 1, (I, I)), RNG.uniform(-1, 1, I)
    assert np.allclose(oracle.forward(e, [x]), np.diag(x) ** 2, rtol=0, atol=1e-15)
    (dx,) = oracle.backward(e, [x], df)
    assert np.array_equal(dx, np.diag(df * 2 * np.diag(x)))


def test_intro_index_sum_exp():
    # f_ij = exp x_{i+j}  ->  dx_k = sum_i df_{i,k-i} exp x_k   (Sec. 1)
    I, J = 6, 9
    e = wl.index_sum_exp_expr(I, J, "f64")
    x, df = RNG.uniform(-1, 1, I + J - 1), RNG.uniform(-1, 1, (I, J))
    f = oracle.forward(e, [x])
    assert np.allclose(f, np.exp(x[np.add.outer(np.arange(I), np.arange(J))]), rtol=1e-15)
    (dx,) = oracle.backward(e, [x], df)
    ref = np.array([sum(df[i, k - i] for i in range(I) if 0 <= k - i < J) * np.exp(x[k])
                    for k in range(I + J - 1)])
    assert np.allclose(dx, ref, rtol=1e-13, atol=1e-15)


# ---------------------------------------------------------------- Sec. 5 examples f^1 .. f^5

def test_sec5_f1_sin():
    N = 13
    e = _expr("sin", (N,), [], [("x", (N,), [[1]])])
    x, dg = RNG.uniform(-2, 2, N), RNG.uniform(-1, 1, N)
    (dx,) = oracle.backward(e, [x], dg)
    assert np.allclose(dx, dg * np.cos(x), rtol=1e-14)


def test_sec5_f2_product():
    # f_ij = x_i y_ij: dx_i = sum_j dg_ij y_ij, dy_ij = dg_ij x_i
    N = 6
    e = _expr("mul", (N, N), [], [("x", (N,), [[1, 0]]), ("y", (N, N), [[1, 0], [0, 1]])])
    x, y, dg = RNG.uniform(-1, 1, N), RNG.uniform(-1, 1, (N, N)), RNG.uniform(-1, 1, (N, N))
    assert np.allclose(oracle.forward(e, [x, y]), x[:, None] * y, rtol=1e-15)
    dx, dy = oracle.backward(e, [x, y], dg)
    assert np.allclose(dx, (dg * y).sum(1), rtol=1e-13)
    assert np.allclose(dy, dg * x[:, None], rtol=1e-15)


def test_sec5_f3_diagonal_cube():
    N = 5
    e = _expr("cube", (N,), [], [("x", (N, N), [[1], [1]])])
    x, dg = RNG.uniform(-1, 1, (N, N)), RNG.uniform(-1, 1, N)
    (dx,) = oracle.backward(e, [x], dg)
    assert np.allclose(dx, np.diag(dg * 3 * np.diag(x) ** 2), rtol=1e-14)


def test_sec5_f4_matmul_reduces_to_textbook():
    # f_ij = sum_k x_ik y_kj: dx = dg y^T, dy = x^T dg
    I, K, J = 5, 7, 4
    e = _expr("mul", (I, J), [(0, K - 1)],
              [("x", (I, K), [[1, 0, 0], [0, 0, 1]]), ("y", (K, J), [[0, 0, 1], [0, 1, 0]])])
    x, y, dg = RNG.uniform(-1, 1, (I, K)), RNG.uniform(-1, 1, (K, J)), RNG.uniform(-1, 1, (I, J))
    assert np.allclose(oracle.forward(e, [x, y]), x @ y, rtol=1e-13)
    dx, dy = oracle.backward(e, [x, y], dg)
    assert np.allclose(dx, dg @ y.T, rtol=1e-13, atol=1e-15)
    assert np.allclose(dy, x.T @ dg, rtol=1e-13, atol=1e-15)


def test_sec5_f5_linear_combination():
    # f_ij = exp x_{M i + j}: dx_i' = sum_i dg_{i, i'-M i} exp x_i'
    N, M = 4, 3
    e = _expr("exp", (N, M), [], [("x", (N * M,), [[M, 1]])])
    x, dg = RNG.uniform(-1, 1, N * M), RNG.uniform(-1, 1, (N, M))
    (dx,) = oracle.backward(e, [x], dg)
    assert np.allclose(dx, dg.reshape(-1) * np.exp(x), rtol=1e-14)


# ---------------------------------------------------------------- Sec. 6 printed derivatives

def _read_limits():
    lim, cond = {}, {}
    for line in open(os.path.join(GOLDEN, "worked_expression_limits.txt")):
        if line.startswith("#") or not line.strip():
            continue
        g, kind, *rest = line.split()
        if kind == "condition":
            cond[g] = rest[0]
        elif kind != "index":
            lim.setdefault(g, {})[kind] = (rest[0], rest[1])
    return lim, cond


def _lim(txt, m=0):
    mm = re.fullmatch(r"(max|min)\((-?\d+),m(-\d+)?\)", txt)
    if mm:
        other = m + int(mm.group(3) or 0)
        return (max if mm.group(1) == "max" else min)(int(mm.group(2)), other)
    return int(txt)


def test_printed_derivatives_of_worked_expression():
    """Gather-form expressions with the printed limits at the paper's shapes (3,4,5,8)."""
    lim, cond = _read_limits()
    assert cond["dc"] == "dc_0-dc_1=0"
    I, J, K = 3, 4, 5
    e = wl.worked_expr(I, J, K, "f64", d_len=8)
    w = wl.random_inputs(e, 99)
    a, b, c, d = w.arg_list()
    c = np.abs(c)
    df = w.df
    f = oracle.forward(e, [a, b, c, d])
    # forward against the definition typed out directly
    fref = np.array([[np.exp(-sum((a[i, k] + b[j, k]) ** 2 * c[i, i] + d[i + k] ** 3 for k in range(K)))
                      for j in range(J)] for i in range(I)])
    assert np.allclose(f, fref, rtol=1e-14)
    da, db, dc, dd = oracle.backward(e, [a, b, c, d], df)

    g = -(df * f)
    lo, hi = (_lim(t) for t in lim["da"]["z0"])
    assert (lo, hi) == (0, J - 1)
    ref = np.array([[sum(g[i, z] * c[i, i] * 2 * (a[i, k] + b[z, k]) for z in range(lo, hi + 1))
                     for k in range(K)] for i in range(I)])
    assert np.allclose(da, ref, rtol=1e-13, atol=1e-16)

    lo, hi = (_lim(t) for t in lim["db"]["z0"])
    assert (lo, hi) == (0, I - 1)
    ref = np.array([[sum(g[z, j] * c[z, z] * 2 * (a[z, k] + b[j, k]) for z in range(lo, hi + 1))
                     for k in range(K)] for j in range(J)])
    assert np.allclose(db, ref, rtol=1e-13, atol=1e-16)

    l1, h1 = (_lim(t) for t in lim["dc"]["z1"])
    l0, h0 = (_lim(t) for t in lim["dc"]["z0"])
    ref = np.zeros((I, I))
    for i in range(I):
        ref[i, i] = sum((a[i, z1] + b[z0, z1]) ** 2 * g[i, z0]
                        for z1 in range(l1, h1 + 1) for z0 in range(l0, h0 + 1))
    assert np.allclose(dc, ref, rtol=1e-13, atol=1e-16)
    assert np.count_nonzero(dc - np.diag(np.diag(dc))) == 0

    ref = np.zeros(8)
    for m in range(8):
        l1, h1 = _lim(lim["dd"]["z1"][0], m), _lim(lim["dd"]["z1"][1], m)
        l0, h0 = (_lim(t) for t in lim["dd"]["z0"])
        ref[m] = sum(g[m - z1, z0] * 3 * d[m] ** 2
                     for z1 in range(l1, h1 + 1) for z0 in range(l0, h0 + 1))
    assert np.allclose(dd, ref, rtol=1e-13, atol=1e-16)
    assert dd[7] == 0.0   # d_7 is never referenced: empty range max(0,5)..min(4,7)


# ---------------------------------------------------------------- numeric verification (Sec. 6)

def _loss(expr, args, df):
    return float((oracle.forward(expr, args) * df).sum())


def _fd_grad(expr, args, df, p, h=1e-6):
    x = args[p]
    out = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        idx = it.multi_index
        xp = [a.copy() for a in args]
        xm = [a.copy() for a in args]
        xp[p][idx] += h
        xm[p][idx] -= h
        out[idx] = (_loss(expr, xp, df) - _loss(expr, xm, df)) / (2 * h)
    return out


@pytest.mark.parametrize("make", [
    lambda: wl.config1().expr,
    lambda: wl.worked_expr(3, 4, 5, "f64", d_len=8),
    lambda: wl.strided_tanh_expr(2, 3, 4, 3, 3, 2, "f64"),
    lambda: wl.index_sum_exp_expr(4, 5, "f64"),
    lambda: _expr("exp", (3, 4), [], [("x", (20,), [[2, 4]])]),
    lambda: _expr("sq", (4, 3), [(0, 2)], [("x", (12,), [[2, 1, 1]])]),
])
def test_central_finite_differences(make):
    e = make()
    w = wl.random_inputs(e, 7)
    args = [np.asarray(a, dtype=np.float64) for a in w.arg_list()]
    grads = oracle.backward(e, args, w.df)
    for p, g in enumerate(grads):
        fd = _fd_grad(e, args, w.df, p)
        assert np.allclose(g, fd, rtol=2e-7, atol=2e-8), (e.body, p)


def _fd_grad_tensor(expr, args, df, p, h=1e-6):
    """Central differences with respect to the tensor of operand p: all its occurrences move together."""
    same = [q for q, a in enumerate(expr.args) if q == p or a.same_as == p]
    out = np.zeros_like(args[p])
    it = np.nditer(args[p], flags=["multi_index"])
    for _ in it:
        idx = it.multi_index
        xp = [a.copy() for a in args]
        xm = [a.copy() for a in args]
        for q in same:
            xp[q][idx] += h
            xm[q][idx] -= h
        out[idx] = (_loss(expr, xp, df) - _loss(expr, xm, df)) / (2 * h)
    return out


@pytest.mark.parametrize("make", [
    lambda: wl.matrix_square_expr(4, "f64"),
    lambda: wl.symmetric_product_expr(3, 4, "f64"),
    lambda: wl.autocorrelation_expr(5, 3, "f64"),
    lambda: wl.worked_shared_expr(3, 2, "f64"),
])
def test_repeated_tensor_matches_finite_differences(make):
    e = make()
    w = wl.random_inputs(e, 5)
    args = [np.asarray(a, dtype=np.float64) for a in w.arg_list()]
    grads = oracle.backward_by_tensor(e, args, w.df)
    for p, g in enumerate(grads):
        if e.args[p].same_as is not None:
            assert g is None
            continue
        fd = _fd_grad_tensor(e, args, w.df, p)
        assert np.allclose(g, fd, rtol=2e-7, atol=2e-8), (e.body, p)


def test_matrix_square_closed_form():
    """f = X X: dl/dX = df X^T + X^T df (textbook)."""
    e = wl.matrix_square_expr(6, "f64")
    w = wl.random_inputs(e, 9)
    X = np.asarray(w.arg_list()[0], dtype=np.float64)
    assert np.allclose(oracle.forward(e, [X, X]), X @ X, rtol=1e-13, atol=1e-14)
    g = oracle.backward_by_tensor(e, [X, X], w.df)[0]
    assert np.allclose(g, w.df @ X.T + X.T @ w.df, rtol=1e-12, atol=1e-13)


def test_jacobian_rows_by_one_hot_df():
    """One-hot df picks one row of the Jacobian (Sec. 5.3); compare with central differences of f."""
    e = wl.worked_expr(2, 3, 2, "f64")
    w = wl.random_inputs(e, 3)
    args = [np.asarray(a, dtype=np.float64) for a in w.arg_list()]
    h = 1e-6
    for i in range(2):
        for j in range(3):
            df = np.zeros((2, 3))
            df[i, j] = 1.0
            grads = oracle.backward(e, args, df)
            for p, g in enumerate(grads):
                it = np.nditer(args[p], flags=["multi_index"])
                for _ in it:
                    idx = it.multi_index
                    xp = [a.copy() for a in args]
                    xm = [a.copy() for a in args]
                    xp[p][idx] += h
                    xm[p][idx] -= h
                    fd = (oracle.forward(e, xp)[i, j] - oracle.forward(e, xm)[i, j]) / (2 * h)
                    assert abs(g[idx] - fd) <= 1e-7 * max(1.0, abs(fd))


def test_threads_do_not_change_the_result():
    w = wl.config5("small")
    args = w.arg_list()
    g1 = oracle.backward(w.expr, args, w.df, nthreads=1)
    g3 = oracle.backward(w.expr, args, w.df, nthreads=3)
    for x, y in zip(g1, g3):
        assert np.allclose(x, y, rtol=1e-13, atol=1e-14)


# ---------------------------------------------------------------- index sets

def _fig(name):
    out = {}
    for line in open(os.path.join(GOLDEN, "lattice_figures.txt")):
        if line.startswith(name + " "):
            _, key, *vals = line.split()
            out[key] = [int(v) for v in vals]
    return out


def test_gamma_fig1():
    g = _fig("fig1")
    a1lo, a1hi, a2lo, a2hi = g["box"]
    assert (a1lo, a2lo) == (0, 0)
    e = _expr("sq", (a1hi + 1, a2hi + 1), [], [("x", (1,), [g["A"]])])
    pts = oracle.gamma(e, 0, g["beta"])
    zlo, zhi = g["z"]
    expect = [(-1 + 2 * z, z) for z in range(zlo, zhi + 1)]   # I beta + K z
    assert [tuple(p) for p in pts] == expect


def test_gamma_fig2():
    g = _fig("fig2")
    a1lo, a1hi, a2lo, a2hi = g["box"]
    e = _expr("sq", (a1hi + 1, a2hi + 1), [(-30, 30)], [("x", (1,), [g["A"]])])
    pts = {tuple(p) for p in oracle.gamma(e, 0, g["beta"])}
    assert len(pts) == g["count"][0]
    K = np.array(g["K"]).reshape(2, 3).T
    expect = set()
    for z2 in range(-1, 6):
        for z1 in range(max(-1, -z2), min(1, 4 - z2) + 1):
            expect.add(tuple(np.array([3, 0, 0]) + K @ np.array([z1, z2])))
    assert pts == expect


def test_gamma_counts_match_per_beta_scan():
    e = wl.strided_tanh_expr(2, 3, 4, 3, 3, 2, "f64")
    for p, a in enumerate(e.args):
        counts = oracle.gamma_counts(e, p)
        for beta in np.ndindex(*a.shape):
            assert counts[beta] == len(oracle.gamma(e, p, beta))
        assert counts.sum() == np.prod(e.f_shape) * 9


# ---------------------------------------------------------------- scalar bodies given as programs

@pytest.mark.parametrize("make", [
    lambda: wl.config1(),
    lambda: wl.config2(1, "small"), lambda: wl.config2(2, "small"), lambda: wl.config2(3, "small"),
    lambda: wl.config5("small"),
    lambda: wl.random_inputs(wl.matmul_expr(5, 7, 6, "f64"), 3),
    lambda: wl.random_inputs(_expr("sin", (9,), [], [("x", (9,), [[1]])]), 4),
    lambda: wl.random_inputs(_expr("cube", (5,), [], [("x", (5, 5), [[1], [1]])]), 5),
], ids=["worked", "sq", "diag_sq", "exp", "tanh_dot", "mul", "sin", "cube"])
def test_program_body_equals_builtin_body(make):
    """The postfix interpreter and its dual-number derivatives reproduce every hand-written body
    (whose partial derivatives are pinned above by the paper's printed expressions and by differences)."""
    w = make()
    args = [np.asarray(a, dtype=np.float64) for a in w.arg_list()]
    ep = wl.as_program(w.expr)
    assert np.allclose(oracle.forward(ep, args), oracle.forward(w.expr, args), rtol=1e-14, atol=1e-15)
    for g, r in zip(oracle.backward(ep, args, w.df), oracle.backward(w.expr, args, w.df)):
        assert np.allclose(g, r, rtol=1e-13, atol=1e-14)


def test_program_body_finite_differences():
    """A body with no built-in twin (division, log, sqrt, cos, constants): oracle against central differences."""
    e = wl.softplus_ratio_expr(3, 4, 3, "f64")
    w = wl.random_inputs(e, 12)
    args = [np.asarray(a, dtype=np.float64) for a in w.arg_list()]
    grads = oracle.backward(e, args, w.df)
    for p, g in enumerate(grads):
        assert np.allclose(g, _fd_grad(e, args, w.df, p), rtol=2e-7, atol=2e-8), p


def test_program_body_closed_form():
    """f_i = log(1 + x_i^2): df/dx = 2x / (1 + x^2)."""
    e = wl.ExprSpec("program", (6,), [], [wl.ArgSpec("x", (6,), [[1]])], "f64",
                    [("arg", 0), ("powi", 2)], [("const", 1.0), ("sum",), ("add",), ("log",)])
    x = np.linspace(-1.5, 2.0, 6)
    df = np.linspace(0.5, 1.5, 6)
    assert np.allclose(oracle.forward(e, [x]), np.log1p(x * x), rtol=1e-14)
    assert np.allclose(oracle.backward(e, [x], df)[0], df * 2 * x / (1 + x * x), rtol=1e-13)


def test_program_subtraction_closed_forms():
    """The subtraction rule of the interpreter, as the second operand of the inner function and in the outer one:
    f_i = sum_k (x_ik - y_k)^2 has d/dx = 2 (x - y) df_i and d/dy = -2 sum_i (x - y) df_i (the sign and the order of
    the operands both show); f_i = 3 - s_i with s_i = sum_k (x_ik - y_k) has d/dx = -df_i, d/dy = +sum_i df_i."""
    args = [wl.ArgSpec("x", (5, 4), [[1, 0], [0, 1]]), wl.ArgSpec("y", (4,), [[0, 1]])]
    rng = np.random.default_rng(31)
    x, y, df = rng.uniform(-1, 1, (5, 4)), rng.uniform(-1, 1, 4), rng.uniform(-1, 1, 5)
    sq = wl.ExprSpec("program", (5,), [(0, 3)], args, "f64",
                     [("arg", 0), ("arg", 1), ("sub",), ("powi", 2)], [("sum",)])
    diff = x - y[None, :]
    assert np.allclose(oracle.forward(sq, [x, y]), (diff ** 2).sum(axis=1), rtol=1e-14)
    dx, dy = oracle.backward(sq, [x, y], df)
    assert np.allclose(dx, 2 * diff * df[:, None], rtol=1e-13, atol=1e-15)
    assert np.allclose(dy, -2 * (diff * df[:, None]).sum(axis=0), rtol=1e-13, atol=1e-15)
    lin = wl.ExprSpec("program", (5,), [(0, 3)], args, "f64",
                      [("arg", 0), ("arg", 1), ("sub",)], [("const", 3.0), ("sum",), ("sub",)])
    assert np.allclose(oracle.forward(lin, [x, y]), 3.0 - diff.sum(axis=1), rtol=1e-14)
    dx, dy = oracle.backward(lin, [x, y], df)
    assert np.allclose(dx, -np.broadcast_to(df[:, None], (5, 4)), rtol=1e-14)
    assert np.allclose(dy, np.full(4, df.sum()), rtol=1e-13)


def test_program_temporaries_equal_the_written_out_program():
    """(x + y)^2 + sin(x + y) with x + y kept in a temporary, and the outer function u * exp(u) likewise, against
    the same programs with the shared part written twice; plus the closed form of the forward value."""
    args = [wl.ArgSpec("x", (5, 3), [[1, 0], [0, 1]]), wl.ArgSpec("y", (3,), [[0, 1]])]
    xy = [("arg", 0), ("arg", 1), ("add",)]
    shared = wl.ExprSpec("program", (5,), [(0, 2)], args, "f64",
                         xy + [("store", 3), ("powi", 2), ("load", 3), ("sin",), ("add",)],
                         [("sum",), ("const", 0.25), ("mul",), ("store", 0), ("load", 0), ("exp",), ("mul",)])
    written = wl.ExprSpec("program", (5,), [(0, 2)], args, "f64",
                          xy + [("powi", 2)] + xy + [("sin",), ("add",)],
                          [("sum",), ("const", 0.25), ("mul",), ("sum",), ("const", 0.25), ("mul",), ("exp",), ("mul",)])
    w = wl.random_inputs(written, 21)
    xs = w.arg_list()
    f = oracle.forward(shared, xs)
    u = 0.25 * ((xs[0] + xs[1]) ** 2 + np.sin(xs[0] + xs[1])).sum(axis=1)
    assert np.allclose(f, u * np.exp(u), rtol=1e-14)
    assert np.array_equal(f, oracle.forward(written, xs))
    for g, r in zip(oracle.backward(shared, xs, w.df), oracle.backward(written, xs, w.df)):
        assert np.allclose(g, r, rtol=1e-14, atol=1e-16)
    shared.inner = [("load", 3)] + shared.inner          # read before anything was stored
    with pytest.raises(RuntimeError):
        f = oracle.forward(shared, xs)
        if np.isnan(f).all():
            raise RuntimeError("malformed program")


# ---------------------------------------------------------------- operands of the outer function (Sec. 5.2)

def test_outer_operand_closed_form():
    """f_i = tanh(b_i + sum_k x_ik w_k): a dense layer; textbook gradients."""
    e = wl.biased_tanh_expr(5, 4, "f64")
    rng = np.random.default_rng(8)
    x, w, b, df = rng.uniform(-1, 1, (5, 4)), rng.uniform(-1, 1, 4), rng.uniform(-1, 1, 5), rng.uniform(-1, 1, 5)
    t = np.tanh(b + x @ w)
    assert np.allclose(oracle.forward(e, [x, w, b]), t, rtol=1e-14)
    g = df * (1 - t * t)
    dx, dw, db = oracle.backward(e, [x, w, b], df)
    assert np.allclose(dx, np.outer(g, w), rtol=1e-13, atol=1e-15)
    assert np.allclose(dw, g @ x, rtol=1e-13, atol=1e-15)
    assert np.allclose(db, g, rtol=1e-13, atol=1e-15)


def test_outer_operand_equals_the_factor_inside_the_sum():
    """x_i * sum_k y_ik, with x read by the outer function, is sum_k x_i y_ik."""
    args = [wl.ArgSpec("x", (6,), [[1, 0]]), wl.ArgSpec("y", (6, 3), [[1, 0], [0, 1]])]
    outside = wl.ExprSpec("program", (6,), [(0, 2)], args, "f64", [("arg", 1)], [("arg", 0), ("sum",), ("mul",)])
    inside = wl.ExprSpec("mul", (6,), [(0, 2)], args, "f64")
    w = wl.random_inputs(inside, 9)
    xs = w.arg_list()
    assert np.allclose(oracle.forward(outside, xs), oracle.forward(inside, xs), rtol=1e-14)
    for g, r in zip(oracle.backward(outside, xs, w.df), oracle.backward(inside, xs, w.df)):
        assert np.allclose(g, r, rtol=1e-13, atol=1e-15)


def test_outer_operand_finite_differences():
    """A tensor read inside the sum and by the outer function, one of them through a second occurrence."""
    e = wl.gated_gauss_expr(4, 3, 3, "f64")
    w = wl.random_inputs(e, 10, -0.8, 0.8)
    args = [np.asarray(a, dtype=np.float64) for a in w.arg_list()]
    grads = oracle.backward_by_tensor(e, args, w.df)
    for p in (0, 1):
        assert np.allclose(grads[p], _fd_grad_tensor(e, args, w.df, p), rtol=2e-7, atol=2e-8), p
    # an operand whose index moves with the summation index has no single value per function index
    e.outer[0] = ("arg", 1)
    with pytest.raises(RuntimeError):
        oracle.forward(e, args)


# ---------------------------------------------------------------- summation ranges that depend on other indices

def test_cumulative_sum_closed_form():
    """f_i = exp(sum_{k<=i} x_k): df/dx_k = sum_{i>=k} df_i f_i (reverse cumulative sum)."""
    e = wl.cumulative_sum_expr(9, "f64")
    rng = np.random.default_rng(1)
    x, df = rng.uniform(-1, 1, 9), rng.uniform(-1, 1, 9)
    f = oracle.forward(e, [x])
    assert np.allclose(f, np.exp(np.cumsum(x)), rtol=1e-14)
    assert np.allclose(oracle.backward(e, [x], df)[0], np.cumsum((df * f)[::-1])[::-1], rtol=1e-13)


def test_causal_convolution_reduces_to_library_routine():
    e = wl.causal_convolution_expr(11, 4, "f64")
    rng = np.random.default_rng(2)
    x, w, df = rng.uniform(-1, 1, 11), rng.uniform(-1, 1, 4), rng.uniform(-1, 1, 11)
    assert np.allclose(oracle.forward(e, [x, w]), np.convolve(x, w)[:11], rtol=1e-13, atol=1e-14)
    dx, dw = oracle.backward(e, [x, w], df)
    assert np.allclose(dx, np.correlate(df, w, "full")[3:], rtol=1e-13, atol=1e-14)          # dx_m = sum_k df_{m+k} w_k
    assert np.allclose(dw, [np.dot(df[k:], x[:11 - k]) for k in range(4)], rtol=1e-13, atol=1e-14)


def test_triangular_matmul_closed_form():
    e = wl.triangular_matmul_expr(4, 6, "f64")
    rng = np.random.default_rng(3)
    x, y, df = rng.uniform(-1, 1, (4, 6)), rng.uniform(-1, 1, (6, 6)), rng.uniform(-1, 1, (4, 6))
    yu = np.triu(y)
    assert np.allclose(oracle.forward(e, [x, y]), x @ yu, rtol=1e-13, atol=1e-14)
    dx, dy = oracle.backward(e, [x, y], df)
    assert np.allclose(dx, df @ yu.T, rtol=1e-13, atol=1e-14)
    assert np.allclose(dy, np.triu(x.T @ df), rtol=1e-13, atol=1e-14)
    assert np.all(np.tril(dy, -1) == 0)


def test_moving_window_finite_differences():
    e = wl.band_expr(8, 2, "f64")
    w = wl.random_inputs(e, 6)
    args = [np.asarray(a, dtype=np.float64) for a in w.arg_list()]
    for p, g in enumerate(oracle.backward(e, args, w.df)):
        assert np.allclose(g, _fd_grad(e, args, w.df, p), rtol=2e-7, atol=2e-8), p


# ---------------------------------------------------------------- the rounding bound used for long sums

def test_rounding_bound_covers_another_summation_order_and_stays_small():
    """The element-wise bound for long sums (rounding_bound.py) against a second evaluation that adds in another
    order (numpy's pairwise / blocked sums): every difference lies below the bound, the bound itself stays a
    modest multiple of n * 2^-53 * sum|term|, and it grows with the number of terms."""
    import rounding_bound
    worst = []
    for K in (300, 2400):
        e = wl.matmul_expr(7, 5, K, "f64")
        w = wl.random_inputs(e, 61)
        x, y = w.arg_list()
        bound_f, (bound_x, bound_y) = rounding_bound.bounds(e, [x, y], w.df)
        f = oracle.forward(e, [x, y])
        dx, dy = oracle.backward(e, [x, y], w.df)
        assert np.all(np.abs(f - x @ y) <= bound_f)
        assert np.all(np.abs(dx - w.df @ y.T) <= bound_x) and np.all(np.abs(dy - x.T @ w.df) <= bound_y)
        mags = np.abs(x) @ np.abs(y)
        assert np.all(bound_f <= 2.1 * (K + 2) * 2.0 ** -53 * mags)
        worst.append(float(bound_f.max()))
    assert worst[1] > 10 * worst[0]
    # exp of a cumulative sum: the bound follows the magnification by the outer function
    e = wl.cumulative_sum_expr(900, "f64")
    w = wl.random_inputs(e, 62)
    (x,) = w.arg_list()
    bound_f, (bound_x,) = rounding_bound.bounds(e, [x], w.df)
    f = oracle.forward(e, [x])
    ref = np.exp(np.cumsum(x))
    assert np.all(np.abs(f - ref) <= bound_f) and np.all(bound_f <= 1e-10 * ref)
    dx = oracle.backward(e, [x], w.df)[0]
    assert np.all(np.abs(dx - np.cumsum((w.df * ref)[::-1])[::-1]) <= bound_x)
    # dense layer, matrix form of the same bound
    e = wl.dense_layer_expr(6, 5, 700, "f64")
    w = wl.random_inputs(e, 63)
    x, wt, b = w.arg_list()
    bound_f, bound_g = rounding_bound.dense_layer_bounds("f64", x, wt, b, w.df)
    t = np.tanh(b + x @ wt)
    g = w.df * (1 - t * t)
    assert np.all(np.abs(oracle.forward(e, [x, wt, b]) - t) <= bound_f)
    for got, ref, bd in zip(oracle.backward(e, [x, wt, b], w.df), (g @ wt.T, x.T @ g, g.sum(axis=0)), bound_g):
        assert np.all(np.abs(got - ref) <= bd)
