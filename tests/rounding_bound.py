"""Element-wise rounding-error bounds for long sums (test infrastructure).

Two correct evaluations of  f = outer(s),  s = sum_k t_k  in a floating-point format with unit roundoff u that add
the n terms in different orders differ in s by at most

    delta_s <= 2 (n + 1) u  sum_k |t_k|                                   (each side: gamma_n sum|t|, plus the products)

so the values of f differ by |outer'(s)| delta_s plus the evaluation error of the outer function, and a gradient
element  dx_beta = sum_z g_alpha D_alpha,  g = df outer'(s),  D = d inner / d x,  by

    (2 n_beta + 4) u  sum_z |g_alpha| |D_alpha|   +   sum_z |df_alpha| (|outer''(s_alpha)| delta_s_alpha + e2_alpha) |D_alpha|.

Every quantity on the right is a sum of magnitudes over the same index sets as the expression itself, so it is
obtained by running the CPU oracle on the magnitudes of the inputs with a linear body (the oracle supplies the index
structure; no value it returns for the expression under test enters the bound except through s and f).  The bounds
grow with the number of terms; nothing about the inputs is assumed.
"""
import numpy as np

import oracle
from paper_1711_01348_amd import workloads as wl

UNIT = {"f64": 2.0 ** -53, "f32": 2.0 ** -24}


def _linear_twin(e):
    """Same indices, ranges, conditions and operands; body sum_k x (one operand) or sum_k x y (two operands)."""
    if e.body in ("mul", "tanh_dot"):
        return wl.ExprSpec("mul", e.f_shape, list(e.sums), list(e.args), "f64", constraints=list(e.constraints))
    return wl.ExprSpec("program", e.f_shape, list(e.sums), list(e.args), "f64", [("arg", 0)], [("sum",)],
                       list(e.constraints))


def _outer_terms(body, s, u):
    """(|outer'|, |outer''|, evaluation slack of outer, evaluation slack of outer') at s."""
    if body == "exp":
        f = np.exp(s)
        return f, f, 8 * u * f, 8 * u * f
    if body == "sq":
        return 2 * np.abs(s), np.full_like(s, 2.0), 8 * u * s * s, 16 * u * np.abs(s)
    if body == "cube":
        return 3 * s * s, 6 * np.abs(s), 8 * u * np.abs(s) ** 3, 24 * u * s * s
    if body == "sin":
        return np.abs(np.cos(s)), np.abs(np.sin(s)), np.full_like(s, 8 * u), np.full_like(s, 8 * u)
    if body == "mul":
        return np.ones_like(s), np.zeros_like(s), 2 * u * np.abs(s), np.zeros_like(s)
    if body == "tanh_dot":
        t = np.tanh(s)
        return 1 - t * t, 2 * np.abs(t) * (1 - t * t), np.full_like(s, 8 * u), np.full_like(s, 16 * u)
    raise ValueError(body)


def bounds(e, args, df):
    """(bound on |f_a - f_b|, [bound on |dx_a - dx_b| per operand]) for two evaluations in e.dtype of an expression
    with one of the built-in bodies sq, cube, sin, exp, mul, tanh_dot."""
    u = UNIT[e.dtype]
    lin = _linear_twin(e)
    xs = [np.asarray(a, dtype=np.float64) for a in args]
    mags = [np.abs(x) for x in xs]
    ones = [np.ones_like(x) for x in xs]
    s = oracle.forward(lin, xs)
    mag_s = oracle.forward(lin, mags)
    n_terms = oracle.forward(lin, ones)
    ds = 2 * (n_terms + 1) * u * mag_s
    l1, l2, e1, e2 = _outer_terms(e.body, s, u)
    adf = np.abs(np.asarray(df, dtype=np.float64))
    bound_f = 1.01 * l1 * ds + e1
    t = oracle.backward(lin, mags, adf * l1, nthreads=8)
    n_beta = oracle.backward(lin, ones, np.ones_like(adf), nthreads=8)
    p = oracle.backward(lin, mags, adf * (1.01 * l2 * ds + e2), nthreads=8)
    return bound_f, [(2 * nb + 4) * u * tt + pp for tt, nb, pp in zip(t, n_beta, p)]


def dense_layer_bounds(dtype, x, w, b, df):
    """The same bounds for f_ij = tanh(b_j + sum_k x_ik w_kj), written out with matrix products of magnitudes."""
    u = UNIT[dtype]
    x, w, b, df = (np.asarray(v, dtype=np.float64) for v in (x, w, b, df))
    n = x.shape[1] + 1
    s = x @ w + b
    ds = 2 * (n + 1) * u * (np.abs(x) @ np.abs(w) + np.abs(b))
    l1, l2, e1, e2 = _outer_terms("tanh_dot", s, u)
    adf = np.abs(df)
    g, q = adf * l1, adf * (1.01 * l2 * ds + e2)
    I, J = s.shape
    return 1.01 * l1 * ds + e1, [(2 * J + 4) * u * (g @ np.abs(w).T) + q @ np.abs(w).T,
                                 (2 * I + 4) * u * (np.abs(x).T @ g) + np.abs(x).T @ q,
                                 (2 * I + 4) * u * g.sum(axis=0) + q.sum(axis=0)]
