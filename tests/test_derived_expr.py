"""A gradient written out as an element-wise defined tensor of its own (Sec. 5.3: derived expressions have the
form of the input again, so they can be evaluated and differentiated once more).  Host logic only, no GPU:
the emitted expression is checked term by term against the brute-force scan of the original expression, and
its values, computed by a few lines of numpy here, against the oracle's scatter gradient of the original.
For the second level an expression that has passed this check takes the place of the original."""
import itertools
import math

import numpy as np
import pytest

import oracle
from paper_1711_01348_amd import binding as B
from paper_1711_01348_amd import workloads as wl


def _expr(body, f_shape, sums, args, dtype="f64", **kw):
    return wl.ExprSpec(body, tuple(f_shape), list(sums), [wl.ArgSpec(n, tuple(s), A) for n, s, A in args], dtype, **kw)


def _slots(e):
    """(tensor operand, occurrence number, operand slot) of every occurrence."""
    out = []
    for p, a in enumerate(e.args):
        root = p if a.same_as is None else a.same_as
        out.append((root, sum(1 for r, _, _ in out if r == root), p))
    return out


def _ext_points(spec, beta):
    """Extended indices [beta z] of the terms of `spec` at function index beta."""
    for z in itertools.product(*[range(lo, hi + 1) for lo, hi in spec.sums]):
        ext = list(beta) + list(z)
        if all(sum(c * v for c, v in zip(coef, ext)) + const >= 0 for coef, const in spec.constraints):
            yield ext


def _terms_of(spec, beta):
    """Per term: the index tuple of every operand (operand 0 is df)."""
    out = []
    for ext in _ext_points(spec, beta):
        t = tuple(tuple(sum(a * v for a, v in zip(row, ext)) for row in arg.A) for arg in spec.args)
        for idx, arg in zip(t, spec.args):
            assert all(0 <= i < n for i, n in zip(idx, arg.shape)), (beta, ext, arg.name, idx)
        out.append(t)
    return sorted(out)


def _terms_brute(e, slot, beta, operands):
    """The same from the scan of the original box: function index and the indices of the kept operands."""
    nf = len(e.f_shape)
    out = []
    for x in oracle.gamma(e, slot, beta):
        t = [tuple(int(v) for v in x[:nf])]
        for q in operands[1:]:
            t.append(tuple(int(np.dot(row, x)) for row in e.args[q].A))
        out.append(tuple(t))
    return sorted(out)


def _run_postfix(prog, values, total=0.0):
    st, tmp = [], {}
    una = {"neg": lambda a: -a, "exp": math.exp, "log": math.log, "sin": math.sin, "cos": math.cos,
           "tanh": math.tanh, "sqrt": math.sqrt}
    for t in prog:
        if t[0] == "const": st.append(float(t[1]))
        elif t[0] == "arg": st.append(values[t[1]])
        elif t[0] == "sum": st.append(total)
        elif t[0] == "powi": st.append(st.pop() ** t[1])
        elif t[0] == "store": tmp[t[1]] = st[-1]
        elif t[0] == "load": st.append(tmp[t[1]])
        elif t[0] in una: st.append(una[t[0]](st.pop()))
        else:
            b, a = st.pop(), st.pop()
            st.append({"add": a + b, "sub": a - b, "mul": a * b, "div": a / b if t[0] == "div" else 0.0}[t[0]])
    assert len(st) == 1
    return st[0]


def _evaluate(spec, tensors):
    """f of a program expression by its definition (the outer function may read operands at the function index)."""
    f = np.zeros(spec.f_shape)
    nf = len(spec.f_shape)
    reads = {t[1] for t in spec.outer if t[0] == "arg"}
    for beta in itertools.product(*[range(n) for n in spec.f_shape]):
        s = 0.0
        for ext in _ext_points(spec, beta):
            vals = [t[tuple(sum(a * v for a, v in zip(row, ext)) for row in arg.A)] for t, arg in zip(tensors, spec.args)]
            s += _run_postfix(spec.inner, vals)
        at = [tensors[p][tuple(sum(a * v for a, v in zip(row[:nf], beta)) for row in arg.A)] if p in reads else None
              for p, arg in enumerate(spec.args)]
        f[beta] = _run_postfix(spec.outer, at, s)
    return f


def _nonlinear(I, J, K):
    """f_ij = sum_k exp(x_ik) sqrt(y_kj^2 + 1) / (2 + cos(z_{i+k})): the inner function of a body without a
    built-in twin, summed without an outer function."""
    e = wl.softplus_ratio_expr(I, J, K, "f64")
    e.outer = [("sum",)]
    return e


def _triple(N):
    """f_i = sum_{j <= i} x_j x_{i-j} x_i: one tensor three times, a range that depends on i."""
    return wl.ExprSpec("program", (N,), [(0, N - 1)],
                       [wl.ArgSpec("x", (N,), [[0, 1]]), wl.ArgSpec("x2", (N,), [[1, -1]], same_as=0),
                        wl.ArgSpec("x3", (N,), [[1, 0]], same_as=0)], "f64",
                       inner=[("arg", 0), ("arg", 1), ("mul",), ("arg", 2), ("mul",)], outer=[("sum",)],
                       constraints=[([1, -1], 0)])


def _status(fn):
    try:
        fn()
    except B.TadError as e:
        return e.status
    return 0


CASES = [
    ("matmul", lambda: wl.matmul_expr(3, 4, 5, "f64")),
    ("matmul_transposed", lambda: wl.matmul_expr(4, 3, 2, "f64", True, True, True)),
    ("broadcast_sq", lambda: wl.broadcast_sq_expr(4, 5, "f64")),
    ("diagonal_cube", lambda: _expr("cube", (4,), [], [("x", (4, 6), [[1], [1]])])),          # cokernel condition
    ("antidiagonal", lambda: _expr("mul", (6, 5), [], [("x", (10,), [[1, 1]]), ("y", (6,), [[1, 0]])])),
    ("plane", lambda: _expr("sin", (3, 3, 2), [], [("x", (12,), [[1, 2, 3]])])),               # kernel dimension 2
    ("skew_plane", lambda: _expr("mul", (4, 3), [(0, 2)], [("x", (9, 3), [[2, 1, 0], [0, 0, 1]]),
                                                           ("y", (6,), [[1, 0, 1]])])),
    ("causal_conv", lambda: wl.causal_convolution_expr(9, 4, "f64")),
    ("triangular", lambda: wl.triangular_matmul_expr(3, 5, "f64")),
    ("skew_condition", lambda: wl.ExprSpec("mul", (5, 6), [(0, 3)],
                                           [wl.ArgSpec("x", (5, 4), [[1, 0, 0], [0, 0, 1]]),
                                            wl.ArgSpec("y", (12,), [[0, 1, 2]])], "f64",
                                           constraints=[([2, 1, -3], -1)])),
    ("matrix_square", lambda: wl.matrix_square_expr(4, "f64")),
    ("symmetric_product", lambda: wl.symmetric_product_expr(3, 5, "f64")),
    ("autocorrelation", lambda: wl.autocorrelation_expr(6, 3, "f64")),
    ("nonlinear", lambda: _nonlinear(3, 4, 2)),
    ("triple", lambda: _triple(6)),
    # Smith divisors above one: divisibility masks
    ("stride2", lambda: _expr("sq", (4,), [], [("x", (9,), [[2]])])),
    ("stride2_broadcast", lambda: _expr("cube", (4, 3), [], [("x", (8,), [[2, 0]])])),
    ("stride_2_4", lambda: _expr("sin", (4, 3), [], [("x", (16,), [[2, 4]])])),
    ("stride_mixed_sum", lambda: _expr("mul", (3, 4), [(0, 2)], [("x", (7, 9), [[2, 0, 1], [0, 2, 1]]),
                                                                   ("y", (3,), [[0, 0, 1]])])),
    ("stride_3_1", lambda: _expr("exp", (4, 3), [], [("x", (12,), [[3, 1]])])),
    # outer functions other than the identity: the gradient is a seed expression followed by a derived one
    ("worked", lambda: wl.worked_expr(3, 4, 2, "f64")),
    ("worked_shared", lambda: wl.worked_shared_expr(3, 2, "f64")),
    ("cumsum_exp", lambda: wl.cumulative_sum_expr(5, "f64")),
    ("tanh_stencil", lambda: wl.strided_tanh_expr(1, 3, 3, 2, 2, 1, "f64")),
    ("softplus", lambda: wl.softplus_ratio_expr(3, 2, 2, "f64")),
    # the outer function reads operands: the gradient of such an operand has a second part
    ("biased_tanh", lambda: wl.biased_tanh_expr(4, 3, "f64")),
    ("gated_gauss", lambda: wl.gated_gauss_expr(3, 2, 2, "f64")),
    ("biased_causal_conv", lambda: wl.biased_causal_conv_expr(6, 3, "f64")),
]


def _check_against_original(e, depth, refused=None):
    """Every derived expression of `e` has exactly the terms of the brute-force scan, its values (with the seed
    expressions evaluated first where the outer function is not the identity) add up to the oracle's gradient,
    and (depth > 0) the same holds for the expressions derived from those.  Expressions the limits refuse at the
    lower level are recorded in `refused`."""
    plan = B.Plan(e)
    w = wl.random_inputs(e, 17 + depth, -0.9, 0.9)
    tensors = w.arg_list()
    want = oracle.backward(e, tensors, w.df)
    fused = not e.sums and not e.constraints
    nf = len(e.f_shape)
    seeds = {}

    def seed(which):
        if which not in seeds:
            sspec = plan.seed_expr(which)
            assert [a.name for a in sspec.args] == ["df"] + [a.name for a in e.args]
            seeds[which] = (sspec, _evaluate(sspec, [w.df] + tensors))
        return seeds[which][1]

    below = []
    for root, occ, slot in _slots(e):
        try:
            spec, operands = plan.derived_expr(root, occ)
        except B.TadError as err:
            assert err.status == -5 and refused is not None
            refused.append(slot)
            continue
        assert spec.args[0].shape == tuple(e.f_shape) and spec.f_shape == tuple(e.args[slot].shape)
        assert spec.outer == [("sum",)] and spec.inner[0] == ("arg", 0)
        identity = e.body == "mul" or (e.body == "program" and e.outer == [("sum",)])
        assert operands[0] == (-1 if identity or fused else -2)
        for beta in itertools.product(*[range(n) for n in spec.f_shape]):
            assert _terms_of(spec, beta) == _terms_brute(e, slot, beta, operands), (slot, beta)
        try:
            first = w.df if operands[0] == -1 else seed(-1)
            second = seed(slot) if plan.query(root, occ)["in_outer"] and not fused else None
        except B.TadError as err:
            assert err.status == -5 and refused is not None
            refused.append(("no seed", slot))
            continue
        got = _evaluate(spec, [first] + [tensors[q] for q in operands[1:]])
        parts = [spec]
        if plan.query(root, occ)["in_outer"] and not fused:
            spec1, operands1 = plan.derived_expr(root, occ, 1)
            assert operands1 == [-3 - slot] and spec1.inner == [("arg", 0)] and spec1.outer == [("sum",)]
            for beta in itertools.product(*[range(n) for n in spec1.f_shape]):
                brute = sorted((alpha,) for alpha in itertools.product(*[range(n) for n in e.f_shape])
                               if all(sum(a * v for a, v in zip(row[:nf], alpha)) == b
                                      for row, b in zip(e.args[slot].A, beta)))
                assert _terms_of(spec1, beta) == brute, (slot, beta)
            got = got + _evaluate(spec1, [second])
            parts.append(spec1)
        else:
            assert _status(lambda: plan.derived_expr(root, occ, 1)) == -1
        np.testing.assert_allclose(got, want[slot], rtol=1e-12, atol=1e-13)
        # occurrences of one tensor among the kept operands stay one tensor
        for q, a in enumerate(spec.args):
            if a.same_as is not None:
                r0 = lambda p: p if e.args[p].same_as is None else e.args[p].same_as
                assert r0(operands[q]) == r0(operands[a.same_as]) and spec.args[a.same_as].same_as is None
        for part in parts:
            # it is a valid expression again; if its own derivatives outgrow the device form, at least as a forward pass
            if _status(lambda: B.Plan(part)) != 0:
                assert _status(lambda: B.Plan(part)) == -5 and depth == 0
                B.Plan(part, needs_grad=[False] * len(part.args))
            if depth > 0:
                inner_refused = []
                _check_against_original(part, depth - 1, inner_refused)
                below.append((slot, inner_refused))
    if depth > 0:
        for which, (sspec, _) in sorted(seeds.items()):
            inner_refused = []
            _check_against_original(sspec, depth - 1, inner_refused)
            below.append(("seed", which, inner_refused))
        if refused is not None:
            refused.extend(below)


@pytest.mark.parametrize("name,make", CASES, ids=[c[0] for c in CASES])
def test_derived_expression_is_the_gradient(name, make):
    refused = []
    _check_against_original(make(), 1, refused)
    # nothing is refused at either level: shared sub-expressions are kept in temporaries, so even the second
    # derivatives of the body with divisions and square roots fit the program length
    assert all(entry[-1] == [] for entry in refused), refused


@pytest.mark.parametrize("seed", range(24))
def test_random_expressions_have_exact_derived_expressions(seed):
    refused = []
    _check_against_original(wl.random_expr(seed), 0, refused)
    assert refused == []


def test_scalar_part_is_df_times_the_symbolic_partial_derivative():
    e = _nonlinear(2, 2, 2)
    plan = B.Plan(e)
    rng = np.random.default_rng(5)
    for p in range(3):
        spec, operands = plan.derived_expr(p)
        dplan = B.Plan(spec)
        for _ in range(20):
            vals = rng.uniform(-1, 1, 3)
            g = rng.uniform(-1, 1)
            got = dplan.program_eval(-1, [g] + [vals[q] for q in operands[1:]])
            assert got == pytest.approx(g * plan.program_eval(p, vals), rel=1e-14, abs=1e-15)
    # d (x y) / d x = y: the factor 1 from the seed of the backward sweep is not written out
    spec, operands = B.Plan(wl.matmul_expr(2, 2, 2, "f64")).derived_expr(0)
    assert spec.inner == [("arg", 0), ("arg", 1), ("mul",)] and operands == [-1, 1]
    # a derivative that is the constant 1 leaves df alone: f_ij = sum_k (x_ik + y_kj)
    e = wl.matmul_expr(2, 3, 4, "f64")
    e = wl.ExprSpec("program", e.f_shape, e.sums, e.args, "f64", [("arg", 0), ("arg", 1), ("add",)], [("sum",)])
    spec, operands = B.Plan(e).derived_expr(1)
    assert spec.inner == [("arg", 0)] and operands == [-1] and len(spec.args) == 1


def test_product_programs_run_on_the_matrix_cores():
    """The derived expressions of a matrix product are matrix products again."""
    plan = B.Plan(wl.matmul_expr(8, 12, 16, "f32"))
    for p in range(2):
        spec, _ = plan.derived_expr(p)
        assert B.Plan(spec).forward_family == "contraction"
        assert B.Plan(spec, generic_only=True, keep_program=True).forward_family == "program"
        assert B.Plan(spec, generic_only=True).forward_family == "generic"      # recognised as the product body
    assert B.Plan(wl.as_program(wl.matmul_expr(8, 12, 16, "f32"))).forward_family == "contraction"
    assert B.Plan(wl.as_program(wl.matmul_expr(8, 12, 16, "f64")), keep_program=True).forward_family == "program"
    assert B.Plan(wl.as_program(wl.matmul_expr(8, 12, 16, "f64"))).forward_family == "generic"   # recognised as the product body


def test_derived_expression_rules():
    # an outer function puts a second, nested sum into the gradient: operand 0 is then the seed g, not df
    assert B.Plan(wl.config1().expr).derived_expr(0)[1][0] == -2
    assert B.Plan(wl.as_program(wl.config1().expr), keep_program=True).derived_expr(3)[1] == [-2, 3]
    assert B.Plan(wl.matmul_expr(2, 2, 2, "f64")).derived_expr(0)[1][0] == -1
    # without a summation outer(inner(x)) is one function: f_ij = x_i^2 needs no seed
    assert B.Plan(wl.broadcast_sq_expr(3, 4, "f64")).derived_expr(0)[1] == [-1, 0]
    plan = B.Plan(wl.biased_tanh_expr(3, 2, "f64"))
    assert [plan.query(p)["in_outer"] for p in range(3)] == [False, False, True]
    assert _status(lambda: plan.derived_expr(0, 0, 1)) == -1      # the outer function does not read x
    assert _status(lambda: plan.derived_expr(2, 0, 2)) == -1
    assert _status(lambda: plan.seed_expr(0)) == -1 and _status(lambda: plan.seed_expr(3)) == -1
    assert plan.seed_expr(2).outer[0] == ("arg", 0)
    # a Smith divisor above 1: the quotient becomes a summation index tied to beta by two conditions
    e = _expr("sq", (4,), [], [("x", (8,), [[2]])])
    spec, _ = B.Plan(e).derived_expr(0)
    assert spec.sums == [(0, 3)] and sorted(spec.constraints) == sorted([([1, -2], 0), ([-1, 2], 0)])
    plan = B.Plan(wl.matrix_square_expr(3, "f64"))
    assert _status(lambda: plan.derived_expr(1)) == -1           # an alias operand is reached through its tensor
    assert _status(lambda: plan.derived_expr(0, 2)) == -1
    assert _status(lambda: B.Plan(wl.matmul_expr(2, 2, 2, "f64"), needs_grad=[False, True]).derived_expr(0)) == -1
    # df would be an operand of rank 5
    e = _expr("sin", (2, 2, 2, 2, 2), [], [("x", (2, 2, 2, 4), [[1, 0, 0, 0, 0], [0, 1, 0, 0, 0], [0, 0, 1, 0, 0],
                                                                 [0, 0, 0, 1, 1]])])
    assert _status(lambda: B.Plan(e).derived_expr(0)) == -5
    # rank 4 with a cokernel row and a three-dimensional kernel: 4 + 3 indices are one too many
    e = _expr("mul", (2, 2, 2, 2), [(0, 1), (0, 1)],
              [("x", (2, 2, 2, 2), [[1, 0, 0, 0, 0, 0], [1, 0, 0, 0, 0, 0], [0, 1, 0, 0, 0, 0], [0, 0, 1, 0, 0, 0]]),
               ("y", (2, 2, 2), [[0, 0, 0, 1, 0, 0], [0, 0, 0, 0, 1, 0], [0, 0, 0, 0, 0, 1]])])
    assert _status(lambda: B.Plan(e).derived_expr(0)) == -5
    assert _status(lambda: B.Plan(e).derived_expr(1)) == 0


def test_gradient_graph_counts_and_misuse():
    """tad_derived_create on the host: how many seed expressions and parts the gradient of a tensor consists of."""
    from paper_1711_01348_amd import binding as B
    from paper_1711_01348_amd import workloads as wl
    cases = [
        # (expression, tensor, seeds, parts)
        (wl.matmul_expr(5, 4, 3, "f64"), 0, 0, 1),                       # outer function = the sum: no seed
        (wl.worked_expr(4, 5, 3, "f64"), 2, 1, 1),                        # exp(-s): g is a seed
        (wl.matrix_square_expr(6, "f64"), 0, 0, 2),                       # two occurrences, one part each
        (wl.dense_layer_expr(5, 4, 3, "f64"), 2, 1, 1),                   # bias: only read by the outer function ...
        (wl.gated_gauss_expr(4, 3, 2, "f64"), 0, 2, 2),                   # x inside the sum and outside: g and h, two parts
        (wl.broadcast_sq_expr(5, 6, "f64"), 0, 0, 1),                     # no sum, no condition: one fused function
    ]
    for e, arg, n_seeds, n_parts in cases:
        plan = B.Plan(e)
        dg = B.DerivedGradient(plan, arg)
        if e is cases[3][0]:
            # the bias does not occur inside the sum: part 0 sums an inner derivative that is identically zero
            assert dg.counts[1] in (1, 2)
        else:
            assert dg.counts == (n_seeds, n_parts), (e.body, arg, dg.counts)
        assert dg.workspace_bytes >= 0
    e = wl.matrix_square_expr(6, "f64")
    plan = B.Plan(e)
    with pytest.raises(B.TadError):
        B.DerivedGradient(plan, 1)          # an alias has no gradient of its own
    with pytest.raises(B.TadError):
        B.DerivedGradient(plan, 7)
    assert B.lib.tad_derived_workspace_bytes(None) == 0
    assert B.lib.tad_eval_derived(None, None, None, None, None, 0, None) == -1
