"""GPU parity: HIP path (through the C ABI) against the fp64 CPU oracle, element by element."""
import numpy as np
import pytest

import oracle
import rounding_bound
from paper_1711_01348_amd import check
from paper_1711_01348_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _expr(body, f_shape, sums, args, dtype="f64"):
    return wl.ExprSpec(body, tuple(f_shape), list(sums),
                       [wl.ArgSpec(n, tuple(s), A) for n, s, A in args], dtype)


def _to_dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def run_gpu(w, generic_only=False, wanted=None, keep_program=True, term_lists=True):
    """keep_program: a body given as programs stays on the interpreter kernels even where it spells out a built-in
    body (most tests here give built-in bodies as programs precisely to exercise those kernels).
    term_lists=False: a small expression is not expanded into term lists at plan time; the device walks its ranges."""
    import torch
    from paper_1711_01348_amd import binding as B
    plan = B.Plan(w.expr, generic_only=generic_only, keep_program=keep_program, term_lists=term_lists)
    args = [_to_dev(a) for a in w.arg_list()]
    f = plan.forward(args)
    grads = plan.backward(args, f, _to_dev(w.df), wanted=wanted)
    torch.cuda.synchronize()
    return plan, f.cpu().numpy(), [None if g is None else g.cpu().numpy() for g in grads]


def assert_parity(w, f, grads, f_ref, g_ref, tag=""):
    dt = w.expr.dtype
    e = check.errors(f, f_ref)
    assert check.within(f, f_ref, dt), (w.name, tag, "f", e)
    for a, g, r in zip(w.expr.args, grads, g_ref):
        if g is None:
            continue
        e = check.errors(g, r)
        assert check.within(g, r, dt), (w.name, tag, "d" + a.name, e)
        # structural zeros (cokernel mask, unreferenced elements) must be exact zeros
        assert np.all(g[r == 0] == 0), (w.name, tag, "d" + a.name, "mask")


def assert_within_rounding_bounds(w, f, grads, f_ref, g_ref, bound_f, bound_g, tag=""):
    """Long sums: the element-wise difference stays below the bound that follows from the number of terms and the
    sum of their magnitudes (rounding_bound.py); returns the largest floored relative error seen, for the record."""
    worst = 0.0
    for what, got, ref, bound in [("f", f, f_ref, bound_f)] + [("d" + a.name, g, r, b) for a, g, r, b in
                                                                zip(w.expr.args, grads, g_ref, bound_g) if g is not None]:
        diff = np.abs(np.asarray(got, dtype=np.float64) - ref)
        assert np.all(np.isfinite(diff)), (w.name, tag, what, "not finite")
        over = diff > bound
        assert not over.any(), (w.name, tag, what, "difference", float(diff[over].max()), "bound", float(bound[over].min()),
                                check.errors(got, ref))
        assert np.all(np.asarray(got)[ref == 0] == 0), (w.name, tag, what, "mask")
        worst = max(worst, check.errors(got, ref)["floored"])
    return worst


def oracle_all(w, nthreads=8):
    args = w.arg_list()
    return oracle.forward(w.expr, args), oracle.backward_by_tensor(w.expr, args, w.df, nthreads=nthreads)


@pytest.mark.parametrize("generic_only", [True, False], ids=["generic", "selected"])
@pytest.mark.parametrize("w", wl.all_configs("small"), ids=lambda w: w.name)
def test_configs_small(w, generic_only):
    f_ref, g_ref = oracle_all(w)
    plan, f, grads = run_gpu(w, generic_only)
    assert_parity(w, f, grads, f_ref, g_ref, "generic" if generic_only else "selected")
    if plan.query(0)["listed"]:   # small enough for term lists: also with the ranges walked on the device
        plan, f, grads = run_gpu(w, generic_only, term_lists=False)
        assert not plan.query(0)["listed"]
        assert_parity(w, f, grads, f_ref, g_ref, "ranges walked on the device")


EXPECTED_FAMILY = {"cfg1": "generic", "cfg2_1": "row_reduce", "cfg2_2": "diagonal", "cfg2_3": "antidiagonal",
                   "cfg3": "worked", "cfg4": "worked_mfma", "cfg5": "strided"}


@pytest.mark.parametrize("w", wl.all_configs("small") + [wl.config3(), wl.config4(), wl.config5()],
                         ids=lambda w: w.name)
def test_selected_kernel_family(w):
    """The benchmark configurations must run on their specialised kernels, not on the generic fallback."""
    from paper_1711_01348_amd import binding as B
    plan = B.Plan(w.expr)
    key = next(k for k in sorted(EXPECTED_FAMILY, key=len, reverse=True) if w.name.startswith(k))
    assert plan.forward_family == EXPECTED_FAMILY[key], w.name
    for p in range(len(w.expr.args)):
        assert plan.query(p)["family"] == EXPECTED_FAMILY[key], (w.name, p)
    assert B.Plan(w.expr, generic_only=True).forward_family == "generic"


@pytest.mark.parametrize("term_lists", [True, False], ids=["terms listed", "ranges walked"])
def test_config1_fp64_tight(term_lists):
    w = wl.config1()
    f_ref, g_ref = oracle_all(w, 1)
    plan, f, grads = run_gpu(w, term_lists=term_lists)
    assert [plan.query(p)["listed"] for p in range(4)] == [term_lists] * 4
    for got, ref in [(f, f_ref)] + list(zip(grads, g_ref)):
        e = check.errors(got, ref)
        assert e["floored"] <= 1e-12 and e["raw"] <= 1e-12, e   # the plain element-wise relative error holds here too
    dc = grads[2]
    assert np.count_nonzero(dc - np.diag(np.diag(dc))) == 0


def _padded_strided(N, I, J, U, V, stride, more_rows, more_cols):
    """The strided map with an x that is larger than the range the map reaches: the gradient there is exactly zero."""
    e = wl.strided_tanh_expr(N, I, J, U, V, stride, "f32")
    x = e.args[0]
    e.args[0] = wl.ArgSpec(x.name, (x.shape[0], x.shape[1] + more_rows, x.shape[2] + more_cols), x.A)
    return e


ASSORTED = [
    lambda: _expr("sin", (13,), [], [("x", (13,), [[1]])]),
    lambda: _expr("cube", (5,), [], [("x", (5, 5), [[1], [1]])]),
    lambda: _expr("mul", (6, 6), [], [("x", (6,), [[1, 0]]), ("y", (6, 6), [[1, 0], [0, 1]])]),
    lambda: _expr("mul", (37, 29), [(0, 40)], [("x", (37, 41), [[1, 0, 0], [0, 0, 1]]),
                                              ("y", (41, 29), [[0, 0, 1], [0, 1, 0]])]),
    lambda: _expr("exp", (5,), [], [("x", (9,), [[2]])]),
    lambda: _expr("exp", (5, 4), [], [("x", (9,), [[2, 0]])]),
    lambda: _expr("exp", (4, 3), [], [("x", (20,), [[2, 4]])]),
    lambda: _expr("exp", (4, 3), [], [("x", (12,), [[3, 1]])]),
    lambda: _expr("exp", (3, 4), [(0, 2)], [("x", (7, 9), [[2, 0, 1], [0, 2, 1]])]),
    lambda: _expr("exp", (3, 3, 3), [], [("x", (5, 5), [[1, 1, 0], [0, 1, 1]])]),
    lambda: _expr("exp", (6,), [(0, 3), (0, 2)], [("x", (30,), [[3, 2, 4]])]),
    # masks that leave few elements: the kernels run over the transformed index y instead of over all beta
    # (a stride of 5; a diagonal with stride 3 in a matrix with room to spare; a sum that reaches the same element
    # of a strided diagonal several times)
    lambda: _expr("sq", (40,), [], [("x", (300,), [[5]])]),
    lambda: _expr("exp", (9,), [], [("x", (31, 40), [[3], [3]])], "f32"),
    lambda: _expr("exp", (7, 4), [(0, 2)], [("x", (50, 60), [[4, 0, 2], [4, 0, 2]])]),
    lambda: wl.worked_expr(4, 3, 5, "f64", d_len=11, c_shape=(6, 5)),
    lambda: wl.worked_expr(3, 4, 5, "f64", d_len=8),
    lambda: wl.worked_expr(70, 1301, 5, "f32"),          # row length not a multiple of 4: generic kernels
    lambda: wl.worked_expr(130, 520, 3, "f32", d_len=140, c_shape=(133, 131)),
    # pattern families with other bodies, arguments longer than the referenced range, ragged tiles
    lambda: _expr("sin", (70, 1028), [], [("x", (75,), [[1, 0]])], "f32"),
    lambda: _expr("cube", (259,), [], [("x", (263, 264), [[1], [1]])], "f32"),
    lambda: _expr("sq", (130, 260), [], [("x", (400,), [[1, 1]])], "f32"),
    lambda: _expr("exp", (65, 1032), [], [("x", (1096,), [[1, 1]])], "f32"),
    lambda: _expr("exp", (33, 517), [], [("x", (33,), [[1, 0]])], "f32"),        # not a multiple of 4: generic
    lambda: wl.strided_tanh_expr(3, 19, 23, 5, 4, 3, "f32"),
    lambda: wl.strided_tanh_expr(2, 30, 41, 2, 2, 1, "f32"),
    lambda: wl.strided_tanh_expr(2, 5, 4, 2, 3, 3, "f64"),
    lambda: wl.strided_tanh_expr(2, 5, 130, 7, 7, 8, "f32"),     # 49 taps, stride 8: general range divisors
    lambda: wl.strided_tanh_expr(2, 9, 200, 3, 3, 2, "f32"),
    lambda: wl.strided_tanh_expr(1, 6, 70, 4, 5, 1, "f32"),      # stride 1: up to 20 terms per gradient element
    lambda: wl.strided_tanh_expr(1, 3, 4, 3, 3, 2, "f32"),       # one wavefront's worth of columns, one n
    lambda: wl.strided_tanh_expr(5, 40, 132, 3, 3, 1, "f32"),    # stride 1 under a 3 x 3 filter: three values per range
    lambda: wl.strided_tanh_expr(2, 70, 96, 2, 2, 3, "f32"),     # stride 3 under a 2 x 2 filter: rows and columns of x nobody reads
    lambda: _padded_strided(3, 33, 60, 3, 3, 2, 4, 7),           # x with rows and columns beyond the referenced range
    # few gradient elements with long sums: one block per element shares the z loops
    lambda: _expr("exp", (40, 3001), [], [("x", (40,), [[1, 0]])], "f32"),                 # one range, split in pieces
    lambda: _expr("exp", (7, 50, 61), [(0, 4)], [("x", (11,), [[1, 0, 0, 1]])], "f64"),     # three kernel coordinates
    lambda: wl.as_program(_expr("exp", (40, 3001), [], [("x", (40,), [[1, 0]])], "f32")),
    lambda: wl.as_program(wl.strided_tanh_expr(2, 40, 37, 3, 3, 2, "f64")),
    # a tensor that occurs twice: the gradient is the sum over both occurrences
    lambda: wl.matrix_square_expr(23, "f64"),
    lambda: wl.matrix_square_expr(67, "f32"),
    lambda: wl.symmetric_product_expr(19, 21, "f64"),
    lambda: wl.autocorrelation_expr(300, 17, "f32"),
    lambda: wl.worked_shared_expr(41, 5, "f32"),
    lambda: wl.worked_shared_expr(9, 3, "f64"),
]


@pytest.mark.parametrize("make", ASSORTED)
def test_assorted_index_maps_fp64(make):
    e = make()
    w = wl.random_inputs(e, 11, -0.9, 0.9)
    f_ref, g_ref = oracle_all(w, 1)
    plan, f, grads = run_gpu(w)
    assert_parity(w, f, grads, f_ref, g_ref)
    if plan.query(0)["listed"]:
        _, f, grads = run_gpu(w, term_lists=False)
        assert_parity(w, f, grads, f_ref, g_ref, "ranges walked on the device")


@pytest.mark.parametrize("seed", range(40))
def test_random_expressions(seed):
    """Seeded random expressions (index matrices, ranks, summation ranges, conditions, bodies) on the plan-driven
    kernels, and the same expression with its body given as programs."""
    e = wl.random_expr(seed, "f64" if seed % 2 else "f32")
    w = wl.random_inputs(e, 100 + seed, -0.6, 0.6)
    f_ref, g_ref = oracle_all(w, 2)
    plan, f, grads = run_gpu(w)
    assert_parity(w, f, grads, f_ref, g_ref, "random %d" % seed)
    if plan.query(0)["listed"]:
        _, f, grads = run_gpu(w, term_lists=False)
        assert_parity(w, f, grads, f_ref, g_ref, "random %d, ranges walked on the device" % seed)
    wp = wl.Workload(w.name, wl.as_program(e), w.inputs, w.df)
    plan, f, grads = run_gpu(wp)
    assert plan.forward_family in ("program", "contraction")
    assert_parity(wp, f, grads, f_ref, g_ref, "random %d as program" % seed)


@pytest.mark.parametrize("seed", range(32))
def test_random_expressions_with_a_long_index(seed):
    """The same random expressions with one index of 1100..2600 values: gradients (or function elements) that sum
    thousands of terms, so that the plan-driven kernels lay their threads out in every way they know (one workgroup
    per element, several per element, one thread per element with shared sums, unmasked elements only).  fp32,
    values small enough that exp of the sum stays inside fp32."""
    e = wl.random_expr(seed, "f32", long_index=True)
    terms = int(np.prod([hi - lo + 1 for lo, hi in e.sums])) if e.sums else 1
    span = min(0.03, 2.0 / terms) if e.body == "exp" else 0.03     # exp of the sum must stay inside fp32
    w = wl.random_inputs(e, 300 + seed, -span, span)
    f_ref, g_ref = oracle_all(w, 8)
    _, f, grads = run_gpu(w)
    assert_parity(w, f, grads, f_ref, g_ref, "random %d with a long index" % seed)
    wp = wl.Workload(w.name, wl.as_program(e), w.inputs, w.df)
    plan, f, grads = run_gpu(wp)
    assert plan.forward_family in ("program", "contraction")
    assert_parity(wp, f, grads, f_ref, g_ref, "random %d with a long index, as program" % seed)


@pytest.mark.parametrize("seed", range(32))
def test_random_expressions_with_a_long_index_fp64(seed):
    """The long-index expressions in fp64 on values of order one (the range of the short random expressions, not
    shrunk).  The kernels add thousands of terms in another order than the oracle, which shows beyond 1e-12 on
    some elements; what must hold is the bound that grows with the number of terms, 2 (n + 1) 2^-53 sum |term|
    carried through the outer function and the gradient sums, element by element."""
    e = wl.random_expr(seed, "f64", long_index=True)
    terms = int(np.prod([hi - lo + 1 for lo, hi in e.sums])) if e.sums else 1
    span = min(0.6, 600.0 / terms) if e.body == "exp" else 0.6     # exp of the sum must stay finite in fp64
    w = wl.random_inputs(e, 300 + seed, -span, span)
    f_ref, g_ref = oracle_all(w, 8)
    assert np.all(np.isfinite(f_ref)) and all(np.all(np.isfinite(g)) for g in g_ref if g is not None)
    bound_f, bound_g = rounding_bound.bounds(e, w.arg_list(), w.df)
    _, f, grads = run_gpu(w)
    worst = assert_within_rounding_bounds(w, f, grads, f_ref, g_ref, bound_f, bound_g, "long index %d, fp64" % seed)
    wp = wl.Workload(w.name, wl.as_program(e), w.inputs, w.df)
    plan, f, grads = run_gpu(wp)
    assert plan.forward_family in ("program", "contraction")
    worst = max(worst, assert_within_rounding_bounds(wp, f, grads, f_ref, g_ref, bound_f, bound_g, "as program"))
    print("long index %d fp64: largest floored relative error %.2e" % (seed, worst))


LONG_SUMS = [
    ("matmul_f64", lambda: wl.matmul_expr(12, 9, 1500, "f64")),                       # plan-driven kernels (fp64)
    ("matmul_program_f32", lambda: wl.as_program(wl.matmul_expr(10, 7, 1300, "f32", True, False))),
    ("cumsum_exp_f64", lambda: wl.cumulative_sum_expr(1500, "f64")),                  # a condition on every term
    ("two_sums_f32", lambda: _expr("exp", (5,), [(0, 39), (1, 40)], [("x", (60, 45), [[1, 1, 0], [0, 0, 1]])], "f32")),
    ("dense_layer_f64", lambda: wl.dense_layer_expr(6, 5, 1100, "f64")),              # outer operand, long sum
    # few function indices: several blocks share one, a second pass adds their sums and applies the outer function
    ("matmul_few_f64", lambda: wl.matmul_expr(3, 2, 9000, "f64")),
    ("matmul_few_program_f32", lambda: wl.as_program(wl.matmul_expr(3, 2, 9000, "f32", True, False))),
    ("dense_layer_few_f64", lambda: wl.dense_layer_expr(2, 3, 9000, "f64")),
    ("dense_layer_few_f32", lambda: wl.dense_layer_expr(1, 2, 70000, "f32")),
]


@pytest.mark.parametrize("name,make", LONG_SUMS, ids=[c[0] for c in LONG_SUMS])
def test_long_sums_per_function_index(name, make):
    """At least 1024 terms per function index: the forward kernels give one block to every function index.
    Inputs are uniform in [-1, 1] throughout (only the fp32 exp of 1600 terms draws from [-0.5, 0.5] to stay inside
    the format); the results are held to the element-wise bound that follows from the number of terms and the sum
    of their magnitudes, and the fp32 ones to the normwise limit as well."""
    e = make()
    w = wl.random_inputs(e, 41, -0.5, 0.5) if name == "two_sums_f32" else wl.random_inputs(e, 41)
    f_ref, g_ref = oracle_all(w, 4)
    if name.startswith("dense_layer"):
        bound_f, bound_g = rounding_bound.dense_layer_bounds(e.dtype, *w.arg_list(), w.df)
    else:
        plain = e if e.body != "program" else wl.matmul_expr(*e.f_shape, e.sums[0][1] + 1, e.dtype, True, False)
        bound_f, bound_g = rounding_bound.bounds(plain, w.arg_list(), w.df)
    plan, f, grads = run_gpu(w)
    worst = assert_within_rounding_bounds(w, f, grads, f_ref, g_ref, bound_f, bound_g, name)
    if e.dtype == "f32":
        for got, ref in [(f, f_ref)] + list(zip(grads, g_ref)):
            assert check.errors(got, ref)["normwise"] <= check.LIMITS["f32"][1], (name, check.errors(got, ref))
    print("%s: largest floored relative error %.2e" % (name, worst))


FEW_ELEMENTS = [
    # (name, expression, generic kernels only, value range)
    # a 3 x 3 filter summed over 4 * 40 * 40 positions, and the worked expression with 8 rows: c has 64 elements
    # of which the 8 on the diagonal are not masked, d has 10
    ("filter_generic_f32", lambda: wl.strided_tanh_expr(4, 81, 81, 3, 3, 2, "f32"), True, 0.9),
    ("worked_generic_f32", lambda: wl.worked_expr(8, 20000, 3, "f32"), True, 0.6),
    ("worked_generic_f64", lambda: wl.worked_expr(3, 30000, 2, "f64"), True, 0.6),
    ("filter_program_f32", lambda: wl.as_program(wl.strided_tanh_expr(4, 81, 81, 3, 3, 2, "f32")), False, 0.9),
    # weights (54 elements) through the sum, bias (6 elements) through the outer function
    ("dense_layer_program_f32", lambda: wl.dense_layer_expr(9000, 6, 9, "f32"), False, 0.5),
    ("dense_layer_program_f64", lambda: wl.dense_layer_expr(7000, 3, 4, "f64"), False, 0.5),
    # sums down the columns of f (db of the worked expression, dy of a matrix product): neighbouring elements read
    # neighbouring f, successive terms lie a row apart -- one thread per element, the rows shared by several blocks
    ("column_sums_generic_f32", lambda: wl.worked_expr(1100, 60, 3, "f32"), True, 0.6),
    ("column_sums_program_f32", lambda: wl.as_program(wl.worked_expr(1100, 60, 3, "f32")), False, 0.6),
    ("matmul_columns_generic_f64", lambda: wl.matmul_expr(1500, 40, 9, "f64"), True, 0.9),
]


@pytest.mark.parametrize("name,make,generic_only,span", FEW_ELEMENTS, ids=[c[0] for c in FEW_ELEMENTS])
def test_few_elements_with_long_sums(name, make, generic_only, span):
    """Gradients whose elements each sum a thousand terms or more and that are few (a filter, a bias, a small
    matrix) or read f across its contiguous direction: several blocks share an element, their partial sums are
    added in a fixed order by a finishing pass; elements that a mask zeroes stay exact zeros; two runs give
    identical bits."""
    from paper_1711_01348_amd import binding as B
    e = make()
    w = wl.random_inputs(e, 77, -span, span)
    if "worked" in name:
        w.inputs["c"] = np.abs(w.inputs["c"]) * 0.3
    plan, f, grads = run_gpu(w, generic_only=generic_only)
    assert plan.forward_family in ("generic", "program")
    if plan.forward_family == "generic":
        assert plan.workspace_bytes > 0          # room for the partial sums of the shared elements
    f_ref, g_ref = oracle_all(w, 8)
    assert_parity(w, f, grads, f_ref, g_ref, name)
    _, _, again = run_gpu(w, generic_only=generic_only)
    for a, b in zip(grads, again):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("rows,dtype", [(4097, "f32"), (4095, "f32"), (4400, "f64")])
def test_many_elements_with_long_sums(rows, dtype):
    """A gradient with thousands of elements that each sum more than a thousand terms (dx_ik = sum_j df_ij y_kj with
    one k): from 4096 elements on the cooperative layout gives every element a wavefront (four to a workgroup, the
    last workgroup not full), below that a workgroup; against the oracle, twice with identical bits."""
    from paper_1711_01348_amd import binding as B
    e = wl.matmul_expr(rows, 1500, 1, dtype)
    w = wl.random_inputs(e, 83, -0.9, 0.9)
    plan, f, grads = run_gpu(w, generic_only=True)
    q = plan.query(0)
    assert q["family"] == "generic" and q["gather_layout"] == "blocks" and q["gather_elements"] == rows
    f_ref, g_ref = oracle_all(w, 8)
    assert_parity(w, f, grads, f_ref, g_ref, "rows %d" % rows)
    _, _, again = run_gpu(w, generic_only=True)
    for x, y in zip(grads, again):
        assert np.array_equal(x, y)


def test_backward_is_deterministic_and_skips_unwanted():
    import torch
    w = wl.config3("small")
    _, f1, g1 = run_gpu(w)
    _, f2, g2 = run_gpu(w)
    assert np.array_equal(f1, f2)
    for a, b in zip(g1, g2):
        assert np.array_equal(a, b)
    _, _, g3 = run_gpu(w, wanted=[True, False, False, True])
    assert g3[1] is None and g3[2] is None
    assert np.array_equal(g3[0], g1[0]) and np.array_equal(g3[3], g1[3])


# ---------------------------------------------------------------- full benchmark sizes

def _full(w, nthreads=16):
    f_ref, g_ref = oracle_all(w, nthreads)
    _, f, grads = run_gpu(w)
    assert_parity(w, f, grads, f_ref, g_ref, "full")


@pytest.mark.parametrize("make", [lambda: wl.config2(1), lambda: wl.config2(2), lambda: wl.config2(3),
                                  lambda: wl.config5()], ids=["cfg2_1", "cfg2_2", "cfg2_3", "cfg5"])
def test_full_size_small_workloads(make):
    _full(make())


def test_full_size_config3():
    """8192 x 8192 x 5: every element of f and of the four gradients against the oracle."""
    _full(wl.config3())


@pytest.mark.parametrize("make", [lambda: wl.config2(1), lambda: wl.config2(3), lambda: wl.config5(), lambda: wl.config3()],
                         ids=["cfg2_1", "cfg2_3", "cfg5", "cfg3"])
def test_full_size_on_the_plan_driven_kernels(make):
    """The same workloads with the specialised families switched off: the cooperative layouts (every die a range of
    elements of its own, batches of terms, operands that stand still along a run) at the sizes they are meant for."""
    w = make()
    f_ref, g_ref = oracle_all(w, 16)
    plan, f, grads = run_gpu(w, generic_only=True)
    assert plan.forward_family == "generic"
    assert_parity(w, f, grads, f_ref, g_ref, "full, generic")


def test_full_size_config4():
    """4096 x 4096 x 256 in the benchmark's launch configuration (matrix-core family, the collapsed indices split
    over 8 chunks of workgroups): every element of f, da, db, dc and dd against the oracle, which visits all
    4.3e9 extended indices.  dd is looked at once more on its own: the elements whose window
    max(0, m - (I-1)) .. min(K-1, m) of Sec. 6 is complete (K-1 <= m <= I-1) and the clipped ones at both ends."""
    w = wl.config4()
    I, J = w.expr.f_shape
    K = w.expr.sums[0][1] + 1
    f_ref, g_ref = oracle_all(w, 16)
    plan, f, grads = run_gpu(w)
    assert plan.forward_family == "worked_mfma"
    assert_parity(w, f, grads, f_ref, g_ref, "full")
    dd, dd_ref = grads[3], g_ref[3]
    assert dd.shape == (I + K - 1,)
    for lo, hi, what in ((0, K - 1, "clipped below"), (K - 1, I, "complete window"), (I, I + K - 1, "clipped above")):
        assert check.within(dd[lo:hi], dd_ref[lo:hi], "f32"), (what, check.errors(dd[lo:hi], dd_ref[lo:hi]))
    dc = grads[2]
    assert np.count_nonzero(dc) <= I and np.count_nonzero(dc - np.diag(np.diag(dc))) == 0


def test_determinism_full_config3():
    w = wl.config3()
    _, f1, g1 = run_gpu(w)
    _, f2, g2 = run_gpu(w)
    assert np.array_equal(f1, f2)
    for x, y in zip(g1, g2):
        assert np.array_equal(x, y)


def test_device_entry_points_reject_misuse():
    """Host-side checks of the device entry points: no kernel is launched on any of these paths."""
    import ctypes
    import torch
    from paper_1711_01348_amd import binding as B
    w = wl.config3("small")
    plan = B.Plan(w.expr)
    args = [_to_dev(a) for a in w.arg_list()]
    f = torch.empty(tuple(w.expr.f_shape), dtype=torch.float32, device="cuda")
    ptrs = (ctypes.c_void_p * 4)(*[t.data_ptr() for t in args])
    assert plan.workspace_bytes > 0
    # workspace missing / too small
    assert B.lib.tad_eval_forward(plan._h, ptrs, f.data_ptr(), None, 0, None) == -7
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    dptr = (ctypes.c_void_p * 4)(*[t.data_ptr() for t in args])
    assert B.lib.tad_eval_backward(plan._h, ptrs, f.data_ptr(), f.data_ptr(), dptr, small.data_ptr(), 16, None) == -7
    # NULL argument pointer
    bad = (ctypes.c_void_p * 4)(args[0].data_ptr(), None, args[2].data_ptr(), args[3].data_ptr())
    assert B.lib.tad_eval_forward(plan._h, bad, f.data_ptr(), small.data_ptr(), 16, None) == -1
    # a gradient that was not planned
    plan2 = B.Plan(w.expr, needs_grad=[True, True, False, True])
    ws = plan2.workspace()
    assert B.lib.tad_eval_backward(plan2._h, ptrs, f.data_ptr(), f.data_ptr(), dptr, ws.data_ptr(), ws.numel(), None) == -1
    # the binding refuses wrong dtypes, shapes and host tensors before calling the library
    with pytest.raises(ValueError):
        plan.forward([a.double() for a in args])
    with pytest.raises(ValueError):
        plan.forward([a.cpu() for a in args])
    with pytest.raises(ValueError):
        plan.forward([args[0][:-1].contiguous()] + args[1:])
    torch.cuda.synchronize()


def test_runs_on_a_side_stream():
    """Kernels are enqueued on the caller's stream."""
    import torch
    from paper_1711_01348_amd import binding as B
    w = wl.config5("small")
    plan = B.Plan(w.expr)
    f_ref, g_ref = oracle_all(w, 1)
    s = torch.cuda.Stream()
    args = [_to_dev(a) for a in w.arg_list()]
    df = _to_dev(w.df)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        f = plan.forward(args)
        grads = plan.backward(args, f, df)
    s.synchronize()
    assert_parity(w, f.cpu().numpy(), [g.cpu().numpy() for g in grads], f_ref, g_ref, "side stream")


GRAPH_CASES = [
    ("generic_f64", lambda: wl.config1()),
    ("worked_f32", lambda: wl.config3("small")),
    ("mfma_f32", lambda: wl.config4("small")),
    ("strided_f32", lambda: wl.config5("small")),
    ("antidiagonal_f32", lambda: wl.config2(3, "small")),
    ("program_outer_operand_f64", lambda: wl.random_inputs(wl.dense_layer_expr(70, 33, 5, "f64"), 13)),
]


@pytest.mark.parametrize("name,make", GRAPH_CASES, ids=[c[0] for c in GRAPH_CASES])
def test_captured_graph_replays_match_eager_calls(name, make):
    """Both evaluation calls only enqueue kernels (no allocation, no synchronisation, no memset node), so a step
    can be captured once and replayed: every replay, with new input values and eager work in between, gives
    exactly what the eager calls give."""
    import torch
    from paper_1711_01348_amd import binding as B
    w = make()
    plan = B.Plan(w.expr)
    args = [_to_dev(a) for a in w.arg_list()]
    df = _to_dev(w.df)
    ws, ws2 = plan.workspace(), plan.workspace()
    f = torch.empty(tuple(w.expr.f_shape), dtype=df.dtype, device="cuda")
    is_alias = [a.same_as is not None for a in w.expr.args]
    grads = [None if al else torch.empty_like(a) for a, al in zip(args, is_alias)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):           # warm-up on the capturing side stream
        plan.forward(args, out=f, ws=ws)
        plan.backward(args, f, df, out=grads, ws=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        plan.forward(args, out=f, ws=ws)
        plan.backward(args, f, df, out=grads, ws=ws)
    rng = np.random.Generator(np.random.PCG64(wl.SEED_BASE + 99))
    for replay in range(3):
        for t in [a for a, al in zip(args, is_alias) if not al] + [df]:     # new values in the captured buffers
            t.mul_(float(rng.uniform(0.7, 1.1)))
        f.zero_()
        for g in grads:
            if g is not None:
                g.fill_(7.0)
        graph.replay()
        torch.cuda.synchronize()
        f_eager = plan.forward(args, ws=ws2)
        g_eager = plan.backward(args, f_eager, df, ws=ws2)
        torch.cuda.synchronize()
        assert torch.equal(f, f_eager), (name, replay, "f")
        for a, g, ge in zip(w.expr.args, grads, g_eager):
            if g is not None:
                assert torch.equal(g, ge), (name, replay, "d" + a.name)


CONTRACTIONS = [(xt, yt, sw) for xt in (False, True) for yt in (False, True) for sw in (False, True)]


@pytest.mark.gpu
@pytest.mark.parametrize("xt,yt,sw", CONTRACTIONS)
def test_contraction_family_all_memory_orders(xt, yt, sw):
    """Matrix product and its two derived products on the matrix cores, every storage order of the operands,
    sizes that are not multiples of the tile."""
    e = wl.matmul_expr(132, 260, 72, "f32", xt, yt, sw)
    w = wl.random_inputs(e, 21)
    f_ref, g_ref = oracle_all(w, 4)
    plan, f, grads = run_gpu(w)
    assert plan.forward_family == "contraction"
    assert [plan.query(p)["family"] for p in range(2)] == ["contraction", "contraction"]
    assert_parity(w, f, grads, f_ref, g_ref)
    _, f2, grads2 = run_gpu(w, generic_only=True)
    assert_parity(w, f2, grads2, f_ref, g_ref, "generic")


@pytest.mark.gpu
@pytest.mark.parametrize("xt,yt,sw", CONTRACTIONS)
@pytest.mark.parametrize("I,J,K", [(260, 384, 160), (288, 260, 256)])
def test_contraction_whole_tiles_beside_ragged_ones(I, J, K, xt, yt, sw):
    """Shapes where some workgroups own tiles wholly inside the operands (they run the loop without bounds checks, an
    odd and an even number of contraction tiles) and others a ragged edge, in the product and in one derived
    product each, every storage order."""
    e = wl.matmul_expr(I, J, K, "f32", xt, yt, sw)
    w = wl.random_inputs(e, 29)
    f_ref, g_ref = oracle_all(w, 8)
    plan, f, grads = run_gpu(w)
    assert plan.forward_family == "contraction"
    assert_parity(w, f, grads, f_ref, g_ref)


@pytest.mark.gpu
@pytest.mark.parametrize("I,J,K,xt,yt", [(128, 256, 4096, False, False), (64, 68, 8192, True, False),
                                          (132, 60, 2100, False, True), (4096, 64, 96, False, False)])
def test_contraction_with_a_split_summation_index(I, J, K, xt, yt):
    """Few output tiles and a long summation index (or, in the gradients, a long collapsed function index): the
    index is cut into pieces for separate workgroups; against the fp64 matrix products."""
    import torch
    from paper_1711_01348_amd import binding as B
    e = wl.matmul_expr(I, J, K, "f32", xt, yt)
    w = wl.random_inputs(e, 23)
    plan = B.Plan(e)
    assert plan.forward_family == "contraction" and plan.workspace_bytes > 0
    x, y = w.arg_list()
    args = [_to_dev(x), _to_dev(y)]
    f = plan.forward(args)
    dx, dy = plan.backward(args, f, _to_dev(w.df))
    torch.cuda.synchronize()
    X = (x.T if xt else x).astype(np.float64)
    Y = (y.T if yt else y).astype(np.float64)
    D = w.df.astype(np.float64)
    gx, gy = D @ Y.T, X.T @ D
    for got, ref, what in ((f, X @ Y, "f"), (dx, gx.T if xt else gx, "dx"), (dy, gy.T if yt else gy, "dy")):
        got = got.cpu().numpy()
        assert check.within(got, ref, "f32"), (what, check.errors(got, ref))


def test_contraction_full_size_against_sampled_rows():
    """4096^3 product: the oracle computes sampled rows of f, dx and dy one by one (fp64 dot products)."""
    w = wl.matmul_workload(4096)
    plan, f, grads = run_gpu(w)
    assert plan.forward_family == "contraction"
    x, y = [np.asarray(a, dtype=np.float64) for a in w.arg_list()]
    df = np.asarray(w.df, dtype=np.float64)
    rng = np.random.default_rng(5)
    rows = sorted(set(rng.integers(0, 4096, size=6).tolist() + [0, 127, 128, 4095]))
    for r in rows:
        # restrict the expression to one row of f / dx (a 1 x J x K problem) and one row of dy
        e1 = wl.matmul_expr(1, 4096, 4096, "f32")
        f_row = oracle.forward(e1, [x[r:r + 1], y])[0]
        assert check.within(f[r], f_row, "f32"), ("f", r, check.errors(f[r], f_row))
        dx_row = oracle.backward(e1, [x[r:r + 1], y], df[r:r + 1], wanted=[True, False])[0][0]
        assert check.within(grads[0][r], dx_row, "f32"), ("dx", r, check.errors(grads[0][r], dx_row))
        # dy[r, :] = sum_i x[i, r] df[i, :]: the expression with K restricted to index r
        e2 = wl.matmul_expr(4096, 4096, 1, "f32")
        dy_row = oracle.backward(e2, [x[:, r:r + 1], y[r:r + 1]], df, wanted=[False, True], nthreads=8)[1][0]
        assert check.within(grads[1][r], dy_row, "f32"), ("dy", r, check.errors(grads[1][r], dy_row))


def _alias_program():
    e = wl.matrix_square_expr(31, "f64")
    return wl.as_program(e)


PROGRAM_CASES = [
    ("worked_f64", lambda: wl.Workload("p", wl.as_program(wl.config1().expr), wl.config1().inputs, wl.config1().df)),
    ("worked_f32", lambda: wl.random_inputs(wl.as_program(wl.worked_expr(37, 52, 5, "f32")), 2, -0.9, 0.9)),
    ("sq_f32", lambda: wl.random_inputs(wl.as_program(wl.broadcast_sq_expr(50, 72, "f32")), 3)),
    ("diag_f32", lambda: wl.random_inputs(wl.as_program(wl.diagonal_sq_expr(77, "f32")), 4)),
    ("exp_f32", lambda: wl.random_inputs(wl.as_program(wl.index_sum_exp_expr(40, 33, "f32")), 5)),
    ("strided_f32", lambda: wl.random_inputs(wl.as_program(wl.strided_tanh_expr(2, 9, 11, 3, 3, 2, "f32")), 6)),
    ("matmul_f64", lambda: wl.random_inputs(wl.as_program(wl.matmul_expr(12, 9, 14, "f64")), 7)),
    ("softplus_f64", lambda: wl.random_inputs(wl.softplus_ratio_expr(9, 13, 6, "f64"), 8)),
    ("softplus_f32", lambda: wl.random_inputs(wl.softplus_ratio_expr(33, 21, 17, "f32"), 9)),
    ("alias_f64", lambda: wl.random_inputs(_alias_program(), 10)),
    # the outer function reads operands (Sec. 5.2): bias of a dense layer (few bias elements, long sums over the
    # batch: cooperative gather), an operand read inside the sum and outside it, one tensor read both ways
    # through two occurrences, a range that depends on the function index
    ("biased_tanh_f64", lambda: wl.random_inputs(wl.biased_tanh_expr(301, 7, "f64"), 11)),
    ("dense_layer_f32", lambda: wl.random_inputs(wl.dense_layer_expr(2500, 6, 9, "f32"), 12, -0.7, 0.7)),
    ("dense_layer_f64", lambda: wl.random_inputs(wl.dense_layer_expr(70, 33, 5, "f64"), 13)),
    ("gated_gauss_f64", lambda: wl.random_inputs(wl.gated_gauss_expr(37, 29, 4, "f64"), 14, -0.8, 0.8)),
    ("gated_gauss_f32", lambda: wl.random_inputs(wl.gated_gauss_expr(130, 70, 3, "f32"), 15, -0.8, 0.8)),
    ("biased_causal_conv_f64", lambda: wl.random_inputs(wl.biased_causal_conv_expr(400, 9, "f64"), 16)),
    # more values alive at once than the interpreter's register form holds: the kernels with one temporary per
    # operation run the forward pass, the register form the gradients
    ("many_live_f64", lambda: wl.random_inputs(wl.many_live_values_expr(45, 7, "f64"), 17, -0.9, 0.9)),
    ("many_live_f32", lambda: wl.random_inputs(wl.many_live_values_expr(300, 5, "f32"), 18, -0.9, 0.9)),
    ("many_live_long_f32", lambda: wl.random_inputs(wl.many_live_values_expr(3, 2100, "f32"), 19, -0.9, 0.9)),
]


@pytest.mark.gpu
@pytest.mark.parametrize("name,make", PROGRAM_CASES, ids=[c[0] for c in PROGRAM_CASES])
def test_program_bodies(name, make):
    """Scalar part given as postfix programs: derivatives derived by reverse accumulation at plan time and
    interpreted by the kernels, against the oracle's own interpreter with forward-mode derivatives."""
    w = make()
    f_ref, g_ref = oracle_all(w, 2)
    plan, f, grads = run_gpu(w)
    assert plan.forward_family == "program"
    assert_parity(w, f, grads, f_ref, g_ref, name)


RECOGNISED = [
    ("worked", lambda: wl.config3("small"), "worked"),
    ("worked_mfma", lambda: wl.config4("small"), "worked_mfma"),
    ("strided", lambda: wl.config5("small"), "strided"),
    ("antidiagonal", lambda: wl.config2(3, "small"), "antidiagonal"),
    ("row_reduce", lambda: wl.config2(1, "small"), "row_reduce"),
    ("product", lambda: wl.random_inputs(wl.matmul_expr(132, 260, 72, "f32"), 21), "contraction"),
]


@pytest.mark.gpu
@pytest.mark.parametrize("name,make,family", RECOGNISED, ids=[c[0] for c in RECOGNISED])
def test_program_that_spells_out_a_builtin_body_reaches_its_kernels(name, make, family):
    """A body given as postfix programs that are the built-in body's own functions (here also with the operands of
    its sums and products swapped) is planned as that body: same kernel family, same bits as the built-in form."""
    from paper_1711_01348_amd import binding as B
    w = make()
    ep = wl.as_program(w.expr)
    if name.startswith("worked"):       # (b + a)^2, c on the left of the product, d^3 first
        ep.inner = [("arg", 3), ("powi", 3), ("arg", 2), ("arg", 1), ("arg", 0), ("add",), ("powi", 2), ("mul",), ("add",)]
    wp = wl.Workload(w.name, ep, w.inputs, w.df)
    plan, f, grads = run_gpu(wp, keep_program=False)
    assert plan.forward_family == family
    _, f_ref, g_ref = run_gpu(w)
    assert np.array_equal(f, f_ref)
    for g, r in zip(grads, g_ref):
        assert np.array_equal(g, r)
    # a different function must not match: (a + b)^2 c + d^2
    if name == "worked":
        ep.inner[1] = ("powi", 2)
        assert B.Plan(ep).forward_family == "program"


@pytest.mark.gpu
@pytest.mark.parametrize("K", [1, 2, 4, 6, 7, 8])
def test_worked_family_every_short_sum_length(K):
    """The fused kernels are instantiated per length of the summed index (1..8)."""
    e = wl.worked_expr(261, 520, K, "f32")
    w = wl.random_inputs(e, 30 + K, -0.8, 0.8)
    w.inputs["c"] = np.abs(w.inputs["c"]) * np.float32(0.5)
    f_ref, g_ref = oracle_all(w, 4)
    plan, f, grads = run_gpu(w)
    assert plan.forward_family == "worked"
    assert_parity(w, f, grads, f_ref, g_ref, "K=%d" % K)


@pytest.mark.gpu
@pytest.mark.parametrize("I,J,K", [(256, 512, 5), (512, 1024, 3), (768, 512, 4), (512, 1536, 5), (512, 1024, 6),
                                   (512, 1024, 2)])
def test_worked_family_whole_tiles(I, J, K):
    """Shapes made of whole backward tiles (256 rows x 512 columns), where no load of the backward pass needs a
    predicate: one tile, several tiles each way."""
    e = wl.worked_expr(I, J, K, "f32")
    w = wl.random_inputs(e, 60 + K, -0.8, 0.8)
    w.inputs["c"] = np.abs(w.inputs["c"]) * np.float32(0.5)
    f_ref, g_ref = oracle_all(w, 4)
    plan, f, grads = run_gpu(w)
    assert plan.forward_family == "worked"
    assert_parity(w, f, grads, f_ref, g_ref, "%dx%dx%d" % (I, J, K))


@pytest.mark.gpu
@pytest.mark.parametrize("I,J,K", [(70, 132, 32), (129, 260, 96), (64, 64, 64)])
def test_mfma_family_other_shapes(I, J, K):
    """Long summed index (a multiple of 32): matrix-core kernels on ragged tiles and on exactly one tile."""
    e = wl.worked_expr(I, J, K, "f32")
    w = wl.random_inputs(e, 40 + K, -0.5, 0.5)
    w.inputs["c"] = np.abs(w.inputs["c"]) * np.float32(4.0 / K)
    w.inputs["d"] = w.inputs["d"] * np.float32(0.4)
    f_ref, g_ref = oracle_all(w, 4)
    plan, f, grads = run_gpu(w)
    assert plan.forward_family == "worked_mfma"
    assert_parity(w, f, grads, f_ref, g_ref, "%dx%dx%d" % (I, J, K))


CONDITIONED = [
    ("cumsum_f64", lambda: wl.cumulative_sum_expr(97, "f64")),
    ("cumsum_f32", lambda: wl.cumulative_sum_expr(600, "f32")),
    ("causal_conv_f32", lambda: wl.causal_convolution_expr(5000, 33, "f32")),
    ("causal_conv_f64", lambda: wl.causal_convolution_expr(61, 7, "f64")),
    ("triangular_f32", lambda: wl.triangular_matmul_expr(40, 70, "f32")),
    ("triangular_f64", lambda: wl.triangular_matmul_expr(9, 12, "f64")),
    ("window_f32", lambda: wl.band_expr(3000, 5, "f32")),
    ("window_program_f64", lambda: wl.as_program(wl.band_expr(50, 4, "f64"))),
    ("never_f64", lambda: wl.ExprSpec("exp", (4,), [(0, 3)], [wl.ArgSpec("x", (4,), [[0, 1]])], "f64",
                                      constraints=[([-1, -1], -1)])),
]


@pytest.mark.gpu
@pytest.mark.parametrize("name,make", CONDITIONED, ids=[c[0] for c in CONDITIONED])
def test_sums_with_index_dependent_ranges(name, make):
    e = make()
    lim = 0.02 if name == "cumsum_f32" else 0.9       # keep exp(sum of 600 values) in range
    w = wl.random_inputs(e, 50, -lim, lim)
    f_ref, g_ref = oracle_all(w, 2)
    plan, f, grads = run_gpu(w)
    assert plan.forward_family in ("generic", "program")
    assert_parity(w, f, grads, f_ref, g_ref, name)


@pytest.mark.gpu
def test_direct_and_expanded_forward_forms_agree():
    """Long summed index: the direct form on the vector ALUs and the expanded square on the matrix cores both
    meet the fp32 tolerance against the oracle (small case element by element, full size on sampled rows)."""
    import torch
    from paper_1711_01348_amd import binding as B
    w = wl.config4("small")
    f_ref = oracle.forward(w.expr, w.arg_list())
    args = [_to_dev(a) for a in w.arg_list()]
    for direct in (False, True):
        plan = B.Plan(w.expr, direct_form=direct)
        assert plan.forward_family == "worked_mfma"
        f = plan.forward(args).cpu().numpy()
        assert check.within(f, f_ref, "f32"), (direct, check.errors(f, f_ref))
    w = wl.config4()
    args = [_to_dev(a) for a in w.arg_list()]
    fd = B.Plan(w.expr, direct_form=True).forward(args).cpu().numpy()
    fe = B.Plan(w.expr).forward(args).cpu().numpy()
    a, b, c, d = [np.asarray(x, dtype=np.float64) for x in w.arg_list()]
    for i in (0, 63, 64, 2047, 4095):
        s = ((a[i][None, :] + b) ** 2).sum(axis=1) * c[i, i] + (d[i:i + 256] ** 3).sum()
        e1 = wl.worked_expr(1, 4096, 256, "f32", d_len=256 + 0, c_shape=(1, 1))
        row = oracle.forward(e1, [a[i:i + 1], b, c[i:i + 1, i:i + 1], d[i:i + 256]])[0]
        assert np.allclose(row, np.exp(-s), rtol=1e-12)
        assert check.within(fd[i], row, "f32"), ("direct", i, check.errors(fd[i], row))
        assert check.within(fe[i], row, "f32"), ("expanded", i, check.errors(fe[i], row))


# ---- a gradient evaluated as an expression of its own, and differentiated once more (Sec. 5.3) ---------------

def _nonlinear_sum(I, J, K, dtype):
    e = wl.softplus_ratio_expr(I, J, K, dtype)
    e.outer = [("sum",)]
    return e


DERIVED = [
    ("matmul_f64", lambda: wl.matmul_expr(23, 17, 31, "f64")),
    ("matmul_f32", lambda: wl.matmul_expr(37, 29, 41, "f32", True, False, True)),
    ("broadcast_sq_f32", lambda: wl.broadcast_sq_expr(70, 300, "f32")),
    ("diagonal_cube_f64", lambda: _expr("cube", (33,), [], [("x", (33, 40), [[1], [1]])])),
    ("causal_conv_f64", lambda: wl.causal_convolution_expr(300, 17, "f64")),
    ("triangular_f32", lambda: wl.triangular_matmul_expr(40, 50, "f32")),
    ("matrix_square_f64", lambda: wl.matrix_square_expr(21, "f64")),
    ("autocorrelation_f32", lambda: wl.autocorrelation_expr(500, 33, "f32")),
    ("nonlinear_f64", lambda: _nonlinear_sum(19, 23, 7, "f64")),
    ("skew_plane_f64", lambda: _expr("mul", (14, 9), [(0, 5)], [("x", (40, 6), [[2, 1, 0], [0, 0, 1]]),
                                                                ("y", (19,), [[1, 0, 1]])])),
    # Smith divisors above one (the quotient becomes a summation index of the derived expression)
    ("stride_mixed_f64", lambda: _expr("mul", (13, 11), [(0, 4)], [("x", (29, 25), [[2, 0, 1], [0, 2, 1]]),
                                                                   ("y", (5,), [[0, 0, 1]])])),
    ("stride3_exp_f32", lambda: _expr("exp", (40, 3), [], [("x", (120,), [[3, 1]])], "f32")),
    # outer functions: seed expression, then the derived one; operands of the outer function: a second part
    ("worked_f64", lambda: wl.worked_expr(19, 23, 5, "f64")),
    ("worked_f32", lambda: wl.worked_expr(40, 52, 5, "f32")),
    ("worked_wide_f64", lambda: wl.worked_expr(9, 1100, 3, "f64")),      # derived expressions with long sums
    ("cumsum_exp_f64", lambda: wl.cumulative_sum_expr(200, "f64")),
    ("dense_layer_f32", lambda: wl.dense_layer_expr(300, 12, 9, "f32")),
    ("gated_gauss_f64", lambda: wl.gated_gauss_expr(21, 17, 4, "f64")),
    ("biased_causal_conv_f64", lambda: wl.biased_causal_conv_expr(150, 7, "f64")),
]


@pytest.mark.parametrize("name,make", DERIVED, ids=[d[0] for d in DERIVED])
def test_derived_expressions(name, make):
    """tad_eval_derived: the gradient of every tensor, evaluated by the library through its derived expressions
    (seed expressions first where the outer function is not the identity, one part per occurrence, a second part for
    operands the outer function reads, the parts added by the library), is the oracle's gradient of the original
    expression.  Then the derived expression of every occurrence is differentiated once more: its gradients (second
    order) are the oracle's gradients of that expression, whose terms the host tests check against the scan of the
    original."""
    import torch
    from paper_1711_01348_amd import binding as B
    e = make()
    w = wl.random_inputs(e, 31, -0.9, 0.9)
    tensors = w.arg_list()
    npdt = tensors[0].dtype
    want = oracle.backward_by_tensor(e, tensors, w.df, nthreads=8)
    plan = B.Plan(e)
    dev_args = [_to_dev(x) for x in tensors]
    dev_df = _to_dev(w.df)
    fused = not e.sums and not e.constraints
    occurrences = {}
    for p, a in enumerate(e.args):
        occurrences.setdefault(p if a.same_as is None else a.same_as, []).append(p)
    for root, slots in occurrences.items():
        dg = B.DerivedGradient(plan, root)
        n_second = sum(1 for sl in slots if plan.query(root, slots.index(sl))["in_outer"] and not fused)
        assert dg.counts[1] == len(slots) + n_second, (name, root, dg.counts)
        got = dg.evaluate(dev_args, dev_df)
        torch.cuda.synchronize()
        got = got.cpu().numpy()
        assert check.within(got, want[root], e.dtype), (name, root, check.errors(got, want[root]))
        again = dg.evaluate(dev_args, dev_df).cpu().numpy()
        assert np.array_equal(got, again), (name, root, "not deterministic")

    # second order: v . dx (the part through the sum) differentiated with respect to df / g and the kept operands
    rng = np.random.Generator(np.random.PCG64(wl.SEED_BASE + 77))
    seeds = {}

    def seed():
        """g = df * d outer / d sum on the device (by the library) and on the host (by the oracle, rounded)"""
        if not seeds:
            sspec = plan.seed_expr(-1)
            ins = [w.df] + tensors
            on_gpu = B.Plan(sspec, needs_grad=[False] * len(ins)).forward([_to_dev(x) for x in ins])
            ref = oracle.forward(sspec, ins)
            torch.cuda.synchronize()
            assert check.within(on_gpu.cpu().numpy(), ref, e.dtype), (name, "seed")
            seeds[-1] = ref.astype(npdt)
        return seeds[-1]

    for root, slots in occurrences.items():
        for occ in range(len(slots)):
            spec, operands = plan.derived_expr(root, occ)
            dplan = B.Plan(spec)
            kept = [tensors[q] for q in operands[1:]]
            ins = [w.df if operands[0] == -1 else seed()] + kept
            dev = [_to_dev(x) for x in ins]
            v = rng.uniform(-1, 1, spec.f_shape).astype(npdt)
            grads = dplan.backward(dev, dplan.forward(dev), _to_dev(v))
            torch.cuda.synchronize()
            ref = oracle.backward_by_tensor(spec, ins, v, nthreads=8)
            for a, g, r in zip(spec.args, grads, ref):
                if r is None:
                    continue
                g = g.cpu().numpy()
                assert check.within(g, r, e.dtype), (name, root, occ, "d" + a.name, check.errors(g, r))


def test_second_order_matrix_product_closed_form_on_the_matrix_cores():
    """dx = df y^T for f = x y; with a weight v on dx: d(v . dx)/d df = v y and d(v . dx)/d y = v^T df."""
    import torch
    from paper_1711_01348_amd import binding as B
    I, J, K = 192, 136, 260
    e = wl.matmul_expr(I, J, K, "f32")
    w = wl.random_inputs(e, 5)
    x, y = w.arg_list()
    spec, operands = B.Plan(e).derived_expr(0)
    assert operands == [-1, 1]
    dplan = B.Plan(spec)
    assert dplan.forward_family == "contraction"
    rng = np.random.Generator(np.random.PCG64(wl.SEED_BASE + 78))
    v = rng.uniform(-1, 1, (I, K)).astype(np.float32)
    dev = [_to_dev(w.df), _to_dev(y)]
    dx = dplan.forward(dev)
    g_df, g_y = dplan.backward(dev, dx, _to_dev(v))
    torch.cuda.synchronize()
    df64, y64, v64 = w.df.astype(np.float64), y.astype(np.float64), v.astype(np.float64)
    for got, ref, what in ((dx, df64 @ y64.T, "dx"), (g_df, v64 @ y64, "d df"), (g_y, v64.T @ df64, "d y")):
        got = got.cpu().numpy()
        assert check.within(got, ref, "f32"), (what, check.errors(got, ref))
