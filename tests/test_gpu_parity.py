"""GPU parity: HIP path (through the C ABI) against the fp64 CPU oracle, element by element."""
import numpy as np
import pytest

import oracle
from paper_1711_01348_amd import check
from paper_1711_01348_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _expr(body, f_shape, sums, args, dtype="f64"):
    return wl.ExprSpec(body, tuple(f_shape), list(sums),
                       [wl.ArgSpec(n, tuple(s), A) for n, s, A in args], dtype)


def _to_dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def run_gpu(w, generic_only=False, wanted=None):
    import torch
    from paper_1711_01348_amd import binding as B
    plan = B.Plan(w.expr, generic_only=generic_only)
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


def oracle_all(w, nthreads=8):
    args = w.arg_list()
    return oracle.forward(w.expr, args), oracle.backward(w.expr, args, w.df, nthreads=nthreads)


@pytest.mark.parametrize("generic_only", [True, False], ids=["generic", "selected"])
@pytest.mark.parametrize("w", wl.all_configs("small"), ids=lambda w: w.name)
def test_configs_small(w, generic_only):
    f_ref, g_ref = oracle_all(w)
    plan, f, grads = run_gpu(w, generic_only)
    assert_parity(w, f, grads, f_ref, g_ref, "generic" if generic_only else "selected")


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


def test_config1_fp64_tight():
    w = wl.config1()
    f_ref, g_ref = oracle_all(w, 1)
    _, f, grads = run_gpu(w)
    for got, ref in [(f, f_ref)] + list(zip(grads, g_ref)):
        assert check.errors(got, ref)["floored"] <= 1e-12
    dc = grads[2]
    assert np.count_nonzero(dc - np.diag(np.diag(dc))) == 0


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
]


@pytest.mark.parametrize("make", ASSORTED)
def test_assorted_index_maps_fp64(make):
    e = make()
    w = wl.random_inputs(e, 11, -0.9, 0.9)
    f_ref, g_ref = oracle_all(w, 1)
    _, f, grads = run_gpu(w)
    assert_parity(w, f, grads, f_ref, g_ref)


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
