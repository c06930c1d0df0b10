"""Host-side index plans: integer machinery invariants, paper pins, brute-force parity (no GPU)."""
import itertools
import os
import re
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_1711_01348_amd import binding as B
from paper_1711_01348_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
HEADER = os.path.join(os.path.dirname(os.path.dirname(__file__)), "include", "tad.h")


def _expr(body, f_shape, sums, args, dtype="f64"):
    return wl.ExprSpec(body, tuple(f_shape), list(sums),
                       [wl.ArgSpec(n, tuple(s), A) for n, s, A in args], dtype)


# ---------------------------------------------------------------- ABI surface

def test_library_exports_every_declared_symbol():
    text = open(HEADER).read()
    declared = set(re.findall(r"\b(tad_[a-z_0-9]+)\s*\(", text))
    assert declared, "no declarations found"
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(B.lib, name), name


def test_header_is_plain_c_and_struct_layouts_match(tmp_path):
    """The boundary header compiles as C99 and as C++, and the ctypes mirrors have the C struct sizes."""
    import ctypes
    import subprocess
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", HEADER],
                   check=True)
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c++", HEADER], check=True)
    src = tmp_path / "sizes.c"
    src.write_text('#include <stdio.h>\n#include "%s"\nint main(void){printf("%%zu %%zu %%zu %%zu\\n", sizeof(tad_expr), '
                   'sizeof(tad_arg), sizeof(tad_plan_info), sizeof(tad_op));return 0;}\n' % HEADER)
    exe = tmp_path / "sizes"
    subprocess.run(["gcc", "-std=c99", str(src), "-o", str(exe)], check=True)
    sizes = [int(v) for v in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert sizes == [ctypes.sizeof(B.TadExpr), ctypes.sizeof(B.TadArg), ctypes.sizeof(B.TadPlanInfo), ctypes.sizeof(B.TadOp)]


# ---------------------------------------------------------------- Sec. 4.1: Euclid and Smith

def test_extended_gcd_bezout_identity():
    rng = np.random.default_rng(1)
    pairs = [(0, 0), (0, 7), (-7, 0), (12, 18), (-12, 18), (12, -18), (-12, -18), (1, 1), (2**40, 2**20 * 3)]
    pairs += [tuple(int(v) for v in rng.integers(-10**6, 10**6, 2)) for _ in range(300)]
    for a, b in pairs:
        g, x, y = B.extended_gcd(a, b)
        assert g == int(np.gcd(a, b)) and g >= 0
        assert a * x + b * y == g


def _det(M):
    M = [[Fraction(int(v)) for v in row] for row in M]
    n, d = len(M), Fraction(1)
    for c in range(n):
        piv = next((r for r in range(c, n) if M[r][c] != 0), None)
        if piv is None:
            return Fraction(0)
        if piv != c:
            M[c], M[piv] = M[piv], M[c]
            d = -d
        d *= M[c][c]
        for r in range(c + 1, n):
            f = M[r][c] / M[c][c]
            M[r] = [a - f * b for a, b in zip(M[r], M[c])]
    return d


def _check_smith(A):
    A = np.asarray(A, dtype=np.int64)
    S, U, V, R = B.smith_normal_form(A)
    assert np.array_equal(U.astype(object) @ A.astype(object) @ V.astype(object), S.astype(object))
    assert abs(_det(U)) == 1 and abs(_det(V)) == 1
    off = S.copy()
    for i in range(min(S.shape)):
        off[i, i] = 0
    assert not off.any()
    diag = [int(S[i, i]) for i in range(min(S.shape))]
    assert all(d > 0 for d in diag[:R]) and all(d == 0 for d in diag[R:])
    assert all(diag[i + 1] % diag[i] == 0 for i in range(R - 1))
    assert R == np.linalg.matrix_rank(A.astype(float))
    # pseudo-inverse, kernel, cokernel (Sec. 4.1)
    n, m = A.shape
    Sd = [[Fraction(0)] * n for _ in range(m)]
    for r in range(R):
        Sd[r][r] = Fraction(1, diag[r])
    fr = lambda M: [[Fraction(int(v)) for v in row] for row in M]
    mul = lambda X, Y: [[sum(X[i][k] * Y[k][j] for k in range(len(Y))) for j in range(len(Y[0]))] for i in range(len(X))]
    I = mul(mul(fr(V), Sd), fr(U))
    assert mul(mul(fr(A), I), fr(A)) == fr(A)            # A I A = A
    assert not (A.astype(object) @ V[:, R:].astype(object)).any()   # A K = 0
    assert not (U[R:, :].astype(object) @ A.astype(object)).any()   # C A = 0
    return diag[:R]


def test_smith_known_and_edge_cases():
    assert _check_smith([[2, 4, 4], [-6, 6, 12], [10, -4, -16]]) == [2, 6, 12]
    assert _check_smith([[6, 0], [0, 4]]) == [2, 12]       # needs the divisibility repair
    assert _check_smith([[4, 0, 0], [0, 6, 0], [0, 0, 10]]) == [2, 2, 60]
    assert _check_smith([[1, -2]]) == [1]
    assert _check_smith([[2, 4]]) == [2]
    assert _check_smith([[2], [4], [6]]) == [2]
    assert _check_smith([[0, 0], [0, -3]]) == [3]
    assert _check_smith([[1, 0, 0], [1, 0, 0]]) == [1]
    assert _check_smith([[1, 0, 0, 0, 0], [0, 2, 0, 1, 0], [0, 0, 2, 0, 1]]) == [1, 1, 1]


def test_smith_random_matrices():
    rng = np.random.default_rng(2)
    for _ in range(300):
        n, m = rng.integers(1, 5), rng.integers(1, 6)
        A = rng.integers(-6, 7, (n, m))
        if rng.random() < 0.3 and n > 1:       # force rank deficiency
            A[-1] = A[0] * rng.integers(-2, 3)
        if not A.any():
            continue
        _check_smith(A)


def test_smith_rejects_zero_matrix_and_overflow():
    with pytest.raises(B.TadError) as e:
        B.smith_normal_form([[0, 0], [0, 0]])
    assert e.value.status == -1
    big = 2**62
    with pytest.raises(B.TadError) as e:
        B.smith_normal_form([[big, big - 1], [big - 3, big - 7]])
    assert e.value.status == -4


# ---------------------------------------------------------------- Sec. 4.2 / 5.1: ranges

def _brute(A, lo, hi, beta):
    A = np.asarray(A)
    pts = [x for x in itertools.product(*[range(l, h + 1) for l, h in zip(lo, hi)])
           if np.array_equal(A @ np.array(x), np.asarray(beta))]
    return sorted(pts)


def _fig(name):
    out = {}
    for line in open(os.path.join(GOLDEN, "lattice_figures.txt")):
        if line.startswith(name + " "):
            _, key, *vals = line.split()
            out[key] = [int(v) for v in vals]
    return out


def test_fig1_line_in_a_box():
    g = _fig("fig1")
    lo, hi = [g["box"][0], g["box"][2]], [g["box"][1], g["box"][3]]
    pts = B.lattice_enumerate([g["A"]], lo, hi, g["beta"])
    zlo, zhi = g["z"]
    assert [tuple(p) for p in pts] == [(-1 + 2 * z, z) for z in range(zlo, zhi + 1)]
    # neighbours of the end points l = (0, 0.5), h = (6, 3.5): ceil(0.5) = 1, floor(3.5) = 3
    assert (-1 + 2 * 0, 0) not in map(tuple, pts) and (-1 + 2 * 4, 4) not in map(tuple, pts)


def test_fig2_plane_in_a_box():
    g = _fig("fig2")
    lo, hi = [g["box"][0], g["box"][2], -30], [g["box"][1], g["box"][3], 30]
    pts = {tuple(p) for p in B.lattice_enumerate([g["A"]], lo, hi, g["beta"])}
    K = np.array(g["K"]).reshape(2, 3).T
    expect = {tuple(np.array([3, 0, 0]) + K @ np.array([z1, z2]))
              for z2 in range(-1, 6) for z1 in range(max(-1, -z2), min(1, 4 - z2) + 1)}
    assert len(expect) == g["count"][0]
    assert pts == expect


def test_lattice_enumeration_matches_brute_force_on_random_systems():
    rng = np.random.default_rng(3)
    done = 0
    while done < 150:
        n, m = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        A = rng.integers(-3, 4, (n, m))
        if not A.any():
            continue
        lo = rng.integers(-3, 2, m)
        hi = lo + rng.integers(0, 5, m)
        # a few reachable and a few arbitrary right-hand sides
        betas = [A @ rng.integers(lo, hi + 1) for _ in range(3)] + [rng.integers(-6, 7, n) for _ in range(3)]
        for beta in betas:
            got = [tuple(p) for p in B.lattice_enumerate(A, lo, hi, beta)]
            assert got == _brute(A, lo, hi, beta), (A, lo, hi, beta)
        done += 1


def test_divisibility_condition_is_not_redundant():
    """f_ij = x_{2i}: for odd beta the z range is the full j range, yet there is no integer solution."""
    assert len(B.lattice_enumerate([[2, 0]], [0, 0], [4, 3], [3])) == 0
    assert len(B.lattice_enumerate([[2, 0]], [0, 0], [4, 3], [4])) == 4
    assert len(B.lattice_enumerate([[2]], [0], [4], [3])) == 0
    assert [tuple(p) for p in B.lattice_enumerate([[2, 4]], [0, 0], [5, 5], [10])] == [(1, 2), (3, 1), (5, 0)]
    assert len(B.lattice_enumerate([[2, 4]], [0, 0], [5, 5], [7])) == 0


# ---------------------------------------------------------------- Sec. 6: printed plan of the worked expression

def _read_limits():
    lim = {}
    for line in open(os.path.join(GOLDEN, "worked_expression_limits.txt")):
        if line.startswith("#") or not line.strip():
            continue
        g, kind, *rest = line.split()
        if kind not in ("condition", "index"):
            lim.setdefault(g, {})[kind] = (rest[0], rest[1])
    return lim


def _lim(txt, m=0):
    mm = re.fullmatch(r"(max|min)\((-?\d+),m(-\d+)?\)", txt)
    if mm:
        return (max if mm.group(1) == "max" else min)(int(mm.group(2)), m + int(mm.group(3) or 0))
    return int(txt)


def test_plan_reproduces_printed_limits():
    lim = _read_limits()
    e = wl.worked_expr(3, 4, 5, "f64", d_len=8)
    plan = B.Plan(e)
    rng = lambda g, z, m=0: range(_lim(lim[g][z][0], m), _lim(lim[g][z][1], m) + 1)
    for i in range(3):
        for k in range(5):
            assert [tuple(p) for p in plan.enumerate(0, [i, k])] == [(i, z, k) for z in rng("da", "z0")]
    for j in range(4):
        for k in range(5):
            assert [tuple(p) for p in plan.enumerate(1, [j, k])] == [(z, j, k) for z in rng("db", "z0")]
    for b0 in range(3):
        for b1 in range(3):
            got = [tuple(p) for p in plan.enumerate(2, [b0, b1])]
            want = sorted((b1, z0, z1) for z1 in rng("dc", "z1") for z0 in rng("dc", "z0")) if b0 == b1 else []
            assert got == want
    for m in range(8):
        got = [tuple(p) for p in plan.enumerate(3, [m])]
        want = sorted((m - z1, z0, z1) for z1 in rng("dd", "z1", m) for z0 in rng("dd", "z0"))
        assert got == want
    assert len(plan.enumerate(3, [7])) == 0
    # the parameterisation itself: one cokernel row +-(1, -1) for c; kernel of d spans j and (i down, k up)
    qc, qd = plan.query(2), plan.query(3)
    assert qc["rank"] == 1 and qc["C"].tolist() in ([[1, -1]], [[-1, 1]])
    assert qd["rank"] == 1 and qd["kernel_dim"] == 2
    assert not (np.array([[1, 0, 1]]) @ qd["K"]).any()


def _ranges_from_rows(plan, arg, beta):
    """Evaluate the Fourier-Motzkin rows in the paper's form (over b(beta)) with exact fractions."""
    q = plan.query(arg)
    e = plan.expr
    D, R, kap = plan.n_ext, q["rank"], q["kernel_dim"]
    lo = [0] * len(e.f_shape) + [s[0] for s in e.sums]
    hi = [n - 1 for n in e.f_shape] + [s[1] for s in e.sums]
    U, V = q["U"], q["V"]
    y = [Fraction(int((U[r] * np.array(beta)).sum()), q["smith"][r]) for r in range(R)]
    base = [sum(Fraction(int(V[d, r])) * y[r] for r in range(R)) for d in range(D)]     # I beta
    b = [Fraction(lo[d]) - base[d] for d in range(D)] + [base[d] - Fraction(hi[d]) for d in range(D)]
    for row in plan.bound_rows(arg, B.ROWS_FEASIBILITY):
        if sum(int(c) * v for c, v in zip(row["coef_b"], b)) > 0:
            return None
    return q, b


def test_bound_rows_in_paper_form_give_the_printed_dd_range():
    e = wl.worked_expr(3, 4, 5, "f64", d_len=8)
    plan = B.Plan(e)
    import math
    for m in range(7):
        q, b = _ranges_from_rows(plan, 3, [m])
        outer = q["kernel_dim"] - 1
        lo = max(math.ceil(sum(int(c) * v for c, v in zip(r["coef_b"], b)) / r["scale"])
                 for r in plan.bound_rows(3, B.ROWS_LOWER, outer))
        hi = min(math.floor(sum(int(c) * v for c, v in zip(r["coef_b"], b)) / r["scale"])
                 for r in plan.bound_rows(3, B.ROWS_UPPER, outer))
        # outermost kernel coordinate of d moves k up and i down: printed range max(0, m-2) .. min(4, m)
        col = q["K"][:, outer]
        assert col.tolist() in ([-1, 0, 1], [1, 0, -1])
        if col.tolist() == [-1, 0, 1]:
            assert (lo, hi) == (max(0, m - 2), min(4, m))
        else:
            assert (-hi, -lo) == (max(0, m - 2), min(4, m))


# ---------------------------------------------------------------- plans of the benchmark configurations

def _check_plan_against_scan(expr, sample=40, seed=0):
    plan = B.Plan(expr)
    rng = np.random.default_rng(seed)
    for p, a in enumerate(expr.args):
        counts = oracle.gamma_counts(expr, p)
        assert np.array_equal(plan.count_all(p), counts), (expr.body, p)
        total = int(np.prod(a.shape))
        picks = range(total) if total <= sample else rng.choice(total, sample, replace=False)
        for lin in picks:
            beta = np.unravel_index(int(lin), a.shape)
            assert np.array_equal(plan.enumerate(p, beta), oracle.gamma(expr, p, beta)), (expr.body, p, beta)


@pytest.mark.parametrize("w", wl.all_configs("small")[:5] + [wl.config5("small")], ids=lambda w: w.name)
def test_config_plans_match_exhaustive_scan_small(w):
    _check_plan_against_scan(w.expr)


def test_config4_plan_matches_scan_reduced_rows():
    _check_plan_against_scan(wl.worked_expr(9, 7, 256, "f32"), sample=25)


@pytest.mark.parametrize("make", [
    lambda: _expr("exp", (5,), [], [("x", (9,), [[2]])]),
    lambda: _expr("exp", (5, 4), [], [("x", (9,), [[2, 0]])]),
    lambda: _expr("exp", (4, 3), [], [("x", (20,), [[2, 4]])]),
    lambda: _expr("exp", (4, 3), [], [("x", (12,), [[3, 1]])]),
    lambda: _expr("exp", (3, 4), [(0, 2)], [("x", (7, 9), [[2, 0, 1], [0, 2, 1]])]),
    lambda: _expr("mul", (5, 4), [(1, 6)], [("x", (5, 7), [[1, 0, 0], [0, 0, 1]]), ("y", (7, 4), [[0, 0, 1], [0, 1, 0]])]),
    lambda: _expr("exp", (3, 3, 3), [], [("x", (5, 5), [[1, 1, 0], [0, 1, 1]])]),
    lambda: _expr("exp", (6,), [(0, 3), (0, 2)], [("x", (30,), [[3, 2, 4]])]),
    lambda: wl.worked_expr(4, 3, 5, "f64", d_len=11, c_shape=(6, 5)),     # arguments larger than the referenced range
])
def test_assorted_index_maps_match_scan(make):
    _check_plan_against_scan(make(), sample=1000)


@pytest.mark.parametrize("seed", range(40))
def test_random_expressions_match_scan(seed):
    """Seeded random index matrices (ranks 1..3, coefficients 0..3, a negative one under a condition, slack in the
    shapes): every plan visits exactly what the scan of the box finds."""
    _check_plan_against_scan(wl.random_expr(seed), sample=60, seed=seed)


def test_counts_at_full_size():
    """Bit-exact counts for every gradient element at the full benchmark sizes (cfg 2, 3, 5)."""
    for w in [wl.config2(1), wl.config2(2), wl.config2(3), wl.config3(), wl.config5()]:
        plan = B.Plan(w.expr)
        for p in range(len(w.expr.args)):
            assert np.array_equal(plan.count_all(p), oracle.gamma_counts(w.expr, p)), (w.name, p)


# ---------------------------------------------------------------- error paths (host only)

def _status(fn):
    with pytest.raises(B.TadError) as e:
        fn()
    return e.value.status


def test_error_paths():
    ok = _expr("exp", (4, 4), [], [("x", (7,), [[1, 1]])])
    B.Plan(ok)
    assert _status(lambda: B.Plan(_expr("exp", (4, 4), [], [("x", (7,), [[0, 0]])]))) == -1       # zero matrix
    assert _status(lambda: B.Plan(_expr("exp", (4, 4), [], [("x", (6,), [[1, 1]])]))) == -2       # leaves shape
    assert _status(lambda: B.Plan(_expr("exp", (4, 4), [], [("x", (7,), [[1, -1]])]))) == -2      # negative index
    assert _status(lambda: B.Plan(_expr("exp", (4, 4), [(3, 2)], [("x", (9,), [[1, 1, 1]])]))) == -2   # lo > hi
    assert _status(lambda: B.Plan(_expr("sq", (4,), [(0, 1)], [("x", (9,), [[1, 1]])]))) == -5     # sq takes no sum
    assert _status(lambda: B.Plan(_expr("mul", (4,), [], [("x", (4,), [[1]])]))) == -1             # argument count
    assert _status(lambda: B.Plan(_expr("exp", (4, 0), [], [("x", (7,), [[1, 1]])]))) == -2        # empty f
    big = 2**40
    assert _status(lambda: B.Plan(_expr("exp", (4,), [], [("x", (3 * big + 1,), [[big]])]))) == -4  # int32 range


def test_null_and_misuse_at_the_abi():
    import ctypes
    e = _expr("exp", (4, 4), [], [("x", (7,), [[1, 1]])])
    ce, ca = B.pack_expr(e), B.pack_args(e)
    h = ctypes.c_void_p()
    assert B.lib.tad_plan_derive(None, ca, 1, 1, 0, ctypes.byref(h)) == -1
    assert B.lib.tad_plan_derive(ctypes.byref(ce), None, 1, 1, 0, ctypes.byref(h)) == -1
    assert B.lib.tad_plan_derive(ctypes.byref(ce), ca, 1, 1, 0, None) == -1
    assert B.lib.tad_plan_derive(ctypes.byref(ce), ca, 1, 7, 0, ctypes.byref(h)) == -1
    ca[0].alias = 1        # an operand cannot be an alias of itself or of a later operand
    assert B.lib.tad_plan_derive(ctypes.byref(ce), ca, 1, 1, 0, ctypes.byref(h)) == -1
    ca[0].alias = -1
    assert B.lib.tad_plan_derive(ctypes.byref(ce), ca, 1, 1, 0, ctypes.byref(h)) == -1
    ca[0].alias = 0
    ca[0].needs_grad = 0
    assert B.lib.tad_plan_derive(ctypes.byref(ce), ca, 1, 1, 0, ctypes.byref(h)) == 0
    info = B.TadPlanInfo()
    assert B.lib.tad_plan_query(h, 0, 0, ctypes.byref(info)) == -1      # gradient was not planned
    assert B.lib.tad_plan_query(h, 5, 0, ctypes.byref(info)) == -1
    assert B.lib.tad_eval_forward(h, None, None, None, 0, None) == -1
    assert B.lib.tad_eval_backward(h, None, None, None, None, None, 0, None) == -1
    B.lib.tad_plan_free(h)
    B.lib.tad_plan_free(None)
    assert B.strerror(-4) == "integer overflow"


def test_size_limits():
    # 2^32 function elements: beyond the int32 element index of the kernels
    assert _status(lambda: B.Plan(wl.broadcast_sq_expr(65536, 65536, "f32"))) == -4
    # too many indices / too high rank are rejected before the library is called or by it
    with pytest.raises(B.TadError):
        B.Plan(_expr("exp", (2, 2, 2, 2, 2, 2, 2), [], [("x", (2,), [[1, 0, 0, 0, 0, 0, 0]])]))
    # kernel dimension 5 > TAD_MAX_KERNEL
    assert _status(lambda: B.Plan(_expr("exp", (2, 2, 2, 2, 2, 2), [], [("x", (2,), [[1, 0, 0, 0, 0, 0]])]))) == -5
    # the largest benchmark shapes derive fine
    for w in (wl.config3(), wl.config4(), wl.config2(2)):
        assert B.Plan(w.expr).workspace_bytes >= 0


def test_workspace_sizes_are_reported():
    assert B.Plan(wl.config1().expr).workspace_bytes == 0          # generic kernels need none
    assert B.Plan(wl.config3().expr).workspace_bytes > 0
    # the plan-driven kernels keep partial sums only for gradients whose elements are shared by several blocks:
    # here db (40960 elements, sums down the columns of f, 13 blocks per element: fp64 partial sums and one flag
    # per element, each part rounded up to 256 bytes)
    assert B.Plan(wl.config3().expr, generic_only=True).workspace_bytes == 40960 * 13 * 8 + 40960 * 4
    assert B.Plan(wl.worked_expr(20, 30, 3, "f32"), generic_only=True).workspace_bytes == 0   # short sums: none


# ---- a tensor that occurs several times (Sec. 5.3: one plan per occurrence) ---------------------

REPEATED = [
    ("matrix_square", lambda: wl.matrix_square_expr(5, "f64")),
    ("symmetric_product", lambda: wl.symmetric_product_expr(4, 6, "f64")),
    ("autocorrelation", lambda: wl.autocorrelation_expr(7, 4, "f64")),
    ("worked_shared", lambda: wl.worked_shared_expr(5, 3, "f64")),
]


@pytest.mark.parametrize("name,make", REPEATED, ids=[r[0] for r in REPEATED])
def test_each_occurrence_has_its_own_exact_plan(name, make):
    """Every occurrence's plan visits exactly the extended indices that the brute-force scan of the box
    finds for that occurrence's index map."""
    import itertools
    e = make()
    plan = B.Plan(e)
    assert plan.forward_family == "generic"
    root = 0
    alias = [p for p, a in enumerate(e.args) if a.same_as == root]
    assert len(alias) == 1
    for occ, slot in enumerate([root] + alias):
        for beta in itertools.product(*[range(n) for n in e.args[root].shape]):
            got = plan.enumerate(root, beta, occ=occ)
            want = oracle.gamma(e, slot, beta)
            assert got.shape == want.shape and (got == want).all(), (name, occ, beta)


def test_alias_rules():
    e = wl.matrix_square_expr(4, "f64")
    e.args[1].shape = (4, 5)
    assert _status(lambda: B.Plan(e)) == -2          # alias with another shape
    e = wl.worked_shared_expr(4, 2, "f64")
    e.args[2].same_as = 1                            # alias of an alias
    assert _status(lambda: B.Plan(e)) in (-1, -2)
    e = wl.matrix_square_expr(4, "f64")
    plan = B.Plan(e)
    assert _status(lambda: plan.query(1)) == -1      # an alias operand is reached through its tensor
    q0, q1 = plan.query(0), plan.query(0, occ=1)
    assert q0["kernel_dim"] == 1 and q1["kernel_dim"] == 1
    assert _status(lambda: plan.query(0, occ=2)) == -1


def test_contraction_family_is_selected_only_for_exact_matrix_products():
    assert B.Plan(wl.matmul_expr(8, 12, 16, "f32")).forward_family == "contraction"
    assert B.Plan(wl.matmul_expr(8, 12, 16, "f32", True, True, True)).forward_family == "contraction"
    assert B.Plan(wl.matmul_expr(8, 12, 16, "f64")).forward_family == "generic"        # fp32 only
    assert B.Plan(wl.matmul_expr(8, 12, 18, "f32")).forward_family == "generic"        # rows not 16-byte multiples
    assert B.Plan(wl.matrix_square_expr(8, "f32")).forward_family == "generic"         # repeated tensor
    e = wl.matmul_expr(8, 12, 16, "f32")
    e.args[0].shape = (9, 16)                                                           # longer than the range
    assert B.Plan(e).forward_family == "generic"


# ---- scalar bodies given as programs: symbolic reverse accumulation on the host (Sec. 2) ---------

def _scalar_expr(inner, outer, n_operands):
    """f_0 = outer(inner(v_0..)) on one-element tensors: the gradient is outer' * d inner / d v_p."""
    args = [wl.ArgSpec("v%d" % p, (1,), [[1]]) for p in range(n_operands)]
    return wl.ExprSpec("program", (1,), [], args, "f64", list(inner), list(outer))


PROGRAMS = [
    (wl.PROGRAM_OF_BODY["worked"][0], wl.PROGRAM_OF_BODY["worked"][1], 4),
    (wl.PROGRAM_OF_BODY["tanh_dot"][0], wl.PROGRAM_OF_BODY["tanh_dot"][1], 2),
    (wl.softplus_ratio_expr(2, 2, 2, "f64").inner, wl.softplus_ratio_expr(2, 2, 2, "f64").outer, 3),
    # x / (y - x) + sin(x y) - sqrt(y) * x^5, repeated operands and every derivative rule with two inputs
    ([("arg", 0), ("arg", 1), ("arg", 0), ("sub",), ("div",), ("arg", 0), ("arg", 1), ("mul",), ("sin",), ("add",),
      ("arg", 1), ("sqrt",), ("arg", 0), ("powi", 5), ("mul",), ("sub",)], [("sum",), ("cos",), ("neg",), ("exp",)], 2),
    # an operand the function does not depend on, and a constant function of the sum
    ([("arg", 0), ("const", 3.0), ("mul",)], [("const", 2.5)], 2),
    ([("arg", 1), ("powi", 1)], [("sum",), ("powi", 1)], 2),
    # the outer function reads operands (no summation index here, so every operand has one value per f index):
    # v2 + tanh(s) * v0 / (1 + v1^2) with s = v0 v1 + sin(v2)
    ([("arg", 0), ("arg", 1), ("mul",), ("arg", 2), ("sin",), ("add",)],
     [("arg", 2), ("sum",), ("tanh",), ("arg", 0), ("mul",), ("const", 1.0), ("arg", 1), ("powi", 2), ("add",),
      ("div",), ("add",)], 3),
    # 18 values alive at once: no register form for the inner program, one for its derivatives
    (wl.many_live_values_expr(2, 2, "f64").inner, wl.many_live_values_expr(2, 2, "f64").outer, 2),
]


@pytest.mark.parametrize("inner,outer,nop", PROGRAMS, ids=["worked", "tanh_dot", "softplus", "mixed", "unused", "powi1", "outer_operands", "many_live"])
def test_symbolic_derivatives_match_forward_mode_oracle(inner, outer, nop):
    """The programs derived by reverse accumulation, evaluated on the host, against the oracle's dual numbers."""
    e = _scalar_expr(inner, outer, nop)
    plan = B.Plan(e, keep_program=True)
    rng = np.random.default_rng(8)
    for _ in range(20):
        v = rng.uniform(0.2, 1.4, size=nop)      # positive: sqrt and log stay real, y - x may be either sign
        if abs(v[-1] - v[0]) < 0.05:
            continue
        args = [np.array([x]) for x in v]
        total = plan.program_eval(-1, v)
        f_ref = oracle.forward(e, args)[0]
        reads = any(t[0] == "arg" for t in outer)
        vo = v if reads else None
        assert abs(plan.program_eval(-2, vo, total) - f_ref) <= 1e-13 * max(1.0, abs(f_ref))
        g_ref = oracle.backward(e, args, np.array([1.0]))
        for p in range(nop):
            got = plan.program_eval(-3, vo, total) * plan.program_eval(p, v) + plan.program_eval(-4 - p, vo, total)
            assert abs(got - g_ref[p][0]) <= 1e-12 * max(1.0, abs(g_ref[p][0])), (p, got, g_ref[p][0])


def test_gather_layouts_of_the_plan_driven_kernels():
    """How the plan-driven kernels lay their threads over a gradient, as the query reports it: one thread per
    element for short sums; one workgroup per element for long sums that run along the contiguous direction of
    f; one thread per element with the sum shared by workgroups where f is contiguous along the elements instead
    (a column sum); several workgroups per element where the elements are few."""
    big = B.Plan(wl.config3().expr, generic_only=True)          # 8192 x 8192 x 5
    a, b, c, d = (big.query(p) for p in range(4))
    assert (a["gather_layout"], a["gather_splits"]) == ("blocks", 1)       # da_ik: 8192 terms along a row of f
    assert (b["gather_layout"], b["gather_splits"]) == ("lanes", 13)       # db_jk: 8192 terms down a column of f
    # dc: 67 million elements, all but the diagonal masked: the launch runs over the 8192 values of y = i instead
    assert (c["gather_layout"], c["gather_splits"], c["gather_elements"]) == ("blocks", 1, 8192)
    assert a["gather_elements"] == 8192 * 5 and d["gather_elements"] == 8196
    assert (d["gather_layout"], d["gather_splits"]) == ("blocks", 1)       # dd_m: 5 x 8192 terms, 8196 elements
    small = B.Plan(wl.config1().expr)
    assert all(small.query(p)["gather_layout"] == "threads" and small.query(p)["gather_splits"] == 1 for p in range(4))
    conv = B.Plan(wl.config5().expr, generic_only=True)         # x: at most 4 terms; w: 9 elements, 524288 terms each
    assert conv.query(0)["gather_layout"] == "threads"
    assert (conv.query(1)["gather_layout"], conv.query(1)["gather_splits"]) == ("blocks", 114)
    # a gradient with a divisibility mask: f_i = x_{5i}: the launch runs over y = beta / 5 (a box of at most a
    # quarter of the elements is worth the separate clearing pass; f_i = x_{3i} runs over all beta)
    fifth = B.Plan(_expr("sq", (40,), [], [("x", (300,), [[5]])], "f64"))
    assert fifth.query(0)["gather_elements"] == 60            # y = 0 .. 59 (beta up to 299), 40 of them used
    assert B.Plan(_expr("sq", (40,), [], [("x", (130,), [[3]])], "f64")).query(0)["gather_elements"] == 130
    # no mask: all elements
    assert B.Plan(_expr("sq", (40,), [], [("x", (40,), [[1]])], "f64")).query(0)["gather_elements"] == 40
    mm = B.Plan(wl.matmul_expr(1500, 40, 9, "f64"), generic_only=True)     # dy_kj = sum_i x_ik df_ij: down the columns
    assert (mm.query(1)["gather_layout"], mm.query(1)["gather_splits"]) == ("lanes", 5)
    assert mm.query(0)["gather_layout"] == "threads"                       # dx_ik: 40 terms


def test_program_register_form():
    """Registers assigned to the temporaries of the derived programs by live range: operands, constants and the sum
    take none (they are read where they are used); as many as values are alive at once; -1 beyond 16 -- the
    kernels then fall back to one temporary per operation.  Both forms evaluate alike (the host evaluator uses the
    register form when there is one; the oracle comparison above covers the values)."""
    plan = B.Plan(_scalar_expr(wl.many_live_values_expr(2, 2, "f64").inner, [("sum",)], 2))
    assert plan.program_registers(-1) == -1                                        # 18 function values alive at once
    assert 1 <= plan.program_registers(0) <= 16 and 1 <= plan.program_registers(1) <= 16
    assert plan.program_registers(-2) == 0 and plan.program_registers(-3) == 0     # the sum itself; the constant 1
    assert plan.program_registers(-4) == 0                                         # d outer / d operand: zero
    # x * y: one operation on two operands
    plan = B.Plan(_scalar_expr([("arg", 0), ("arg", 1), ("mul",)], [("sum",)], 2), keep_program=True)
    assert plan.program_registers(-1) == 1
    assert plan.program_registers(0) == 0 and plan.program_registers(1) == 0       # d/dx = y, d/dy = x: operands
    # a chain of unary operations needs one register however long it is
    plan = B.Plan(_scalar_expr([("arg", 0)] + [("sin",), ("exp",), ("tanh",)] * 5, [("sum",)], 1))
    assert plan.program_registers(-1) == 1
    # (x + y) * (x - y): two values alive before the product
    plan = B.Plan(_scalar_expr([("arg", 0), ("arg", 1), ("add",), ("arg", 0), ("arg", 1), ("sub",), ("mul",)], [("sum",)], 2))
    assert plan.program_registers(-1) == 2
    assert _status(lambda: plan.program_registers(2)) == -1
    assert _status(lambda: plan.program_registers(-6)) == -1
    assert _status(lambda: B.Plan(wl.config1().expr).program_registers(-1)) == -1   # not a program plan


def test_program_rules():
    ok_in, ok_out = [("arg", 0)], [("sum",)]
    mk = lambda i, o, n=1: B.Plan(_scalar_expr(i, o, n))
    mk(ok_in, ok_out)
    assert _status(lambda: mk([("arg", 1)], ok_out)) == -1                      # operand index out of range
    assert _status(lambda: mk([("sum",)], ok_out)) == -1                        # the sum is not an inner input
    mk(ok_in, [("arg", 0)])                                   # the outer function may read an operand that has one value per f index
    moving = wl.ExprSpec("program", (3,), [(0, 2)], [wl.ArgSpec("x", (5,), [[1, 1]]), wl.ArgSpec("b", (3,), [[1, 0]])],
                         "f64", [("arg", 0)], [("sum",), ("arg", 0), ("mul",)])
    assert _status(lambda: B.Plan(moving)) == -1                                # ... not one that moves with the summation index
    moving.outer = [("sum",), ("arg", 1), ("mul",)]
    B.Plan(moving)
    assert _status(lambda: mk(ok_in, [("arg", 1)])) == -1
    assert _status(lambda: mk([("arg", 0), ("add",)], ok_out)) == -1            # stack underflow
    assert _status(lambda: mk([("arg", 0), ("arg", 0)], ok_out)) == -1          # two values left
    assert _status(lambda: mk([("arg", 0), ("powi", 0)], ok_out)) == -1
    assert _status(lambda: mk([("const", float("inf"))], ok_out)) == -1
    assert _status(lambda: mk(ok_in, [])) == -1
    assert _status(lambda: mk([("arg", 0)] + [("neg",)] * 64, ok_out)) == -1    # longer than TAD_MAX_PROGRAM
    mk([("arg", 0), ("store", 15), ("load", 15), ("mul",)], ok_out)             # a temporary: x * x
    assert _status(lambda: mk([("load", 0), ("arg", 0), ("mul",)], ok_out)) == -1    # read before it is stored
    assert _status(lambda: mk([("arg", 0), ("store", 16)], ok_out)) == -1            # beyond TAD_MAX_TEMPS
    assert _status(lambda: mk([("store", 0), ("arg", 0)], ok_out)) == -1             # nothing on the stack to keep
    assert _status(lambda: mk([("arg", 0), ("store", 0)], [("load", 0)])) == -1      # temporaries belong to one program
    # a derivative too long for the device form is refused, not truncated
    long_inner = [("arg", 0)] + [("arg", 0), ("div",), ("sin",)] * 7
    assert _status(lambda: mk(long_inner, ok_out)) in (0, -5)
    plan = B.Plan(wl.as_program(wl.config1().expr), keep_program=True)
    assert plan.forward_family == "program" and plan.workspace_bytes >= 8 * 6 * 8
    # without the flag a program that spells out a built-in body is planned as that body
    assert B.Plan(wl.as_program(wl.config1().expr)).forward_family == "generic"
    assert B.Plan(wl.as_program(wl.config3("small").expr)).forward_family == "worked"
    assert _status(lambda: B.Plan(wl.config1().expr).program_eval(-1, np.zeros(4))) == -1   # not a program plan
    plan = B.Plan(wl.biased_tanh_expr(3, 2, "f64"), needs_grad=[True, False, True])
    assert _status(lambda: plan.program_eval(-2, None, 0.3)) == -1             # the outer function needs the operand values
    assert _status(lambda: plan.program_eval(1, np.zeros(3))) == -1            # derivative not planned
    assert _status(lambda: plan.program_eval(-4 - 1, np.zeros(3), 0.3)) == -1
    assert plan.program_eval(-4 - 2, np.zeros(3), 0.0) == 1.0                  # d tanh(b + s) / d b at 0
    assert _status(lambda: plan.program_eval(-4 - 3, np.zeros(3), 0.3)) == -1
    assert plan.workspace_bytes >= 2 * 3 * 8                                    # g and the sums


# ---- summation ranges that depend on other indices: extra linear conditions in the constraint system --------

CONDITIONED = [
    ("cumsum", lambda: wl.cumulative_sum_expr(7, "f64")),
    ("causal_conv", lambda: wl.causal_convolution_expr(9, 4, "f64")),
    ("triangular", lambda: wl.triangular_matmul_expr(3, 5, "f64")),
    ("window", lambda: wl.band_expr(8, 2, "f64")),
    ("window_program", lambda: wl.as_program(wl.band_expr(6, 3, "f64"))),
    # a condition that couples three indices with coefficients other than one: 2 i + j - 3 k >= 1
    ("skew", lambda: wl.ExprSpec("mul", (5, 6), [(0, 3)],
                                 [wl.ArgSpec("x", (5, 4), [[1, 0, 0], [0, 0, 1]]), wl.ArgSpec("y", (12,), [[0, 1, 2]])],
                                 "f64", constraints=[([2, 1, -3], -1)])),
    # no extended index satisfies the condition at all
    ("never", lambda: wl.ExprSpec("exp", (4,), [(0, 3)], [wl.ArgSpec("x", (4,), [[0, 1]])], "f64",
                                  constraints=[([-1, -1], -1)])),
]


@pytest.mark.parametrize("name,make", CONDITIONED, ids=[c[0] for c in CONDITIONED])
def test_conditioned_sums_match_brute_force(name, make):
    e = make()
    plan = B.Plan(e)
    assert plan.forward_family in ("generic", "program")
    for arg, a in enumerate(e.args):
        assert (plan.count_all(arg) == oracle.gamma_counts(e, arg)).all(), (name, arg)
        for beta in itertools.product(*[range(n) for n in a.shape]):
            got, want = plan.enumerate(arg, beta), oracle.gamma(e, arg, beta)
            assert got.shape == want.shape and (got == want).all(), (name, arg, beta)


def test_condition_rules():
    e = wl.cumulative_sum_expr(5, "f64")
    rows = B.Plan(e).bound_rows(0, B.ROWS_LOWER) + B.Plan(e).bound_rows(0, B.ROWS_UPPER)
    assert any(r["coef_c"].any() for r in rows)            # the condition shows up in the range rows
    e.constraints = e.constraints * 9
    assert _status(lambda: B.Plan(e)) == -1                 # more than TAD_MAX_CONSTRAINTS
    # x_{i-k} without the condition k <= i leaves the tensor; with it, it does not
    e = wl.causal_convolution_expr(6, 3, "f64")
    B.Plan(e)
    e.constraints = []
    assert _status(lambda: B.Plan(e)) == -2
    # conditions keep the specialised families off
    e = wl.matmul_expr(8, 8, 8, "f32")
    e.constraints = [([0, 1, -1], 0)]
    assert B.Plan(e).forward_family == "generic"


def test_small_expressions_get_term_lists():
    """Sec. 5.1: a small expression on the plan-driven kernels has its sets Gamma-hat(beta) written out at plan time
    (tad_plan_query reports it); larger ones, program bodies and expressions with aliases keep the ranges."""
    from paper_1711_01348_amd import binding as B
    w = wl.config1()
    assert all(B.Plan(w.expr).query(p)["listed"] for p in range(4))
    assert not any(B.Plan(w.expr, term_lists=False).query(p)["listed"] for p in range(4))
    assert not B.Plan(wl.config3("small").expr, generic_only=True).query(0)["listed"]      # too many terms
    assert not B.Plan(wl.as_program(w.expr), keep_program=True).query(0)["listed"]          # program body
    assert not B.Plan(wl.matrix_square_expr(5, "f64")).query(0)["listed"]                   # alias operand
    small = B.Plan(wl.config3("small").expr)                                                # specialised family: no list
    assert small.query(0)["family"] == "worked" and not small.query(0)["listed"]
