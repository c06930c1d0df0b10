// Index-plan derivation on the host (Sec. 5.3, index half of the element-wise
// derivation algorithm) and the host-only entry points of the C ABI.
#include "plan.hpp"

#include <algorithm>
#include <cstring>
#include <new>

namespace tad {

int body_arg_count(int body) {
    switch (body) {
    case TAD_BODY_SQ: case TAD_BODY_CUBE: case TAD_BODY_SIN: case TAD_BODY_EXP: return 1;
    case TAD_BODY_MUL: case TAD_BODY_TANH_DOT: return 2;
    case TAD_BODY_WORKED: return 4;
    default: return -1;
    }
}

static const int64_t kInt32Safe = (int64_t)1 << 30;

static int32_t fit32(int64_t v) {
    if (v >= kInt32Safe || v <= -kInt32Safe) throw overflow_error();
    return (int32_t)v;
}

// Solve  A x = beta,  lo <= x <= hi  once for all beta with |beta_r| < extent[r]: Smith parts, constraints
// Inverse of a unimodular integer matrix: integer Gauss-Jordan on [M | 1] with row operations (the pivots end
// as +-1).  False if M is not unimodular.
static bool unimodular_inverse(const IMat &M, IMat &Inv) {
    const int D = M.rows;
    IMat W = M;
    Inv = IMat::identity(D);
    for (int c = 0; c < D; ++c) {
        for (;;) {
            int piv = -1;
            int64_t best = 0;
            for (int i = c; i < D; ++i) {
                int64_t v = cabs(W(i, c));
                if (v != 0 && (piv < 0 || v < best)) { best = v; piv = i; }
            }
            if (piv < 0) return false;
            detail::swap_rows(W, c, piv); detail::swap_rows(Inv, c, piv);
            bool clean = true;
            for (int i = c + 1; i < D; ++i) {
                if (W(i, c) == 0) continue;
                int64_t f = W(i, c) / W(c, c);
                detail::sub_row(W, i, c, f); detail::sub_row(Inv, i, c, f);
                if (W(i, c) != 0) clean = false;
            }
            if (clean) break;
        }
        if (W(c, c) < 0)
            for (int j = 0; j < D; ++j) { W(c, j) = cneg(W(c, j)); Inv(c, j) = cneg(Inv(c, j)); }
        if (W(c, c) != 1) return false;
    }
    for (int c = D - 1; c >= 0; --c)   // back substitution: clear the entries above each pivot
        for (int i = 0; i < c; ++i) {
            int64_t f = W(i, c);
            if (f == 0) continue;
            detail::sub_row(W, i, c, f); detail::sub_row(Inv, i, c, f);
        }
    return true;
}

// Omega', Fourier-Motzkin rows and the folded device form (masks, transformed index, ranges).
// Extra conditions  cons[e][0..D) . x + cons[e][D] >= 0  (n_cons of them) are further rows of the constraint system.
static int derive_lattice(const IMat &A, const int64_t *lo, const int64_t *hi, const int64_t *extent,
                          ArgPlan &ap, int n_cons = 0, const int64_t (*cons_in)[TAD_MAX_EXT + 1] = nullptr) {
    const int D = A.cols, N = A.rows, E = n_cons;
    bool nonzero = false;
    for (int64_t v : A.a) nonzero |= v != 0;
    if (!nonzero) return TAD_EINVAL;  // the Smith algorithm is defined for non-zero matrices only

    ap.smith = smith_normal_form(A);
    const int R = ap.smith.R, kappa = D - R;
    if (kappa > TAD_MAX_KERNEL) return TAD_EUNSUPPORTED;
    ap.diag.resize(R);
    for (int r = 0; r < R; ++r) ap.diag[r] = ap.smith.S(r, r);
    ap.UR = IMat(R, N);
    ap.C = IMat(N - R, N);
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < N; ++j) {
            if (i < R) ap.UR(i, j) = ap.smith.U(i, j);
            else ap.C(i - R, j) = ap.smith.U(i, j);
        }
    ap.VR = IMat(D, R);
    ap.K = IMat(D, kappa);
    for (int i = 0; i < D; ++i)
        for (int j = 0; j < D; ++j) {
            if (j < R) ap.VR(i, j) = ap.smith.V(i, j);
            else ap.K(i, j - R) = ap.smith.V(i, j);
        }

    // Omega': [K ; -K] z >= b(beta),  b = [lo - I beta ; I beta - hi]  (Sec. 5.1, zero-based box); an extra
    // condition c . x + c0 >= 0 with x = I beta + K z adds the row (c K) z >= -c0 - c . (I beta)
    IMat cons(2 * D + E, kappa), B = IMat::identity(2 * D + E);
    for (int d = 0; d < D; ++d)
        for (int m = 0; m < kappa; ++m) {
            cons(d, m) = ap.K(d, m);
            cons(D + d, m) = cneg(ap.K(d, m));
        }
    for (int e = 0; e < E; ++e)
        for (int m = 0; m < kappa; ++m) {
            int64_t v = 0;
            for (int d = 0; d < D; ++d) v = cadd(v, cmul(cons_in[e][d], ap.K(d, m)));
            cons(2 * D + e, m) = v;
        }
    ap.fm = fourier_motzkin(cons, 2 * D + E, B);
    if (!ap.fm.bounded) return TAD_EINVAL;  // a kernel direction that is bounded from one side only

    // ---- fold into the device form -------------------------------------------------------------
    GatherPlan &g = ap.dev;
    std::memset(&g, 0, sizeof g);
    g.rank = N;
    for (int r = 0; r < N; ++r) g.shape[r] = fit32(extent[r]);
    g.R = R; g.kappa = kappa; g.nC = N - R;
    for (int r = 0; r < R; ++r) {
        g.diag[r] = fit32(ap.diag[r]);
        for (int d = 0; d < N; ++d) g.U[r][d] = fit32(ap.UR(r, d));
    }
    for (int c = 0; c < N - R; ++c)
        for (int d = 0; d < N; ++d) g.C[c][d] = fit32(ap.C(c, d));

    // A gradient with a cokernel or a divisibility mask is zero except at beta = U^{-1} [alpha y ; 0] for integer
    // y (Sec. 4.1: the masks say exactly that U beta has this form).  Where these elements are few, the
    // plan-driven kernels run over the box of y instead of over all beta and never visit a masked element.
    bool masked = N - R > 0;
    for (int r = 0; r < R; ++r) masked = masked || ap.diag[r] != 1;
    IMat Uinv;
    if (masked && unimodular_inverse(ap.smith.U, Uinv)) {
        long double box = 1, count = 1;
        for (int d = 0; d < N; ++d) count *= (long double)extent[d];
        for (int r = 0; r < R; ++r) {
            int64_t mn = 0, mx = 0;
            for (int d = 0; d < N; ++d) {
                const int64_t v = cmul(ap.UR(r, d), csub(extent[d], 1));
                if (v < 0) mn = cadd(mn, v); else mx = cadd(mx, v);
            }
            const int64_t y_lo = ceil_div(mn, ap.diag[r]), y_hi = floor_div(mx, ap.diag[r]);
            g.y_lo[r] = fit32(y_lo);
            g.y_n[r] = fit32(csub(y_hi, y_lo) + 1);
            box *= (long double)g.y_n[r];
            for (int d = 0; d < N; ++d) g.B[d][r] = fit32(cmul(Uinv(d, r), ap.diag[r]));
        }
        if (box * 4 <= count && box < 2147483647.0L) {
            g.live = 1;
            g.live_count = (int32_t)box;
        }
    }

    // Magnitude bounds of y and z over all beta, to prove that int32 arithmetic on the device cannot
    // overflow.  |y_r| <= |U beta|_r.  [y z] = V^{-1} [alpha k] with V unimodular, so |z_m| is bounded by
    // row R+m of V^{-1} applied to the box extents.
    int64_t ymax[kMaxRank] = {0}, zmax = 0;
    for (int r = 0; r < R; ++r) {
        int64_t s = 0;
        for (int d = 0; d < N; ++d) s = cadd(s, cmul(cabs(ap.UR(r, d)), extent[d]));
        ymax[r] = s;
        fit32(s);
    }
    for (int c = 0; c < N - R; ++c) {
        int64_t s = 0;
        for (int d = 0; d < N; ++d) s = cadd(s, cmul(cabs(ap.C(c, d)), extent[d]));
        fit32(s);
    }
    {
        IMat Inv;
        if (!unimodular_inverse(ap.smith.V, Inv)) return TAD_EINVAL;
        for (int m = 0; m < kappa; ++m) {
            int64_t s = 0;
            for (int d = 0; d < D; ++d)
                s = cadd(s, cmul(cabs(Inv(R + m, d)), std::max(cabs(lo[d]), cabs(hi[d]))));
            zmax = std::max(zmax, s);
        }
        fit32(zmax);
        ap.Vinv = Inv;
    }

    auto fold = [&](int64_t scale, const std::vector<int64_t> &cb, const std::vector<int64_t> *cz) {
        GRow row;
        std::memset(&row, 0, sizeof row);
        row.scale = fit32(scale);
        int64_t k0 = 0;
        for (int d = 0; d < D; ++d)
            k0 = cadd(k0, csub(cmul(cb[d], lo[d]), cmul(cb[D + d], hi[d])));
        for (int e = 0; e < E; ++e) k0 = csub(k0, cmul(cb[2 * D + e], cons_in[e][D]));
        row.k0 = fit32(k0);
        int64_t mag = cabs(k0);
        for (int r = 0; r < R; ++r) {
            int64_t s = 0;
            for (int d = 0; d < D; ++d) s = cadd(s, cmul(csub(cb[D + d], cb[d]), ap.VR(d, r)));
            for (int e = 0; e < E; ++e) {
                int64_t cv = 0;
                for (int d = 0; d < D; ++d) cv = cadd(cv, cmul(cons_in[e][d], ap.VR(d, r)));
                s = csub(s, cmul(cb[2 * D + e], cv));
            }
            row.ky[r] = fit32(s);
            mag = cadd(mag, cmul(cabs(s), ymax[r]));
        }
        if (cz)
            for (int m = 0; m < kappa; ++m) {
                row.kz[m] = fit32((*cz)[m]);
                mag = cadd(mag, cmul(cabs((*cz)[m]), zmax));
            }
        fit32(mag);
        return row;
    };

    int nrows = 0;
    for (int k = 0; k < kappa; ++k) {
        const auto &lo = ap.fm.lower[k];
        const auto &hi = ap.fm.upper[k];
        if (nrows + (int)lo.size() + (int)hi.size() > kMaxRows) return TAD_EUNSUPPORTED;
        g.lo_begin[k] = (uint8_t)nrows;
        for (const FMRow &r : lo) g.rows[nrows++] = fold(r.scale, r.coef_b, &r.coef_z);
        g.lo_end[k] = (uint8_t)nrows;
        g.hi_begin[k] = (uint8_t)nrows;
        for (const FMRow &r : hi) g.rows[nrows++] = fold(r.scale, r.coef_b, &r.coef_z);
        g.hi_end[k] = (uint8_t)nrows;
    }
    // only the original variable-free constraints need an explicit test; derived rows of F are implied
    // by the loop ranges being empty
    g.nF = 0;
    for (size_t f = 0; f < ap.fm.feasibility.size(); ++f) {
        if (!ap.fm.feasibility_original[f]) continue;
        if (g.nF == kMaxFeas) return TAD_EUNSUPPORTED;
        g.feas[g.nF++] = fold(1, ap.fm.feasibility[f], nullptr);
    }
    ap.derived = true;
    return TAD_OK;
}

// Range of the linear form a . x over the rational relaxation of { lo <= x <= hi, extra conditions } by
// Fourier-Motzkin projection (variables x_0..x_{D-1} eliminated first, the form's value t last).  Returns false
// if the set is empty (then every range is fine).  The integer range is inside [tmin, tmax].
bool linear_form_range(const int64_t *a, int D, const int64_t *lo, const int64_t *hi, int E,
                              const int64_t (*cons_in)[TAD_MAX_EXT + 1], int64_t &tmin, int64_t &tmax) {
    const int M = D + 1, rows = 2 * D + E + 2;
    IMat A(rows, M), B(rows, 1);
    for (int d = 0; d < D; ++d) {
        A(d, d) = 1; B(d, 0) = lo[d];                 //  x_d >= lo_d
        A(D + d, d) = -1; B(D + d, 0) = cneg(hi[d]);  // -x_d >= -hi_d
    }
    for (int e = 0; e < E; ++e) {
        for (int d = 0; d < D; ++d) A(2 * D + e, d) = cons_in[e][d];
        B(2 * D + e, 0) = cneg(cons_in[e][D]);
    }
    for (int d = 0; d < D; ++d) {
        A(2 * D + E, d) = cneg(a[d]);                 //  t - a . x >= 0
        A(2 * D + E + 1, d) = a[d];                   // -t + a . x >= 0
    }
    A(2 * D + E, D) = 1;
    A(2 * D + E + 1, D) = -1;
    const FMResult fm = fourier_motzkin(A, 1, B);
    for (const auto &f : fm.feasibility)
        if (f[0] > 0) return false;                   // F b <= 0 violated: no point at all
    bool have_lo = false, have_hi = false;
    for (const FMRow &r : fm.lower[D]) {
        const int64_t v = ceil_div(r.coef_b[0], r.scale);
        tmin = have_lo ? std::max(tmin, v) : v;
        have_lo = true;
    }
    for (const FMRow &r : fm.upper[D]) {
        const int64_t v = floor_div(r.coef_b[0], r.scale);
        tmax = have_hi ? std::min(tmax, v) : v;
        have_hi = true;
    }
    if (!have_lo || !have_hi) throw overflow_error();   // cannot happen for a bounded box
    return tmin <= tmax;
}

// Index plan of one argument of an expression (one pass of the loop body of the derivation algorithm).
static int derive_arg(const tad_plan &pl, int p, ArgPlan &ap) {
    const tad_arg &arg = pl.args[p];
    const int D = pl.n_ext, N = arg.rank;
    IMat A(N, D);
    for (int r = 0; r < N; ++r)
        for (int d = 0; d < D; ++d) A(r, d) = arg.index[r][d];
    int rc = derive_lattice(A, pl.lo, pl.hi, arg.shape, ap, pl.expr.n_constraints, pl.expr.constraint);
    if (rc) return rc;
    GatherPlan &g = ap.dev;
    const int R = ap.smith.R, kappa = D - R;

    // memory offsets, linear in the extended index, re-expressed in (y, z)
    for (int s = 0; s < kSlots; ++s) {
        int64_t lin[TAD_MAX_EXT] = {0};
        if (s < (int)pl.args.size()) {
            const tad_arg &q = pl.args[s];
            int64_t stride = 1;
            for (int r = q.rank - 1; r >= 0; --r) {
                for (int d = 0; d < D; ++d) lin[d] = cadd(lin[d], cmul(stride, q.index[r][d]));
                stride = cmul(stride, q.shape[r]);
            }
        } else if (s == kSlotF) {
            int64_t stride = 1;
            for (int d = pl.expr.n_f - 1; d >= 0; --d) {
                lin[d] = stride;
                stride = cmul(stride, pl.expr.f_shape[d]);
            }
        } else {
            continue;
        }
        for (int r = 0; r < R; ++r) {
            int64_t v = 0;
            for (int d = 0; d < D; ++d) v = cadd(v, cmul(lin[d], ap.VR(d, r)));
            g.offY[s][r] = v;
        }
        for (int m = 0; m < kappa; ++m) {
            int64_t v = 0;
            for (int d = 0; d < D; ++d) v = cadd(v, cmul(lin[d], ap.K(d, m)));
            g.offZ[s][m] = v;
        }
    }
    ap.derived = true;
    return TAD_OK;
}

// Plan of an operand the outer function reads, over the function indices alone: its index ignores the
// summation indices and the extra conditions do not apply (the outer function is evaluated once per function
// index whatever the sum contains).  Offsets are filled in for f and for the operands the outer function reads.
static int derive_arg_outer(const tad_plan &pl, int p, ArgPlan &ap) {
    const tad_arg &arg = pl.args[p];
    const int D = pl.expr.n_f, N = arg.rank;
    IMat A(N, D);
    for (int r = 0; r < N; ++r)
        for (int d = 0; d < D; ++d) A(r, d) = arg.index[r][d];
    int rc = derive_lattice(A, pl.lo, pl.hi, arg.shape, ap);
    if (rc) return rc;
    GatherPlan &g = ap.dev;
    const int R = ap.smith.R, kappa = D - R;
    for (int s = 0; s < kSlots; ++s) {
        int64_t lin[TAD_MAX_EXT] = {0};
        if (s < (int)pl.args.size()) {
            if (!((pl.prog.outer_mask >> s) & 1u)) continue;
            const tad_arg &q = pl.args[s];
            int64_t stride = 1;
            for (int r = q.rank - 1; r >= 0; --r) {
                for (int d = 0; d < D; ++d) lin[d] = cadd(lin[d], cmul(stride, q.index[r][d]));
                stride = cmul(stride, q.shape[r]);
            }
        } else if (s == kSlotF) {
            int64_t stride = 1;
            for (int d = D - 1; d >= 0; --d) {
                lin[d] = stride;
                stride = cmul(stride, pl.expr.f_shape[d]);
            }
        } else {
            continue;
        }
        for (int r = 0; r < R; ++r) {
            int64_t v = 0;
            for (int d = 0; d < D; ++d) v = cadd(v, cmul(lin[d], ap.VR(d, r)));
            g.offY[s][r] = v;
        }
        for (int m = 0; m < kappa; ++m) {
            int64_t v = 0;
            for (int d = 0; d < D; ++d) v = cadd(v, cmul(lin[d], ap.K(d, m)));
            g.offZ[s][m] = v;
        }
    }
    return TAD_OK;
}

static void list_terms(tad_plan &pl);

int derive_plan(const tad_expr *expr, const tad_arg *args, int n_args, tad_dtype dt, uint32_t flags,
                tad_plan **out) {
    if (!expr || !args || !out) return TAD_EINVAL;
    *out = nullptr;
    if (dt != TAD_F32 && dt != TAD_F64) return TAD_EINVAL;
    // a program body that spells out one of the built-in bodies is planned as that body: the expression then reaches
    // the kernels written for it (and their hand-written partial derivatives, the same functions)
    tad_expr as_builtin;
    if (expr->body == TAD_BODY_PROGRAM && !(flags & TAD_PLAN_KEEP_PROGRAM) && expr->n_operands >= 1 &&
        expr->n_operands <= TAD_MAX_ARGS && expr->n_sum >= 0) {
        const int id = matching_builtin_body(*expr);
        if (id >= 0) {
            as_builtin = *expr;
            as_builtin.body = id;
            expr = &as_builtin;
        }
    }
    const int want = expr->body == TAD_BODY_PROGRAM ? expr->n_operands : body_arg_count(expr->body);
    if (want < 0) return TAD_EUNSUPPORTED;
    if (expr->body == TAD_BODY_PROGRAM && (want < 1 || want > TAD_MAX_ARGS)) return TAD_EINVAL;
    if (n_args != want) return TAD_EINVAL;
    if (expr->n_f < 1 || expr->n_sum < 0 || expr->n_f + expr->n_sum > TAD_MAX_EXT) return TAD_EINVAL;
    if (expr->n_constraints < 0 || expr->n_constraints > TAD_MAX_CONSTRAINTS) return TAD_EINVAL;
    if (expr->n_sum > 0 &&
        (expr->body == TAD_BODY_SQ || expr->body == TAD_BODY_CUBE || expr->body == TAD_BODY_SIN))
        return TAD_EUNSUPPORTED;

    tad_plan *pl = new (std::nothrow) tad_plan();
    if (!pl) return TAD_ENOMEM;
    struct Guard {
        tad_plan *p;
        ~Guard() { delete p; }
    } guard{pl};

    pl->expr = *expr;
    if (expr->body == TAD_BODY_PROGRAM) {
        // the outer program may read the operands whose index ignores the summation indices
        uint32_t constant_in_k = 0, wanted = 0;
        for (int p = 0; p < n_args; ++p) {
            const int root = (args[p].alias > 0 && args[p].alias <= p) ? args[p].alias - 1 : p;
            if (args[root].needs_grad) wanted |= 1u << p;
            bool zero = args[p].rank >= 1 && args[p].rank <= TAD_MAX_RANK;
            for (int r = 0; zero && r < args[p].rank; ++r)
                for (int s = 0; s < expr->n_sum; ++s) zero = zero && args[p].index[r][expr->n_f + s] == 0;
            if (zero) constant_in_k |= 1u << p;
        }
        const int rc = build_program_body(*expr, pl->prog, constant_in_k, wanted);
        if (rc) return rc;
    }
    pl->args.assign(args, args + n_args);
    pl->dtype = dt;
    pl->flags = flags;
    pl->n_ext = expr->n_f + expr->n_sum;
    const int D = pl->n_ext;
    pl->f_count = 1;
    for (int d = 0; d < expr->n_f; ++d) {
        if (expr->f_shape[d] < 1) return TAD_ESHAPE;
        pl->lo[d] = 0;
        pl->hi[d] = expr->f_shape[d] - 1;
        pl->f_count = cmul(pl->f_count, expr->f_shape[d]);
    }
    for (int s = 0; s < expr->n_sum; ++s) {
        if (expr->sum_lo[s] > expr->sum_hi[s]) return TAD_ESHAPE;
        pl->lo[expr->n_f + s] = expr->sum_lo[s];
        pl->hi[expr->n_f + s] = expr->sum_hi[s];
    }
    if (pl->f_count >= ((int64_t)1 << 31)) return TAD_EOVERFLOW;
    pl->terms_total = (double)pl->f_count;
    for (int s = 0; s < expr->n_sum; ++s) pl->terms_total *= (double)(expr->sum_hi[s] - expr->sum_lo[s] + 1);

    pl->arg_count.resize(n_args);
    pl->root.resize(n_args);
    for (int p = 0; p < n_args; ++p) {
        const tad_arg &a = args[p];
        if (a.rank < 1 || a.rank > TAD_MAX_RANK) return TAD_EINVAL;
        if (a.alias < 0 || a.alias > p) return TAD_EINVAL;
        pl->root[p] = a.alias ? a.alias - 1 : p;
        if (a.alias) {
            const tad_arg &r = args[a.alias - 1];
            if (r.alias) return TAD_EINVAL;
            if (r.rank != a.rank) return TAD_ESHAPE;
            for (int d = 0; d < a.rank; ++d)
                if (r.shape[d] != a.shape[d]) return TAD_ESHAPE;
            pl->args[p].needs_grad = r.needs_grad;
            pl->has_alias = true;
        }
        int64_t cnt = 1;
        for (int r = 0; r < a.rank; ++r) {
            if (a.shape[r] < 1) return TAD_ESHAPE;
            cnt = cmul(cnt, a.shape[r]);
            // extremes of the linear map over the box (and the extra conditions): every reachable index must
            // lie in the shape
            int64_t mn = 0, mx = 0;
            if (expr->n_constraints == 0) {
                for (int d = 0; d < D; ++d) {
                    int64_t u = cmul(a.index[r][d], pl->lo[d]), v = cmul(a.index[r][d], pl->hi[d]);
                    mn = cadd(mn, std::min(u, v));
                    mx = cadd(mx, std::max(u, v));
                }
            } else if (!linear_form_range(a.index[r], D, pl->lo, pl->hi, expr->n_constraints, expr->constraint, mn,
                                          mx)) {
                mn = mx = 0;   // no extended index satisfies the conditions: nothing is read
            }
            if (mn < 0 || mx >= a.shape[r]) return TAD_ESHAPE;
        }
        if (cnt >= ((int64_t)1 << 31)) return TAD_EOVERFLOW;
        pl->arg_count[p] = cnt;
    }

    // forward plan: linear element offsets of every argument in the extended index
    ForwardPlan &fw = pl->fwd;
    std::memset(&fw, 0, sizeof fw);
    fw.n_f = expr->n_f;
    fw.n_sum = expr->n_sum;
    for (int d = 0; d < expr->n_f; ++d) fw.f_shape[d] = fit32(expr->f_shape[d]);
    for (int s = 0; s < expr->n_sum; ++s) {
        fw.sum_lo[s] = fit32(expr->sum_lo[s]);
        fw.sum_n[s] = fit32(csub(expr->sum_hi[s], expr->sum_lo[s]) + 1);
    }
    for (int p = 0; p < n_args; ++p) {
        int64_t stride = 1;
        for (int r = args[p].rank - 1; r >= 0; --r) {
            for (int d = 0; d < D; ++d)
                fw.off[p][d] = cadd(fw.off[p][d], cmul(stride, args[p].index[r][d]));
            stride = cmul(stride, args[p].shape[r]);
        }
    }

    for (int p = 0; p < n_args; ++p) {
        for (int s = 0; s < expr->n_sum; ++s)
            fw.base0[p] = cadd(fw.base0[p], cmul(fw.off[p][expr->n_f + s], expr->sum_lo[s]));
        fw.last_stride[p] = expr->n_sum > 0 ? fw.off[p][expr->n_f + expr->n_sum - 1] : 0;
    }

    fw.n_cons = expr->n_constraints;
    for (int e = 0; e < expr->n_constraints; ++e) {
        int64_t mag = cabs(expr->constraint[e][D]);
        for (int d = 0; d <= D; ++d) fw.cons[e][d] = fit32(expr->constraint[e][d]);
        for (int d = 0; d < D; ++d)
            mag = cadd(mag, cmul(cabs(expr->constraint[e][d]), std::max(cabs(pl->lo[d]), cabs(pl->hi[d]))));
        fit32(mag);   // the kernels evaluate the condition in int32
    }

    pl->ap.resize(n_args);
    pl->ap_outer.resize(n_args);
    for (int p = 0; p < n_args; ++p) {
        if (!pl->args[p].needs_grad) continue;
        int rc = derive_arg(*pl, p, pl->ap[p]);
        if (rc) return rc;
        if (expr->body == TAD_BODY_PROGRAM && ((pl->prog.outer_mask >> p) & 1u)) {
            rc = derive_arg_outer(*pl, p, pl->ap_outer[p]);
            if (rc) return rc;
        }
    }
    select_families(*pl);
    list_terms(*pl);
    guard.p = nullptr;
    *out = pl;
    return TAD_OK;
}

template <class Fn>
static void visit_beta(int n_ext, const ArgPlan &ap, const int32_t *beta, Fn &&fn);

// Visit every extended index of the element with transformed index y through the ranges and the maps V_R y + K z.
template <class Fn>
static void visit_y(int n_ext, const ArgPlan &ap, const int32_t *y, Fn &&fn) {
    const GatherPlan &g = ap.dev;
    int32_t z[kMaxKernel] = {0}, hi[kMaxKernel] = {0};
    auto emit = [&]() {
        int64_t ext[TAD_MAX_EXT];
        for (int d = 0; d < n_ext; ++d) {
            int64_t v = 0;
            for (int r = 0; r < g.R; ++r) v += ap.VR(d, r) * (int64_t)y[r];
            for (int m = 0; m < g.kappa; ++m) v += ap.K(d, m) * (int64_t)z[m];
            ext[d] = v;
        }
        fn(ext);
    };
    if (g.kappa == 0) { emit(); return; }
    int lvl = g.kappa - 1;
    gather_bounds(g, lvl, y, z, z[lvl], hi[lvl]);
    for (;;) {
        if (z[lvl] > hi[lvl]) {
            if (++lvl == g.kappa) break;
            ++z[lvl];
            continue;
        }
        if (lvl == 0) { emit(); ++z[0]; }
        else { --lvl; gather_bounds(g, lvl, y, z, z[lvl], hi[lvl]); }
    }
}

// The same for beta, through the masks.
template <class Fn>
static void visit_beta(int n_ext, const ArgPlan &ap, const int32_t *beta, Fn &&fn) {
    int32_t y[kMaxRank] = {0};
    if (!gather_prepare(ap.dev, beta, y)) return;
    visit_y(n_ext, ap, y, fn);
}

// Small expressions on the plan-driven kernels: write out, per gradient element, the extended indices that the
// plan's masks and ranges enumerate (exactly what the device would walk), as offsets into the tensors.
static void list_terms(tad_plan &pl) {
    if ((pl.flags & TAD_PLAN_NO_TERM_LISTS) || pl.expr.body == TAD_BODY_PROGRAM || pl.has_alias) return;
    const int n_args = (int)pl.args.size();
    if (n_args > kListSlots - 1) return;
    long long elements = 0;
    int n_grad = 0;
    for (int q = 0; q < n_args; ++q) {
        if (!pl.ap[q].derived) continue;
        if (pl.ap[q].family != TAD_FAMILY_GENERIC) return;
        elements += pl.arg_count[q];
        ++n_grad;
    }
    if (n_grad == 0 || elements > kListElements || pl.terms_total * n_grad > (double)kListTerms) return;
    TermList L{};
    int e = 0, t = 0;
    bool fits = true;
    for (int q = 0; q < n_args && fits; ++q) {
        if (!pl.ap[q].derived) continue;
        const int g = L.n_grad++;
        L.first_element[g] = e;
        L.operand[g] = q;
        const tad_arg &a = pl.args[q];
        for (int64_t lin = 0; lin < pl.arg_count[q] && fits; ++lin, ++e) {
            int32_t beta[kMaxRank] = {0};
            int64_t r = lin;
            for (int d = a.rank - 1; d >= 0; --d) { beta[d] = (int32_t)(r % a.shape[d]); r /= a.shape[d]; }
            L.first_term[e] = (uint16_t)t;
            visit_beta(pl.n_ext, pl.ap[q], beta, [&](const int64_t *ext) {
                if (t >= kListTerms) { fits = false; return; }
                for (int s = 0; s < n_args; ++s) {
                    int64_t o = 0;
                    for (int d = 0; d < pl.n_ext; ++d) o += pl.fwd.off[s][d] * ext[d];
                    if (o < 0 || o > INT32_MAX) fits = false;
                    L.off[t][s] = (int32_t)o;
                }
                int64_t of = 0;
                for (int d = 0; d < pl.expr.n_f; ++d) of = of * pl.expr.f_shape[d] + ext[d];
                if (of < 0 || of > INT32_MAX) fits = false;
                L.off[t][kListSlots - 1] = (int32_t)of;
                ++t;
            });
        }
    }
    if (!fits) return;
    for (int g = L.n_grad; g <= kMaxArgs; ++g) L.first_element[g] = e;
    for (int x = e; x <= kListElements; ++x) L.first_term[x] = (uint16_t)t;
    pl.term_list.push_back(L);
}

// plan of occurrence `occ` of the tensor given as operand `arg` (0: the operand itself, k: its k-th alias)
const ArgPlan *get_arg(const tad_plan *plan, int arg, int occ, int *slot_out) {
    if (!plan || arg < 0 || arg >= (int)plan->ap.size() || occ < 0 || plan->root[arg] != arg) return nullptr;
    int slot = -1;
    for (int p = arg, k = 0; p < (int)plan->ap.size(); ++p)
        if (plan->root[p] == arg && k++ == occ) { slot = p; break; }
    if (slot < 0) return nullptr;
    if (slot_out) *slot_out = slot;
    return plan->ap[slot].derived ? &plan->ap[slot] : nullptr;
}

}  // namespace tad

using namespace tad;

extern "C" {

int tad_plan_derive(const tad_expr *expr, const tad_arg *args, int n_args, tad_dtype dt, uint32_t flags,
                    tad_plan **out) {
    try {
        return derive_plan(expr, args, n_args, dt, flags, out);
    } catch (const overflow_error &) {
        return TAD_EOVERFLOW;
    } catch (const std::bad_alloc &) {
        return TAD_ENOMEM;
    } catch (...) {
        return TAD_EINVAL;
    }
}

void tad_plan_free(tad_plan *plan) { delete plan; }

size_t tad_plan_workspace_bytes(const tad_plan *plan) { return plan ? plan->ws_bytes : 0; }

int tad_plan_forward_family(const tad_plan *plan) { return plan ? plan->fwd_family : TAD_EINVAL; }

int tad_plan_query(const tad_plan *plan, int arg, int occ, tad_plan_info *out) {
    const ArgPlan *ap = get_arg(plan, arg, occ);
    if (!ap || !out) return TAD_EINVAL;
    std::memset(out, 0, sizeof *out);
    const int N = plan->args[arg].rank, D = plan->n_ext, R = ap->smith.R;
    out->rank = R;
    out->kernel_dim = D - R;
    out->n_cokernel = N - R;
    for (int r = 0; r < R; ++r) out->smith[r] = ap->diag[r];
    for (int i = 0; i < N; ++i)
        for (int j = 0; j < N; ++j) out->U[i][j] = ap->smith.U(i, j);
    for (int i = 0; i < D; ++i)
        for (int j = 0; j < D; ++j) out->V[i][j] = ap->smith.V(i, j);
    for (int i = 0; i < D; ++i)
        for (int m = 0; m < D - R; ++m) out->K[i][m] = ap->K(i, m);
    for (int c = 0; c < N - R; ++c)
        for (int j = 0; j < N; ++j) out->C[c][j] = ap->C(c, j);
    for (int k = 0; k < D - R; ++k) {
        out->n_lower[k] = (int32_t)ap->fm.lower[k].size();
        out->n_upper[k] = (int32_t)ap->fm.upper[k].size();
    }
    out->n_feasibility = (int32_t)ap->fm.feasibility.size();
    out->family = ap->family;
    int slot = -1;
    get_arg(plan, arg, occ, &slot);
    out->in_outer = plan->expr.body == TAD_BODY_PROGRAM && ((plan->prog.outer_mask >> slot) & 1u) ? 1 : 0;
    {
        const GatherShape shape = gather_shape(ap->dev, gather_launch_count(ap->dev, plan->arg_count[(size_t)plan->root[slot]]),
                                               plan->terms_total);
        out->gather_layout = shape.layout;
        out->gather_splits = shape.splits;
        out->gather_elements = gather_launch_count(ap->dev, plan->arg_count[(size_t)plan->root[slot]]);
    }
    out->listed = plan->term_list.empty() ? 0 : 1;
    return TAD_OK;
}

int tad_plan_bound_row(const tad_plan *plan, int arg, int kind, int level, int row, int64_t *scale,
                       int64_t *coef_b, int64_t *coef_z, int64_t *coef_c) {
    const ArgPlan *ap = get_arg(plan, arg, 0);
    if (!ap || !scale || !coef_b || !coef_z) return TAD_EINVAL;
    const int D = plan->n_ext, kappa = D - ap->smith.R;
    std::fill(coef_b, coef_b + 2 * TAD_MAX_EXT, 0);
    std::fill(coef_z, coef_z + TAD_MAX_KERNEL, 0);
    if (coef_c) std::fill(coef_c, coef_c + TAD_MAX_CONSTRAINTS, 0);
    auto put_b = [&](const std::vector<int64_t> &cb) {
        for (int d = 0; d < D; ++d) {
            coef_b[d] = cb[d];
            coef_b[TAD_MAX_EXT + d] = cb[D + d];
        }
        if (coef_c)
            for (int e = 0; e < plan->expr.n_constraints; ++e) coef_c[e] = cb[2 * D + e];
    };
    if (kind == TAD_ROWS_FEASIBILITY) {
        if (row < 0 || row >= (int)ap->fm.feasibility.size()) return TAD_EINVAL;
        *scale = 1;
        put_b(ap->fm.feasibility[row]);
        return TAD_OK;
    }
    if (level < 0 || level >= kappa) return TAD_EINVAL;
    const std::vector<FMRow> &rows = kind == TAD_ROWS_LOWER ? ap->fm.lower[level] : ap->fm.upper[level];
    if (kind != TAD_ROWS_LOWER && kind != TAD_ROWS_UPPER) return TAD_EINVAL;
    if (row < 0 || row >= (int)rows.size()) return TAD_EINVAL;
    *scale = rows[row].scale;
    put_b(rows[row].coef_b);
    for (int m = 0; m < kappa; ++m) coef_z[m] = rows[row].coef_z[m];
    return TAD_OK;
}

int tad_plan_enumerate(const tad_plan *plan, int arg, int occ, const int64_t *beta, int64_t *alpha_out,
                       size_t cap, size_t *n) {
    const ArgPlan *ap = get_arg(plan, arg, occ);
    if (!ap || !beta || !n) return TAD_EINVAL;
    const int N = plan->args[arg].rank, D = plan->n_ext;
    int32_t b32[kMaxRank];
    *n = 0;
    for (int r = 0; r < N; ++r) {
        if (beta[r] < 0 || beta[r] >= plan->args[arg].shape[r]) return TAD_ESHAPE;
        b32[r] = (int32_t)beta[r];
    }
    std::vector<std::vector<int64_t>> pts;
    try {
        visit_beta(D, *ap, b32, [&](const int64_t *ext) { pts.emplace_back(ext, ext + D); });
        std::sort(pts.begin(), pts.end());
    } catch (const std::bad_alloc &) {
        return TAD_ENOMEM;
    }
    *n = pts.size();
    if (alpha_out)
        for (size_t i = 0; i < pts.size() && i < cap; ++i)
            std::copy(pts[i].begin(), pts[i].end(), alpha_out + i * D);
    return TAD_OK;
}

int tad_plan_count_all(const tad_plan *plan, int arg, int64_t *counts) {
    const ArgPlan *ap = get_arg(plan, arg, 0);
    if (!ap || !counts) return TAD_EINVAL;
    // the way the plan-driven kernels run over the gradient: element numbers of the launch (all of the tensor, or
    // the unmasked elements only), each mapped to its position and its transformed index
    const int64_t total = plan->arg_count[arg];
    for (int64_t lin = 0; lin < total; ++lin) counts[lin] = 0;
    const int64_t numbers = gather_launch_count(ap->dev, total);
    for (int64_t idx = 0; idx < numbers; ++idx) {
        int32_t y[kMaxRank] = {0};
        int lin = -1;
        if (!gather_element_index(ap->dev, (int)idx, &lin, y)) continue;
        int64_t c = 0;
        visit_y(plan->n_ext, *ap, y, [&](const int64_t *) { ++c; });
        counts[lin] += c;
    }
    return TAD_OK;
}

int tad_plan_program_eval(const tad_plan *plan, int which, const double *values, double sum, double *out) {
    if (!plan || !out || plan->expr.body != TAD_BODY_PROGRAM) return TAD_EINVAL;
    const ProgramBody &pb = plan->prog;
    if (which <= -2) {
        if (which < -3 - pb.n_operands) return TAD_EINVAL;
        if (which <= -4 && !plan->ap[-4 - which].derived) return TAD_EINVAL;   // derivative not planned
        const DevProg &prog = which == -2 ? pb.outer : which == -3 ? pb.douter : pb.douter_arg[-4 - which];
        if (!values && reads_operands(prog)) return TAD_EINVAL;
        *out = eval_host(prog, values, sum);
        return TAD_OK;
    }
    if (!values || which >= pb.n_operands) return TAD_EINVAL;
    if (which >= 0 && !plan->ap[which].derived) return TAD_EINVAL;             // derivative not planned
    *out = eval_host(which < 0 ? pb.inner : pb.dinner[which], values, 0.0);
    return TAD_OK;
}

int tad_plan_program_registers(const tad_plan *plan, int which, int *registers_out) {
    if (!plan || !registers_out || plan->expr.body != TAD_BODY_PROGRAM) return TAD_EINVAL;
    const ProgramBody &pb = plan->prog;
    if (which < -3 - pb.n_operands || which >= pb.n_operands) return TAD_EINVAL;
    const int operand = which >= 0 ? which : which <= -4 ? -4 - which : -1;
    if (operand >= 0 && !plan->ap[operand].derived) return TAD_EINVAL;   // derivative not planned
    const DevProg &prog = which == -1 ? pb.inner : which >= 0 ? pb.dinner[which] : which == -2 ? pb.outer
                          : which == -3 ? pb.douter : pb.douter_arg[operand];
    *registers_out = prog.result < 0 ? 0 : prog.n_regs;   // < 0: no register form
    return TAD_OK;
}

int tad_extended_gcd(int64_t a, int64_t b, int64_t *g, int64_t *x, int64_t *y) {
    if (!g || !x || !y) return TAD_EINVAL;
    try {
        Bezout bz = egcd(a, b);
        *g = bz.g; *x = bz.x; *y = bz.y;
        return TAD_OK;
    } catch (const overflow_error &) {
        return TAD_EOVERFLOW;
    }
}

int tad_smith_normal_form(const int64_t *A, int n, int m, int64_t *S, int64_t *U, int64_t *V, int *rank) {
    if (!A || !S || !U || !V || !rank || n < 1 || m < 1 || n > 16 || m > 16) return TAD_EINVAL;
    try {
        IMat a(n, m);
        bool nonzero = false;
        for (int i = 0; i < n * m; ++i) { a.a[i] = A[i]; nonzero |= A[i] != 0; }
        if (!nonzero) return TAD_EINVAL;
        Smith w = smith_normal_form(a);
        std::copy(w.S.a.begin(), w.S.a.end(), S);
        std::copy(w.U.a.begin(), w.U.a.end(), U);
        std::copy(w.V.a.begin(), w.V.a.end(), V);
        *rank = w.R;
        return TAD_OK;
    } catch (const overflow_error &) {
        return TAD_EOVERFLOW;
    } catch (...) {
        return TAD_ENOMEM;
    }
}

int tad_lattice_enumerate(const int64_t *A, int n, int m, const int64_t *lo, const int64_t *hi,
                          const int64_t *beta, int64_t *x_out, size_t cap, size_t *count) {
    if (!A || !lo || !hi || !beta || !count || n < 1 || n > TAD_MAX_RANK || m < 1 || m > TAD_MAX_EXT)
        return TAD_EINVAL;
    *count = 0;
    try {
        IMat a(n, m);
        for (int i = 0; i < n * m; ++i) a.a[i] = A[i];
        int64_t extent[TAD_MAX_RANK];
        int32_t b32[kMaxRank] = {0};
        for (int r = 0; r < n; ++r) {
            int64_t s = 1;
            for (int d = 0; d < m; ++d) {
                if (lo[d] > hi[d]) return TAD_ESHAPE;
                s = cadd(s, cmul(cabs(a(r, d)), std::max(cabs(lo[d]), cabs(hi[d]))));
            }
            extent[r] = s;
            if (cabs(beta[r]) >= s) return TAD_OK;   // beyond every reachable value: no solution
            b32[r] = (int32_t)beta[r];
        }
        ArgPlan ap;
        int rc = derive_lattice(a, lo, hi, extent, ap);
        if (rc) return rc;
        std::vector<std::vector<int64_t>> pts;
        visit_beta(m, ap, b32, [&](const int64_t *x) { pts.emplace_back(x, x + m); });
        std::sort(pts.begin(), pts.end());
        *count = pts.size();
        if (x_out)
            for (size_t i = 0; i < pts.size() && i < cap; ++i)
                std::copy(pts[i].begin(), pts[i].end(), x_out + i * m);
        return TAD_OK;
    } catch (const overflow_error &) {
        return TAD_EOVERFLOW;
    } catch (...) {
        return TAD_ENOMEM;
    }
}

const char *tad_strerror(int status) {
    switch (status) {
    case TAD_OK: return "ok";
    case TAD_EINVAL: return "invalid argument";
    case TAD_ESHAPE: return "index leaves a tensor's shape, or empty range";
    case TAD_EINFEASIBLE: return "constraint system has no solution";
    case TAD_EOVERFLOW: return "integer overflow";
    case TAD_EUNSUPPORTED: return "unsupported body or index pattern";
    case TAD_EDEVICE: return "device error";
    case TAD_ENOMEM: return "out of memory or workspace too small";
    default: return "unknown status";
    }
}

}  // extern "C"
