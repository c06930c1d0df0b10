// Gradients written out as expressions of their own (Sec. 5.3: the derived expressions have the form of the input
// again, so the derivation can be applied to its own output): seed expressions for the factor all gradients share,
// derived expressions for the sum over the kernel coordinates.  Host only.
#include <algorithm>
#include <cstring>

#include "derived.hpp"
#include "launch_geom.h"
#include "plan.hpp"

namespace tad {

// Inner and outer function of any body as postfix programs.
static bool body_programs(const tad_plan &pl, std::vector<tad_op> &inner, std::vector<tad_op> &outer, int &n_operands) {
    if (pl.expr.body == TAD_BODY_PROGRAM) {
        inner.assign(pl.expr.inner, pl.expr.inner + pl.expr.n_inner);
        outer.assign(pl.expr.outer, pl.expr.outer + pl.expr.n_outer);
        n_operands = pl.expr.n_operands;
        return true;
    }
    n_operands = body_arg_count(pl.expr.body);
    return builtin_body_programs(pl.expr.body, inner, outer);
}

// How the scalar part of the gradients is organised.
struct ScalarForm {
    Graph g;                 // inner function, and (fused) the outer function applied to it
    int inner = -1;          // node of the inner function (fused: of outer(inner))
    std::vector<int> dinner; // per operand: d inner / d operand (fused: d outer(inner) / d operand), -1 = zero
    bool fused = false;      // no summation and no condition: f = outer(inner(x)) is one function of the operands
    bool identity = false;   // the outer function is the sum itself
    Graph go;                // outer function (not fused)
    std::vector<int> douter; // per operand, then the sum: d outer / d input, -1 = zero
    uint32_t outer_mask = 0; // operands the outer function reads (not fused)
    int n_ops = 0;
};

static int scalar_form(const tad_plan &pl, ScalarForm &f) {
    std::vector<tad_op> inner, outer;
    if (!body_programs(pl, inner, outer, f.n_ops)) return TAD_EUNSUPPORTED;
    const uint32_t all = (1u << f.n_ops) - 1u;
    f.inner = parse_postfix(inner.data(), (int)inner.size(), false, f.n_ops, f.g);
    if (f.inner < 0) return f.inner;
    f.fused = pl.expr.n_sum == 0 && pl.expr.n_constraints == 0;
    if (f.fused) {
        // the sum has exactly one term: replace the sum node of the outer function by the inner function
        Graph tmp;
        const int ro = parse_postfix(outer.data(), (int)outer.size(), true, f.n_ops, tmp, all);
        if (ro < 0) return ro;
        std::vector<int> at(tmp.nodes.size());
        for (size_t i = 0; i < tmp.nodes.size(); ++i) {
            Node nd = tmp.nodes[i];
            if (nd.op == P_SUM) { at[i] = f.inner; continue; }
            if (nd.a >= 0) nd.a = at[nd.a];
            if (nd.b >= 0) nd.b = at[nd.b];
            f.g.nodes.push_back(nd);
            at[i] = (int)f.g.nodes.size() - 1;
        }
        f.inner = at[ro];
        f.identity = true;
    } else {
        uint32_t allowed = 0;
        for (int p = 0; p < f.n_ops; ++p) {
            bool zero = true;
            for (int r = 0; r < pl.args[p].rank; ++r)
                for (int q = 0; q < pl.expr.n_sum; ++q) zero = zero && pl.args[p].index[r][pl.expr.n_f + q] == 0;
            if (zero) allowed |= 1u << p;
        }
        const int ro = parse_postfix(outer.data(), (int)outer.size(), true, f.n_ops, f.go, allowed);
        if (ro < 0) return ro;
        for (const tad_op &o : outer)
            if (o.op == TAD_OP_ARG) f.outer_mask |= 1u << o.iarg;
        const std::vector<int> alias = simplify(f.go);
        f.identity = f.go.nodes[alias[ro]].op == P_SUM;
        reverse_accumulate(f.go, ro, f.n_ops, f.douter);
    }
    reverse_accumulate(f.g, f.inner, f.n_ops, f.dinner);
    return TAD_OK;
}

// Postfix form of `node` of graph g (a constant zero if node < 0); is_one: the expression is the constant 1.
static bool postfix_of(const Graph &g, int node, std::vector<tad_op> &out, bool &is_one, size_t cap) {
    is_one = false;
    if (node < 0) {
        tad_op zero{};
        zero.op = TAD_OP_CONST;
        out.push_back(zero);
        return true;
    }
    const std::vector<int> alias = simplify(g);
    const Node &top = g.nodes[alias[node]];
    is_one = top.op == P_CONST && top.c == 1.0;
    return is_one || emit_postfix(g, alias, node, out, cap);
}

// Index part of a derived expression.  The solutions of A x = beta are x = V_R y + K z with y_r = (U beta)_r / alpha_r
// for every beta with C beta = 0 and every division exact.  Rows with alpha_r = 1 give y_r = (U beta)_r directly;
// for a row with alpha_r > 1 the quotient becomes one more summation index t with the pair of conditions
// (U beta)_r - alpha_r t >= 0 and <= 0, a sum of at most one term (the divisibility mask written as a sum).  So
// x = M [beta z t]: the new function indices are beta, the new summation indices z and t with their extremes
// over the old box as constant limits, and what the old box and conditions still demand become the new
// conditions.  (D, lo, hi, E, cons): the old index space.
static int derived_index(const ArgPlan &ap, int D, const tad_arg &arg, const int64_t *lo, const int64_t *hi, int E,
                         const int64_t (*cons)[TAD_MAX_EXT + 1], tad_expr *eo, IMat &M) {
    const int N = arg.rank, R = ap.smith.R, kappa = D - R;
    int col_of_row[TAD_MAX_RANK], n_quot = 0;   // column of t for a row with a divisor above one, else -1
    for (int r = 0; r < R; ++r) col_of_row[r] = ap.diag[r] != 1 ? N + kappa + n_quot++ : -1;
    const int D2 = N + kappa + n_quot;
    if (D2 > TAD_MAX_EXT) return TAD_EUNSUPPORTED;
    M = IMat(D, D2);
    for (int d = 0; d < D; ++d) {
        for (int j = 0; j < N; ++j) {
            int64_t v = 0;
            for (int r = 0; r < R; ++r)
                if (col_of_row[r] < 0) v = cadd(v, cmul(ap.VR(d, r), ap.UR(r, j)));
            M(d, j) = v;
        }
        for (int m = 0; m < kappa; ++m) M(d, N + m) = ap.K(d, m);
        for (int r = 0; r < R; ++r)
            if (col_of_row[r] >= 0) M(d, col_of_row[r]) = ap.VR(d, r);
    }
    eo->n_f = N;
    for (int j = 0; j < N; ++j) eo->f_shape[j] = arg.shape[j];
    eo->n_sum = kappa + n_quot;
    int64_t blo[TAD_MAX_EXT], bhi[TAD_MAX_EXT];   // box of the new extended index [beta z t]
    for (int j = 0; j < N; ++j) { blo[j] = 0; bhi[j] = arg.shape[j] - 1; }
    auto limits_of = [&](int vinv_row, int col) {
        // the coordinate is a row of V^{-1} applied to the old extended index: its extremes over the old box
        int64_t row[TAD_MAX_EXT], mn = 0, mx = 0;
        for (int d = 0; d < D; ++d) row[d] = ap.Vinv(vinv_row, d);
        if (!linear_form_range(row, D, lo, hi, E, cons, mn, mx)) mn = mx = 0;
        eo->sum_lo[col - N] = blo[col] = mn;
        eo->sum_hi[col - N] = bhi[col] = mx;
    };
    for (int m = 0; m < kappa; ++m) limits_of(R + m, N + m);
    for (int r = 0; r < R; ++r)
        if (col_of_row[r] >= 0) limits_of(r, col_of_row[r]);
    // conditions c . [beta z] + c0 >= 0; one that holds on the whole new box, or is there already, is left out
    eo->n_constraints = 0;
    auto add_condition = [&](const int64_t *c, int64_t c0) {
        int64_t mn = c0;
        bool any = false;
        for (int j = 0; j < D2; ++j) {
            mn = cadd(mn, std::min(cmul(c[j], blo[j]), cmul(c[j], bhi[j])));
            any |= c[j] != 0;
        }
        if (mn >= 0 || !any) return true;
        for (int e = 0; e < eo->n_constraints; ++e) {
            bool same = eo->constraint[e][D2] == c0;
            for (int j = 0; j < D2; ++j) same = same && eo->constraint[e][j] == c[j];
            if (same) return true;
        }
        if (eo->n_constraints == TAD_MAX_CONSTRAINTS) return false;
        int64_t *dst = eo->constraint[eo->n_constraints++];
        for (int j = 0; j < D2; ++j) dst[j] = c[j];
        dst[D2] = c0;
        return true;
    };
    int64_t c[TAD_MAX_EXT];
    for (int d = 0; d < D; ++d) {
        for (int j = 0; j < D2; ++j) c[j] = M(d, j);
        if (!add_condition(c, cneg(lo[d]))) return TAD_EUNSUPPORTED;          //  x_d - lo_d >= 0
        for (int j = 0; j < D2; ++j) c[j] = cneg(M(d, j));
        if (!add_condition(c, hi[d])) return TAD_EUNSUPPORTED;                // -x_d + hi_d >= 0
    }
    for (int e = 0; e < E; ++e) {
        for (int j = 0; j < D2; ++j) {
            int64_t v = 0;
            for (int d = 0; d < D; ++d) v = cadd(v, cmul(cons[e][d], M(d, j)));
            c[j] = v;
        }
        if (!add_condition(c, cons[e][D])) return TAD_EUNSUPPORTED;
    }
    for (int r = 0; r < N - R; ++r)
        for (int sign = 1; sign >= -1; sign -= 2) {
            for (int j = 0; j < D2; ++j) c[j] = j < N ? cmul(sign, ap.C(r, j)) : 0;
            if (!add_condition(c, 0)) return TAD_EUNSUPPORTED;
        }
    for (int r = 0; r < R; ++r) {
        if (col_of_row[r] < 0) continue;
        for (int sign = 1; sign >= -1; sign -= 2) {   // (U beta)_r = alpha_r t
            for (int j = 0; j < D2; ++j) c[j] = j < N ? cmul(sign, ap.UR(r, j)) : 0;
            c[col_of_row[r]] = cmul(-sign, ap.diag[r]);
            if (!add_condition(c, 0)) return TAD_EUNSUPPORTED;
        }
    }
    return TAD_OK;
}

// operand of a derived expression: tensor `src` read at (rows of its index matrix) . M
static void mapped_operand(const tad_arg &src, int D, const IMat &M, tad_arg &dst) {
    dst.rank = src.rank;
    dst.needs_grad = 1;
    for (int r = 0; r < src.rank; ++r) {
        dst.shape[r] = src.shape[r];
        for (int j = 0; j < M.cols; ++j) {
            int64_t v = 0;
            for (int d = 0; d < D; ++d) v = cadd(v, cmul(src.index[r][d], M(d, j)));
            dst.index[r][j] = v;
        }
    }
}

// f (or df, or a seed tensor of f's shape) as an operand read at the function-index rows of M
static void mapped_f(const tad_plan &pl, const IMat &M, tad_arg &dst) {
    dst.rank = pl.expr.n_f;
    dst.needs_grad = 1;
    for (int r = 0; r < pl.expr.n_f; ++r) {
        dst.shape[r] = pl.expr.f_shape[r];
        for (int j = 0; j < M.cols; ++j) dst.index[r][j] = M(r, j);
    }
}

// The gradient of the occurrence in operand slot `slot` as an expression of its own (Sec. 5.3).
// part 0: the terms through the sum; part 1: the term of an operand the outer function reads.
static int derived_expr(const tad_plan &pl, int slot, int part, tad_expr *eo, tad_arg *ao, int *operand_out, int *n_out) {
    const int D = pl.n_ext, nf = pl.expr.n_f;
    if (nf > TAD_MAX_RANK) return TAD_EUNSUPPORTED;
    ScalarForm sf;
    int rc = scalar_form(pl, sf);
    if (rc) return rc;
    std::memset(eo, 0, sizeof *eo);
    std::memset(ao, 0, sizeof(tad_arg) * TAD_MAX_ARGS);
    eo->body = TAD_BODY_PROGRAM;
    eo->outer[0].op = TAD_OP_SUM;
    eo->n_outer = 1;
    IMat M;
    if (part == 1) {
        // sum over the function indices mapped onto beta of h = df * d outer / d x, h given as operand 0
        if (sf.fused || !((sf.outer_mask >> slot) & 1u) || !pl.ap_outer[slot].derived) return TAD_EINVAL;
        rc = derived_index(pl.ap_outer[slot], nf, pl.args[slot], pl.lo, pl.hi, 0, nullptr, eo, M);
        if (rc) return rc;
        eo->n_operands = 1;
        eo->inner[0].op = TAD_OP_ARG;
        eo->n_inner = 1;
        mapped_f(pl, M, ao[0]);
        if (operand_out) operand_out[0] = -3 - slot;
        *n_out = 1;
        return TAD_OK;
    }
    if (part != 0) return TAD_EINVAL;

    // ---- scalar part: operand 0 (df, or g = df * d outer / d sum) times d inner / d operand `slot` ------------
    std::vector<tad_op> dprog;
    bool is_one = false;
    if (!postfix_of(sf.g, sf.dinner[slot], dprog, is_one, TAD_MAX_PROGRAM - 2)) return TAD_EUNSUPPORTED;
    // operands the derivative depends on, in their original order; new index = 1 + position
    int new_index[TAD_MAX_ARGS], kept[TAD_MAX_ARGS], n_kept = 0;
    for (int q = 0; q < sf.n_ops; ++q) {
        new_index[q] = -1;
        for (const tad_op &o : dprog)
            if (o.op == TAD_OP_ARG && o.iarg == q) new_index[q] = 0;
        if (new_index[q] == 0) {
            if (1 + n_kept >= TAD_MAX_ARGS) return TAD_EUNSUPPORTED;
            kept[n_kept] = q;
            new_index[q] = 1 + n_kept++;
        }
    }
    eo->n_operands = 1 + n_kept;
    int n = 0;
    eo->inner[n].op = TAD_OP_ARG;
    eo->inner[n++].iarg = 0;
    if (!is_one) {
        for (tad_op o : dprog) {
            if (o.op == TAD_OP_ARG) o.iarg = new_index[o.iarg];
            eo->inner[n++] = o;
        }
        eo->inner[n++].op = TAD_OP_MUL;
    }
    eo->n_inner = n;

    // ---- index part and operands: df (or g) through the first n_f rows of M, every kept operand through A^q M ----
    rc = derived_index(pl.ap[slot], D, pl.args[slot], pl.lo, pl.hi, pl.expr.n_constraints, pl.expr.constraint, eo, M);
    if (rc) return rc;
    mapped_f(pl, M, ao[0]);
    if (operand_out) operand_out[0] = sf.identity ? -1 : -2;
    for (int t = 0; t < n_kept; ++t) {
        const int q = kept[t];
        mapped_operand(pl.args[q], D, M, ao[1 + t]);
        for (int u = 0; u < t; ++u)   // a later kept occurrence of the same tensor names the first kept one
            if (pl.root[kept[u]] == pl.root[q]) { ao[1 + t].alias = 1 + u + 1; break; }
        if (operand_out) operand_out[1 + t] = q;
    }
    *n_out = 1 + n_kept;
    return TAD_OK;
}

// The factor all gradients share, as an expression over the function indices of the original one:
// which = -1: g = df * d outer / d sum;  which = p: h = df * d outer / d operand p.  Operand 0 is df, operands
// 1.. are the original operands.
static int seed_expr(const tad_plan &pl, int which, tad_expr *eo, tad_arg *ao, int *n_out) {
    ScalarForm sf;
    int rc = scalar_form(pl, sf);
    if (rc) return rc;
    const int n_ops = sf.n_ops, D = pl.n_ext;
    if (which < -1 || which >= n_ops) return TAD_EINVAL;
    if (1 + n_ops > TAD_MAX_ARGS || pl.expr.n_f > TAD_MAX_RANK) return TAD_EUNSUPPORTED;
    std::vector<tad_op> inner, outer, dprog;
    int dummy = 0;
    body_programs(pl, inner, outer, dummy);
    bool is_one = false;
    if (sf.fused) {
        // one function of the operands: d outer / d sum is taken as 1 and nothing is read outside the sum
        if (which >= 0) return TAD_EINVAL;
        is_one = true;
    } else {
        if (which >= 0 && !((sf.outer_mask >> which) & 1u)) return TAD_EINVAL;
        if (!postfix_of(sf.go, sf.douter[which < 0 ? n_ops : which], dprog, is_one, TAD_MAX_PROGRAM - 2))
            return TAD_EUNSUPPORTED;
    }
    std::memset(eo, 0, sizeof *eo);
    std::memset(ao, 0, sizeof(tad_arg) * TAD_MAX_ARGS);
    eo->body = TAD_BODY_PROGRAM;
    eo->n_f = pl.expr.n_f;
    eo->n_sum = pl.expr.n_sum;
    for (int d = 0; d < pl.expr.n_f; ++d) eo->f_shape[d] = pl.expr.f_shape[d];
    for (int q = 0; q < pl.expr.n_sum; ++q) { eo->sum_lo[q] = pl.expr.sum_lo[q]; eo->sum_hi[q] = pl.expr.sum_hi[q]; }
    eo->n_constraints = pl.expr.n_constraints;
    for (int e = 0; e < pl.expr.n_constraints; ++e)
        for (int d = 0; d <= D; ++d) eo->constraint[e][d] = pl.expr.constraint[e][d];
    eo->n_operands = 1 + n_ops;
    if ((int)inner.size() > TAD_MAX_PROGRAM) return TAD_EUNSUPPORTED;
    for (size_t i = 0; i < inner.size(); ++i) {
        eo->inner[i] = inner[i];
        if (inner[i].op == TAD_OP_ARG) eo->inner[i].iarg = inner[i].iarg + 1;
    }
    eo->n_inner = (int)inner.size();
    int n = 0;
    eo->outer[n].op = TAD_OP_ARG;
    eo->outer[n++].iarg = 0;
    if (!is_one) {
        for (tad_op o : dprog) {
            if (o.op == TAD_OP_ARG) o.iarg += 1;
            eo->outer[n++] = o;
        }
        eo->outer[n++].op = TAD_OP_MUL;
    }
    eo->n_outer = n;
    ao[0].rank = pl.expr.n_f;
    ao[0].needs_grad = 1;
    for (int r = 0; r < pl.expr.n_f; ++r) {
        ao[0].shape[r] = pl.expr.f_shape[r];
        ao[0].index[r][r] = 1;
    }
    for (int q = 0; q < n_ops; ++q) {
        ao[1 + q] = pl.args[q];
        ao[1 + q].needs_grad = 1;
        if (ao[1 + q].alias) ao[1 + q].alias += 1;
    }
    *n_out = 1 + n_ops;
    return TAD_OK;
}

// Plan of one expression of the graph: forward evaluation only, so no gradient plans are derived for it.
static int node_plan(tad_expr &e, tad_arg *a, int n, tad_dtype dt, tad_derived::Node &node) {
    for (int q = 0; q < n; ++q) a[q].needs_grad = 0;
    return tad_plan_derive(&e, a, n, dt, 0, &node.plan);
}

static int build_graph(const tad_plan &pl, int arg, tad_derived &d) {
    ScalarForm sf;
    int rc = scalar_form(pl, sf);
    if (rc) return rc;
    d.dtype = pl.dtype;
    d.arg = arg;
    d.n_original = (int)pl.args.size();
    d.root = pl.root;
    d.count = pl.arg_count[(size_t)arg];
    const size_t es = pl.dtype == TAD_F64 ? 8 : 4;
    size_t ws = 0, sub = 0;
    auto seed_for = [&](int which) -> int {        // which: kSrcSeedG or -3 - p
        for (const auto &s : d.seeds)
            if (s.seed == which) return TAD_OK;
        tad_expr e;
        tad_arg a[TAD_MAX_ARGS];
        int n = 0;
        int r = seed_expr(pl, which == kSrcSeedG ? -1 : -3 - which, &e, a, &n);
        if (r) return r;
        tad_derived::Node node;
        r = node_plan(e, a, n, pl.dtype, node);
        if (r) return r;
        node.seed = which;
        node.src.push_back(kSrcDf);
        for (int q = 0; q < n - 1; ++q) node.src.push_back(q);
        node.out_offset = ws;
        ws += align256((size_t)pl.f_count * es);
        sub = std::max(sub, node.plan->ws_bytes);
        d.seeds.push_back(std::move(node));
        node.plan = nullptr;
        return TAD_OK;
    };
    for (int occ = 0;; ++occ) {
        int slot = -1;
        const ArgPlan *ap = get_arg(&pl, arg, occ, &slot);
        if (!ap) {
            if (occ == 0) return TAD_EINVAL;
            if (slot < 0) break;                 // no further occurrence
            return TAD_EINVAL;                   // an occurrence without a plan
        }
        const bool second = !sf.fused && ((sf.outer_mask >> slot) & 1u);
        for (int part = 0; part < (second ? 2 : 1); ++part) {
            tad_expr e;
            tad_arg a[TAD_MAX_ARGS];
            int src[TAD_MAX_ARGS] = {0}, n = 0;
            rc = derived_expr(pl, slot, part, &e, a, src, &n);
            if (rc) return rc;
            if (src[0] != kSrcDf) {
                rc = seed_for(src[0]);
                if (rc) return rc;
            }
            tad_derived::Node node;
            rc = node_plan(e, a, n, pl.dtype, node);
            if (rc) return rc;
            node.src.assign(src, src + n);
            sub = std::max(sub, node.plan->ws_bytes);
            d.parts.push_back(std::move(node));
            node.plan = nullptr;
        }
    }
    d.tmp_offset = ws;
    if (d.parts.size() > 1) ws += align256((size_t)d.count * es);
    d.sub_offset = ws;
    d.ws_bytes = ws + sub;
    return TAD_OK;
}

}  // namespace tad

using namespace tad;

extern "C" {

int tad_derived_create(const tad_plan *plan, int arg, tad_derived **out) {
    if (!plan || !out || arg < 0 || arg >= (int)plan->args.size() || plan->root[(size_t)arg] != arg) return TAD_EINVAL;
    *out = nullptr;
    tad_derived *d = nullptr;
    try {
        d = new tad_derived();
        const int rc = build_graph(*plan, arg, *d);
        if (rc) { delete d; return rc; }
        *out = d;
        return TAD_OK;
    } catch (const overflow_error &) {
        delete d;
        return TAD_EOVERFLOW;
    } catch (const std::bad_alloc &) {
        delete d;
        return TAD_ENOMEM;
    } catch (...) {
        delete d;
        return TAD_EINVAL;
    }
}

void tad_derived_free(tad_derived *d) { delete d; }

size_t tad_derived_workspace_bytes(const tad_derived *d) { return d ? d->ws_bytes : 0; }

int tad_derived_count(const tad_derived *d, int *n_seeds, int *n_parts) {
    if (!d) return TAD_EINVAL;
    if (n_seeds) *n_seeds = (int)d->seeds.size();
    if (n_parts) *n_parts = (int)d->parts.size();
    return TAD_OK;
}

int tad_plan_derived_expr(const tad_plan *plan, int arg, int occ, int part, tad_expr *expr_out, tad_arg *args_out,
                          int *operand_out, int *n_args_out) {
    int slot = -1;
    const ArgPlan *ap = get_arg(plan, arg, occ, &slot);
    if (!ap || !expr_out || !args_out || !n_args_out) return TAD_EINVAL;
    try {
        // the outputs are written only on success
        tad_expr e;
        tad_arg a[TAD_MAX_ARGS];
        int src[TAD_MAX_ARGS] = {0}, n = 0;
        const int rc = derived_expr(*plan, slot, part, &e, a, src, &n);
        if (rc) return rc;
        *expr_out = e;
        std::copy(a, a + TAD_MAX_ARGS, args_out);
        if (operand_out) std::copy(src, src + TAD_MAX_ARGS, operand_out);
        *n_args_out = n;
        return TAD_OK;
    } catch (const overflow_error &) {
        return TAD_EOVERFLOW;
    } catch (const std::bad_alloc &) {
        return TAD_ENOMEM;
    } catch (...) {
        return TAD_EINVAL;
    }
}

int tad_plan_seed_expr(const tad_plan *plan, int which, tad_expr *expr_out, tad_arg *args_out, int *n_args_out) {
    if (!plan || !expr_out || !args_out || !n_args_out) return TAD_EINVAL;
    try {
        tad_expr e;
        tad_arg a[TAD_MAX_ARGS];
        int n = 0;
        const int rc = seed_expr(*plan, which, &e, a, &n);
        if (rc) return rc;
        *expr_out = e;
        std::copy(a, a + TAD_MAX_ARGS, args_out);
        *n_args_out = n;
        return TAD_OK;
    } catch (const overflow_error &) {
        return TAD_EOVERFLOW;
    } catch (const std::bad_alloc &) {
        return TAD_ENOMEM;
    } catch (...) {
        return TAD_EINVAL;
    }
}

}  // extern "C"
